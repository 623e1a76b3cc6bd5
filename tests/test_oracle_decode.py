"""Pins for the decode oracle (CPU only).

Each test ties the oracle to something other than itself: textbook attention from a library
routine, closed forms, special cases in which Eq. 1 / Eq. 2 of the paper reduce to full attention,
invariants of a softmax, or a brute-force selection written differently.
"""
import math

import numpy as np
import pytest
import torch

from oracle import mp_oracle as O


def _bf16(a):
    return torch.tensor(np.asarray(a), dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def _rand_unit(rng, n=96, d=16, G=3, Cf=8, Cc=3, levels=2, spread=1.0):
    centers = rng.normal(size=(Cf, d)) * 1.5
    fot = rng.integers(0, Cf, size=n).astype(np.int32)
    K = _bf16(centers[fot] + spread * 0.3 * rng.normal(size=(n, d)))
    V = _bf16(rng.normal(size=(n, d)))
    q = _bf16(rng.normal(size=(G, d)))
    cof = rng.integers(0, Cc, size=Cf).astype(np.int32) if levels == 2 else None
    cl = O.clustering_from_assignment(K, V, fot, Cf, cof, Cc if levels == 2 else 0)
    return q, K, V, cl


def _exact_tables(cl):
    """Replace the bf16-rounded centroid tables by exact fp64 member means."""
    K, V, fot = cl["K"], cl["V"], cl["fine_of_token"]
    out = dict(cl)
    Cf = cl["N_f"].shape[0]
    Sk, N = O.member_sums(K, fot, Cf)
    Sv, _ = O.member_sums(V, fot, Cf)
    nz = N > 0
    out["Kc_f"] = np.zeros_like(Sk)
    out["Vc_f"] = np.zeros_like(Sv)
    out["Kc_f"][nz] = Sk[nz] / N[nz, None]
    out["Vc_f"][nz] = Sv[nz] / N[nz, None]
    if cl["levels"] == 2:
        cof = cl["coarse_of_fine"]
        Cc = cl["N_c"].shape[0]
        Sk, N = O.member_sums(K, cof[fot], Cc)
        Sv, _ = O.member_sums(V, cof[fot], Cc)
        nz = N > 0
        out["Kc_c"] = np.zeros_like(Sk)
        out["Vc_c"] = np.zeros_like(Sv)
        out["Kc_c"][nz] = Sk[nz] / N[nz, None]
        out["Vc_c"][nz] = Sv[nz] / N[nz, None]
    return out


def test_full_attention_matches_library_sdpa():
    rng = np.random.default_rng(0)
    G, n, d = 5, 300, 32
    q, K, V = rng.normal(size=(G, d)), rng.normal(size=(n, d)), rng.normal(size=(n, d))
    scale = 0.37
    out, lse = O.full_attention(q, K, V, scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None], torch.tensor(K)[None], torch.tensor(V)[None], scale=scale)[0].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    ref_lse = torch.logsumexp(torch.tensor(q) @ torch.tensor(K).T * scale, dim=-1).numpy()
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-13)


def test_hand_worked_example():
    # d = 1, one query head, q = 1, scale = 1.  Cluster 0 = keys {0, 2} (centroid 1, values 3 and 5,
    # value centroid 4), cluster 1 = key {10} (value 7).  Budget 1 keeps only cluster 1 (the higher
    # score); cluster 0 enters as 2 e^{1} with value 4 (Eq. 2).
    K = np.array([[0.0], [2.0], [10.0]])
    V = np.array([[3.0], [5.0], [7.0]])
    cl = O.clustering_from_assignment(K, V, [0, 0, 1], 2)
    res = O.decode_unit(np.array([[1.0]]), cl, key_budget=1, scale=1.0)
    assert list(res["selected"]) == [0, 1]
    expect = (math.exp(10) * 7 + 2 * math.exp(1) * 4) / (math.exp(10) + 2 * math.exp(1))
    assert res["out"][0, 0] == pytest.approx(expect, rel=1e-14)
    assert res["lse"][0] == pytest.approx(math.log(math.exp(10) + 2 * math.exp(1)), rel=1e-14)
    # Eq. 1 for cluster 1: e^{10} / (2 e^{1} + 1 e^{10}); the rank key is its log
    assert res["r_f"][1] == pytest.approx(math.log(math.exp(10) / (2 * math.exp(1) + math.exp(10))), rel=1e-13)
    assert res["r_f"][0] == pytest.approx(math.log(math.exp(1) / (2 * math.exp(1) + math.exp(10))), rel=1e-13)
    # budget 2 cannot hold cluster 1 (1 key) + cluster 0 (2 keys): still only cluster 1; budget 3 holds both
    assert list(O.decode_unit(np.array([[1.0]]), cl, 2, scale=1.0)["selected"]) == [0, 1]
    res3 = O.decode_unit(np.array([[1.0]]), cl, 3, scale=1.0)
    assert list(res3["selected"]) == [1, 1]
    full = (3 + math.exp(2) * 5 + math.exp(10) * 7) / (1 + math.exp(2) + math.exp(10))
    assert res3["out"][0, 0] == pytest.approx(full, rel=1e-14)


@pytest.mark.parametrize("levels", [1, 2])
def test_budget_covering_everything_is_full_attention(levels):
    rng = np.random.default_rng(1)
    q, K, V, cl = _rand_unit(rng, levels=levels)
    scale = 1 / math.sqrt(q.shape[1])
    res = O.decode_unit(q, cl, key_budget=K.shape[0], coarse_budget=K.shape[0])
    ref, ref_lse = O.full_attention(q, K, V, scale)
    np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(res["lse"], ref_lse, rtol=1e-13)
    assert res["selected"].all() and res["n_sel_keys"] == K.shape[0]


@pytest.mark.parametrize("budget", [0, 1, 7, 40])
@pytest.mark.parametrize("levels", [1, 2])
def test_singleton_clusters_are_exact_for_any_budget(budget, levels):
    rng = np.random.default_rng(2)
    n, d, G = 40, 8, 2
    K, V, q = _bf16(rng.normal(size=(n, d))), _bf16(rng.normal(size=(n, d))), _bf16(rng.normal(size=(G, d)))
    fot = rng.permutation(n).astype(np.int32)
    cof = (np.arange(n) // 8).astype(np.int32) if levels == 2 else None
    cl = O.clustering_from_assignment(K, V, fot, n, cof, 5 if levels == 2 else 0)
    # coarse clusters are not singletons: give the coarse level enough budget that every fine
    # cluster is a candidate, so only singleton terms enter Eq. 2
    res = O.decode_unit(q, cl, key_budget=budget, coarse_budget=n)
    ref, ref_lse = O.full_attention(q, K, V, 1 / math.sqrt(d))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(res["lse"], ref_lse, rtol=1e-13)
    assert res["n_sel_keys"] == budget


@pytest.mark.parametrize("budget,cbudget", [(0, 0), (10, 30), (25, 1000)])
def test_identical_keys_per_cluster_are_exact(budget, cbudget):
    # If all keys of a cluster coincide, N e^{q.Kc} Vc = sum_t e^{q.k_t} v_t: Eq. 2 is exact, at both levels
    # as long as a coarse cluster's children share one key too.
    rng = np.random.default_rng(3)
    Cf, Cc, d, G = 6, 6, 8, 3
    centers = _bf16(rng.normal(size=(Cf, d)))
    fot = np.repeat(np.arange(Cf), [3, 5, 2, 7, 4, 6]).astype(np.int32)
    rng.shuffle(fot)
    K = centers[fot]
    V = _bf16(rng.normal(size=(len(fot), d)))
    q = _bf16(rng.normal(size=(G, d)))
    cl = _exact_tables(O.clustering_from_assignment(K, V, fot, Cf, np.arange(Cf, dtype=np.int32), Cc))
    res = O.decode_unit(q, cl, key_budget=budget, coarse_budget=cbudget)
    ref, ref_lse = O.full_attention(q, K, V, 1 / math.sqrt(d))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(res["lse"], ref_lse, rtol=1e-13)


@pytest.mark.parametrize("levels", [1, 2])
def test_softmax_normalisation_constant_values(levels):
    rng = np.random.default_rng(4)
    q, K, V, cl = _rand_unit(rng, levels=levels)
    const = _bf16(rng.normal(size=K.shape[1]))
    Vc = np.tile(const, (K.shape[0], 1))
    cof = cl.get("coarse_of_fine")
    cl2 = O.clustering_from_assignment(K, Vc, cl["fine_of_token"], cl["N_f"].shape[0], cof,
                                       0 if cof is None else cl["N_c"].shape[0])
    tail_k, tail_v = _bf16(rng.normal(size=(5, K.shape[1]))), np.tile(const, (5, 1))
    for budget in (0, 20, 50):
        res = O.decode_unit(q, cl2, key_budget=budget, coarse_budget=40, Kx=tail_k, Vx=tail_v)
        np.testing.assert_allclose(res["out"], np.tile(const, (q.shape[0], 1)), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("levels", [1, 2])
def test_jensen_denominator_bound_and_convex_hull(levels):
    # N e^{q.mean(k)} <= sum e^{q.k}: with exact means the oracle's denominator never exceeds the true one.
    rng = np.random.default_rng(5)
    for trial in range(5):
        q, K, V, cl = _rand_unit(rng, levels=levels)
        cl = _exact_tables(cl)
        _, ref_lse = O.full_attention(q, K, V, 1 / math.sqrt(q.shape[1]))
        res = O.decode_unit(q, cl, key_budget=20 * trial, coarse_budget=30)
        assert (res["lse"] <= ref_lse + 1e-12).all()
        lo = np.minimum(V.min(0), cl["Vc_f"].min(0))
        hi = np.maximum(V.max(0), cl["Vc_f"].max(0))
        assert ((res["out"] >= lo - 1e-12) & (res["out"] <= hi + 1e-12)).all()


def test_error_vanishes_as_clusters_tighten():
    errs = []
    for spread in (1.0, 0.3, 0.1, 0.0):
        rng = np.random.default_rng(6)
        q, K, V, cl = _rand_unit(rng, n=200, levels=2, spread=spread)
        cl = _exact_tables(cl)
        # equal values inside a cluster isolate the key-side approximation of Eq. 2
        V2 = cl["Vc_f"][cl["fine_of_token"]]
        cl = _exact_tables(O.clustering_from_assignment(K, V2, cl["fine_of_token"], 8, cl["coarse_of_fine"], 3))
        # coarse clusters gather unrelated fine clusters: keep every fine cluster a candidate
        res = O.decode_unit(q, cl, key_budget=30, coarse_budget=10**6)
        ref, _ = O.full_attention(q, K, V2, 1 / math.sqrt(q.shape[1]))
        errs.append(np.abs(res["out"] - ref).max())
    assert errs[0] > errs[1] > errs[2] > errs[3]
    assert errs[3] < 1e-12


def test_two_level_with_unbounded_coarse_budget_equals_one_level():
    rng = np.random.default_rng(7)
    q, K, V, cl2 = _rand_unit(rng, levels=2)
    cl1 = dict(cl2, levels=1)
    for budget in (0, 15, 33, 96):
        a = O.decode_unit(q, cl2, key_budget=budget, coarse_budget=K.shape[0])
        b = O.decode_unit(q, cl1, key_budget=budget)
        np.testing.assert_array_equal(a["selected"], b["selected"])
        np.testing.assert_allclose(a["out"], b["out"], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(a["r_f"], b["r_f"], rtol=1e-13)


def _brute_select(scores, N, budget):
    """Selection written without a sort: cluster i is kept iff the token count of all clusters
    ranked at or before it (higher score, or equal score and lower index) fits in the budget."""
    C = len(scores)
    keep = np.zeros(C, dtype=np.uint8)
    for i in range(C):
        if N[i] == 0:
            continue
        tot = 0
        for j in range(C):
            if N[j] == 0:
                continue
            before = scores[j] > scores[i] or (scores[j] == scores[i] and j <= i)
            if before:
                tot += N[j]
        keep[i] = tot <= budget
    return keep


def test_selection_against_brute_force_linear_domain():
    # Rank by Eq. 1 averaged over the heads of the group, computed directly (no logs), and select by brute force.
    rng = np.random.default_rng(8)
    for trial in range(20):
        q, K, V, cl = _rand_unit(rng, n=80, Cf=10, levels=1)
        scale = 1 / math.sqrt(q.shape[1])
        N = cl["N_f"].astype(np.float64)
        e = np.exp(scale * q @ cl["Kc_f"].T)                       # [G, Cf]
        S = e / (e * N[None, :]).sum(1, keepdims=True)             # Eq. 1 per head
        score = np.where(N > 0, S.mean(0), -1.0)                   # averaged over the group
        budget = int(rng.integers(0, 90))
        res = O.decode_unit(q, cl, key_budget=budget)
        np.testing.assert_array_equal(res["selected"], _brute_select(score, cl["N_f"], budget))
        got = np.exp(res["r_f"][cl["N_f"] > 0])
        np.testing.assert_allclose(got, score[cl["N_f"] > 0], rtol=1e-12)


def test_selection_two_level_against_brute_force():
    rng = np.random.default_rng(9)
    for trial in range(20):
        q, K, V, cl = _rand_unit(rng, n=120, Cf=12, Cc=4, levels=2)
        scale = 1 / math.sqrt(q.shape[1])
        Nc, Nf, cof = cl["N_c"], cl["N_f"], cl["coarse_of_fine"]
        ec = np.exp(scale * q @ cl["Kc_c"].T)
        Sc = (ec / (ec * Nc[None, :]).sum(1, keepdims=True)).mean(0)
        cb, kb = int(rng.integers(0, 130)), int(rng.integers(0, 130))
        prom = _brute_select(np.where(Nc > 0, Sc, -1.0), Nc, cb)
        cand = (Nf > 0) & (prom[cof] == 1)
        ef = np.exp(scale * q @ cl["Kc_f"].T)
        den = (ef * Nf[None, :] * cand[None, :]).sum(1) + (ec * Nc[None, :] * (1 - prom)[None, :]).sum(1)
        Sf = (ef / den[:, None]).mean(0)
        sel = _brute_select(np.where(cand, Sf, -1.0), np.where(cand, Nf, 0), kb)
        res = O.decode_unit(q, cl, key_budget=kb, coarse_budget=cb)
        np.testing.assert_array_equal(res["promising"], prom)
        np.testing.assert_array_equal(res["selected"], sel)
        np.testing.assert_allclose(np.exp(res["r_c"][Nc > 0]), Sc[Nc > 0], rtol=1e-12)
        np.testing.assert_allclose(np.exp(res["r_f"][cand]), Sf[cand], rtol=1e-12)
        assert np.isnan(res["r_f"][~cand]).all()


def test_tie_break_lowest_index_first():
    # two identical clusters (same centroid, same size): the lower id wins the last budget slot
    K = np.array([[1.0, 0.0]] * 2 + [[1.0, 0.0]] * 2 + [[-1.0, 0.0]] * 2)
    V = np.arange(12, dtype=np.float64).reshape(6, 2)
    cl = O.clustering_from_assignment(K, V, [0, 0, 1, 1, 2, 2], 3)
    res = O.decode_unit(np.array([[1.0, 0.0]]), cl, key_budget=2, scale=1.0)
    assert list(res["selected"]) == [1, 0, 0]
    assert res["r_f"][0] == res["r_f"][1]


def test_relabelling_clusters_keeps_the_selected_tokens():
    rng = np.random.default_rng(10)
    q, K, V, cl = _rand_unit(rng, levels=1)
    Cf = cl["N_f"].shape[0]
    perm = rng.permutation(Cf).astype(np.int32)
    cl_p = O.clustering_from_assignment(K, V, perm[cl["fine_of_token"]], Cf)
    for budget in (10, 30, 60):
        a = O.decode_unit(q, cl, key_budget=budget)
        b = O.decode_unit(q, cl_p, key_budget=budget)
        tok_a = a["selected"][cl["fine_of_token"]]
        tok_b = b["selected"][cl_p["fine_of_token"]]
        np.testing.assert_array_equal(tok_a, tok_b)
        np.testing.assert_allclose(a["out"], b["out"], rtol=1e-12, atol=1e-14)


def test_larger_budget_selects_superset():
    rng = np.random.default_rng(11)
    q, K, V, cl = _rand_unit(rng, n=200, Cf=16, Cc=4, levels=2)
    prev = np.zeros(16, dtype=np.uint8)
    for budget in range(0, 200, 13):
        sel = O.decode_unit(q, cl, key_budget=budget, coarse_budget=200)["selected"]
        assert ((sel | prev) == sel).all()
        assert (cl["N_f"] * sel).sum() <= budget
        prev = sel


def test_no_multipole_terms_is_attention_over_retrieved_keys():
    rng = np.random.default_rng(12)
    q, K, V, cl = _rand_unit(rng, levels=2)
    Kx, Vx = _bf16(rng.normal(size=(4, K.shape[1]))), _bf16(rng.normal(size=(4, K.shape[1])))
    res = O.decode_unit(q, cl, key_budget=40, coarse_budget=70, Kx=Kx, Vx=Vx, mp_terms=False)
    keep = res["selected"][cl["fine_of_token"]] == 1
    ref, ref_lse = O.full_attention(q, np.concatenate([K[keep], Kx]), np.concatenate([V[keep], Vx]),
                                    1 / math.sqrt(q.shape[1]))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(res["lse"], ref_lse, rtol=1e-13)


def test_extras_are_always_exact_and_outside_the_budget():
    rng = np.random.default_rng(13)
    q, K, V, cl = _rand_unit(rng, levels=1)
    Kx, Vx = _bf16(rng.normal(size=(7, K.shape[1]))), _bf16(rng.normal(size=(7, K.shape[1])))
    res = O.decode_unit(q, cl, key_budget=K.shape[0], Kx=Kx, Vx=Vx)
    ref, _ = O.full_attention(q, np.concatenate([K, Kx]), np.concatenate([V, Vx]), 1 / math.sqrt(q.shape[1]))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)
    assert res["n_sel_keys"] == K.shape[0]


def test_empty_clusters_and_large_logits():
    rng = np.random.default_rng(14)
    n, d = 50, 8
    fot = rng.integers(0, 4, size=n).astype(np.int32) * 2          # odd ids stay empty
    K = _bf16(rng.normal(size=(n, d)) * 30)                        # logits of several hundred
    V = _bf16(rng.normal(size=(n, d)))
    q = _bf16(rng.normal(size=(2, d)) * 30)
    cl = O.clustering_from_assignment(K, V, fot, 8, (np.arange(8) // 2).astype(np.int32), 4)
    res = O.decode_unit(q, cl, key_budget=20, coarse_budget=30)
    assert np.isfinite(res["out"]).all() and np.isfinite(res["lse"]).all()
    assert not res["selected"][1::2].any() and np.isnan(res["r_f"][1::2]).all()
    full = O.decode_unit(q, cl, key_budget=n, coarse_budget=n)
    ref, _ = O.full_attention(q, K, V, 1 / math.sqrt(d))
    np.testing.assert_allclose(full["out"], ref, rtol=1e-12, atol=1e-14)


def test_inconsistent_clustering_is_rejected():
    rng = np.random.default_rng(15)
    q, K, V, cl = _rand_unit(rng, levels=2)
    bad = dict(cl, N_f=cl["N_f"] + 1)
    with pytest.raises(ValueError):
        O.decode_unit(q, bad, key_budget=10, coarse_budget=10)


def test_more_heads_than_clusters():
    # one token, one fine and one coarse cluster, seven heads: every head attends to the only token
    # whatever the budgets, with or without centroid terms (the centroid IS the token)
    rng = np.random.default_rng(77)
    K, V, q = _bf16(rng.normal(size=(1, 16))), _bf16(rng.normal(size=(1, 16))), _bf16(rng.normal(size=(7, 16)))
    cl = dict(K=K, V=V, levels=2, fine_of_token=np.zeros(1, np.int32), Kc_f=K.copy(), Vc_f=V.copy(), N_f=np.ones(1, np.int32),
              coarse_of_fine=np.zeros(1, np.int32), Kc_c=K.copy(), Vc_c=V.copy(), N_c=np.ones(1, np.int32))
    for kb, cb in [(0, 0), (1, 1), (5, 0), (0, 5)]:
        r = O.decode_unit(q, cl, kb, cb)
        np.testing.assert_allclose(r["out"], np.repeat(V, 7, axis=0), rtol=1e-14)
        np.testing.assert_allclose(r["lse"], (q @ K[0]) / np.sqrt(16), rtol=1e-13, atol=1e-13)
    r = O.decode_unit(q, cl, 1, 1, mp_terms=False)
    np.testing.assert_allclose(r["out"], np.repeat(V, 7, axis=0), rtol=1e-14)


def test_batch_entry_points_equal_a_loop_over_units():
    """mpo_decode_batch / mpo_full_attention_batch (what the benchmark times on the host) against a
    loop of the per-unit functions that all other pins rest on: bit-identical."""
    rng = np.random.default_rng(21)
    U, G, d, n, kf, kc = 5, 3, 16, 300, 20, 4

    def bf16(a):
        import torch
        return torch.tensor(np.asarray(a), dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()

    cls, qs, Kxs, Vxs = [], [], [], []
    blocks = O.plan_blocks(n, 0, 0, kf, kc)
    for u in range(U):
        centers = rng.normal(size=(8, d)) * 2
        K = bf16(centers[rng.integers(0, 8, n)] + 0.3 * rng.normal(size=(n, d)))
        V = bf16(rng.normal(size=(n, d)))
        cls.append(O.cluster_unit(K, V, blocks, rng.choice(n, kf, replace=False), rng.choice(kf, kc, replace=False), 2, 2))
        qs.append(bf16(0.5 * centers[rng.integers(0, 8, G)] + 0.3 * rng.normal(size=(G, d))))
        Kxs.append(bf16(rng.normal(size=(7, d))))
        Vxs.append(bf16(rng.normal(size=(7, d))))
    q, Kx, Vx = np.stack(qs), np.stack(Kxs), np.stack(Vxs)
    for kb, cb, tail, terms in [(60, 150, True, True), (0, 0, False, True), (40, 100, True, False), (10 ** 6, 10 ** 6, False, True)]:
        out, lse, prom, sel = O.decode_batch(q, cls, kb, cb, Kx if tail else None, Vx if tail else None, mp_terms=terms)
        for u in range(U):
            r = O.decode_unit(q[u], cls[u], kb, cb, Kx[u] if tail else None, Vx[u] if tail else None, mp_terms=terms)
            np.testing.assert_array_equal(out[u], r["out"])
            np.testing.assert_array_equal(lse[u], r["lse"])
            np.testing.assert_array_equal(prom[u], r["promising"])
            np.testing.assert_array_equal(sel[u], r["selected"])
    K, V = np.stack([c["K"] for c in cls]), np.stack([c["V"] for c in cls])
    out, lse = O.full_attention_batch(q, K, V, 0.25)
    for u in range(U):
        o, l = O.full_attention(q[u], K[u], V[u], 0.25)
        np.testing.assert_array_equal(out[u], o)
        np.testing.assert_array_equal(lse[u], l)
