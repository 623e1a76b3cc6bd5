"""Pins for the online-update oracle (CPU only)."""
import numpy as np
import torch

from oracle import mp_oracle as O


def _bf16(a):
    return torch.tensor(np.asarray(a), dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def _setup(rng, n=600, d=16, kf=24, kc=4, W=0, alpha=0, levels=2):
    centers = rng.normal(size=(12, d)) * 2
    K = _bf16(centers[rng.integers(0, 12, n)] + 0.3 * rng.normal(size=(n, d)))
    V = _bf16(rng.normal(size=(n, d)))
    blocks = O.plan_blocks(n, W, alpha, kf, kc if levels == 2 else 0)
    init_f = np.concatenate([rng.choice(b["t1"] - b["t0"], b["f1"] - b["f0"], replace=False) for b in blocks])
    init_c = np.concatenate([rng.choice(b["f1"] - b["f0"], b["c1"] - b["c0"], replace=False) for b in blocks]) \
        if levels == 2 else None
    cl = O.cluster_unit(K, V, blocks, init_f, init_c, 3, levels)
    return cl, centers


def _new_tokens(rng, centers, n_new, d=16):
    Kn = _bf16(centers[rng.integers(0, 12, n_new)] + 0.3 * rng.normal(size=(n_new, d)))
    return Kn, _bf16(rng.normal(size=(n_new, d)))


def _check_consistent(cl):
    K, V, fot, Nf = cl["K"], cl["V"], cl["fine_of_token"], cl["N_f"]
    assert fot.shape[0] == K.shape[0] and (np.bincount(fot, minlength=Nf.shape[0]) == Nf).all()
    for f in np.flatnonzero(Nf):
        np.testing.assert_array_equal(cl["Kc_f"][f], _bf16(K[fot == f].sum(0) / Nf[f]))
        np.testing.assert_array_equal(cl["Vc_f"][f], _bf16(V[fot == f].sum(0) / Nf[f]))
    for b in cl["blocks"]:
        f = fot[b["t0"]:b["t1"]]
        assert f.min() >= b["f0"] and f.max() < b["f1"]
    if cl["levels"] == 2:
        cof = cl["coarse_of_fine"]
        assert (np.bincount(cof, weights=Nf, minlength=cl["N_c"].shape[0]) == cl["N_c"]).all()
        for b in cl["blocks"]:
            c = cof[b["f0"]:b["f1"]]
            assert (np.diff(c) >= 0).all() and c.min() >= b["c0"] and c.max() < b["c1"]
    assert cl["blocks"][-1]["t1"] == K.shape[0] and cl["blocks"][-1]["f1"] == Nf.shape[0]


def test_one_shot_update_without_refinement_keeps_old_assignments_and_takes_exact_means():
    rng = np.random.default_rng(0)
    cl, centers = _setup(rng, levels=1)
    Kn, Vn = _new_tokens(rng, centers, 32)
    out = O.update_unit(cl, Kn, Vn, 0, 0, [], 0, 0, 0)
    np.testing.assert_array_equal(out["fine_of_token"][:600], cl["fine_of_token"])
    # appended tokens went to the nearest stored centroid (library argmin as the independent check)
    from sklearn.metrics import pairwise_distances_argmin
    np.testing.assert_array_equal(out["fine_of_token"][600:], pairwise_distances_argmin(Kn, cl["Kc_f"]))
    _check_consistent(out)    # stored centroid = exact mean of old and new members (closed form)
    assert out["N_f"].sum() == 632


def test_new_seed_clusters_capture_their_seed_token():
    rng = np.random.default_rng(1)
    cl, centers = _setup(rng, levels=2)
    Kn, Vn = _new_tokens(rng, centers, 64)
    Kn[5] = 40.0      # far from everything: seeding a centroid there must capture exactly that token
    Kn = _bf16(Kn)
    out = O.update_unit(cl, Kn, Vn, 2, 1, [5, 9, 0], 2, 0, 0)
    _check_consistent(out)
    assert out["N_f"].shape[0] == 26 and out["N_c"].shape[0] == 5
    f = out["fine_of_token"][600 + 5]
    assert out["N_f"][f] == 1 and (out["Kc_f"][f] == 40.0).all()


def test_refinement_equals_lloyd_from_the_one_shot_centroids():
    rng = np.random.default_rng(2)
    cl, centers = _setup(rng, levels=1)
    Kn, Vn = _new_tokens(rng, centers, 48)
    out0 = O.update_unit(cl, Kn, Vn, 3, 0, [1, 2, 3], 0, 0, 0)
    out2 = O.update_unit(cl, Kn, Vn, 3, 0, [1, 2, 3], 2, 0, 0)
    _check_consistent(out2)
    # inertia of the refined clustering is not worse than that of the one-shot one
    def inertia(c):
        return ((c["K"] - c["Kc_f"][c["fine_of_token"]]) ** 2).sum()
    assert inertia(out2) <= inertia(out0) * (1 + 1e-3)


def test_running_mean_closed_form_on_exactly_representable_data():
    # cluster 0 = {0, 2} (centroid 1), cluster 1 = {8}; append 3, 1 and 4: all nearest to cluster 0.
    K = np.array([[0.0], [2.0], [8.0]])
    V = np.zeros((3, 1))
    cl = O.clustering_from_assignment(K, V, [0, 0, 1], 2)
    new = np.array([[3.0], [1.0], [4.0]])
    out = O.update_unit(cl, new, np.zeros((3, 1)), 0, 0, [], 0, 0, 0)
    np.testing.assert_array_equal(out["fine_of_token"], [0, 0, 1, 0, 0, 0])
    np.testing.assert_array_equal(out["Kc_f"][:, 0], [(0 + 2 + 3 + 1 + 4) / 5, 8.0])
    # a token at equal distance from both centroids (4.5: 3.5 from 1 and from 8) goes to the lower id
    tie = O.update_unit(cl, np.array([[4.5]]), np.zeros((1, 1)), 0, 0, [], 0, 0, 0)
    assert tie["fine_of_token"][3] == 0
    # with one refinement pass the assignment is made against the running means:
    # (2*1 + 3 + 1 + 4)/5 = 2 and 8, so the token 5.5 appended next would go to cluster 1 (2.5 vs 3.5)
    out1 = O.update_unit(cl, new, np.zeros((3, 1)), 0, 0, [], 1, 0, 0)
    np.testing.assert_array_equal(out1["fine_of_token"], [0, 0, 1, 0, 0, 0])
    nxt = O.update_unit(out1, np.array([[5.5]]), np.zeros((1, 1)), 0, 0, [], 0, 0, 0)
    assert nxt["fine_of_token"][6] == 1


def test_split_when_last_block_reaches_w_plus_alpha():
    rng = np.random.default_rng(3)
    W, alpha = 256, 128
    cl, centers = _setup(rng, n=352, kf=22, kc=4, W=W, alpha=alpha, levels=2)    # one block of 352 tokens
    assert len(cl["blocks"]) == 1
    Kn, Vn = _new_tokens(rng, centers, 32)
    counts = O.update_seed_counts(cl["blocks"], 32, 4, 1, W, alpha, 2)
    assert counts == [4, 1, 26 * 256 // 384, 26 - 26 * 256 // 384, 5 * 256 // 384, 5 - 5 * 256 // 384]
    seeds = np.concatenate([rng.choice(32, 4, replace=False), rng.choice(4, 1, replace=False),
                            rng.choice(256, counts[2], replace=False), rng.choice(128, counts[3], replace=False),
                            rng.choice(counts[2], counts[4], replace=False),
                            rng.choice(counts[3], counts[5], replace=False)])
    out = O.update_unit(cl, Kn, Vn, 4, 1, seeds, 2, W, alpha, split_iters=3)
    _check_consistent(out)
    assert [(b["t0"], b["t1"]) for b in out["blocks"]] == [(0, 256), (256, 384)]
    # the split result is exactly a fresh clustering of the two parts with those seeds
    blocks = [dict(t0=0, t1=256, f0=0, f1=counts[2], c0=0, c1=counts[4]),
              dict(t0=256, t1=384, f0=counts[2], f1=26, c0=counts[4], c1=5)]
    cuts = np.cumsum([0] + counts)
    ref = O.cluster_unit(out["K"], out["V"], blocks, np.concatenate([seeds[cuts[2]:cuts[3]], seeds[cuts[3]:cuts[4]]]),
                         np.concatenate([seeds[cuts[4]:cuts[5]], seeds[cuts[5]:cuts[6]]]), 3, 2)
    for key in ("fine_of_token", "coarse_of_fine", "N_f", "N_c", "Kc_f", "Vc_f", "Kc_c", "Vc_c"):
        np.testing.assert_array_equal(out[key], ref[key])
    # one token short of W + alpha: no split
    cl2, _ = _setup(np.random.default_rng(3), n=351, kf=22, kc=4, W=W, alpha=alpha, levels=2)
    assert O.update_seed_counts(cl2["blocks"], 32, 4, 1, W, alpha, 2)[2:] == [0, 0, 0, 0]


def test_update_of_a_later_block_leaves_frozen_blocks_untouched():
    rng = np.random.default_rng(4)
    cl, centers = _setup(rng, n=700, kf=40, kc=8, W=256, alpha=128, levels=2)
    assert len(cl["blocks"]) == 3
    Kn, Vn = _new_tokens(rng, centers, 16)
    out = O.update_unit(cl, Kn, Vn, 2, 1, [3, 7, 1], 3, 256, 128)
    _check_consistent(out)
    lb = cl["blocks"][-1]
    np.testing.assert_array_equal(out["fine_of_token"][:lb["t0"]], cl["fine_of_token"][:lb["t0"]])
    np.testing.assert_array_equal(out["Kc_f"][:lb["f0"]], cl["Kc_f"][:lb["f0"]])
    np.testing.assert_array_equal(out["Kc_c"][:lb["c0"]], cl["Kc_c"][:lb["c0"]])
    q = _bf16(rng.normal(size=(2, 16)))
    res = O.decode_unit(q, out, key_budget=716, coarse_budget=716)
    ref, _ = O.full_attention(q, out["K"], out["V"], 0.25)
    np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)


def test_coarse_refresh_assigns_every_fine_centroid_to_its_nearest_stored_coarse_centroid():
    """Coarse level of an update (Sec. 3.4 applied to Sec. 3.3), no refinement, no new coarse seed:
    one Lloyd step of the block's fine working centroids from the stored coarse key centroids.
    Every appended token seeds a cluster of its own, so the working centroids are known without any
    arithmetic (stored fine centroids, then the appended keys); the library argmin gives the parents;
    the stable renumbering and the stored means follow from their definitions."""
    from sklearn.metrics import pairwise_distances_argmin
    rng = np.random.default_rng(11)
    cl, centers = _setup(rng, n=600, kf=24, kc=4, levels=2)
    n_new = 6
    Kn, Vn = _new_tokens(rng, centers, n_new)
    out = O.update_unit(cl, Kn, Vn, n_new, 0, list(range(n_new)), 0, 0, 0)
    _check_consistent(out)
    Cw = np.concatenate([cl["Kc_f"], Kn])                      # working fine centroids, old numbering
    parent = pairwise_distances_argmin(Cw, cl["Kc_c"])         # nearest stored coarse centroid
    order = np.argsort(parent, kind="stable")                  # children contiguous, stable in the old id
    np.testing.assert_array_equal(out["coarse_of_fine"], parent[order])
    old_fot = np.concatenate([cl["fine_of_token"], 24 + np.arange(n_new)])    # each appended token: its own cluster
    new_of_old = np.empty(30, dtype=np.int64)
    new_of_old[order] = np.arange(30)
    np.testing.assert_array_equal(out["fine_of_token"], new_of_old[old_fot])
    # stored coarse tables = member counts and bf16 means of all member keys / values
    tok_parent = parent[old_fot]
    for c in range(4):
        m = tok_parent == c
        assert out["N_c"][c] == m.sum()
        np.testing.assert_array_equal(out["Kc_c"][c], _bf16(out["K"][m].sum(0) / m.sum()))
        np.testing.assert_array_equal(out["Vc_c"][c], _bf16(out["V"][m].sum(0) / m.sum()))


def test_coarse_refresh_with_separated_families_and_a_far_new_coarse_seed():
    """Two families of fine clusters far apart: after any update each fine cluster must hang under its
    family's coarse cluster, and a new coarse cluster seeded with a far-away new fine cluster captures
    exactly that fine cluster."""
    rng = np.random.default_rng(12)
    d = 16
    fam = np.zeros((2, d)); fam[0, 0] = -50.0; fam[1, 0] = 50.0
    n = 400
    side = (np.arange(n) % 2)                       # tokens alternate between the families
    K = _bf16(fam[side] + rng.normal(size=(n, d)))
    V = _bf16(rng.normal(size=(n, d)))
    # seeds: 5 fine clusters per family, one coarse seed in each family
    init_f = np.array([0, 2, 4, 6, 8, 1, 3, 5, 7, 9])
    blocks = O.plan_blocks(n, 0, 0, 10, 2)
    cl = O.cluster_unit(K, V, blocks, init_f, np.array([0, 5]), 3, 2)
    np.testing.assert_array_equal(cl["coarse_of_fine"], [0] * 5 + [1] * 5)
    # append 8 ordinary tokens and one far away from both families; it seeds a fine and a coarse cluster
    Kn = _bf16(fam[np.arange(9) % 2] + rng.normal(size=(9, d)))
    Kn[8] = 0.0; Kn[8, 1] = 200.0
    Vn = _bf16(rng.normal(size=(9, d)))
    for refine in (0, 2):
        out = O.update_unit(cl, Kn, Vn, 1, 1, [8, 0], refine, 0, 0)
        _check_consistent(out)
        assert out["N_c"].tolist() == [204, 204, 1]
        np.testing.assert_array_equal(out["coarse_of_fine"], [0] * 5 + [1] * 5 + [2])
        f_far = out["fine_of_token"][n + 8]
        assert f_far == 10 and out["N_f"][10] == 1
        np.testing.assert_array_equal(out["Kc_c"][2], Kn[8])
        np.testing.assert_array_equal(out["Vc_c"][2], Vn[8])
        # every token hangs under the coarse cluster of its family
        tok_c = out["coarse_of_fine"][out["fine_of_token"]]
        np.testing.assert_array_equal(tok_c[:n], side)
        np.testing.assert_array_equal(tok_c[n:n + 8], np.arange(8) % 2)


def test_update_seed_counts_values():
    b1 = [dict(t0=0, t1=600, f0=0, f1=24, c0=0, c1=4)]
    assert O.update_seed_counts(b1, 32, 3, 1, 0, 0, 2) == [3, 1, 0, 0, 0, 0]          # one block for ever: never a split
    assert O.update_seed_counts(b1, 32, 3, 1, 0, 0, 1) == [3, 0, 0, 0, 0, 0]          # one level: no coarse seeds
    # W = 512, alpha = 128: 600 + 40 = 640 tokens reach W + alpha; 24 + 4 = 28 fine and 4 + 2 = 6 coarse clusters are
    # shared out as 28 * 512 // 640 = 22 / 6 and 6 * 512 // 640 = 4 / 2
    assert O.update_seed_counts(b1, 40, 4, 2, 512, 128, 2) == [4, 2, 22, 6, 4, 2]
    assert O.update_seed_counts(b1, 40, 4, 2, 512, 128, 1) == [4, 0, 22, 6, 0, 0]
    assert O.update_seed_counts(b1, 39, 4, 2, 512, 128, 2) == [4, 2, 0, 0, 0, 0]      # 639 tokens: one short
    # only the last block counts
    b2 = [dict(t0=0, t1=512, f0=0, f1=32, c0=0, c1=4), dict(t0=512, t1=700, f0=32, f1=44, c0=4, c1=6)]
    assert O.update_seed_counts(b2, 452, 8, 1, 512, 128, 2) == [8, 1, (12 + 8) * 512 // 640, 20 - 20 * 512 // 640, 3 * 512 // 640, 3 - 3 * 512 // 640]


def test_coarse_refresh_runs_max_1_refine_iters_lloyd_steps():
    """Hand-worked on a line: fine clusters at 0, 0, 0, 0 and 6, stored coarse key centroids 3.5 and 9.
    One Lloyd step over the fine centroids puts all five under coarse 0 (6 is 2.5 from 3.5, 3 from 9) and
    moves that centroid to 6/5; only a second step hands the fine cluster at 6 to coarse 1 (4.8 against 3)."""
    K = np.array([[0.0], [0.0], [0.0], [0.0], [6.0]])
    V = np.arange(5, dtype=np.float64)[:, None]
    cl = O.clustering_from_assignment(K, V, [0, 1, 2, 3, 4], 5, [0, 0, 0, 0, 1], 2)
    cl["Kc_c"] = np.array([[3.5], [9.0]])          # what an earlier history may have left behind
    new_k, new_v = np.array([[0.0]]), np.array([[7.0]])
    out = O.update_unit(cl, new_k, new_v, 0, 0, [], 0, 0, 0)          # no refinement: ONE coarse step
    np.testing.assert_array_equal(out["coarse_of_fine"], [0, 0, 0, 0, 0])
    np.testing.assert_array_equal(out["N_c"], [6, 0])
    assert out["Kc_c"][1, 0] == 9.0 and out["Kc_c"][0, 0] == 1.0      # empty: keeps its centroid; mean key of six tokens
    assert out["fine_of_token"][5] == 0                                # equal distances: lowest id
    out = O.update_unit(cl, new_k, new_v, 0, 0, [], 2, 0, 0)          # two refinement iterations: TWO coarse steps
    np.testing.assert_array_equal(out["coarse_of_fine"], [0, 0, 0, 0, 1])
    np.testing.assert_array_equal(out["N_c"], [5, 1])
    np.testing.assert_array_equal(out["Kc_c"][:, 0], [0.0, 6.0])
