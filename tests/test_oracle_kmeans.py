"""Pins for the k-means / index-construction oracle (CPU only)."""
import numpy as np
import pytest
import torch
from sklearn.cluster import KMeans
from sklearn.metrics import pairwise_distances_argmin

from oracle import mp_oracle as O


def _bf16(a):
    return torch.tensor(np.asarray(a), dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def _mixture(rng, n, k, d, noise=0.3):
    centers = rng.normal(size=(k, d)) * 2
    lab = rng.integers(0, k, size=n)
    return _bf16(centers[lab] + noise * rng.normal(size=(n, d))), centers, lab


def test_round_bf16_matches_library_conversion():
    rng = np.random.default_rng(0)
    x32 = (rng.normal(size=20000) * np.exp(rng.normal(size=20000) * 8)).astype(np.float32)
    ref = torch.tensor(x32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_bf16(x32.astype(np.float64)), ref)


def test_round_bf16_ties_to_even_and_single_rounding():
    u = 2.0 ** -8                                   # half an ulp of bf16 at 1.0 is 2^-8
    assert O.round_bf16(np.array([1 + u]))[0] == 1.0            # tie -> even mantissa (1.0)
    assert O.round_bf16(np.array([1 + 3 * u]))[0] == 1 + 4 * u  # tie -> even mantissa
    assert O.round_bf16(np.array([1 + u + 2.0 ** -40]))[0] == 1 + 2 * u   # just above the tie: up
    # rounding first to fp32 would land exactly on the tie and then go to even: single rounding must not
    assert O.round_bf16(np.array([-(1 + u + 2.0 ** -40)]))[0] == -(1 + 2 * u)
    assert O.round_bf16(np.array([0.0]))[0] == 0.0
    assert O.round_bf16(np.array([255.5]))[0] == 256.0


def test_assign_matches_library_argmin():
    rng = np.random.default_rng(1)
    X, centers, _ = _mixture(rng, 500, 12, 24)
    Cn = _bf16(centers)
    np.testing.assert_array_equal(O.assign(X, Cn), pairwise_distances_argmin(X, Cn))


def test_assign_ties_go_to_lowest_index():
    X = np.array([[0.0, 0.0], [5.0, 5.0], [0.0, 3.0]])
    Cn = np.array([[2.0, 0.0], [0.0, 2.0], [0.0, 2.0], [5.0, 5.0], [5.0, 5.0]])
    assert list(O.assign(X, Cn)) == [0, 3, 1]


def test_single_cluster_is_global_mean():
    rng = np.random.default_rng(2)
    X, _, _ = _mixture(rng, 300, 4, 16)
    Cn, a, cnt = O.lloyd(X, [17], 3)
    assert (a == 0).all() and cnt[0] == 300
    np.testing.assert_array_equal(Cn[0], _bf16(X.mean(0)))


def test_separated_modes_recovered_in_one_step():
    rng = np.random.default_rng(3)
    k, d = 6, 16
    X, centers, lab = _mixture(rng, 400, k, d, noise=0.01)
    seeds = [int(np.flatnonzero(lab == j)[0]) for j in range(k)]
    Cn, a, cnt = O.lloyd(X, seeds, 1)
    np.testing.assert_array_equal(a, lab)
    for j in range(k):
        np.testing.assert_allclose(Cn[j], X[lab == j].mean(0), rtol=2.0 ** -8, atol=1e-6)


def test_one_lloyd_iteration_matches_sklearn():
    rng = np.random.default_rng(4)
    X, _, _ = _mixture(rng, 600, 10, 20)
    seeds = rng.choice(600, size=10, replace=False).astype(np.int32)
    Cn, a, cnt = O.lloyd(X, seeds, 1)
    km = KMeans(n_clusters=10, init=X[seeds], n_init=1, algorithm="lloyd", tol=0, max_iter=1).fit(X)
    assert cnt.min() > 0
    np.testing.assert_allclose(Cn, km.cluster_centers_, rtol=2.0 ** -8, atol=1e-6)
    # sklearn's labels_ are the assignment to the updated centers = our second assignment
    _, a2, _ = O.lloyd(X, seeds, 2)
    agree = (a2 == km.labels_).mean()
    assert agree > 0.99        # centers differ by bf16 rounding only


def test_inertia_never_increases_without_rounding():
    rng = np.random.default_rng(5)
    X, _, _ = _mixture(rng, 500, 8, 12, noise=1.0)
    Cn = X[rng.choice(500, 8, replace=False)].copy()
    last = np.inf
    for it in range(8):
        a = O.assign(X, Cn)
        inertia_assign = ((X - Cn[a]) ** 2).sum()
        assert inertia_assign <= last + 1e-9
        S, cnt = O.member_sums(X, a, 8)
        Cn = np.where(cnt[:, None] > 0, S / np.maximum(cnt, 1)[:, None], Cn)
        last = ((X - Cn[a]) ** 2).sum()
        assert last <= inertia_assign + 1e-9
        assert cnt.sum() == 500


def test_member_sums_and_empty_clusters_keep_centroid():
    X = _bf16(np.array([[0.0, 0.0], [0.5, 0.0], [10.0, 10.0]]))
    # seeds: points 0 and 1 and 2 -> after one step all are singletons; force an empty cluster with duplicates
    Xd = np.concatenate([X, X[:1]])
    Cn, a, cnt = O.lloyd(Xd, [0, 3, 2], 1)          # seeds 0 and 3 coincide -> cluster 1 gets nothing
    assert list(cnt) == [3, 0, 1] and list(a) == [0, 0, 2, 0]
    np.testing.assert_array_equal(Cn[1], Xd[3])     # an empty cluster keeps its centroid
    np.testing.assert_array_equal(Cn[0], _bf16(np.array([0.5 / 3, 0.0])))
    S, c2 = O.member_sums(Xd, a, 3)
    np.testing.assert_array_equal(c2, cnt)
    for j in range(3):
        np.testing.assert_allclose(S[j], Xd[a == j].sum(0) if (a == j).any() else 0)


def test_plan_blocks():
    b = O.plan_blocks(131072, 8192, 4096, 4096, 256)
    assert len(b) == 16 and all(x["t1"] - x["t0"] == 8192 for x in b)
    assert all(x["f1"] - x["f0"] == 256 and x["c1"] - x["c0"] == 16 for x in b)
    b = O.plan_blocks(8192, 8192, 4096, 256, 32)
    assert len(b) == 1 and b[0]["t1"] == 8192
    b = O.plan_blocks(12288, 8192, 4096, 768, 96)            # W + alpha: first W tokens become a block
    assert [(x["t0"], x["t1"]) for x in b] == [(0, 8192), (8192, 12288)]
    assert [(x["f0"], x["f1"]) for x in b] == [(0, 512), (512, 768)]
    b = O.plan_blocks(12287, 8192, 4096, 768, 96)
    assert len(b) == 1
    b = O.plan_blocks(4096, 0, 0, 64, 0)
    assert len(b) == 1 and b[0]["f1"] == 64
    b = O.plan_blocks(30000, 8192, 4096, 1000, 100)
    assert [x["t1"] - x["t0"] for x in b] == [8192, 8192, 8192, 5424]
    assert b[-1]["f1"] == 1000 and b[-1]["c1"] == 100


@pytest.mark.parametrize("levels", [1, 2])
def test_cluster_unit_structure(levels):
    rng = np.random.default_rng(6)
    n, d = 700, 16
    X, _, _ = _mixture(rng, n, 20, d)
    V = _bf16(rng.normal(size=(n, d)))
    blocks = O.plan_blocks(n, 256, 128, 40, 8 if levels == 2 else 0)
    assert len(blocks) == 3
    init_f = np.concatenate([rng.choice(b["t1"] - b["t0"], b["f1"] - b["f0"], replace=False) for b in blocks])
    init_c = np.concatenate([rng.choice(b["f1"] - b["f0"], b["c1"] - b["c0"], replace=False) for b in blocks]) \
        if levels == 2 else None
    cl = O.cluster_unit(X, V, blocks, init_f, init_c, 4, levels)
    fot, Nf = cl["fine_of_token"], cl["N_f"]
    assert Nf.sum() == n and (np.bincount(fot, minlength=40) == Nf).all()
    for b in blocks:                                   # clusters never span blocks
        f = fot[b["t0"]:b["t1"]]
        assert f.min() >= b["f0"] and f.max() < b["f1"]
    for f in range(40):                                # stored centroids are the member means
        if Nf[f]:
            np.testing.assert_array_equal(cl["Kc_f"][f], _bf16(X[fot == f].sum(0) / Nf[f]))
            np.testing.assert_array_equal(cl["Vc_f"][f], _bf16(V[fot == f].sum(0) / Nf[f]))
    if levels == 2:
        cof, Nc = cl["coarse_of_fine"], cl["N_c"]
        for b in blocks:                               # children of a coarse cluster are contiguous, ids ascending
            c = cof[b["f0"]:b["f1"]]
            assert (np.diff(c) >= 0).all() and c.min() >= b["c0"] and c.max() < b["c1"]
        assert (np.bincount(cof, weights=Nf, minlength=8) == Nc).all()
        tok_c = cof[fot]
        for c in range(8):
            if Nc[c]:
                np.testing.assert_allclose(cl["Kc_c"][c], X[tok_c == c].mean(0), rtol=2.0 ** -8, atol=1e-6)
                np.testing.assert_allclose(cl["Vc_c"][c], V[tok_c == c].mean(0), rtol=2.0 ** -8, atol=2e-3)
        # the clustering is a valid decode input and a full budget gives full attention
        q = _bf16(rng.normal(size=(2, d)))
        res = O.decode_unit(q, cl, key_budget=n, coarse_budget=n)
        ref, _ = O.full_attention(q, X, V, 1 / np.sqrt(d))
        np.testing.assert_allclose(res["out"], ref, rtol=1e-12, atol=1e-14)


def test_fine_assignment_is_the_nearest_kmeans_centroid_of_the_last_iteration():
    rng = np.random.default_rng(7)
    X, _, _ = _mixture(rng, 300, 6, 8)
    seeds = rng.choice(300, 6, replace=False)
    C3, a3, _ = O.lloyd(X, seeds, 3)
    C2, _, _ = O.lloyd(X, seeds, 2)
    np.testing.assert_array_equal(a3, pairwise_distances_argmin(X, C2))
    Cc, ac, _ = O.lloyd_from(X, C2, 1)
    np.testing.assert_array_equal(ac, a3)
    np.testing.assert_array_equal(Cc, C3)


def test_coarse_sums_are_the_childrens_sums_added_in_fine_id_order():
    """The coarse tables come from the fine clusters' fp64 member sums, added in ascending fine id from
    zero.  Magnitudes chosen so that the order shows: fine cluster 0 holds 2^60 and 1, fine cluster 1
    holds -2^60 and 1 (all exact in bf16).  Each child's sum loses its 1 to rounding (2^60 + 1 is not a
    double), so the coarse sum is 0; adding the four rows one after the other would give 1, the exact
    sum is 2."""
    K = np.zeros((4, 128))
    K[:, 0] = [2.0 ** 60, 1.0, -2.0 ** 60, 1.0]
    K[:, 1] = [1.0, 2.0, 3.0, 4.0]                     # an ordinary dimension beside it
    V = np.ones((4, 128))
    fot = np.array([0, 0, 1, 1], dtype=np.int32)
    cl = O.clustering_from_assignment(K, V, fot, 2, coarse_of_fine=np.array([0, 0], dtype=np.int32), n_coarse=1)
    assert cl["N_c"][0] == 4
    assert cl["Kc_c"][0, 0] == 0.0
    assert cl["Kc_c"][0, 1] == 2.5
    np.testing.assert_array_equal(cl["Vc_c"][0], np.ones(128))
    # the helper itself: zero start, ascending id, counts added up
    S_f = np.array([[1.0, 2.0 ** 60], [2.0, 1.0], [4.0, -2.0 ** 60]])
    S_c, N_c = O.sums_of_children(S_f, np.array([3, 0, 5]), np.array([1, 1, 1]), 2)
    np.testing.assert_array_equal(S_c, [[0.0, 0.0], [7.0, 0.0]])      # (2^60 + 1) - 2^60 = 0 in fp64, in this order
    np.testing.assert_array_equal(N_c, [0, 8])
