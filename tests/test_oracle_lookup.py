"""Pins for the lookup keys / lookup query of the oracle (CPU only; Sec. 3.1, last paragraph, and
Sec. 4): clusters are formed on one set of keys and compared with one query, exact attention uses
another.  Each test ties the oracle to something other than itself."""
import math

import numpy as np
import torch

from oracle import mp_oracle as O
from tests.test_oracle_decode import _bf16, _brute_select


def _signed_permutation(rng, d):
    perm = rng.permutation(d)
    sign = rng.choice([-1.0, 1.0], size=d)
    return lambda x: np.asarray(x)[..., perm] * sign


def _data(rng, n=150, d=16, G=3, modes=9, spread=1.0):
    centers = rng.normal(size=(modes, d)) * 2.0
    m = rng.integers(0, modes, size=n)
    K = _bf16(centers[m] + spread * 0.25 * rng.normal(size=(n, d)))
    V = _bf16(rng.normal(size=(n, d)))
    q = _bf16(centers[rng.integers(0, modes, size=G)] + 0.25 * rng.normal(size=(G, d)))
    return q, K, V


def test_lookup_equal_to_the_keys_changes_nothing():
    rng = np.random.default_rng(31)
    q, K, V = _data(rng)
    blocks = O.plan_blocks(150, 0, 0, 12, 3)
    fi, ci = rng.choice(150, 12, replace=False).astype(np.int32), rng.choice(12, 3, replace=False).astype(np.int32)
    a = O.cluster_unit(K, V, blocks, fi, ci, 3, 2)
    b = O.cluster_unit(K, V, blocks, fi, ci, 3, 2, K_lookup=K)
    for key in ("fine_of_token", "coarse_of_fine", "Kc_f", "Vc_f", "Kc_c", "N_f", "N_c"):
        np.testing.assert_array_equal(a[key], b[key])
    ra = O.decode_unit(q, a, 40, 90)
    rb = O.decode_unit(q, b, 40, 90, q_lookup=q)
    np.testing.assert_array_equal(ra["out"], rb["out"])
    np.testing.assert_array_equal(ra["selected"], rb["selected"])


def test_a_signed_permutation_of_lookup_keys_and_lookup_query_is_invisible():
    # Dot products and distances do not change under a signed permutation of the coordinates (up to
    # the order of an fp64 sum): same clusters, same selection, same output, although the exact
    # part works on entirely different-looking vectors than the lookup.
    rng = np.random.default_rng(32)
    for trial in range(5):
        q, K, V = _data(rng)
        A = _signed_permutation(rng, K.shape[1])
        blocks = O.plan_blocks(150, 0, 0, 10, 3)
        fi, ci = rng.choice(150, 10, replace=False).astype(np.int32), rng.choice(10, 3, replace=False).astype(np.int32)
        plain = O.cluster_unit(K, V, blocks, fi, ci, 4, 2)
        look = O.cluster_unit(K, V, blocks, fi, ci, 4, 2, K_lookup=A(K))
        np.testing.assert_array_equal(plain["fine_of_token"], look["fine_of_token"])
        np.testing.assert_array_equal(plain["coarse_of_fine"], look["coarse_of_fine"])
        np.testing.assert_array_equal(A(plain["Kc_f"]), look["Kc_f"])
        np.testing.assert_array_equal(plain["Vc_f"], look["Vc_f"])
        for kb, cb in ((0, 0), (35, 80), (150, 150)):
            r0 = O.decode_unit(q, plain, kb, cb)
            r1 = O.decode_unit(q, look, kb, cb, q_lookup=A(q))
            np.testing.assert_array_equal(r0["selected"], r1["selected"])
            np.testing.assert_array_equal(r0["promising"], r1["promising"])
            np.testing.assert_allclose(r0["out"], r1["out"], rtol=1e-11, atol=1e-13)


def test_which_query_meets_which_keys_brute_force():
    # One level, written out from Eq. 1 / Eq. 2: centroid logits from the lookup query and the means
    # of the lookup keys; exact logits from the query and the stored keys.
    rng = np.random.default_rng(33)
    for trial in range(10):
        q, K, V = _data(rng, n=90, modes=7)
        KL = _bf16(K[:, ::-1] * 0.5 + 0.3 * rng.normal(size=K.shape))     # unrelated-looking lookup keys
        ql = _bf16(rng.normal(size=q.shape))
        fot = rng.integers(0, 7, size=90).astype(np.int32)
        cl = O.clustering_from_assignment(K, V, fot, 7, K_lookup=KL)
        N = cl["N_f"].astype(np.float64)
        Sk, _ = O.member_sums(KL, fot, 7)
        np.testing.assert_array_equal(cl["Kc_f"][N > 0], _bf16(Sk[N > 0] / N[N > 0, None]))
        scale = 1 / math.sqrt(q.shape[1])
        e = np.exp(scale * ql @ cl["Kc_f"].T)
        S = (e / (e * N[None]).sum(1, keepdims=True)).mean(0)
        budget = int(rng.integers(0, 95))
        sel = _brute_select(np.where(N > 0, S, -1.0), cl["N_f"], budget).astype(bool)
        tok = sel[fot]
        p_exact = np.exp(scale * q @ K[tok].T)                          # [G, selected tokens]
        rest = (~sel) & (N > 0)
        w_cent = e[:, rest] * N[None, rest]
        num = p_exact @ V[tok] + w_cent @ cl["Vc_f"][rest]
        den = p_exact.sum(1) + w_cent.sum(1)
        res = O.decode_unit(q, cl, budget, q_lookup=ql)
        np.testing.assert_array_equal(res["selected"].astype(bool), sel)
        np.testing.assert_allclose(res["out"], num / den[:, None], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(res["lse"], np.log(den), rtol=1e-12)


def test_update_runs_on_lookup_keys_and_stores_the_keys():
    rng = np.random.default_rng(34)
    q, K, V = _data(rng, n=120)
    A = _signed_permutation(rng, K.shape[1])
    blocks = O.plan_blocks(120, 0, 0, 8, 2)
    fi, ci = rng.choice(120, 8, replace=False).astype(np.int32), rng.choice(8, 2, replace=False).astype(np.int32)
    plain = O.cluster_unit(K, V, blocks, fi, ci, 3, 2)
    look = O.cluster_unit(K, V, blocks, fi, ci, 3, 2, K_lookup=A(K))
    _, Kn, Vn = _data(rng, n=20)
    seeds = np.array([3, 11, 0], dtype=np.int32)               # 2 new fine clusters, 1 new coarse cluster
    p2 = O.update_unit(plain, Kn, Vn, 2, 1, seeds, 2, 0, 0)
    l2 = O.update_unit(look, Kn, Vn, 2, 1, seeds, 2, 0, 0, K_new_lookup=A(Kn))
    np.testing.assert_array_equal(p2["fine_of_token"], l2["fine_of_token"])
    np.testing.assert_array_equal(A(p2["Kc_f"]), l2["Kc_f"])
    np.testing.assert_array_equal(A(p2["Kc_c"]), l2["Kc_c"])
    np.testing.assert_array_equal(l2["K"], np.concatenate([K, Kn]))          # stored keys: as given
    np.testing.assert_array_equal(l2["KL"], np.concatenate([A(K), A(Kn)]))
    r0 = O.decode_unit(q, p2, 50, 100)
    r1 = O.decode_unit(q, l2, 50, 100, q_lookup=A(q))
    np.testing.assert_array_equal(r0["selected"], r1["selected"])
    np.testing.assert_allclose(r0["out"], r1["out"], rtol=1e-11, atol=1e-13)
