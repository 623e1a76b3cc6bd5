"""TEST INFRASTRUCTURE, NOT PRODUCT CODE: Python face of the fp64 CPU oracle.

Loads ``libmp_oracle.so`` (plain C, built from ``mp_oracle.c`` by :func:`build`) and adds the
orchestration that is easier to read in numpy than in C: the blockwise / two-level index
construction (Sec. 3.1, 3.3, 3.4 of the paper) and the online cluster update (Sec. 3.3).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this module.  It imports nothing from the GPU package.

All arrays are float64 numpy arrays holding bf16-representable values (inputs are bf16 tensors
widened exactly); cluster ids are int32.

Also here: the quantiser of the 8-bit cache (e4m3 codes with one fp32 scale a row, keys as residuals
from their cluster's centroid).  The paper names no storage format (Sec. 2.3 only calls KV
quantisation complementary), so the choice of format is "parity unpinned" by the paper; the
arithmetic of the format itself is pinned against the library's float8 conversion
(tests/test_oracle_fp8.py).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mp_oracle.c")
_LIB = os.path.join(_HERE, "libmp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU code, no HIP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int32)
_bp = C.POINTER(C.c_uint8)


def _d(a):
    return None if a is None else a.ctypes.data_as(_dp)


def _i(a):
    return None if a is None else a.ctypes.data_as(_ip)


def _b(a):
    return None if a is None else a.ctypes.data_as(_bp)


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.mpo_round_bf16.restype = C.c_double
        _lib.mpo_round_bf16.argtypes = [C.c_double]
        _lib.mpo_decode_unit.restype = C.c_int
        _lib.mpo_decode_batch.restype = C.c_int
        _lib.mpo_num_threads.restype = C.c_int
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().mpo_num_threads())


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Element-wise round-to-nearest-even of fp64 to bf16 values (returned as fp64)."""
    x = _f64(x)
    out = np.empty_like(x)
    lib().mpo_round_bf16_array(_d(x), _d(out), C.c_int64(x.size))
    return out


def full_attention(q, K, V, scale):
    """Textbook softmax attention of G query rows over all n keys.  Returns (out [G,d], lse [G])."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    G, d = q.shape
    n = K.shape[0]
    out = np.zeros((G, d))
    lse = np.zeros(G)
    lib().mpo_full_attention(_d(q), _d(K), _d(V), C.c_int(G), C.c_int(n), C.c_int(d), C.c_double(scale),
                             _d(out), _d(lse))
    return out, lse


def decode_unit(q, cl, key_budget, coarse_budget=0, Kx=None, Vx=None, scale=None, mp_terms=True, q_lookup=None):
    """One Multipole Attention decode step for one unit (Eq. 1, Eq. 2, Sec. 3.4).

    ``cl`` is a clustering dict as produced by :func:`cluster_unit` or
    :func:`clustering_from_assignment`.  ``q_lookup`` (default: q) is the query used against the
    centroids when the clusters were formed on lookup keys (Sec. 3.1, last paragraph).  Returns a
    dict with out, lse, promising, selected, r_c, r_f, n_sel_keys.
    """
    q = _f64(q)
    ql = q if q_lookup is None else _f64(q_lookup)
    assert ql.shape == q.shape
    G, d = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    K, V = _f64(cl["K"]), _f64(cl["V"])
    n = K.shape[0]
    fot = _i32(cl["fine_of_token"])
    Kc_f, Vc_f, N_f = _f64(cl["Kc_f"]), _f64(cl["Vc_f"]), _i32(cl["N_f"])
    Cf = N_f.shape[0]
    levels = int(cl["levels"])
    if levels == 2:
        cof, Kc_c, Vc_c, N_c = _i32(cl["coarse_of_fine"]), _f64(cl["Kc_c"]), _f64(cl["Vc_c"]), _i32(cl["N_c"])
        Cc = N_c.shape[0]
    else:
        cof = Kc_c = Vc_c = N_c = None
        Cc = 0
    nx = 0 if Kx is None else int(np.asarray(Kx).shape[0])
    Kx = _f64(Kx) if nx else None
    Vx = _f64(Vx) if nx else None
    out = np.zeros((G, d))
    lse = np.zeros(G)
    promising = np.zeros(max(Cc, 1), dtype=np.uint8)
    selected = np.zeros(max(Cf, 1), dtype=np.uint8)
    r_c = np.full(max(Cc, 1), np.nan)
    r_f = np.full(max(Cf, 1), np.nan)
    nsel = C.c_int64(0)
    rc = lib().mpo_decode_unit(
        _d(q), _d(ql), C.c_int(G), C.c_int(d), C.c_double(scale), _d(K), _d(V), C.c_int(n), _i(fot),
        C.c_int(Cf), _d(Kc_f), _d(Vc_f), _i(N_f), C.c_int(levels), C.c_int(Cc), _i(cof), _d(Kc_c), _d(Vc_c),
        _i(N_c), _d(Kx), _d(Vx), C.c_int(nx), C.c_int64(int(key_budget)), C.c_int64(int(coarse_budget)),
        C.c_int(1 if mp_terms else 0), _d(out), _d(lse), _b(promising), _b(selected), _d(r_c), _d(r_f),
        C.byref(nsel))
    if rc != 0:
        raise ValueError("clustering is inconsistent (N_f / N_c do not match the assignments)")
    return dict(out=out, lse=lse, promising=promising[:Cc], selected=selected[:Cf], r_c=r_c[:Cc],
                r_f=r_f[:Cf], n_sel_keys=int(nsel.value))


def stack_units(cls):
    """The clustering dicts of a batch of units of identical shape as one dict of arrays with a
    leading unit axis (what :func:`decode_batch` works on; worth keeping when it is called repeatedly)."""
    levels = int(cls[0]["levels"])
    st = lambda key, conv: conv(np.stack([np.asarray(c[key]) for c in cls]))
    b = dict(U=len(cls), levels=levels, K=st("K", _f64), V=st("V", _f64), fine_of_token=st("fine_of_token", _i32),
             Kc_f=st("Kc_f", _f64), Vc_f=st("Vc_f", _f64), N_f=st("N_f", _i32))
    if levels == 2:
        b.update(coarse_of_fine=st("coarse_of_fine", _i32), Kc_c=st("Kc_c", _f64), Vc_c=st("Vc_c", _f64), N_c=st("N_c", _i32))
    return b


def decode_batch(q, cls, key_budget, coarse_budget=0, Kx=None, Vx=None, scale=None, mp_terms=True):
    """:func:`decode_unit` for a batch of units of identical shape, one OpenMP thread per unit (what
    the benchmark times as its CPU baseline).  q [U,G,d]; cls: list of U clustering dicts, or the
    result of :func:`stack_units`; Kx, Vx [U,nx,d] or None.  Returns out [U,G,d], lse [U,G],
    promising [U,Cc] (or None), selected [U,Cf]."""
    q = _f64(q)
    U, G, d = q.shape
    b = cls if isinstance(cls, dict) else stack_units(cls)
    assert b["U"] == U
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    levels = b["levels"]
    K, V, fot, Kc_f, Vc_f, N_f = b["K"], b["V"], b["fine_of_token"], b["Kc_f"], b["Vc_f"], b["N_f"]
    n, Cf = K.shape[1], N_f.shape[1]
    if levels == 2:
        cof, Kc_c, Vc_c, N_c = b["coarse_of_fine"], b["Kc_c"], b["Vc_c"], b["N_c"]
        Cc = N_c.shape[1]
    else:
        cof = Kc_c = Vc_c = N_c = None
        Cc = 0
    nx = 0 if Kx is None else int(np.asarray(Kx).shape[1])
    Kx = _f64(Kx) if nx else None
    Vx = _f64(Vx) if nx else None
    out = np.zeros((U, G, d))
    lse = np.zeros((U, G))
    promising = np.zeros((U, max(Cc, 1)), dtype=np.uint8)
    selected = np.zeros((U, max(Cf, 1)), dtype=np.uint8)
    fails = lib().mpo_decode_batch(
        C.c_int(U), _d(q), C.c_int(G), C.c_int(d), C.c_double(scale), _d(K), _d(V), C.c_int(n), _i(fot), C.c_int(Cf),
        _d(Kc_f), _d(Vc_f), _i(N_f), C.c_int(levels), C.c_int(Cc), _i(cof), _d(Kc_c), _d(Vc_c), _i(N_c), _d(Kx), _d(Vx),
        C.c_int(nx), C.c_int64(int(key_budget)), C.c_int64(int(coarse_budget)), C.c_int(1 if mp_terms else 0), _d(out),
        _d(lse), _b(promising), _b(selected))
    if fails:
        raise ValueError(f"{fails} units with an inconsistent clustering")
    return out, lse, (promising if levels == 2 else None), selected


def full_attention_batch(q, K, V, scale):
    """:func:`full_attention` for a batch of units, one OpenMP thread per unit.  q [U,G,d], K, V [U,n,d]."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    U, G, d = q.shape
    n = K.shape[1]
    out = np.zeros((U, G, d))
    lse = np.zeros((U, G))
    lib().mpo_full_attention_batch(C.c_int(U), _d(q), _d(K), _d(V), C.c_int(G), C.c_int(n), C.c_int(d), C.c_double(scale),
                                   _d(out), _d(lse))
    return out, lse


# --------------------------------------------------------------------------------------------
# 8-bit storage of the exactly attended keys and values (the KV quantisation that Sec. 2.3 names as
# complementary to the method).  Format: OCP e4m3 ("fn": 4 exponent bits with bias 7, 3 mantissa
# bits, subnormals, no infinities, largest magnitude 448), one fp32 scale per stored row:
#   scale = fp32(max_d |x_d|) / fp32(448)            (fp32 division; 1 for an all-zero row)
#   code_d = nearest e4m3 value to fp32(x_d) / scale  (fp32 division, then round to nearest, ties to
#            the even code, magnitudes above 448 clamp to 448)
# and the row stands for code_d * scale from then on.  Value rows are stored this way.  A key row is
# stored as its RESIDUAL from the key centroid of its fine cluster (the index already holds that
# centroid and the decode step already has q . centroid): r_d = fp32(k_d) - fp32(c_d), one fp32
# subtraction, quantised as above; the key then stands for c_d + code_d * scale.  The decode oracle
# is simply run on those dequantised rows (fp64); centroids are still means of the original rows.
# --------------------------------------------------------------------------------------------

def e4m3_magnitudes():
    """The 127 non-negative finite e4m3 values in code order (code 0..126; code 127 is NaN)."""
    v = np.zeros(127)
    for code in range(1, 127):
        e, m = code >> 3, code & 7
        v[code] = (m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return v


def quantize_rows_e4m3(X):
    """X [n, d] (bf16 values) -> (codes uint8 [n, d], scale float32 [n]) as defined above."""
    X32 = np.asarray(X, dtype=np.float32)
    amax = np.abs(X32).max(axis=1)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    y = (X32 / scale[:, None]).astype(np.float32)
    mag = np.minimum(np.abs(y).astype(np.float64), 448.0)
    tab = e4m3_magnitudes()
    hi = np.searchsorted(tab, mag, side="left").clip(1, 126)       # tab[hi-1] <= mag <= tab[hi] (mag > 0)
    lo = hi - 1
    d_lo, d_hi = mag - tab[lo], tab[hi] - mag
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(mag == 0, 0, code).astype(np.uint8)
    code |= (np.signbit(y).astype(np.uint8) << 7)
    return code, scale


def dequantize_rows_e4m3(codes, scale):
    """code * scale as float64 [n, d] (exact: a 4-bit significand times an fp32)."""
    tab = e4m3_magnitudes()
    mag = tab[(codes & 0x7f).astype(np.int64)]
    sign = np.where(codes & 0x80, -1.0, 1.0)
    return sign * mag * np.asarray(scale, dtype=np.float64)[:, None]


def quantize_keys_e4m3(K, centroid_of_row):
    """Key rows K [n, d] and the key centroid of each row's fine cluster [n, d] (both bf16 values) ->
    (codes, scale) of the fp32 residuals."""
    r = np.asarray(K, dtype=np.float32) - np.asarray(centroid_of_row, dtype=np.float32)
    return quantize_rows_e4m3(r)


def dequantize_keys_e4m3(codes, scale, centroid_of_row):
    """centroid + code * scale as float64 [n, d]."""
    return np.asarray(centroid_of_row, dtype=np.float64) + dequantize_rows_e4m3(codes, scale)


def assign(X, Cn):
    """Nearest-centroid assignment, squared Euclidean distance, ties to the lowest index."""
    X, Cn = _f64(X), _f64(Cn)
    a = np.zeros(X.shape[0], dtype=np.int32)
    lib().mpo_assign(_d(X), C.c_int(X.shape[0]), _d(Cn), C.c_int(Cn.shape[0]), C.c_int(X.shape[1]), _i(a))
    return a


def member_sums(X, a, k):
    X, a = _f64(X), _i32(a)
    S = np.zeros((k, X.shape[1]))
    cnt = np.zeros(k, dtype=np.int32)
    lib().mpo_member_sums(_d(X), C.c_int(X.shape[0]), _i(a), C.c_int(k), C.c_int(X.shape[1]), _d(S), _i(cnt))
    return S, cnt


def lloyd(X, init_idx, iters):
    """Lloyd k-means from explicit seeds; returns (centroids bf16-valued [k,d], assignment, counts)."""
    X, init_idx = _f64(X), _i32(init_idx)
    k = init_idx.shape[0]
    Cn = np.zeros((k, X.shape[1]))
    a = np.zeros(X.shape[0], dtype=np.int32)
    cnt = np.zeros(k, dtype=np.int32)
    lib().mpo_lloyd(_d(X), C.c_int(X.shape[0]), C.c_int(X.shape[1]), _i(init_idx), C.c_int(k), C.c_int(iters),
                    _d(Cn), _i(a), _i(cnt))
    return Cn, a, cnt


def lloyd_from(X, Cn, iters):
    """Lloyd iterations continuing from the given centroids; returns (centroids, assignment, counts)."""
    X = _f64(X)
    Cn = _f64(Cn).copy()
    k = Cn.shape[0]
    a = np.zeros(X.shape[0], dtype=np.int32)
    cnt = np.zeros(k, dtype=np.int32)
    lib().mpo_lloyd_from(_d(X), C.c_int(X.shape[0]), C.c_int(X.shape[1]), C.c_int(k), C.c_int(iters), _d(Cn),
                         _i(a), _i(cnt))
    return Cn, a, cnt


# --------------------------------------------------------------------------------------------
# Blockwise, hierarchical index construction (Sec. 3.3 blocks of W tokens with a final block of
# alpha .. W+alpha tokens; Sec. 3.4 second level obtained by clustering the fine centroids).
# --------------------------------------------------------------------------------------------

def plan_blocks(n_tokens, block_w, block_alpha, n_fine, n_coarse):
    """Token ranges and per-block cluster counts.

    Blocks hold W tokens except the last, which holds between alpha and W+alpha-1 tokens (all of
    them when there are fewer than W+alpha, or when block_w == 0).  The per-unit totals n_fine and
    n_coarse are shared out in proportion to the token ranges by cumulative integer division, so
    that the counts sum exactly to the totals.
    """
    if block_w <= 0 or n_tokens < block_w + block_alpha:
        bounds = [0, n_tokens]
    else:
        m = (n_tokens - block_alpha) // block_w
        bounds = [i * block_w for i in range(m + 1)] + [n_tokens]
    blocks = []
    for b in range(len(bounds) - 1):
        t0, t1 = bounds[b], bounds[b + 1]
        f0, f1 = (n_fine * t0) // n_tokens, (n_fine * t1) // n_tokens
        c0, c1 = (n_coarse * t0) // n_tokens, (n_coarse * t1) // n_tokens
        blocks.append(dict(t0=t0, t1=t1, f0=f0, f1=f1, c0=c0, c1=c1))
    return blocks


def _mean_bf16(S, cnt):
    out = np.zeros_like(S)
    nz = cnt > 0
    out[nz] = round_bf16(S[nz] / cnt[nz, None].astype(np.float64))
    return out


def sums_of_children(S_f, N_f, coarse_of_fine, kc):
    """Member sums and counts of the coarse clusters from those of their fine clusters: the children's
    fp64 sums are added one after the other in ascending fine id, starting from zero (Sec. 3.4: a
    coarse centroid is the mean of all keys below it; the order of the additions is this reading's)."""
    S_c = np.zeros((kc, S_f.shape[1]), dtype=np.float64)
    N_c = np.zeros(kc, dtype=np.int32)
    for f in range(S_f.shape[0]):
        c = int(coarse_of_fine[f])
        S_c[c] = S_c[c] + S_f[f]
        N_c[c] += int(N_f[f])
    return S_c, N_c


def finalize_block(Kb, Vb, a_fine, Cf_kmeans, parent, kc, Cc_kmeans):
    """Renumber a block's fine clusters so that the children of each coarse cluster are contiguous
    (stable in the old id), and compute the stored tables: key/value centroid = mean of the member
    keys/values (Sec. 3.1, 3.2) rounded to bf16; an empty cluster keeps its k-means centroid as
    key centroid, a zero value centroid, and N = 0."""
    kf = Cf_kmeans.shape[0]
    if parent is None:
        order = np.arange(kf)
    else:
        order = np.argsort(parent, kind="stable")
    new_of_old = np.empty(kf, dtype=np.int32)
    new_of_old[order] = np.arange(kf, dtype=np.int32)
    a_new = new_of_old[a_fine]
    Sk, N_f = member_sums(Kb, a_new, kf)
    Sv, _ = member_sums(Vb, a_new, kf)
    Kc_f = _mean_bf16(Sk, N_f)
    Kc_f[N_f == 0] = Cf_kmeans[order][N_f == 0]
    Vc_f = _mean_bf16(Sv, N_f)
    res = dict(fine_of_token=a_new, Kc_f=Kc_f, Vc_f=Vc_f, N_f=N_f, Sk_f=Sk, Sv_f=Sv)
    if parent is not None:
        cof = parent[order].astype(np.int32)
        # member sums of a coarse cluster: its fine clusters' sums (each in sequence order), added in
        # ascending (new) fine id
        Skc, N_c = sums_of_children(Sk, N_f, cof, kc)
        Svc, _ = sums_of_children(Sv, N_f, cof, kc)
        Kc_c = _mean_bf16(Skc, N_c)
        Kc_c[N_c == 0] = Cc_kmeans[N_c == 0]
        Vc_c = _mean_bf16(Svc, N_c)
        res.update(coarse_of_fine=cof, Kc_c=Kc_c, Vc_c=Vc_c, N_c=N_c)
    return res


def cluster_block(Kb, Vb, init_fine, init_coarse, iters, levels):
    """k-means on one block's keys, then (two-level) k-means on the resulting fine centroids."""
    Cf_km, a, _ = lloyd(Kb, init_fine, iters)
    if levels == 2:
        Cc_km, parent, _ = lloyd(Cf_km, init_coarse, iters)
        return finalize_block(Kb, Vb, a, Cf_km, parent, len(init_coarse), Cc_km)
    return finalize_block(Kb, Vb, a, Cf_km, None, 0, None)


def _concat_blocks(K, V, levels, blocks, parts):
    cl = dict(K=K, V=V, levels=levels, blocks=[dict(b) for b in blocks])
    fot = np.zeros(K.shape[0], dtype=np.int32)
    for b, p in zip(blocks, parts):
        fot[b["t0"]:b["t1"]] = p["fine_of_token"] + b["f0"]
    cl["fine_of_token"] = fot
    for key in ("Kc_f", "Vc_f", "N_f"):
        cl[key] = np.concatenate([p[key] for p in parts], axis=0)
    if levels == 2:
        cl["coarse_of_fine"] = np.concatenate([p["coarse_of_fine"] + b["c0"] for b, p in zip(blocks, parts)])
        for key in ("Kc_c", "Vc_c", "N_c"):
            cl[key] = np.concatenate([p[key] for p in parts], axis=0)
    return cl


def cluster_unit(K, V, blocks, init_fine, init_coarse, iters, levels, K_lookup=None):
    """Build the clustered index of one unit.

    blocks: from :func:`plan_blocks`.  init_fine: int32 [n_fine], block-local token indices of the
    seeds, laid out block after block; init_coarse: int32 [n_coarse], block-local fine-cluster
    indices of the coarse seeds (ignored for one level).  K_lookup: the keys the clusters are
    formed on and the key centroids are means of (Sec. 3.1, last paragraph: keys rotated to a
    fixed relative position); K itself is then only attended exactly.  Default: K.
    """
    K, V = _f64(K), _f64(V)
    KL = K if K_lookup is None else _f64(K_lookup)
    assert KL.shape == K.shape
    parts = []
    for b in blocks:
        Kb, Vb = KL[b["t0"]:b["t1"]], V[b["t0"]:b["t1"]]
        fi = _i32(init_fine[b["f0"]:b["f1"]])
        ci = _i32(init_coarse[b["c0"]:b["c1"]]) if levels == 2 else None
        parts.append(cluster_block(Kb, Vb, fi, ci, iters, levels))
    cl = _concat_blocks(K, V, levels, blocks, parts)
    if K_lookup is not None:
        cl["KL"] = KL
    return cl


def clustering_from_assignment(K, V, fine_of_token, n_fine, coarse_of_fine=None, n_coarse=0, K_lookup=None):
    """Stored tables for a given assignment (single block, ids used as given): centroid = bf16(mean
    of members); empty clusters get zero centroids and N = 0.  K_lookup as in :func:`cluster_unit`."""
    K, V = _f64(K), _f64(V)
    KL = K if K_lookup is None else _f64(K_lookup)
    fot = _i32(fine_of_token)
    Sk, N_f = member_sums(KL, fot, n_fine)
    Sv, _ = member_sums(V, fot, n_fine)
    cl = dict(K=K, V=V, levels=1 if coarse_of_fine is None else 2, fine_of_token=fot,
              Kc_f=_mean_bf16(Sk, N_f), Vc_f=_mean_bf16(Sv, N_f), N_f=N_f,
              blocks=[dict(t0=0, t1=K.shape[0], f0=0, f1=n_fine, c0=0, c1=n_coarse)])
    if coarse_of_fine is not None:
        cof = _i32(coarse_of_fine)
        Skc, N_c = sums_of_children(Sk, N_f, cof, n_coarse)      # (see finalize_block)
        Svc, _ = sums_of_children(Sv, N_f, cof, n_coarse)
        cl.update(coarse_of_fine=cof, Kc_c=_mean_bf16(Skc, N_c), Vc_c=_mean_bf16(Svc, N_c), N_c=N_c)
    if K_lookup is not None:
        cl["KL"] = KL
    return cl



# --------------------------------------------------------------------------------------------
# Online cluster update (Sec. 3.3): append tokens to the last block, seed extra centroids from the
# appended tokens, assign the appended tokens once to their nearest centroid and move the touched
# centroids by a running mean, then run a few full Lloyd iterations over the last block; the
# coarse level is refreshed the same way on the block's fine centroids; when the last block reaches
# W + alpha tokens its first W tokens are split off and both parts are clustered afresh.
# --------------------------------------------------------------------------------------------

def update_seed_counts(blocks, n_new, n_new_fine, n_new_coarse, block_w, block_alpha, levels):
    """Sizes of the seed lists one update consumes, in order: new fine seeds (indices into the
    appended tokens), new coarse seeds (indices into the new fine clusters), and -- only if the
    update makes the last block reach W+alpha tokens -- fresh fine seeds for its first W tokens
    (token indices inside that part), for the remaining tokens, then fresh coarse seeds for the two
    parts (fine-cluster indices inside each part)."""
    b = blocks[-1]
    nb = b["t1"] - b["t0"] + n_new
    kf = b["f1"] - b["f0"] + n_new_fine
    kc = (b["c1"] - b["c0"] + n_new_coarse) if levels == 2 else 0
    counts = [n_new_fine, n_new_coarse if levels == 2 else 0, 0, 0, 0, 0]
    if block_w > 0 and nb >= block_w + block_alpha:
        kf1 = kf * block_w // nb
        kc1 = kc * block_w // nb
        counts[2:] = [kf1, kf - kf1, kc1, kc - kc1]
    return counts


def _replace_last_block(cl, K, V, blocks, parts, KL=None):
    """New clustering dict: all blocks but the last as they are, the last one replaced by `parts`
    (one or two finalized blocks whose ranges are blocks[-len(parts):])."""
    levels = int(cl["levels"])
    old_last = cl["blocks"][-1]
    t0, f0, c0 = old_last["t0"], old_last["f0"], old_last["c0"]
    out = dict(K=K, V=V, levels=levels, blocks=[dict(b) for b in blocks])
    if KL is not None:
        out["KL"] = KL
    fot = np.concatenate([cl["fine_of_token"][:t0]] +
                         [p["fine_of_token"] + b["f0"] for b, p in zip(blocks[-len(parts):], parts)]).astype(np.int32)
    out["fine_of_token"] = fot
    for key in ("Kc_f", "Vc_f", "N_f"):
        out[key] = np.concatenate([cl[key][:f0]] + [p[key] for p in parts], axis=0)
    if levels == 2:
        out["coarse_of_fine"] = np.concatenate(
            [cl["coarse_of_fine"][:f0]] + [p["coarse_of_fine"] + b["c0"] for b, p in zip(blocks[-len(parts):], parts)]
        ).astype(np.int32)
        for key in ("Kc_c", "Vc_c", "N_c"):
            out[key] = np.concatenate([cl[key][:c0]] + [p[key] for p in parts], axis=0)
    return out


def update_unit(cl, K_new, V_new, n_new_fine, n_new_coarse, seeds, refine_iters, block_w, block_alpha,
                split_iters=10, K_new_lookup=None):
    """Apply one online update to the clustering dict `cl` of a unit; returns the new dict.
    seeds: int32 list laid out as described by :func:`update_seed_counts`.  K_new_lookup: lookup
    keys of the appended tokens, required iff the index was built on lookup keys; all clustering
    arithmetic below then runs on lookup keys, K_new is only stored."""
    K_new, V_new = _f64(K_new), _f64(V_new)
    has_lookup = "KL" in cl
    assert has_lookup == (K_new_lookup is not None)
    X_new = _f64(K_new_lookup) if has_lookup else K_new
    levels = int(cl["levels"])
    blocks = [dict(b) for b in cl["blocks"]]
    b = blocks[-1]
    t0, t1, f0, f1, c0, c1 = b["t0"], b["t1"], b["f0"], b["f1"], b["c0"], b["c1"]
    n_new = K_new.shape[0]
    counts = update_seed_counts(blocks, n_new, n_new_fine, n_new_coarse, block_w, block_alpha, levels)
    seeds = np.asarray(seeds, dtype=np.int64)
    assert seeds.shape[0] == sum(counts)
    cuts = np.cumsum([0] + counts)
    sd = [seeds[cuts[i]:cuts[i + 1]] for i in range(6)]
    K = np.concatenate([cl["K"], K_new])
    V = np.concatenate([cl["V"], V_new])
    X = np.concatenate([cl["KL"], X_new]) if has_lookup else K     # the keys the clusters are formed on
    Kb, Vb = X[t0:], V[t0:]
    nb = Kb.shape[0]
    kf_old, kf = f1 - f0, f1 - f0 + n_new_fine
    kc_old, kc = c1 - c0, c1 - c0 + (n_new_coarse if levels == 2 else 0)

    # working centroids of the block: the stored fine key centroids, plus the new seeds
    Cw = np.concatenate([cl["Kc_f"][f0:f1], X_new[sd[0]]]) if n_new_fine else cl["Kc_f"][f0:f1].copy()
    Nw = np.concatenate([cl["N_f"][f0:f1], np.zeros(n_new_fine, dtype=np.int32)]).astype(np.int64)
    # one-shot assignment of the appended tokens against frozen centroids
    a_new = assign(X_new, Cw)
    # running mean of the touched centroids: c <- bf16((N c + sum of newly assigned keys) / (N + n))
    Cw = Cw.copy()
    for j in np.unique(a_new):
        s = Nw[j] * Cw[j]
        members = np.flatnonzero(a_new == j)
        for t in members:
            s = s + X_new[t]
        Cw[j] = round_bf16(s / float(Nw[j] + members.size))
    a = np.concatenate([cl["fine_of_token"][t0:t1] - f0, a_new]).astype(np.int32)
    # refinement: full Lloyd iterations over the last block
    if refine_iters > 0:
        Cw, a, _ = lloyd_from(Kb, Cw, refine_iters)
    parent = Ccw = None
    if levels == 2:
        Ccw = cl["Kc_c"][c0:c1]
        if n_new_coarse:
            Ccw = np.concatenate([Ccw, Cw[kf_old + sd[1]]])
        Ccw, parent, _ = lloyd_from(Cw, Ccw, max(1, refine_iters))
    part = finalize_block(Kb, Vb, a, Cw, parent, kc, Ccw)
    b.update(t1=t0 + nb, f1=f0 + kf, c1=c0 + kc)
    KL = X if has_lookup else None
    out = _replace_last_block(cl, K, V, blocks, [part], KL)

    if counts[2] > 0:   # the last block reached W + alpha tokens: split it
        W = block_w
        b1 = dict(t0=t0, t1=t0 + W, f0=f0, f1=f0 + counts[2], c0=c0, c1=c0 + counts[4])
        b2 = dict(t0=t0 + W, t1=t0 + nb, f0=b1["f1"], f1=f0 + kf, c0=b1["c1"], c1=c0 + kc)
        p1 = cluster_block(Kb[:W], Vb[:W], _i32(sd[2]), _i32(sd[4]) if levels == 2 else None, split_iters, levels)
        p2 = cluster_block(Kb[W:], Vb[W:], _i32(sd[3]), _i32(sd[5]) if levels == 2 else None, split_iters, levels)
        out = _replace_last_block(cl, K, V, blocks[:-1] + [b1, b2], [p1, p2], KL)
    return out
