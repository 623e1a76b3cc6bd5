"""Helpers of the GPU parity tests: run the oracle on the same tensors and compare to the bar.

Bar (from the benchmark definition): selected / promising sets bit-exact except where the rank keys
at the cut differ by less than 1e-5 (relative difference of scores = absolute difference of their
logs); outputs within max-abs 2e-2 and mean-rel 5e-3 of the fp64 oracle.
"""
import math

import numpy as np
import torch

from oracle import mp_oracle as O

MAX_ABS = 2e-2
MEAN_REL = 5e-3
NEAR_TIE = 1e-5


def f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def i32(t):
    return t.detach().cpu().numpy().astype(np.int32)


def unit_clustering_from_ctx(ctx, K, V, u):
    """Oracle-side clustering dict of unit u from the library's own tables (so that decode parity
    does not depend on k-means parity).  K, V: [U, n, 128] bf16 tensors in sequence order."""
    if not hasattr(ctx, "_cache_tables"):
        fot, cof = ctx.mp_get_assignments()
        kc_f, vc_f, n_f = ctx.mp_get_centroids(0)
        tabs = dict(fot=i32(fot), kc_f=f64(kc_f), vc_f=f64(vc_f), n_f=i32(n_f))
        if ctx.cfg.levels == 2:
            kc_c, vc_c, n_c = ctx.mp_get_centroids(1)
            tabs.update(cof=i32(cof), kc_c=f64(kc_c), vc_c=f64(vc_c), n_c=i32(n_c))
        torch.cuda.synchronize()
        ctx._cache_tables = tabs
    t = ctx._cache_tables
    cl = dict(K=f64(K[u]), V=f64(V[u]), levels=int(ctx.cfg.levels), fine_of_token=t["fot"][u], Kc_f=t["kc_f"][u],
              Vc_f=t["vc_f"][u], N_f=t["n_f"][u])
    if ctx.cfg.levels == 2:
        cl.update(coarse_of_fine=t["cof"][u], Kc_c=t["kc_c"][u], Vc_c=t["vc_c"][u], N_c=t["n_c"][u])
    return cl


def sets_match(got, want, r, label):
    """Bit-exact, or the differing clusters sit within NEAR_TIE of the cut.  Returns True if exact."""
    got = np.asarray(got).astype(bool)
    want = np.asarray(want).astype(bool)
    if (got == want).all():
        return True
    diff = np.flatnonzero(got != want)
    took = ~np.isnan(r)
    sel_r = r[want & took]
    uns_r = r[(~want) & took]
    edges = []
    if sel_r.size:
        edges.append(sel_r.min())
    if uns_r.size:
        edges.append(uns_r.max())
    for d in diff:
        assert took[d], f"{label}: cluster {d} differs but took no part in ranking"
        gap = min(abs(r[d] - e) for e in edges)
        assert gap < NEAR_TIE, f"{label}: cluster {d} differs, {gap:.3e} away from the cut"
    return False


def check_output(out, ref, label=""):
    err = np.abs(out - ref)
    assert err.max() <= MAX_ABS, f"{label}: max abs err {err.max():.4e}"
    rel = err.mean() / max(np.abs(ref).mean(), 1e-30)
    assert rel <= MEAN_REL, f"{label}: mean rel err {rel:.4e}"
    return err.max(), rel


def rope(x, pos, base=10000.0):
    """Rotary position embedding of x [..., n, d] at the integer positions pos [n] (channel j pairs
    with channel j + d/2), rounded to bf16.  Input generation for the lookup-key tests: the stored
    keys carry their own position, the lookup keys one fixed position."""
    d = x.shape[-1]
    inv = base ** (-torch.arange(0, d // 2, device=x.device, dtype=torch.float64) * 2 / d)
    ang = pos.to(device=x.device, dtype=torch.float64)[:, None] * inv[None, :]
    c, s = torch.cos(ang), torch.sin(ang)
    x = x.to(torch.float64)
    a, b = x[..., : d // 2], x[..., d // 2:]
    return torch.cat([a * c - b * s, a * s + b * c], -1).to(torch.bfloat16)


def signed_permutation(d, seed, device):
    """x -> x[..., perm] * sign: exact in bf16, keeps every dot product and distance."""
    g = torch.Generator().manual_seed(seed)
    perm = torch.randperm(d, generator=g).to(device)
    sign = (torch.randint(0, 2, (d,), generator=g) * 2 - 1).to(device=device, dtype=torch.bfloat16)
    return lambda x: (x[..., perm] * sign).contiguous()


def compare_decode(ctx, q, K, V, key_budget, coarse_budget=0, k_tail=None, v_tail=None, units=None, flags=0,
                   label="", q_lookup=None):
    """Run mp_decode_attention and the oracle on the same inputs; assert the parity bar.
    q [B,Hq,128], K/V [B,Hkv,n,128] (sequence order, the stored keys), tails [B,Hkv,nt,128];
    q_lookup [B,Hq,128]: the query the centroids are compared with (contexts with lookup keys)."""
    B, Hq, d = q.shape
    U, G = ctx.U, ctx.G
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    out = ctx.mp_decode_attention(q, key_budget, coarse_budget, k_tail, v_tail, lse=lse, flags=flags, q_lookup=q_lookup)
    sel = ctx.mp_get_selection()
    cnt = ctx.mp_get_counters()
    torch.cuda.synchronize()
    out64 = f64(out).reshape(U, G, d)
    lse64 = f64(lse).reshape(U, G)
    q64 = f64(q).reshape(U, G, d)
    ql64 = f64(q_lookup).reshape(U, G, d) if q_lookup is not None else None
    Ku, Vu = K.reshape(U, -1, d), V.reshape(U, -1, d)
    fs, rf = sel["fine_selected"].cpu().numpy(), sel["r_fine"].cpu().numpy()
    two = ctx.cfg.levels == 2
    if two:
        cp, rc = sel["coarse_promising"].cpu().numpy(), sel["r_coarse"].cpu().numpy()
    cnt = cnt.cpu().numpy()
    n_exempt = 0
    worst = (0.0, 0.0)
    for u in (range(U) if units is None else units):
        cl = unit_clustering_from_ctx(ctx, Ku, Vu, u)
        Kx = f64(k_tail.reshape(U, -1, d)[u]) if k_tail is not None else None
        Vx = f64(v_tail.reshape(U, -1, d)[u]) if v_tail is not None else None
        res = O.decode_unit(q64[u], cl, key_budget, coarse_budget, Kx, Vx, scale=1 / math.sqrt(d),
                            mp_terms=not (flags & 1), q_lookup=None if ql64 is None else ql64[u])
        exact = True
        if two:
            exact &= sets_match(cp[u], res["promising"], res["r_c"], f"{label} unit {u} coarse")
            both = ~np.isnan(res["r_c"]) & ~np.isnan(rc[u])
            assert (np.isnan(res["r_c"]) == np.isnan(rc[u])).all(), f"{label} unit {u}: coarse rank participation differs"
            np.testing.assert_allclose(rc[u][both], res["r_c"][both], rtol=1e-11, atol=1e-11)
        if exact:
            exact &= sets_match(fs[u], res["selected"], res["r_f"], f"{label} unit {u} fine")
            both = ~np.isnan(res["r_f"]) & ~np.isnan(rf[u])
            assert (np.isnan(res["r_f"]) == np.isnan(rf[u])).all(), f"{label} unit {u}: fine rank participation differs"
            np.testing.assert_allclose(rf[u][both], res["r_f"][both], rtol=1e-11, atol=1e-11)
        if not exact:
            n_exempt += 1
            continue
        nx = 0 if Kx is None else Kx.shape[0]
        assert cnt[u, 0] == res["n_sel_keys"] + nx, f"{label} unit {u}: exact-key counter"
        if np.isinf(res["lse"]).any():
            assert (out64[u] == 0).all()
            continue
        e = check_output(out64[u], res["out"], f"{label} unit {u}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        np.testing.assert_allclose(lse64[u], res["lse"], rtol=3e-5, atol=3e-4)
    return dict(exempt=n_exempt, max_abs=worst[0], mean_rel=worst[1], out=out)
