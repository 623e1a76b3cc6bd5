"""GPU parity: a generation loop through mp_decode_step (library-managed local buffer of L .. 2L
recent tokens plus sink tokens, cluster refresh every L steps; Sec. 4, Sec. 5.1) against the
oracle composed step by step: decode over the oracle's clustering with the buffer as exact extra
tokens, and the oracle's online update whenever the buffer is full."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _loop(levels, steps, L, n_sink, n_recent0, lookup=False, eight_bit=False):
    """lookup: the stored keys carry a rotary embedding of their own position, the lookup keys and
    the lookup query one of a fixed position (Sec. 3.1, last paragraph).
    eight_bit: the clustered cache holds e4m3 codes; the oracle then attends the dequantised rows
    (keys = their fine cluster's key centroid + dequantised residual), the buffer stays bf16."""
    from paper_2506_13059_amd import binding as mp, inputs
    from oracle import mp_oracle as O
    from tests.gpu_util import f64, check_output, sets_match, rope

    def stored_and_lookup(X, pos0):
        if not lookup:
            return X, None
        return rope(X, pos0 + torch.arange(X.shape[-2])), rope(X, torch.full((X.shape[-2],), 4096))
    def attended(cl):
        if not eight_bit:
            return cl
        cen = cl["Kc_f"][cl["fine_of_token"]]
        view = dict(cl)
        view["K"] = O.dequantize_keys_e4m3(*O.quantize_keys_e4m3(cl["K"], cen), cen)
        view["V"] = O.dequantize_rows_e4m3(*O.quantize_rows_e4m3(cl["V"]))
        return view
    B, Hq, Hkv, n0, W, alpha = 1, 4, 2, 700, 512, 256
    nf, nc = 44, 6
    U, G = B * Hkv, Hq // Hkv
    seed = 41
    centers = inputs.make_modes(U, 40, "cuda", seed)
    K, V = inputs.draw_tokens(centers, n0, seed + 1)
    K, KL = stored_and_lookup(K, 0)
    blocks = mp.mp_plan_blocks(n0, W, alpha, nf, nc if levels == 2 else 0)
    init_f, init_c = inputs.draw_seeds(U, blocks, levels, seed + 3)
    cap = n0 + steps + 2 * L
    ctx = mp.MpContext(B, Hq, Hkv, max_tokens=cap, levels=levels, max_fine=nf + 8 * (steps // L + 2),
                       max_coarse=(nc + 2 * (steps // L + 2)) if levels == 2 else 0, block_w=W, block_alpha=alpha,
                       max_tail=n_sink + 2 * L, lookup_keys=lookup, kv_format=mp.MP_KV_E4M3 if eight_bit else mp.MP_KV_BF16)
    ctx.mp_cluster_kv(K.view(B, Hkv, n0, 128), V.view(B, Hkv, n0, 128), nf, nc, iters=4, init_fine=init_f,
                      init_coarse=init_c if levels == 2 else None, k_lookup=KL.view(B, Hkv, n0, 128) if lookup else None)
    K64, V64 = f64(K), f64(V)
    KL64 = f64(KL) if lookup else [None] * U
    cls = [O.cluster_unit(K64[u], V64[u], blocks, init_f[u].numpy(), init_c[u].numpy() if levels == 2 else None, 4, levels,
                          K_lookup=KL64[u]) for u in range(U)]
    g = torch.Generator(device="cuda").manual_seed(seed + 5)
    ks = torch.randn(B, Hkv, n_sink, 128, generator=g, device="cuda").to(torch.bfloat16)
    vs = torch.randn(B, Hkv, n_sink, 128, generator=g, device="cuda").to(torch.bfloat16)
    kr, vr = inputs.draw_tokens(centers, max(n_recent0, 1), seed + 6)
    kr, krl = stored_and_lookup(kr[:, :n_recent0], n0)
    kr, vr = kr.reshape(B, Hkv, n_recent0, 128), vr[:, :n_recent0].reshape(B, Hkv, n_recent0, 128)
    ctx.mp_local_buffer_init(L, ks if n_sink else None, vs if n_sink else None, kr.contiguous() if n_recent0 else None,
                             vr.contiguous() if n_recent0 else None,
                             k_recent_lookup=krl.reshape(B, Hkv, n_recent0, 128).contiguous() if lookup and n_recent0 else None)
    # the oracle's view of the buffer: per unit lists of rows (fp64)
    sink_k, sink_v = f64(ks).reshape(U, n_sink, 128), f64(vs).reshape(U, n_sink, 128)
    rec_k = [list(f64(kr).reshape(U, n_recent0, 128)[u]) for u in range(U)]
    rec_v = [list(f64(vr).reshape(U, n_recent0, 128)[u]) for u in range(U)]
    rec_kl = [list(f64(krl).reshape(U, n_recent0, 128)[u]) if lookup else [] for u in range(U)]
    rng = np.random.default_rng(seed)
    kb, cb = 96, 260
    refreshes = 0
    for t in range(steps):
        centers = inputs.drift_modes(centers, seed + 100 + t)
        kn, vn = inputs.draw_tokens(centers, 1, seed + 200 + t)
        q = inputs.draw_queries(centers, G, 1, seed + 300 + t, softness=0.4).view(B, Hq, 128)
        pos = n0 + n_recent0 + t
        kn, knl = stored_and_lookup(kn, pos)
        q, ql = (rope(q, torch.full((Hq,), pos)), rope(q, torch.full((Hq,), 4100))) if lookup else (q, None)
        size = ctx.mp_local_buffer_size()
        assert size == dict(window=L, n_sink=n_sink, n_recent=len(rec_k[0]))
        will_refresh = size["n_recent"] + 1 == 2 * L
        seeds = None
        if will_refresh:
            counts = ctx.mp_update_seed_counts(L, 3, 1 if levels == 2 else 0)
            nb = cls[0]["blocks"][-1]["t1"] - cls[0]["blocks"][-1]["t0"] + L
            lims = [L, 3, W, nb - W, counts[2], counts[3]]
            seeds = np.stack([np.concatenate([rng.choice(max(l, 1), c, replace=False) for l, c in zip(lims, counts)])
                              for _ in range(U)]).astype(np.int32)
        print(f"step {t}: recent {size['n_recent']} refresh {will_refresh}", flush=True)
        lse = torch.empty(B, Hq, dtype=torch.float32, device="cuda")
        out = ctx.mp_decode_step(q, kn.view(B, Hkv, 1, 128), vn.view(B, Hkv, 1, 128), kb, cb, n_new_fine=3,
                                 n_new_coarse=1 if levels == 2 else 0, refine_iters=2, split_iters=4,
                                 seeds=None if seeds is None else torch.tensor(seeds), lse=lse, q_lookup=ql,
                                 k_new_lookup=knl.view(B, Hkv, 1, 128) if lookup else None)
        sel = ctx.mp_get_selection() if not will_refresh else None      # (the refresh re-numbers clusters)
        torch.cuda.synchronize()
        kn64, vn64, q64 = f64(kn).reshape(U, 128), f64(vn).reshape(U, 128), f64(q).reshape(U, G, 128)
        knl64, ql64 = (f64(knl).reshape(U, 128), f64(ql).reshape(U, G, 128)) if lookup else (None, [None] * U)
        for u in range(U):
            rec_k[u].append(kn64[u])
            rec_v[u].append(vn64[u])
            if lookup:
                rec_kl[u].append(knl64[u])
            Kx = np.concatenate([sink_k[u], np.stack(rec_k[u])]) if n_sink else np.stack(rec_k[u])
            Vx = np.concatenate([sink_v[u], np.stack(rec_v[u])]) if n_sink else np.stack(rec_v[u])
            res = O.decode_unit(q64[u], attended(cls[u]), kb, cb, Kx, Vx, q_lookup=ql64[u])
            check_output(f64(out).reshape(U, G, 128)[u], res["out"], f"step {t} unit {u}")
            np.testing.assert_allclose(lse.view(U, G)[u].cpu().numpy(), res["lse"], rtol=3e-5, atol=3e-4)
            if sel is not None:
                assert sets_match(sel["fine_selected"][u].cpu().numpy(), res["selected"], res["r_f"], f"step {t} unit {u}")
            if will_refresh:
                cls[u] = O.update_unit(cls[u], np.stack(rec_k[u][:L]), np.stack(rec_v[u][:L]), 3, 1 if levels == 2 else 0,
                                       seeds[u], 2, W, alpha, split_iters=4,
                                       K_new_lookup=np.stack(rec_kl[u][:L]) if lookup else None)
                rec_k[u], rec_v[u], rec_kl[u] = rec_k[u][L:], rec_v[u][L:], rec_kl[u][L:]
        refreshes += will_refresh
    sizes = ctx.mp_get_sizes()
    assert sizes["n_tokens"] == n0 + refreshes * L == cls[0]["K"].shape[0]
    fot, _ = ctx.mp_get_assignments()
    torch.cuda.synchronize()
    for u in range(U):
        np.testing.assert_array_equal(fot[u].cpu().numpy(), cls[u]["fine_of_token"])
    ctx.close()
    return refreshes, sizes


def test_generation_two_levels_with_sinks_and_a_split():
    # one block of 700 tokens (W = 512, alpha = 256) grows by 16 per refresh; the fifth refresh makes it
    # reach W + alpha = 768 tokens and splits it
    refreshes, sizes = _loop(levels=2, steps=80, L=16, n_sink=3, n_recent0=20)
    assert refreshes == 5 and sizes["n_blocks"] == 2


def test_generation_with_the_8bit_cache_through_refreshes_and_a_split():
    refreshes, sizes = _loop(levels=2, steps=80, L=16, n_sink=3, n_recent0=20, eight_bit=True)
    assert refreshes == 5 and sizes["n_blocks"] == 2


def test_generation_one_level_from_an_empty_buffer():
    refreshes, sizes = _loop(levels=1, steps=40, L=8, n_sink=0, n_recent0=0)
    assert refreshes == 4


def test_local_buffer_argument_errors():
    from paper_2506_13059_amd import binding as mp
    ctx = mp.MpContext(1, 2, 1, max_tokens=64, levels=1, max_fine=4, max_tail=8)
    z = torch.zeros(1, 1, 4, 128, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(1, 2, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mp.MpError) as e:
        ctx.mp_local_buffer_size()
    assert e.value.status == mp.MP_ESTATE
    with pytest.raises(mp.MpError) as e:
        ctx.mp_local_buffer_init(5)                       # 2 * 5 > max_tail
    assert e.value.status == mp.MP_ECAPACITY
    with pytest.raises(mp.MpError) as e:
        ctx.mp_local_buffer_init(2, k_recent=z, v_recent=z)    # n_recent must stay below 2 * window
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_local_buffer_init(2)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_decode_step(q, z[:, :, :1].contiguous(), z[:, :, :1].contiguous(), 8)   # no index yet
    assert e.value.status == mp.MP_ESTATE
    ctx.close()


def test_generation_with_lookup_keys_and_a_lookup_query():
    refreshes, sizes = _loop(levels=2, steps=80, L=16, n_sink=3, n_recent0=20, lookup=True)
    assert refreshes == 5 and sizes["n_blocks"] == 2
