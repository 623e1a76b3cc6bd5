"""GPU parity of the 8-bit (e4m3 + per-row scale) clustered cache: stored codes and scales against the
oracle's quantiser (bit-exact; value rows as they are, key rows as residuals from their fine cluster's key
centroid), the index against the bf16 context's (identical), and the decode step against the fp64 oracle
run on the dequantised rows (the usual output bar)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _unit_rows(ctx, K, V, u):
    """Sequence-order rows of unit u as fp64 and the key centroid of each row's fine cluster."""
    from tests.gpu_util import f64, i32
    if not hasattr(ctx, "_fp8_tabs"):
        fot, _ = ctx.mp_get_assignments()
        kc, _, _ = ctx.mp_get_centroids(0)
        torch.cuda.synchronize()
        ctx._fp8_tabs = (i32(fot), f64(kc))
    fot, kc = ctx._fp8_tabs
    U = ctx.U
    return f64(K.reshape(U, -1, 128)[u]), f64(V.reshape(U, -1, 128)[u]), kc[u][fot[u]]


def _dequantised(ctx, K, V, units=None):
    """What an 8-bit context attends instead of K, V (sequence order), per unit, fp64 on the host: keys =
    centroid of the fine cluster + dequantised residual, values = dequantised rows."""
    from oracle import mp_oracle as O
    Kd, Vd = {}, {}
    for u in (range(ctx.U) if units is None else units):
        Ku, Vu, cen = _unit_rows(ctx, K, V, u)
        Kd[u] = torch.tensor(O.dequantize_keys_e4m3(*O.quantize_keys_e4m3(Ku, cen), cen))
        Vd[u] = torch.tensor(O.dequantize_rows_e4m3(*O.quantize_rows_e4m3(Vu)))
    return _UnitRows(Kd), _UnitRows(Vd)


def _check_codes(ctx, K, V, units=None):
    from oracle import mp_oracle as O
    kp, vp, perm, _ = ctx.mp_get_layout()
    assert kp is None and vp is None
    kc, vc, sc = ctx.mp_get_kv_codes()
    torch.cuda.synchronize()
    if hasattr(ctx, "_fp8_tabs"):
        del ctx._fp8_tabs                        # (the index may have changed since the last look)
    for u in (range(ctx.U) if units is None else units):
        Ku, Vu, cen = _unit_rows(ctx, K, V, u)
        idx = perm[u].cpu().numpy()
        want_c, want_s = O.quantize_keys_e4m3(Ku[idx], cen[idx])
        np.testing.assert_array_equal(sc[u, :, 0].cpu().numpy(), want_s)
        np.testing.assert_array_equal(kc[u].cpu().numpy(), want_c)
        want_c, want_s = O.quantize_rows_e4m3(Vu[idx])
        np.testing.assert_array_equal(sc[u, :, 1].cpu().numpy(), want_s)
        np.testing.assert_array_equal(vc[u].cpu().numpy(), want_c)


class _UnitRows:
    """Stands in for a [U, n, 128] tensor where only some units' rows were worked out."""
    def __init__(self, rows):
        self.rows = rows

    def reshape(self, *shape):
        return self

    def __getitem__(self, u):
        return self.rows[u]


CASES = [
    dict(name="one_level_g4", B=1, Hq=4, Hkv=1, n=4096, modes=64, levels=1, nf=64, nc=0,
         budgets=[(256, 0), (0, 0), (4096, 0), (1000, 0)], tail=0),
    dict(name="two_level_ragged_g4", B=1, Hq=8, Hkv=2, n=3001, modes=96, levels=2, nf=96, nc=12,
         budgets=[(400, 1200), (0, 0), (3001, 3001), (150, 3001), (2, 3001)], tail=37),
    dict(name="group5", B=2, Hq=5, Hkv=1, n=1500, modes=48, levels=2, nf=48, nc=6, budgets=[(200, 600)], tail=130),
    dict(name="group8", B=1, Hq=8, Hkv=1, n=2100, modes=32, levels=1, nf=70, nc=0, budgets=[(300, 0), (2100, 0)], tail=5),
    dict(name="group1_many_units", B=3, Hq=3, Hkv=3, n=900, modes=30, levels=2, nf=40, nc=5, budgets=[(100, 400)], tail=0),
    dict(name="group6", B=1, Hq=6, Hkv=1, n=1000, modes=40, levels=2, nf=50, nc=6, budgets=[(120, 480)], tail=17),
    # long streams: chunks of 512 rows and more (the eight-iteration strips of the value pass)
    dict(name="long_g4", B=1, Hq=4, Hkv=1, n=20000, modes=200, levels=2, nf=400, nc=40,
         budgets=[(6000, 12000), (20000, 20000)], tail=0),
    dict(name="long_g2", B=1, Hq=2, Hkv=1, n=9000, modes=100, levels=1, nf=150, nc=0, budgets=[(5000, 0)], tail=0),
    dict(name="group3", B=1, Hq=3, Hkv=1, n=1000, modes=40, levels=1, nf=50, nc=0, budgets=[(200, 0)], tail=0),
    dict(name="group7", B=1, Hq=7, Hkv=1, n=1000, modes=40, levels=1, nf=50, nc=0, budgets=[(333, 0)], tail=9),
    # more entries per level than the scoring kernel keeps in LDS: its working arrays, and the logit shares it
    # hands to the value pass, come from the global-memory instantiation
    dict(name="one_level_1300_clusters", B=1, Hq=4, Hkv=1, n=5200, modes=400, levels=1, nf=1300, nc=0,
         budgets=[(700, 0), (5200, 0)], tail=0),
    dict(name="two_level_1300_candidates", B=1, Hq=4, Hkv=1, n=7800, modes=500, levels=2, nf=2600, nc=40,
         budgets=[(900, 3900), (300, 7800)], tail=9),
]


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_decode_on_8bit_rows_matches_oracle_on_dequantised_rows(case):
    from paper_2506_13059_amd import binding as mp
    from tests.gpu_util import compare_decode
    from tests.test_gpu_decode import _mk, _oracle_clusterings, _install
    c = case
    print(f"case {c['name']}", flush=True)
    K, V, q = _mk(c["B"], c["Hq"], c["Hkv"], c["n"], c["modes"], seed=700 + c["n"], softness=0.5, n_sets=1)
    # rows of very different magnitude, an all-zero key row and an all-zero value row
    K = K.clone(); V = V.clone()
    V[:, :, 7::11] *= 16
    K[:, :, 5] = 0
    V[:, :, 6] = 0
    K[:, :, 9] = K[:, :, 8]                       # (two equal keys: one of them may be its cluster's centroid)
    cls = _oracle_clusterings(K, V, c["levels"], c["nf"], c["nc"], iters=2, seed=c["n"])
    kw = dict(max_tokens=c["n"] + 64, levels=c["levels"], max_fine=c["nf"] + 8,
              max_coarse=c["nc"] + 3 if c["levels"] == 2 else 0, max_tail=max(c["tail"], 1))
    ctx = mp.MpContext(c["B"], c["Hq"], c["Hkv"], kv_format=mp.MP_KV_E4M3, **kw)
    ref = mp.MpContext(c["B"], c["Hq"], c["Hkv"], **kw)
    _install(ctx, K, V, cls, c["levels"])
    _install(ref, K, V, cls, c["levels"])
    # the index does not depend on the storage format
    for lvl in range(c["levels"]):
        for a, b in zip(ctx.mp_get_centroids(lvl), ref.mp_get_centroids(lvl)):
            assert torch.equal(a, b)
    for a, b in zip(ctx.mp_get_layout()[2:], ref.mp_get_layout()[2:]):
        assert torch.equal(a, b)
    ref.close()
    _check_codes(ctx, K, V)
    Kd, Vd = _dequantised(ctx, K, V)
    kt = vt = None
    if c["tail"]:
        g = torch.Generator(device="cuda").manual_seed(9)
        kt = (K[:, :, :c["tail"]].float() + 0.1 * torch.randn(K[:, :, :c["tail"]].shape, generator=g, device="cuda")
              ).to(torch.bfloat16).contiguous()
        vt = torch.randn(kt.shape, generator=g, device="cuda").to(torch.bfloat16)
    for kb, cb in c["budgets"]:
        r = compare_decode(ctx, q[0].contiguous(), Kd, Vd, kb, cb, kt, vt, label=f"{c['name']} kb={kb} cb={cb}")
        assert r["exempt"] == 0
    ctx.close()


def test_kmeans_build_and_online_update_store_8bit_rows():
    """mp_cluster_kv (blockwise) and mp_update_clusters write the quantised rows of the layout they produce,
    and that layout equals the bf16 context's."""
    from paper_2506_13059_amd import binding as mp
    from tests.test_gpu_decode import _mk
    B, Hq, Hkv, n, n_new = 1, 4, 2, 2600, 128
    K, V, q = _mk(B, Hq, Hkv, n + n_new, 60, seed=41)
    kw = dict(max_tokens=n + n_new, levels=2, max_fine=200, max_coarse=24, block_w=1024, block_alpha=512)
    ctx = mp.MpContext(B, Hq, Hkv, kv_format=mp.MP_KV_E4M3, **kw)
    ref = mp.MpContext(B, Hq, Hkv, **kw)
    K0, V0 = K[:, :, :n].contiguous(), V[:, :, :n].contiguous()
    K1, V1 = K[:, :, n:].contiguous(), V[:, :, n:].contiguous()
    for c in (ctx, ref):
        c.mp_cluster_kv(K0, V0, 160, 20, iters=3, seed=5)
    _check_codes(ctx, K0, V0)
    for c in (ctx, ref):
        c.mp_update_clusters(K1, V1, 8, 1, refine_iters=2, seed=6)
    for a, b in zip(ctx.mp_get_layout()[2:], ref.mp_get_layout()[2:]):
        assert torch.equal(a, b)
    for lvl in (0, 1):
        for a, b in zip(ctx.mp_get_centroids(lvl), ref.mp_get_centroids(lvl)):
            assert torch.equal(a, b)
    _check_codes(ctx, K, V)
    ctx.close(); ref.close()


def test_getters_reject_the_other_format():
    from paper_2506_13059_amd import binding as mp
    from tests.test_gpu_decode import _mk
    K, V, q = _mk(1, 2, 1, 300, 8, seed=3)
    a = mp.MpContext(1, 2, 1, max_tokens=300, levels=1, max_fine=8)
    a.mp_cluster_kv(K, V, 8, iters=1, seed=1)
    with pytest.raises(mp.MpError) as e:
        a.mp_get_kv_codes()
    assert e.value.status == 1
    a.close()
    with pytest.raises(mp.MpError) as e:
        mp.MpContext(1, 2, 1, max_tokens=300, levels=1, max_fine=8, kv_format=7)
    assert e.value.status == 1


@pytest.mark.parametrize("kb", [8192, 4096])
def test_full_size_decode_on_8bit_rows_sampled_units_match_oracle(kb):
    """The benchmark's workload (batch 16, 32/8 heads, 131072 tokens, 4096 + 256 clusters, W = 8192) with
    the 8-bit cache, in the launch configuration bench.py times, on sampled units."""
    from paper_2506_13059_amd import binding as mp, inputs
    from tests.gpu_util import compare_decode
    free, total = torch.cuda.mem_get_info()
    if free < 40 * 2 ** 30:
        pytest.skip("needs 40 GiB of free device memory")
    w = inputs.WORKLOADS["cfg3_128k_b16"]
    data = inputs.make_workload(w, "cuda", seed=3100, n_query_sets=1)
    ctx = mp.MpContext(w.batch, w.n_q_heads, w.n_kv_heads, max_tokens=w.context, levels=2, max_fine=w.n_fine,
                       max_coarse=w.n_coarse, block_w=w.block_w, block_alpha=w.block_alpha, max_tail=256,
                       kv_format=mp.MP_KV_E4M3)
    ctx.mp_cluster_kv(data["K"], data["V"], w.n_fine, w.n_coarse, iters=2, init_fine=data["init_fine"],
                      init_coarse=data["init_coarse"])
    units = [1, 70, 126]
    _check_codes(ctx, data["K"], data["V"], units=units)
    Kd, Vd = _dequantised(ctx, data["K"], data["V"], units=units)
    r = compare_decode(ctx, data["q"][0].contiguous(), Kd, Vd, kb, 2 * kb, units=units,
                       label=f"cfg3 8-bit kb={kb}")
    assert r["exempt"] == 0
    ctx.close()


def test_8bit_context_refuses_lookup_keys_and_a_lookup_query():
    from paper_2506_13059_amd import binding as mp
    from tests.test_gpu_decode import _mk
    with pytest.raises(mp.MpError) as e:
        mp.MpContext(1, 2, 1, max_tokens=300, levels=1, max_fine=8, kv_format=mp.MP_KV_E4M3, lookup_keys=True)
    assert e.value.status == 1
    K, V, q = _mk(1, 2, 1, 300, 8, seed=3)
    ctx = mp.MpContext(1, 2, 1, max_tokens=300, levels=1, max_fine=8, kv_format=mp.MP_KV_E4M3)
    ctx.mp_cluster_kv(K, V, 8, iters=1, seed=1)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_decode_attention(q[0].contiguous(), 100, q_lookup=q[0].contiguous())
    assert e.value.status == 1
    ctx.mp_decode_attention(q[0].contiguous(), 100)
    ctx.close()
