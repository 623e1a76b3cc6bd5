"""GPU parity: index tables and the multipole decode step against the fp64 oracle.

The clustering is produced by the oracle's k-means (or drawn at random) and installed with
mp_set_clustering, so these tests isolate layout, scoring, selection, the value pass and the merge.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _mk(B, Hq, Hkv, n, modes, seed, softness=1.0, n_sets=1):
    from paper_2506_13059_amd import inputs
    U = B * Hkv
    centers = inputs.make_modes(U, modes, "cuda", seed)
    K, V = inputs.draw_tokens(centers, n, seed + 1)
    q = inputs.draw_queries(centers, Hq // Hkv, n_sets, seed + 2, softness=softness)
    return (K.view(B, Hkv, n, 128), V.view(B, Hkv, n, 128), q.view(n_sets, B, Hq, 128))


def _oracle_clusterings(K, V, levels, n_fine, n_coarse, iters, seed):
    """Per-unit clusterings from the oracle's k-means (single block)."""
    from oracle import mp_oracle as O
    from tests.gpu_util import f64
    U = K.shape[0] * K.shape[1]
    n = K.shape[2]
    Ku, Vu = f64(K).reshape(U, n, 128), f64(V).reshape(U, n, 128)
    rng = np.random.default_rng(seed)
    cls = []
    blocks = O.plan_blocks(n, 0, 0, n_fine, n_coarse if levels == 2 else 0)
    for u in range(U):
        init_f = rng.choice(n, n_fine, replace=False).astype(np.int32)
        init_c = rng.choice(n_fine, n_coarse, replace=False).astype(np.int32) if levels == 2 else None
        cls.append(O.cluster_unit(Ku[u], Vu[u], blocks, init_f, init_c, iters, levels))
    return cls


def _install(ctx, K, V, cls, levels):
    fot = torch.tensor(np.stack([c["fine_of_token"] for c in cls]), dtype=torch.int32, device="cuda")
    cof = torch.tensor(np.stack([c["coarse_of_fine"] for c in cls]), dtype=torch.int32, device="cuda") \
        if levels == 2 else None
    n_fine = cls[0]["N_f"].shape[0]
    n_coarse = cls[0]["N_c"].shape[0] if levels == 2 else 0
    ctx.mp_set_clustering(K, V, fot, n_fine, cof, n_coarse)


def _check_tables(ctx, K, V, cls, levels):
    """Stored tables and layout against the oracle's (bit-exact) and against their own definition."""
    from tests.gpu_util import f64, i32
    U, n = ctx.U, K.shape[2]
    kc, vc, nm = ctx.mp_get_centroids(0)
    fot, cof = ctx.mp_get_assignments()
    kp, vp, perm, fstart = ctx.mp_get_layout()
    torch.cuda.synchronize()
    kc, vc, nm, fot, perm, fstart = f64(kc), f64(vc), i32(nm), i32(fot), i32(perm), i32(fstart)
    Ku, Vu = K.reshape(U, n, 128), V.reshape(U, n, 128)
    for u in range(U):
        c = cls[u]
        np.testing.assert_array_equal(fot[u], c["fine_of_token"])
        np.testing.assert_array_equal(nm[u], c["N_f"])
        live = c["N_f"] > 0
        np.testing.assert_array_equal(kc[u][live], c["Kc_f"][live])
        np.testing.assert_array_equal(vc[u], c["Vc_f"])
        # layout: cluster after cluster, sequence order inside a cluster, rows are the original rows
        np.testing.assert_array_equal(np.diff(fstart[u]), c["N_f"])
        assert sorted(perm[u].tolist()) == list(range(n))
        f_of_row = c["fine_of_token"][perm[u]]
        assert (np.diff(f_of_row) >= 0).all()
        same = np.diff(f_of_row) == 0
        assert (np.diff(perm[u])[same] > 0).all()
        idx = torch.tensor(perm[u], dtype=torch.long, device="cuda")
        assert torch.equal(kp[u], Ku[u][idx]) and torch.equal(vp[u], Vu[u][idx])
    if levels == 2:
        kcc, vcc, nmc = ctx.mp_get_centroids(1)
        torch.cuda.synchronize()
        kcc, vcc, nmc, cof = f64(kcc), f64(vcc), i32(nmc), i32(cof)
        for u in range(U):
            c = cls[u]
            np.testing.assert_array_equal(cof[u], c["coarse_of_fine"])
            np.testing.assert_array_equal(nmc[u], c["N_c"])
            live = c["N_c"] > 0
            np.testing.assert_array_equal(kcc[u][live], c["Kc_c"][live])
            np.testing.assert_array_equal(vcc[u][live], c["Vc_c"][live])


CASES = [
    # B, Hq, Hkv, n, modes, levels, n_fine, n_coarse, budgets [(key, coarse)], n_tail
    dict(name="cfg0", B=1, Hq=4, Hkv=1, n=4096, modes=64, levels=1, nf=64, nc=0,
         budgets=[(256, 0), (0, 0), (4096, 0), (1000, 0), (1, 0)], tail=0),
    # (a key budget below the smallest cluster: nothing is selected, the selected-key workgroups carry only centroid terms)
    dict(name="two_level_ragged", B=1, Hq=8, Hkv=2, n=3001, modes=96, levels=2, nf=96, nc=12,
         budgets=[(400, 1200), (0, 0), (3001, 3001), (700, 300), (150, 3001), (2, 3001)], tail=37),
    dict(name="group5", B=2, Hq=5, Hkv=1, n=1500, modes=48, levels=2, nf=48, nc=6,
         budgets=[(200, 600), (64, 5000)], tail=130),
    dict(name="group8_one_level", B=1, Hq=8, Hkv=1, n=2100, modes=32, levels=1, nf=70, nc=0,
         budgets=[(300, 0), (2100, 0)], tail=5),
    dict(name="mha_many_units", B=3, Hq=3, Hkv=3, n=900, modes=30, levels=2, nf=40, nc=5,
         budgets=[(100, 400)], tail=0),
    dict(name="group2", B=1, Hq=4, Hkv=2, n=1100, modes=40, levels=2, nf=40, nc=5, budgets=[(150, 500)], tail=3),
    dict(name="group3", B=1, Hq=3, Hkv=1, n=1000, modes=40, levels=1, nf=50, nc=0, budgets=[(200, 0)], tail=0),
    dict(name="group6", B=1, Hq=6, Hkv=1, n=1000, modes=40, levels=2, nf=50, nc=6, budgets=[(120, 480)], tail=17),
    dict(name="group7", B=1, Hq=7, Hkv=1, n=1000, modes=40, levels=1, nf=50, nc=0, budgets=[(333, 0)], tail=0),
    # more entries per level than the scoring kernel keeps in LDS (1024): working arrays in global scratch
    dict(name="one_level_1300_clusters", B=1, Hq=4, Hkv=1, n=5200, modes=400, levels=1, nf=1300, nc=0,
         budgets=[(700, 0), (0, 0), (5200, 0)], tail=0, iters=2),
    dict(name="two_level_1300_candidates", B=1, Hq=4, Hkv=1, n=7800, modes=500, levels=2, nf=2600, nc=40,
         budgets=[(900, 3900), (300, 7800)], tail=9, iters=2),
]


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
@pytest.mark.parametrize("softness", [1.0, 0.1])
def test_decode_matches_oracle(case, softness):
    from paper_2506_13059_amd import binding as mp
    from tests.gpu_util import compare_decode
    c = case
    print(f"case {c['name']} softness {softness}", flush=True)
    K, V, q = _mk(c["B"], c["Hq"], c["Hkv"], c["n"], c["modes"], seed=100 + c["n"], softness=softness, n_sets=2)
    cls = _oracle_clusterings(K, V, c["levels"], c["nf"], c["nc"], iters=2, seed=c["n"])
    ctx = mp.MpContext(c["B"], c["Hq"], c["Hkv"], max_tokens=c["n"] + 64, levels=c["levels"], max_fine=c["nf"] + 8,
                       max_coarse=c["nc"] + 3 if c["levels"] == 2 else 0, max_tail=max(c["tail"], 1))
    _install(ctx, K, V, cls, c["levels"])
    _check_tables(ctx, K, V, cls, c["levels"])
    kt = vt = None
    if c["tail"]:
        g = torch.Generator(device="cuda").manual_seed(9)
        kt = (K[:, :, :c["tail"]].float() + 0.1 * torch.randn(K[:, :, :c["tail"]].shape, generator=g, device="cuda")
              ).to(torch.bfloat16).contiguous()
        vt = torch.randn(kt.shape, generator=g, device="cuda").to(torch.bfloat16)
    exempt = 0
    for s in range(q.shape[0]):
        for kb, cb in c["budgets"]:
            r = compare_decode(ctx, q[s].contiguous(), K, V, kb, cb, kt, vt, label=f"{c['name']} kb={kb} cb={cb}")
            exempt += r["exempt"]
    assert exempt == 0     # fp64 rank keys: no near-tie exemption should ever be needed on these inputs
    ctx.close()


def test_no_multipole_flag_and_empty_clusters():
    from paper_2506_13059_amd import binding as mp
    from tests.gpu_util import compare_decode
    from oracle import mp_oracle as O
    from tests.gpu_util import f64
    K, V, q = _mk(1, 4, 1, 800, 16, seed=7, softness=0.2)
    rng = np.random.default_rng(3)
    fot = (rng.integers(0, 10, size=800) * 2).astype(np.int32)          # odd fine ids stay empty
    cof = (np.arange(20) // 5).astype(np.int32)
    cl = O.clustering_from_assignment(f64(K)[0, 0], f64(V)[0, 0], fot, 20, cof, 5)   # coarse 4 is empty
    ctx = mp.MpContext(1, 4, 1, max_tokens=800, levels=2, max_fine=20, max_coarse=5, max_tail=0)
    ctx.mp_set_clustering(K, V, torch.tensor(fot, device="cuda")[None], 20, torch.tensor(cof, device="cuda")[None], 5)
    _check_tables(ctx, K, V, [cl], 2)
    for flags in (0, mp.MP_DECODE_NO_MULTIPOLE):
        for kb, cb in [(100, 400), (0, 0), (800, 800)]:
            compare_decode(ctx, q[0].contiguous(), K, V, kb, cb, flags=flags, label=f"flags={flags} kb={kb}")
    ctx.close()


def test_exact_ties_take_lower_id_first():
    """Duplicate clusters (same keys) give equal rank keys: the lower id must win the last slot."""
    from paper_2506_13059_amd import binding as mp
    from tests.gpu_util import compare_decode
    g = torch.Generator(device="cuda").manual_seed(5)
    base = torch.randn(1, 1, 8, 128, generator=g, device="cuda")
    K = base.repeat(1, 1, 6, 1).to(torch.bfloat16)                      # 48 tokens: 6 copies of 8 keys
    V = torch.randn(1, 1, 48, 128, generator=g, device="cuda").to(torch.bfloat16)
    q = (base[:, 0, :2] * 0.5).to(torch.bfloat16).contiguous()          # [1, 2, 128]
    fot = (torch.arange(48, device="cuda", dtype=torch.int32) // 8)[None]   # cluster j = copy j: all identical
    ctx = mp.MpContext(1, 2, 1, max_tokens=48, levels=1, max_fine=6, max_tail=0)
    ctx.mp_set_clustering(K, V, fot.contiguous(), 6)
    for kb in (0, 8, 15, 16, 24, 47, 48):
        compare_decode(ctx, q, K, V, kb, label=f"ties kb={kb}")
        sel = ctx.mp_get_selection()["fine_selected"][0].cpu().numpy()
        assert sel.tolist() == [1] * (kb // 8) + [0] * (6 - kb // 8)
    ctx.close()


def test_tail_in_a_buffer_of_fixed_capacity():
    """The first n_tail rows of a larger tail buffer give the same bits as a densely packed tail."""
    from paper_2506_13059_amd import binding as mp
    B, Hq, Hkv, n = 2, 4, 2, 600
    K, V, q = _mk(B, Hq, Hkv, n, 12, seed=21, softness=0.5)
    g = torch.Generator(device="cuda").manual_seed(22)
    fot = torch.randint(0, 12, (B * Hkv, n), generator=g, device="cuda").to(torch.int32)
    ctx = mp.MpContext(B, Hq, Hkv, max_tokens=n, levels=1, max_fine=12, max_tail=32)
    ctx.mp_set_clustering(K, V, fot, 12)
    kt = torch.randn(B, Hkv, 32, 128, generator=g, device="cuda").to(torch.bfloat16)
    vt = torch.randn(B, Hkv, 32, 128, generator=g, device="cuda").to(torch.bfloat16)
    for n_tail in (0, 1, 7, 32):
        a = ctx.mp_decode_attention(q[0].contiguous(), 100, k_tail=kt, v_tail=vt, n_tail=n_tail)
        if n_tail:
            b = ctx.mp_decode_attention(q[0].contiguous(), 100, k_tail=kt[:, :, :n_tail].contiguous(),
                                        v_tail=vt[:, :, :n_tail].contiguous())
        else:
            b = ctx.mp_decode_attention(q[0].contiguous(), 100)
        torch.cuda.synchronize()
        assert torch.equal(a, b), f"n_tail={n_tail}"
    with pytest.raises(mp.MpError):
        lib_call = mp.lib().mp_decode_attention      # 0 < tail_stride < n_tail is refused
        st = lib_call(ctx.h, q[0].contiguous().data_ptr(), None, kt.data_ptr(), vt.data_ptr(), 8, 4, 100, 0, 0,
                      torch.empty_like(q[0]).data_ptr(), None, None)
        mp._check(st, ctx.h)
    ctx.close()


@pytest.mark.parametrize("eight_bit", [False, True], ids=["bf16_cache", "8bit_cache"])
def test_decode_step_in_a_hip_graph(eight_bit):
    """A decode step allocates nothing and never waits for the GPU, so it can be captured once and
    replayed: every replay, with eager work and synchronisations in between, must give the bits of
    an eager call on the same inputs."""
    from paper_2506_13059_amd import binding as mp
    B, Hq, Hkv, n = 2, 8, 2, 2500
    K, V, q = _mk(B, Hq, Hkv, n, 60, seed=31, softness=0.5, n_sets=4)
    g = torch.Generator(device="cuda").manual_seed(32)
    fot = torch.randint(0, 80, (B * Hkv, n), generator=g, device="cuda").to(torch.int32)
    cof = (torch.arange(80, device="cuda", dtype=torch.int32) // 10)[None].repeat(B * Hkv, 1).contiguous()
    ctx = mp.MpContext(B, Hq, Hkv, max_tokens=n, levels=2, max_fine=80, max_coarse=8, max_tail=16,
                       kv_format=mp.MP_KV_E4M3 if eight_bit else mp.MP_KV_BF16)
    ctx.mp_set_clustering(K, V, fot, 80, cof, 8)
    kt = torch.randn(B, Hkv, 16, 128, generator=g, device="cuda").to(torch.bfloat16)
    vt = torch.randn(B, Hkv, 16, 128, generator=g, device="cuda").to(torch.bfloat16)
    q_in = q[0].clone()
    out = torch.empty_like(q_in)
    lse = torch.empty(B, Hq, dtype=torch.float32, device="cuda")
    ctx.mp_decode_attention(q_in, 300, 900, k_tail=kt, v_tail=vt, n_tail=11, out=out, lse=lse)   # warm-up, eager
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.mp_decode_attention(q_in, 300, 900, k_tail=kt, v_tail=vt, n_tail=11, out=out, lse=lse)
    for s in range(4):
        q_in.copy_(q[s])
        graph.replay()
        torch.cuda.synchronize()
        got, got_lse = out.clone(), lse.clone()
        ref_lse = torch.empty_like(lse)
        ref = ctx.mp_decode_attention(q[s].contiguous(), 300, 900, k_tail=kt, v_tail=vt, n_tail=11, lse=ref_lse)
        torch.cuda.synchronize()
        assert torch.equal(got, ref) and torch.equal(got_lse, ref_lse), f"replay {s}"
    ctx.close()


def test_decode_argument_errors():
    from paper_2506_13059_amd import binding as mp
    ctx = mp.MpContext(1, 4, 1, max_tokens=64, levels=1, max_fine=4, max_tail=2)
    q = torch.zeros(1, 4, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mp.MpError) as e:
        ctx.mp_decode_attention(q, 10)
    assert e.value.status == mp.MP_ESTATE
    K = torch.randn(1, 1, 64, 128, device="cuda").to(torch.bfloat16)
    fot = torch.zeros(1, 64, dtype=torch.int32, device="cuda")
    with pytest.raises(mp.MpError) as e:
        ctx.mp_set_clustering(K, K, fot, 9)
    assert e.value.status == mp.MP_ECAPACITY
    ctx.mp_set_clustering(K, K, fot, 4)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_decode_attention(q, -1)
    assert e.value.status == mp.MP_EINVAL
    tail = torch.zeros(1, 1, 3, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mp.MpError) as e:
        ctx.mp_decode_attention(q, 10, k_tail=tail, v_tail=tail)
    assert e.value.status == mp.MP_ECAPACITY
    out = ctx.mp_decode_attention(q, 10)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    ctx.close()


def test_many_units_long_chunks():
    # 128 units x 2048 selected keys: the launch shape of the large workloads (512-row chunks of the
    # selected-key stream, eight-iteration strips), at a size the oracle still checks unit by unit
    from paper_2506_13059_amd import binding as mp
    from tests.gpu_util import compare_decode
    B, Hq, Hkv, n = 16, 16, 8, 4096
    K, V, q = _mk(B, Hq, Hkv, n, 64, seed=91, softness=0.4)
    g = torch.Generator(device="cuda").manual_seed(92)
    fot = torch.randint(0, 128, (B * Hkv, n), generator=g, device="cuda").to(torch.int32)
    cof = (torch.arange(128, device="cuda", dtype=torch.int32) // 8)[None].repeat(B * Hkv, 1).contiguous()
    ctx = mp.MpContext(B, Hq, Hkv, max_tokens=n, levels=2, max_fine=128, max_coarse=16, max_tail=0)
    ctx.mp_set_clustering(K, V, fot, 128, cof, 16)
    r = compare_decode(ctx, q[0], K, V, 2048, 4096, label="many units")
    assert r["exempt"] == 0
    ctx.close()
