"""GPU parity of the lookup keys / lookup query (Sec. 3.1, last paragraph; Sec. 4): the clusters and
their key centroids are formed on the lookup keys, every centroid comparison uses the lookup query,
the exact part uses the query and the stored keys.  Build, decode and online update against the
oracle, and the argument checks that go with the option."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _decode_after_chain(ctx, cls, centers, B, Hq, Hkv, lookup, kb, cb, label):
    from paper_2506_13059_amd import inputs
    from tests.gpu_util import compare_decode, rope, signed_permutation
    G = Hq // Hkv
    n = cls[0]["K"].shape[0]
    q = inputs.draw_queries(centers, G, 1, 5, softness=0.3).view(B, Hq, 128)
    if lookup == "rope":
        q, ql = rope(q, torch.full((Hq,), n)), rope(q, torch.full((Hq,), 4100))
    else:
        ql = signed_permutation(128, 77, "cuda")(q)       # a different map than the keys': the logits differ from q's
    K = torch.tensor(np.stack([c["K"] for c in cls]), dtype=torch.float64, device="cuda").to(torch.bfloat16)
    V = torch.tensor(np.stack([c["V"] for c in cls]), dtype=torch.float64, device="cuda").to(torch.bfloat16)
    for budgets in ((kb, cb), (0, 0), (n, n)):
        if hasattr(ctx, "_cache_tables"):
            del ctx._cache_tables
        r = compare_decode(ctx, q, K.view(B, Hkv, n, 128), V.view(B, Hkv, n, 128), *budgets, label=f"{label} {budgets}",
                           q_lookup=ql)
        assert r["exempt"] == 0
    return q, ql, K, V


def test_rotary_lookup_keys_build_update_split_and_decode():
    # one block of 352 tokens (W = 256, alpha = 128); the second update reaches W + alpha and splits
    from tests.test_gpu_update import _chain
    ctx, cls, centers = _chain(1, 8, 2, 352, 24, 2, 22, 4, 256, 128, iters=3,
                               updates=[(16, 2, 1, 2), (16, 2, 0, 3), (48, 6, 1, 1)], seed=61,
                               max_tokens=1024, max_fine=64, max_coarse=16, lookup="rope")
    assert [(b["t0"], b["t1"]) for b in cls[0]["blocks"]] == [(0, 256), (256, 432)]
    _decode_after_chain(ctx, cls, centers, 1, 8, 2, "rope", 100, 250, "rope lookup")
    ctx.close()


def test_permuted_lookup_keys_multi_block_one_and_two_levels():
    from tests.test_gpu_update import _chain
    ctx, cls, centers = _chain(2, 4, 1, 700, 20, 2, 40, 8, 256, 128, iters=2, updates=[(16, 2, 1, 3), (16, 2, 0, 1)], seed=62,
                               max_tokens=1024, max_fine=64, max_coarse=16, lookup="perm")
    assert len(cls[0]["blocks"]) == 3
    _decode_after_chain(ctx, cls, centers, 2, 4, 1, "perm", 120, 300, "perm lookup, two levels")
    ctx.close()
    ctx, cls, centers = _chain(1, 6, 2, 500, 10, 1, 20, 0, 0, 0, iters=2, updates=[(32, 0, 0, 0), (40, 5, 0, 2)], seed=63,
                               max_tokens=700, max_fine=40, max_coarse=0, lookup="perm")
    _decode_after_chain(ctx, cls, centers, 1, 6, 2, "perm", 90, 0, "perm lookup, one level")
    ctx.close()


def test_set_clustering_takes_centroids_from_the_lookup_keys():
    from paper_2506_13059_amd import binding as mp
    from oracle import mp_oracle as O
    from tests.gpu_util import f64
    g = torch.Generator(device="cuda").manual_seed(64)
    B, Hkv, n, nf = 1, 2, 300, 9
    K = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    KL = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    V = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    fot = torch.randint(0, nf, (B * Hkv, n), generator=g, device="cuda", dtype=torch.int32)
    ctx = mp.MpContext(B, 4, Hkv, max_tokens=n, levels=1, max_fine=nf, lookup_keys=True)
    ctx.mp_set_clustering(K, V, fot, nf, k_lookup=KL)
    kc, vc, nm = ctx.mp_get_centroids(0)
    kp, vp, perm, fstart = ctx.mp_get_layout()
    torch.cuda.synchronize()
    for u in range(B * Hkv):
        cl = O.clustering_from_assignment(f64(K.view(-1, n, 128)[u]), f64(V.view(-1, n, 128)[u]), fot[u].cpu().numpy(), nf,
                                          K_lookup=f64(KL.view(-1, n, 128)[u]))
        np.testing.assert_array_equal(f64(kc)[u], cl["Kc_f"])
        np.testing.assert_array_equal(f64(vc)[u], cl["Vc_f"])
        # the cluster-contiguous rows hold the stored keys, not the lookup keys
        assert torch.equal(kp[u], K.view(-1, n, 128)[u][perm[u].long()])
    ctx.close()


def test_lookup_argument_errors():
    from paper_2506_13059_amd import binding as mp
    K = torch.randn(1, 1, 150, 128, device="cuda").to(torch.bfloat16)
    q = torch.randn(1, 2, 128, device="cuda").to(torch.bfloat16)
    kn = K[:, :, :16].contiguous()
    # a context made without the option takes no lookup keys
    ctx = mp.MpContext(1, 2, 1, max_tokens=300, levels=1, max_fine=20, max_tail=8)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_cluster_kv(K, K, 16, iters=1, seed=1, k_lookup=K)
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_cluster_kv(K, K, 16, iters=1, seed=1)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_update_clusters(kn, kn, 2, k_new_lookup=kn)
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_decode_attention(q, 32, q_lookup=q)            # a lookup query alone is allowed: it only replaces q for the centroids
    ctx.close()
    # a context made with the option requires them wherever keys come in
    ctx = mp.MpContext(1, 2, 1, max_tokens=300, levels=1, max_fine=20, max_tail=8, lookup_keys=True)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_cluster_kv(K, K, 16, iters=1, seed=1)
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_cluster_kv(K, K, 16, iters=1, seed=1, k_lookup=K)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_update_clusters(kn, kn, 2)
    assert e.value.status == mp.MP_EINVAL
    with pytest.raises(mp.MpError) as e:
        ctx.mp_local_buffer_init(4, k_recent=kn[:, :, :3].contiguous(), v_recent=kn[:, :, :3].contiguous())
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_local_buffer_init(4)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_decode_step(q, kn[:, :, :1].contiguous(), kn[:, :, :1].contiguous(), 32)
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_decode_step(q, kn[:, :, :1].contiguous(), kn[:, :, :1].contiguous(), 32, q_lookup=q,
                       k_new_lookup=kn[:, :, :1].contiguous())
    assert ctx.mp_local_buffer_size()["n_recent"] == 1
    ctx.close()
