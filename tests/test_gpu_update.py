"""GPU parity: mp_update_clusters (online cluster update, Sec. 3.3) against the oracle, chained
over several updates from the same seeds, including a split of the last block."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _compare_index(ctx, cls, levels, label, units=None):
    """cls: oracle clusterings of the units listed in `units` (default: all units, in order)."""
    from tests.gpu_util import f64, i32
    fot, cof = ctx.mp_get_assignments()
    kc, vc, nm = ctx.mp_get_centroids(0)
    kp, vp, perm, fstart = ctx.mp_get_layout()
    sizes = ctx.mp_get_sizes()
    torch.cuda.synchronize()
    fot, kc, vc, nm, perm, fstart = i32(fot), f64(kc), f64(vc), i32(nm), i32(perm), i32(fstart)
    if levels == 2:
        kcc, vcc, nmc = ctx.mp_get_centroids(1)
        torch.cuda.synchronize()
        cof, kcc, vcc, nmc = i32(cof), f64(kcc), f64(vcc), i32(nmc)
    for u, cl in zip(range(len(cls)) if units is None else units, cls):
        n = cl["K"].shape[0]
        assert sizes["n_tokens"] == n and sizes["n_fine"] == cl["N_f"].shape[0] and sizes["n_blocks"] == len(cl["blocks"])
        np.testing.assert_array_equal(fot[u], cl["fine_of_token"], err_msg=f"{label} unit {u} fine assignment")
        np.testing.assert_array_equal(nm[u], cl["N_f"])
        np.testing.assert_array_equal(kc[u], cl["Kc_f"], err_msg=f"{label} unit {u} fine key centroids")
        np.testing.assert_array_equal(vc[u], cl["Vc_f"])
        # stored layout: rows are the original rows, cluster after cluster
        assert sorted(perm[u].tolist()) == list(range(n))
        np.testing.assert_array_equal(np.diff(fstart[u]), cl["N_f"])
        assert (np.diff(cl["fine_of_token"][perm[u]]) >= 0).all()
        Ku = torch.tensor(cl["K"], dtype=torch.float64)
        assert torch.equal(kp[u].cpu().to(torch.float64), Ku[torch.tensor(perm[u], dtype=torch.long)])
        if levels == 2:
            np.testing.assert_array_equal(cof[u], cl["coarse_of_fine"], err_msg=f"{label} unit {u} coarse assignment")
            np.testing.assert_array_equal(nmc[u], cl["N_c"])
            live = cl["N_c"] > 0
            np.testing.assert_array_equal(kcc[u][live], cl["Kc_c"][live])
            np.testing.assert_array_equal(vcc[u][live], cl["Vc_c"][live])


def _chain(B, Hq, Hkv, n0, modes, levels, nf, nc, W, alpha, iters, updates, seed, max_tokens, max_fine, max_coarse,
           lookup=None, units=None):
    """updates: list of (n_new, n_new_fine, n_new_coarse, refine_iters).  units: the units the oracle
    follows (default: all; the library always works on all of them).  lookup: None, or how the
    lookup keys relate to the stored keys: "rope" (stored keys rotated to their own position, lookup
    keys to one fixed position, Sec. 3.1 last paragraph) or "perm" (a signed permutation)."""
    from paper_2506_13059_amd import binding as mp, inputs
    from oracle import mp_oracle as O
    from tests.gpu_util import f64, rope, signed_permutation
    U = B * Hkv
    sample = list(range(U)) if units is None else list(units)
    centers = inputs.make_modes(U, modes, "cuda", seed)
    K, V = inputs.draw_tokens(centers, n0, seed + 1)
    A = signed_permutation(128, seed, "cuda")

    def stored_and_lookup(X, pos0):
        if lookup == "rope":
            return rope(X, pos0 + torch.arange(X.shape[1])), rope(X, torch.full((X.shape[1],), 4096))
        if lookup == "perm":
            return X, A(X)
        return X, None

    K, KL = stored_and_lookup(K, 0)
    lk = (lambda t, n: None) if lookup is None else (lambda t, n: t.view(B, Hkv, n, 128))
    blocks = mp.mp_plan_blocks(n0, W, alpha, nf, nc if levels == 2 else 0)
    init_f, init_c = inputs.draw_seeds(U, blocks, levels, seed + 3)
    ctx = mp.MpContext(B, Hq, Hkv, max_tokens=max_tokens, levels=levels, max_fine=max_fine, max_coarse=max_coarse,
                       block_w=W, block_alpha=alpha, max_tail=0, lookup_keys=lookup is not None)
    ctx.mp_cluster_kv(K.view(B, Hkv, n0, 128), V.view(B, Hkv, n0, 128), nf, nc, iters=iters, init_fine=init_f,
                      init_coarse=init_c if levels == 2 else None, k_lookup=lk(KL, n0))
    cls = [O.cluster_unit(f64(K[u]), f64(V[u]), blocks, init_f[u].numpy(), init_c[u].numpy() if levels == 2 else None,
                          iters, levels, K_lookup=f64(KL[u]) if lookup else None) for u in sample]
    _compare_index(ctx, cls, levels, "after build", sample)
    rng = np.random.default_rng(seed)
    for step, (n_new, nnf, nnc, refine) in enumerate(updates):
        print(f"update {step}: +{n_new} tokens, +{nnf} fine, +{nnc} coarse, refine {refine}", flush=True)
        centers = inputs.drift_modes(centers, seed + 100 + step)
        Kn, Vn = inputs.draw_tokens(centers, n_new, seed + 200 + step)
        Kn, KLn = stored_and_lookup(Kn, cls[0]["K"].shape[0])
        counts = ctx.mp_update_seed_counts(n_new, nnf, nnc)
        assert counts == O.update_seed_counts(cls[0]["blocks"], n_new, nnf, nnc, W, alpha, levels)
        nb = cls[0]["blocks"][-1]["t1"] - cls[0]["blocks"][-1]["t0"] + n_new
        lims = [n_new, nnf, W, nb - W, counts[2], counts[3]]
        seeds = np.stack([np.concatenate([rng.choice(max(l, 1), c, replace=False) for l, c in zip(lims, counts)])
                          for _ in range(U)]).astype(np.int32)
        ctx.mp_update_clusters(Kn.view(B, Hkv, n_new, 128), Vn.view(B, Hkv, n_new, 128), nnf, nnc, refine_iters=refine,
                               split_iters=iters, seeds=torch.tensor(seeds), k_new_lookup=lk(KLn, n_new))
        cls = [O.update_unit(cl, f64(Kn[u]), f64(Vn[u]), nnf, nnc, seeds[u], refine, W, alpha, split_iters=iters,
                             K_new_lookup=f64(KLn[u]) if lookup else None) for u, cl in zip(sample, cls)]
        _compare_index(ctx, cls, levels, f"after update {step}", sample)
    return ctx, cls, centers


def test_update_chain_two_levels_with_split():
    # one block of 352 tokens (W = 256, alpha = 128): 2 updates of 16 tokens, the second reaches 384 = W + alpha
    ctx, cls, centers = _chain(1, 8, 2, 352, 24, 2, 22, 4, 256, 128, iters=3,
                               updates=[(16, 2, 1, 2), (16, 2, 0, 3), (48, 6, 1, 1)], seed=21,
                               max_tokens=1024, max_fine=64, max_coarse=16)
    assert [(b["t0"], b["t1"]) for b in cls[0]["blocks"]] == [(0, 256), (256, 432)]
    # decode on the updated index
    from tests.gpu_util import compare_decode
    from paper_2506_13059_amd import inputs
    q = inputs.draw_queries(centers, 4, 1, 5, softness=0.3).view(1, 1, 8, 128)[0].contiguous()
    K = torch.tensor(np.stack([c["K"] for c in cls]), dtype=torch.float64, device="cuda").to(torch.bfloat16)
    V = torch.tensor(np.stack([c["V"] for c in cls]), dtype=torch.float64, device="cuda").to(torch.bfloat16)
    compare_decode(ctx, q, K.view(1, 2, -1, 128), V.view(1, 2, -1, 128), 100, 250, label="after updates")
    ctx.close()


def test_update_one_level_no_refinement_and_no_new_clusters():
    ctx, cls, _ = _chain(2, 2, 1, 500, 10, 1, 20, 0, 0, 0, iters=2, updates=[(32, 0, 0, 0), (40, 5, 0, 0), (8, 8, 0, 2)],
                         seed=22, max_tokens=700, max_fine=40, max_coarse=0)
    ctx.close()


def test_update_later_block_of_a_multi_block_index():
    ctx, cls, _ = _chain(1, 4, 1, 700, 20, 2, 40, 8, 256, 128, iters=2, updates=[(16, 2, 1, 3), (16, 2, 0, 1)], seed=23,
                         max_tokens=1024, max_fine=64, max_coarse=16)
    assert len(cls[0]["blocks"]) == 3
    ctx.close()


def test_update_argument_errors():
    from paper_2506_13059_amd import binding as mp
    ctx = mp.MpContext(1, 2, 1, max_tokens=300, levels=2, max_fine=20, max_coarse=4, block_w=128, block_alpha=64, max_tail=0)
    kn = torch.randn(1, 1, 16, 128, device="cuda").to(torch.bfloat16)
    with pytest.raises(mp.MpError) as e:
        ctx.mp_update_clusters(kn, kn, 2, 1)
    assert e.value.status == mp.MP_ESTATE
    K = torch.randn(1, 1, 150, 128, device="cuda").to(torch.bfloat16)
    ctx.mp_cluster_kv(K, K, 16, 3, iters=1, seed=1)
    for kwargs, status in [(dict(n_new_fine=17), mp.MP_EINVAL), (dict(n_new_fine=2, n_new_coarse=3), mp.MP_EINVAL),
                           (dict(n_new_fine=8, n_new_coarse=0), mp.MP_ECAPACITY),
                           (dict(n_new_fine=2, n_new_coarse=2), mp.MP_ECAPACITY)]:
        with pytest.raises(mp.MpError) as e:
            ctx.mp_update_clusters(kn, kn, **kwargs)
        assert e.value.status == status, kwargs
    with pytest.raises(mp.MpError) as e:
        ctx.mp_update_clusters(kn, kn, 2, 1, seeds=torch.tensor([[3, 3, 0]], dtype=torch.int32))
    assert e.value.status == mp.MP_EINVAL
    ctx.mp_update_clusters(kn, kn, 2, 1, seed=5)
    assert ctx.mp_get_sizes()["n_tokens"] == 166
    ctx.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_update_chains(seed):
    # seeded random shapes: block sizes (or no blocks), cluster ratios, iteration counts, update sizes
    # down to a single token, updates without new clusters, with and without lookup keys
    rng = np.random.default_rng(300 + seed)
    W = int(rng.choice([0, 128, 256]))
    alpha = 0 if W == 0 else int(rng.choice([W // 2, W]))
    n0 = int(rng.integers(200, 600)) if W == 0 else int(rng.integers(W + alpha, 3 * W))
    levels = int(rng.integers(1, 3))
    nf = max(2, n0 // int(rng.choice([8, 16, 32])))
    nc = max(1, nf // 6) if levels == 2 else 0
    iters = int(rng.integers(1, 4))
    updates = []
    for _ in range(3):
        n_new = int(rng.choice([1, 8, 16, 40]))
        nnf = int(rng.integers(0, min(n_new, 6) + 1))
        nnc = int(rng.integers(0, min(nnf, 2) + 1)) if levels == 2 else 0
        updates.append((n_new, nnf, nnc, int(rng.integers(0, 3))))
    lookup = [None, "rope", "perm"][int(rng.integers(0, 3))]
    B, Hkv = int(rng.integers(1, 3)), int(rng.integers(1, 3))
    print(f"seed {seed}: B={B} Hkv={Hkv} n0={n0} W={W} alpha={alpha} levels={levels} nf={nf} nc={nc} iters={iters} "
          f"updates={updates} lookup={lookup}", flush=True)
    ctx, cls, _ = _chain(B, 2 * Hkv, Hkv, n0, 12, levels, nf, nc, W, alpha, iters, updates, seed=400 + seed,
                         max_tokens=n0 + sum(u[0] for u in updates), max_fine=nf + sum(u[1] for u in updates) + 8,
                         max_coarse=(nc + sum(u[2] for u in updates) + 4) if levels == 2 else 0, lookup=lookup)
    ctx.close()
