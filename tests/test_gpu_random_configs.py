"""GPU parity over seeded random configurations of the decode step: shapes, group sizes, cluster
counts (with empty clusters), budgets from zero to beyond the context, tails, both levels, the flag
that drops the centroid terms and a lookup query.  Each case goes through mp_set_clustering with a
random assignment, so the whole range of cluster sizes occurs, and is compared with the oracle to
the usual bar."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(seed, eight_bit=False):
    from paper_2506_13059_amd import binding as mp, inputs
    from tests.gpu_util import compare_decode
    rng = np.random.default_rng(1000 + seed)
    B, Hkv = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    G = int(rng.integers(1, 9))
    Hq = Hkv * G
    n = int(rng.choice([1, 2, 17, 63, 64, 65, 300, 1023, 1500, 2600]))
    levels = int(rng.integers(1, 3))
    nf = int(rng.integers(1, min(n, 180) + 1))
    nc = int(rng.integers(1, min(nf, 24) + 1)) if levels == 2 else 0
    n_tail = int(rng.choice([0, 0, 1, 7, 20]))
    flags = int(rng.choice([0, 0, 0, 1]))
    U = B * Hkv
    centers = inputs.make_modes(U, max(1, min(nf, 40)), "cuda", 5000 + seed)
    K, V = inputs.draw_tokens(centers, n, 6000 + seed)
    K, V = K.view(B, Hkv, n, 128), V.view(B, Hkv, n, 128)
    softness = float(rng.choice([0.1, 0.3, 1.0]))
    q = inputs.draw_queries(centers, G, 1, 7000 + seed, softness=softness).view(B, Hq, 128)
    g = torch.Generator(device="cuda").manual_seed(8000 + seed)
    # assignments: a random subset of the clusters stays empty
    used = max(1, int(nf * rng.choice([1.0, 0.7, 0.3])))
    fot = torch.randint(0, used, (U, n), generator=g, device="cuda").to(torch.int32)
    cof = None
    if levels == 2:
        cof = torch.sort(torch.randint(0, nc, (U, nf), generator=g, device="cuda"), dim=1).values.to(torch.int32).contiguous()
    kt = vt = None
    if n_tail:
        kt = torch.randn(B, Hkv, n_tail, 128, generator=g, device="cuda").to(torch.bfloat16)
        vt = torch.randn(B, Hkv, n_tail, 128, generator=g, device="cuda").to(torch.bfloat16)
    ql = None
    if rng.integers(0, 3) == 0 and not eight_bit:      # (8-bit keys take no lookup query)
        ql = (q.float() + 0.2 * torch.randn(q.shape, generator=g, device="cuda")).to(torch.bfloat16)
    desc = f"seed {seed}: B={B} Hkv={Hkv} G={G} n={n} levels={levels} nf={nf} nc={nc} tail={n_tail} flags={flags} " \
           f"soft={softness} lookup_query={ql is not None}"
    print(desc, flush=True)
    ctx = mp.MpContext(B, Hq, Hkv, max_tokens=n, levels=levels, max_fine=nf, max_coarse=nc, max_tail=max(n_tail, 0),
                       kv_format=mp.MP_KV_E4M3 if eight_bit else mp.MP_KV_BF16)
    ctx.mp_set_clustering(K, V, fot, nf, cof, nc)
    if eight_bit:       # the oracle attends what the 8-bit cache stands for
        from tests.test_gpu_fp8 import _check_codes, _dequantised
        _check_codes(ctx, K, V)
        K, V = _dequantised(ctx, K, V)
    exempt = 0
    for kb, cb in [(0, 0), (int(rng.integers(1, n + 1)), int(rng.integers(1, 2 * n + 1))), (n, n), (n + 5, 3 * n),
                   (max(1, n // 8), max(1, n // 3))]:
        r = compare_decode(ctx, q, K, V, kb, cb if levels == 2 else 0, kt, vt, flags=flags, label=f"{desc} kb={kb} cb={cb}",
                           q_lookup=ql)
        exempt += r["exempt"]
    ctx.close()
    return exempt


@pytest.mark.parametrize("block", range(4))
def test_random_configurations(block):
    exempt = sum(_case(seed) for seed in range(8 * block, 8 * block + 8))
    assert exempt <= 2          # units compared only up to a near-tie at the cut


@pytest.mark.parametrize("block", range(2))
def test_random_configurations_8bit_cache(block):
    exempt = sum(_case(seed, eight_bit=True) for seed in range(100 + 8 * block, 100 + 8 * block + 8))
    assert exempt <= 1
