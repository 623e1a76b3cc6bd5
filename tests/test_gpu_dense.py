"""GPU parity: dense bf16 decode attention (the comparison kernel) against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _oracle_full(q, K, V):
    from oracle import mp_oracle as O
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    q64, K64, V64 = (t.to(torch.float64).cpu().numpy() for t in (q, K, V))
    for b in range(B):
        for kv in range(Hkv):
            o, l = O.full_attention(q64[b, kv * G:(kv + 1) * G], K64[b, kv], V64[b, kv], 1 / math.sqrt(d))
            out[b, kv * G:(kv + 1) * G] = o
            lse[b, kv * G:(kv + 1) * G] = l
    return out, lse


def _check(out, lse, ref, ref_lse):
    o = out.to(torch.float64).cpu().numpy()
    err = np.abs(o - ref)
    assert err.max() <= 2e-2, err.max()
    assert (err.mean() / max(np.abs(ref).mean(), 1e-30)) <= 5e-3
    if lse is not None:
        np.testing.assert_allclose(lse.cpu().numpy(), ref_lse, rtol=2e-5, atol=2e-4)


@pytest.mark.parametrize("B,Hq,Hkv,n", [
    (1, 4, 1, 4096),      # config 0 shape
    (2, 8, 2, 1000),      # ragged: not a multiple of any tile
    (1, 5, 1, 777),       # group of 5 (config 2's ratio)
    (1, 1, 1, 1),         # a single key
    (1, 8, 1, 130),       # group of 8, one strip + 2
    (3, 6, 3, 2049),      # group of 2, chunk boundary + 1
    (1, 7, 1, 515),
    (1, 3, 1, 64),
    (2, 12, 2, 3000),     # group of 6: two half-groups per row stream, several chunks
    (1, 8, 1, 5003),      # group of 8 over several chunks with a ragged end
])
def test_dense_matches_oracle(B, Hq, Hkv, n):
    from paper_2506_13059_amd import binding as mp
    print(f"case B={B} Hq={Hq} Hkv={Hkv} n={n}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(1234 + n)
    q = torch.randn(B, Hq, 128, generator=g, device="cuda").to(torch.bfloat16)
    K = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    V = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    lse = torch.empty(B, Hq, dtype=torch.float32, device="cuda")
    out = mp.mp_dense_attention(q, K, V, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = _oracle_full(q, K, V)
    _check(out, lse, ref, ref_lse)


def test_dense_peaked_workload_keys():
    """Keys and queries from the benchmark's mixture recipe (logits of order 100)."""
    from paper_2506_13059_amd import binding as mp, inputs
    w = inputs.WORKLOADS["cfg0_tiny"]
    d = inputs.make_workload(w, "cuda", seed=5)
    q = d["q"][0]
    lse = torch.empty(w.batch, w.n_q_heads, dtype=torch.float32, device="cuda")
    out = mp.mp_dense_attention(q, d["K"], d["V"], lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = _oracle_full(q, d["K"], d["V"])
    _check(out, lse, ref, ref_lse)


def test_dense_empty_context_gives_zero():
    from paper_2506_13059_amd import binding as mp
    q = torch.randn(1, 4, 128, device="cuda").to(torch.bfloat16)
    K = torch.empty(1, 1, 0, 128, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(1, 4, dtype=torch.float32, device="cuda")
    out = mp.mp_dense_attention(q, K, K, lse=lse)
    torch.cuda.synchronize()
    assert (out == 0).all() and torch.isinf(lse).all() and (lse < 0).all()


def test_dense_rejects_bad_arguments():
    from paper_2506_13059_amd import binding as mp
    q = torch.randn(1, 4, 128, device="cuda").to(torch.bfloat16)
    K = torch.randn(1, 3, 16, 128, device="cuda").to(torch.bfloat16)
    with pytest.raises(mp.MpError) as e:
        mp.mp_dense_attention(q, K, K)
    assert e.value.status == mp.MP_EINVAL
    K = torch.randn(1, 1, 16, 128, device="cuda").to(torch.bfloat16)
    with pytest.raises(mp.MpError):
        mp.mp_dense_attention(q, K, K, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
