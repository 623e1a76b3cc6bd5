"""GPU: mp_dense_attention_static (the entry point that allocates nothing) against mp_dense_attention.

Both run the same kernels on the same partial-result layout, so outputs and log-sum-exps must be
bit-identical; the oracle bounds of the dense kernel are checked as well.  Two calls in a row share
the library's built-in scratch array, the second with a smaller input, so stale contents of the
first call lie behind the second one's partials.
"""
import ctypes as C
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _inputs(B, Hq, Hkv, n, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    q = torch.randn(B, Hq, 128, generator=g, device="cuda").to(torch.bfloat16)
    K = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    V = torch.randn(B, Hkv, n, 128, generator=g, device="cuda").to(torch.bfloat16)
    return q, K, V


def _oracle(q, K, V):
    from oracle import mp_oracle as O
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    q64, K64, V64 = (t.to(torch.float64).cpu().numpy() for t in (q, K, V))
    out = np.zeros((B, Hq, d))
    for b in range(B):
        for kv in range(Hkv):
            out[b, kv * G:(kv + 1) * G] = O.full_attention(q64[b, kv * G:(kv + 1) * G], K64[b, kv], V64[b, kv],
                                                           1 / math.sqrt(d))[0]
    return out


def _both(mp, q, K, V):
    B, Hq, _ = q.shape
    lse_ws = torch.empty(B, Hq, dtype=torch.float32, device="cuda")
    lse_st = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
    out_ws = mp.mp_dense_attention(q, K, V, lse=lse_ws)
    out_st = torch.full_like(q, float("nan"))
    mp.mp_dense_attention_static(q, K, V, out_st, lse=lse_st)
    torch.cuda.synchronize()
    return out_ws, lse_ws, out_st, lse_st


def test_static_scratch_entry_matches_workspace_entry_twice():
    from paper_2506_13059_amd import binding as mp
    assert mp.mp_dense_static_scratch_bytes() == 8 << 20
    # first call: several chunks per unit, group of 4, ragged end; second call: smaller, other group size
    for B, Hq, Hkv, n, seed in [(2, 8, 2, 5003, 11), (1, 5, 1, 777, 12)]:
        print(f"case B={B} Hq={Hq} Hkv={Hkv} n={n}", flush=True)
        assert mp.mp_dense_workspace_bytes(B, Hq, Hkv, n) <= mp.mp_dense_static_scratch_bytes()
        q, K, V = _inputs(B, Hq, Hkv, n, seed)
        out_ws, lse_ws, out_st, lse_st = _both(mp, q, K, V)
        assert torch.equal(out_ws.view(torch.int16), out_st.view(torch.int16))
        assert torch.equal(lse_ws.view(torch.int32), lse_st.view(torch.int32))
        ref = _oracle(q, K, V)
        err = np.abs(out_st.to(torch.float64).cpu().numpy() - ref)
        assert err.max() <= 2e-2, err.max()
        assert err.mean() / np.abs(ref).mean() <= 5e-3


def test_static_scratch_entry_rejects_what_does_not_fit():
    from paper_2506_13059_amd import binding as mp
    # sized on the host only: the call must fail before anything is enqueued, so no big tensors are needed
    B, Hq, Hkv, n = 16, 32, 8, 131072
    assert mp.mp_dense_workspace_bytes(B, Hq, Hkv, n) > mp.mp_dense_static_scratch_bytes()
    q = torch.zeros(B, Hq, 128, dtype=torch.bfloat16, device="cuda")
    small = torch.zeros(1, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros_like(q)
    st = mp.lib().mp_dense_attention_static(C.c_void_p(q.data_ptr()), C.c_void_p(small.data_ptr()),
                                            C.c_void_p(small.data_ptr()), B, Hq, Hkv, n, 0.0,
                                            C.c_void_p(out.data_ptr()), None, None)
    assert st == mp.MP_ECAPACITY
    assert b"scratch" in mp.lib().mp_last_error(None)
    st = mp.lib().mp_dense_attention_static(None, None, None, 1, 4, 1, 16, 0.0, C.c_void_p(out.data_ptr()), None, None)
    assert st == mp.MP_EINVAL
