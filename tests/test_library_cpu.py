"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2506_13059_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def _declared():
    with open(os.path.join(ROOT, "include", "mp.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(mp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2506_13059_amd import binding
    names = _declared()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_version_and_last_error(lib):
    assert lib.mp_version().startswith(b"mp-gfx950")
    assert isinstance(lib.mp_last_error(None), bytes)


def test_plan_blocks_matches_the_oracle_plan(lib):
    from paper_2506_13059_amd import binding, inputs
    from oracle import mp_oracle as O
    for args in [(131072, 8192, 4096, 4096, 256), (8192, 8192, 4096, 256, 32), (12288, 8192, 4096, 768, 96),
                 (12287, 8192, 4096, 768, 96), (4096, 0, 0, 64, 0), (30000, 8192, 4096, 1000, 100), (700, 256, 128, 40, 8)]:
        assert binding.mp_plan_blocks(*args) == O.plan_blocks(*args) == inputs.plan_blocks(*args)
    assert lib.mp_plan_blocks(0, 0, 0, 1, 0, None, 0) == -1


def test_create_rejects_bad_configs_without_a_gpu(lib):
    from paper_2506_13059_amd import binding as mp
    good = dict(batch=1, n_q_heads=4, n_kv_heads=1, max_tokens=128, levels=2, max_fine=16, max_coarse=4)
    bad = [dict(batch=0), dict(n_q_heads=5, n_kv_heads=2), dict(head_dim=64), dict(n_q_heads=9, n_kv_heads=1),
           dict(levels=3), dict(max_tokens=0), dict(max_fine=0), dict(max_fine=10 ** 6), dict(max_coarse=0),
           dict(max_coarse=17), dict(block_w=-1), dict(block_w=8, block_alpha=9), dict(max_tail=-1),
           dict(softmax_scale=-1.0), dict(kv_format=2), dict(kv_format=mp.MP_KV_E4M3, lookup_keys=True)]
    for b in bad:
        with pytest.raises(mp.MpError) as e:
            mp.MpContext(**{**good, **b})
        assert e.value.status == mp.MP_EINVAL, b
        assert len(str(e.value)) > 10


def test_null_context_calls_fail_cleanly(lib):
    from paper_2506_13059_amd import binding as mp
    assert lib.mp_decode_attention(None, None, None, None, None, 0, 0, 0, 0, 0, None, None, None) == mp.MP_EINVAL
    assert lib.mp_cluster_kv(None, None, None, None, 1, 1, 0, 1, 0, None, None, None) == mp.MP_EINVAL
    assert lib.mp_update_clusters(None, None, None, None, 1, 0, 0, 0, 1, 0, None, None) == mp.MP_EINVAL
    assert lib.mp_dense_attention(None, None, None, 1, 1, 1, 1, 0.0, None, None, None, 0, None) == mp.MP_EINVAL
    assert lib.mp_get_kv_codes(None, None, None, None, None) == mp.MP_EINVAL
    assert b"null" in lib.mp_last_error(None)
    lib.mp_destroy(None)
    assert lib.mp_device_bytes(None) == 0


def test_dense_workspace_size(lib):
    from paper_2506_13059_amd import binding as mp
    assert mp.mp_dense_workspace_bytes(1, 4, 1, 4096) == 8 * 4 * 132 * 4
    assert mp.mp_dense_workspace_bytes(1, 5, 2, 10) == 0
    big = mp.mp_dense_workspace_bytes(16, 32, 8, 131072)
    assert 0 < big < 2 ** 28


def test_byte_model_reproduces_the_papers_memory_operation_column():
    # Table 2 of the paper lists memory operations relative to dense attention for one-level
    # multipole attention at 8K / 16K context with budgets 128 / 512 (one centroid per 16 tokens, a
    # 2*128-token local buffer, 10 sink tokens): 0.11, 0.09, 0.16, 0.11.  The benchmark's byte
    # accounting, fed with the counters such a step would produce, must give the same fractions.
    import numpy as np
    import bench
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "table2_memory_operations.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for n, budget, want in [(int(a), int(b), float(c)) for a, b, c in rows]:
        cents = n // 16
        counters = np.array([[budget + 256 + 10, cents, 0, cents]])
        step_bytes, value_pass_bytes = bench.algorithmic_bytes(counters, G=4)
        assert round(step_bytes / (2 * n * 256), 2) == want
        assert value_pass_bytes < step_bytes
