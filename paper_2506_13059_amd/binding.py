"""Thin ctypes binding of libmp.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch supplies device memory
(``tensor.data_ptr()``) and the current stream.  There is no CPU fallback: if the library is
missing, importing or calling fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmp.so")

MP_OK, MP_EINVAL, MP_ENOMEM, MP_ESTATE, MP_ECAPACITY, MP_EHIP = range(6)
MP_DECODE_NO_MULTIPOLE = 1

EXPORTS = [
    "mp_create", "mp_destroy", "mp_last_error", "mp_device_bytes", "mp_plan_blocks", "mp_cluster_kv",
    "mp_set_clustering", "mp_update_clusters", "mp_decode_attention", "mp_get_sizes", "mp_get_assignments",
    "mp_get_centroids", "mp_get_selection", "mp_get_counters", "mp_get_layout", "mp_dense_workspace_bytes",
    "mp_dense_attention", "mp_version", "mp_enable_stage_timing", "mp_get_stage_timing", "mp_update_seed_counts", "mp_local_buffer_init", "mp_local_buffer_size", "mp_decode_step",
    "mp_dense_static_scratch_bytes", "mp_dense_attention_static", "mp_get_kv_codes",
]

MP_KV_BF16, MP_KV_E4M3 = 0, 1


class MpError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"mp status {status}: {msg}")
        self.status = status


class MpConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "max_tokens", "levels", "max_fine", "max_coarse",
        "block_w", "block_alpha", "max_tail", "lookup_keys")] + [("softmax_scale", C.c_float), ("kv_format", C.c_int32)]


_lib = None


def lib():
    """Load libmp.so (built beforehand by paper_2506_13059_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first with `python -m paper_2506_13059_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, u64, u32, f32, sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_uint32, C.c_float, C.c_size_t
        L.mp_version.restype = C.c_char_p
        L.mp_last_error.restype = C.c_char_p
        L.mp_last_error.argtypes = [vp]
        L.mp_create.argtypes = [C.POINTER(MpConfig), C.POINTER(vp)]
        L.mp_destroy.argtypes = [vp]
        L.mp_destroy.restype = None
        L.mp_device_bytes.argtypes = [vp]
        L.mp_device_bytes.restype = sz
        L.mp_plan_blocks.argtypes = [i32, i32, i32, i32, i32, vp, i32]
        L.mp_plan_blocks.restype = i32
        L.mp_cluster_kv.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, u64, vp, vp, vp]
        L.mp_set_clustering.argtypes = [vp, vp, vp, vp, i32, vp, i32, vp, i32, vp]
        L.mp_update_clusters.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, u64, vp, vp]
        L.mp_decode_attention.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, u32, vp, vp, vp]
        L.mp_update_seed_counts.argtypes = [vp, i32, i32, i32, vp]
        L.mp_local_buffer_init.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, i32, vp]
        L.mp_local_buffer_size.argtypes = [vp, vp, vp, vp]
        L.mp_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, u32, i32, i32, i32, i32, u64, vp, vp, vp, vp]
        L.mp_update_seed_counts.restype = i32
        L.mp_enable_stage_timing.argtypes = [vp, i32]
        L.mp_get_stage_timing.argtypes = [vp, vp]
        L.mp_get_sizes.argtypes = [vp, vp, vp, vp, vp]
        L.mp_get_assignments.argtypes = [vp, vp, vp, vp]
        L.mp_get_centroids.argtypes = [vp, i32, vp, vp, vp, vp]
        L.mp_get_selection.argtypes = [vp, vp, vp, vp, vp, vp]
        L.mp_get_counters.argtypes = [vp, vp, vp]
        L.mp_get_layout.argtypes = [vp, vp, vp, vp, vp, vp]
        L.mp_get_kv_codes.argtypes = [vp, vp, vp, vp, vp]
        L.mp_dense_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.mp_dense_workspace_bytes.restype = sz
        L.mp_dense_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, vp, vp, vp, sz, vp]
        L.mp_dense_static_scratch_bytes.argtypes = []
        L.mp_dense_static_scratch_bytes.restype = sz
        L.mp_dense_attention_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, vp, vp, vp]
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors passed to the library must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, ctx=None):
    if status != MP_OK:
        msg = lib().mp_last_error(ctx).decode()
        raise MpError(status, msg)


def _host_i32(t):
    """Host int32 array argument: accepts a CPU int32 tensor (or None)."""
    if t is None:
        return None, None
    t = t.to(dtype=torch.int32, device="cpu").contiguous()
    return t, C.c_void_p(t.data_ptr())


def mp_plan_blocks(n_tokens, block_w, block_alpha, n_fine, n_coarse):
    n = lib().mp_plan_blocks(n_tokens, block_w, block_alpha, n_fine, n_coarse, None, 0)
    if n < 0:
        raise MpError(MP_EINVAL, "mp_plan_blocks: invalid arguments")
    buf = (C.c_int32 * (6 * n))()
    lib().mp_plan_blocks(n_tokens, block_w, block_alpha, n_fine, n_coarse, C.cast(buf, C.c_void_p), n)
    keys = ("t0", "t1", "f0", "f1", "c0", "c1")
    return [dict(zip(keys, buf[6 * i:6 * i + 6])) for i in range(n)]


def mp_dense_workspace_bytes(batch, n_q_heads, n_kv_heads, n):
    return int(lib().mp_dense_workspace_bytes(batch, n_q_heads, n_kv_heads, n))


def mp_dense_attention(q, k, v, out=None, lse=None, workspace=None, softmax_scale=0.0):
    """q [B,Hq,128], k/v [B,Hkv,n,128] bf16 CUDA tensors -> out [B,Hq,128] bf16 (and lse fp32 [B,Hq])."""
    B, Hq, _ = q.shape
    Hkv, n = k.shape[1], k.shape[2]
    need = mp_dense_workspace_bytes(B, Hq, Hkv, n)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty_like(q)
    st = lib().mp_dense_attention(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, n, softmax_scale, _ptr(out), _ptr(lse),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(st)
    return out


def mp_dense_static_scratch_bytes():
    return int(lib().mp_dense_static_scratch_bytes())


def mp_dense_attention_static(q, k, v, out, lse=None, softmax_scale=0.0):
    """mp_dense_attention without a workspace: `out` (and lse) are the caller's, nothing is allocated."""
    B, Hq, _ = q.shape
    Hkv, n = k.shape[1], k.shape[2]
    st = lib().mp_dense_attention_static(_ptr(q), _ptr(k), _ptr(v), B, Hq, Hkv, n, softmax_scale, _ptr(out), _ptr(lse),
                                         _stream())
    _check(st)
    return out


class MpContext:
    """Owns an mp_ctx handle.  Method names and arguments mirror the C entry points."""

    def __init__(self, batch, n_q_heads, n_kv_heads, max_tokens, levels, max_fine, max_coarse=0, block_w=0,
                 block_alpha=0, max_tail=0, softmax_scale=0.0, head_dim=128, lookup_keys=False, kv_format=MP_KV_BF16):
        self.cfg = MpConfig(batch, n_q_heads, n_kv_heads, head_dim, max_tokens, levels, max_fine, max_coarse,
                            block_w, block_alpha, max_tail, 1 if lookup_keys else 0, softmax_scale, kv_format)
        self.kv_format = kv_format
        self.h = C.c_void_p()
        st = lib().mp_create(C.byref(self.cfg), C.byref(self.h))
        _check(st)
        self.U = batch * n_kv_heads
        self.G = n_q_heads // n_kv_heads

    def close(self):
        if getattr(self, "h", None) is not None and self.h.value:
            lib().mp_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def device_bytes(self):
        return int(lib().mp_device_bytes(self.h))

    def mp_cluster_kv(self, k, v, n_fine, n_coarse=0, iters=10, seed=0, init_fine=None, init_coarse=None,
                      k_lookup=None):
        n_tokens = k.shape[2]
        f_keep, f_ptr = _host_i32(init_fine)
        c_keep, c_ptr = _host_i32(init_coarse)
        st = lib().mp_cluster_kv(self.h, _ptr(k), _ptr(k_lookup), _ptr(v), n_tokens, n_fine, n_coarse, iters, seed,
                                 f_ptr, c_ptr, _stream())
        _check(st, self.h)

    def mp_set_clustering(self, k, v, fine_of_token, n_fine, coarse_of_fine=None, n_coarse=0, k_lookup=None):
        n_tokens = k.shape[2]
        st = lib().mp_set_clustering(self.h, _ptr(k), _ptr(k_lookup), _ptr(v), n_tokens, _ptr(fine_of_token), n_fine,
                                     _ptr(coarse_of_fine), n_coarse, _stream())
        _check(st, self.h)

    def mp_update_clusters(self, k_new, v_new, n_new_fine, n_new_coarse=0, refine_iters=3, split_iters=10, seed=0,
                           seeds=None, k_new_lookup=None):
        n_new = k_new.shape[2]
        s_keep, s_ptr = _host_i32(seeds)
        st = lib().mp_update_clusters(self.h, _ptr(k_new), _ptr(k_new_lookup), _ptr(v_new), n_new, n_new_fine, n_new_coarse,
                                      refine_iters, split_iters, seed, s_ptr, _stream())
        _check(st, self.h)

    def mp_local_buffer_init(self, window, k_sink=None, v_sink=None, k_recent=None, v_recent=None,
                             k_recent_lookup=None):
        n_sink = 0 if k_sink is None else k_sink.shape[2]
        n_recent = 0 if k_recent is None else k_recent.shape[2]
        st = lib().mp_local_buffer_init(self.h, window, _ptr(k_sink), _ptr(v_sink), n_sink, _ptr(k_recent),
                                        _ptr(k_recent_lookup), _ptr(v_recent), n_recent, _stream())
        _check(st, self.h)

    def mp_local_buffer_size(self):
        buf = (C.c_int32 * 3)()
        base = C.addressof(buf)
        st = lib().mp_local_buffer_size(self.h, C.c_void_p(base), C.c_void_p(base + 4), C.c_void_p(base + 8))
        _check(st, self.h)
        return dict(window=buf[0], n_sink=buf[1], n_recent=buf[2])

    def mp_decode_step(self, q, k_new, v_new, key_budget, coarse_budget=0, n_new_fine=0, n_new_coarse=0,
                       refine_iters=3, split_iters=10, seed=0, seeds=None, out=None, lse=None, flags=0,
                       q_lookup=None, k_new_lookup=None):
        if out is None:
            out = torch.empty_like(q)
        s_keep, s_ptr = _host_i32(seeds)
        st = lib().mp_decode_step(self.h, _ptr(q), _ptr(q_lookup), _ptr(k_new), _ptr(k_new_lookup), _ptr(v_new),
                                  key_budget, coarse_budget, flags,
                                  n_new_fine, n_new_coarse, refine_iters, split_iters, seed, s_ptr, _ptr(out),
                                  _ptr(lse), _stream())
        _check(st, self.h)
        return out

    def mp_update_seed_counts(self, n_new, n_new_fine, n_new_coarse=0):
        buf = (C.c_int32 * 6)()
        t = lib().mp_update_seed_counts(self.h, n_new, n_new_fine, n_new_coarse, C.cast(buf, C.c_void_p))
        if t < 0:
            raise MpError(MP_EINVAL, "mp_update_seed_counts: invalid arguments or no index yet")
        return list(buf)

    def mp_decode_attention(self, q, key_budget, coarse_budget=0, k_tail=None, v_tail=None, out=None, lse=None,
                            flags=0, n_tail=None, q_lookup=None):
        """k_tail / v_tail [B, Hkv, rows, 128]; n_tail (default: all rows) = rows of every unit in use."""
        tail_stride = 0 if k_tail is None else k_tail.shape[2]
        if n_tail is None:
            n_tail = tail_stride
        if out is None:
            out = torch.empty_like(q)
        st = lib().mp_decode_attention(self.h, _ptr(q), _ptr(q_lookup), _ptr(k_tail), _ptr(v_tail), n_tail, tail_stride, key_budget,
                                       coarse_budget, flags, _ptr(out), _ptr(lse), _stream())
        _check(st, self.h)
        return out

    def mp_enable_stage_timing(self, enable=True):
        _check(lib().mp_enable_stage_timing(self.h, 1 if enable else 0), self.h)

    def mp_get_stage_timing(self):
        buf = (C.c_float * 4)()
        _check(lib().mp_get_stage_timing(self.h, C.cast(buf, C.c_void_p)), self.h)
        return dict(coarse_ms=buf[0], fine_ms=buf[1], value_ms=buf[2], merge_ms=buf[3])

    def mp_get_sizes(self):
        v = [C.c_int32() for _ in range(4)]
        st = lib().mp_get_sizes(self.h, *[C.cast(C.byref(x), C.c_void_p) for x in v])
        _check(st, self.h)
        return dict(n_tokens=v[0].value, n_fine=v[1].value, n_coarse=v[2].value, n_blocks=v[3].value)

    def mp_get_assignments(self):
        s = self.mp_get_sizes()
        dev = torch.device("cuda")
        fot = torch.empty(self.U, s["n_tokens"], dtype=torch.int32, device=dev)
        cof = torch.empty(self.U, max(s["n_fine"], 1), dtype=torch.int32, device=dev) if self.cfg.levels == 2 else None
        st = lib().mp_get_assignments(self.h, _ptr(fot), _ptr(cof), _stream())
        _check(st, self.h)
        return fot, (cof[:, :s["n_fine"]] if cof is not None else None)

    def mp_get_centroids(self, level):
        s = self.mp_get_sizes()
        n = s["n_fine"] if level == 0 else s["n_coarse"]
        dev = torch.device("cuda")
        kc = torch.empty(self.U, n, 128, dtype=torch.bfloat16, device=dev)
        vc = torch.empty(self.U, n, 128, dtype=torch.bfloat16, device=dev)
        nm = torch.empty(self.U, n, dtype=torch.int32, device=dev)
        st = lib().mp_get_centroids(self.h, level, _ptr(kc), _ptr(vc), _ptr(nm), _stream())
        _check(st, self.h)
        return kc, vc, nm

    def mp_get_selection(self):
        s = self.mp_get_sizes()
        dev = torch.device("cuda")
        nf, nc = s["n_fine"], max(s["n_coarse"], 1)
        fs = torch.empty(self.U, nf, dtype=torch.uint8, device=dev)
        cp = torch.empty(self.U, nc, dtype=torch.uint8, device=dev)
        rf = torch.empty(self.U, nf, dtype=torch.float64, device=dev)
        rc = torch.empty(self.U, nc, dtype=torch.float64, device=dev)
        two = self.cfg.levels == 2
        st = lib().mp_get_selection(self.h, _ptr(fs), _ptr(cp) if two else None, _ptr(rf), _ptr(rc) if two else None,
                                    _stream())
        _check(st, self.h)
        return dict(fine_selected=fs, coarse_promising=cp[:, :s["n_coarse"]] if two else None, r_fine=rf,
                    r_coarse=rc[:, :s["n_coarse"]] if two else None)

    def mp_get_counters(self):
        c = torch.empty(self.U, 4, dtype=torch.int32, device="cuda")
        st = lib().mp_get_counters(self.h, _ptr(c), _stream())
        _check(st, self.h)
        return c

    def mp_get_layout(self):
        """(k_perm, v_perm, perm, fine_start); k_perm and v_perm are None for a context with 8-bit rows."""
        s = self.mp_get_sizes()
        dev = torch.device("cuda")
        kp = vp = None
        if self.kv_format == MP_KV_BF16:
            kp = torch.empty(self.U, s["n_tokens"], 128, dtype=torch.bfloat16, device=dev)
            vp = torch.empty_like(kp)
        perm = torch.empty(self.U, s["n_tokens"], dtype=torch.int32, device=dev)
        fs = torch.empty(self.U, s["n_fine"] + 1, dtype=torch.int32, device=dev)
        st = lib().mp_get_layout(self.h, _ptr(kp), _ptr(vp), _ptr(perm), _ptr(fs), _stream())
        _check(st, self.h)
        return kp, vp, perm, fs

    def mp_get_kv_codes(self):
        """(k_codes uint8 [U, n, 128], v_codes, scales fp32 [U, n, 2]) of a context with 8-bit rows."""
        s = self.mp_get_sizes()
        dev = torch.device("cuda")
        kc = torch.empty(self.U, s["n_tokens"], 128, dtype=torch.uint8, device=dev)
        vc = torch.empty_like(kc)
        sc = torch.empty(self.U, s["n_tokens"], 2, dtype=torch.float32, device=dev)
        st = lib().mp_get_kv_codes(self.h, _ptr(kc), _ptr(vc), _ptr(sc), _stream())
        _check(st, self.h)
        return kc, vc, sc
