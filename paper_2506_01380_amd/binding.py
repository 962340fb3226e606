"""ctypes binding of libnfd_attn.so: argument marshalling only.

Function names mirror the C ABI (include/nfd_attn.h).  Tensors are passed as
objects with ``data_ptr()`` (torch tensors) or as raw integer device addresses;
PyTorch is used for device memory and streams only.  There is no fallback: if
the shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libnfd_attn.so")

NFD_BF16, NFD_FP32 = 0, 1
NFD_OK, NFD_ERR_NULL, NFD_ERR_SHAPE, NFD_ERR_UNSUPPORTED = 0, -1, -2, -3
NFD_ERR_CAPACITY, NFD_ERR_HIP, NFD_ERR_ALLOC = -4, -5, -6
_ERR_NAMES = {
    NFD_ERR_NULL: "NFD_ERR_NULL", NFD_ERR_SHAPE: "NFD_ERR_SHAPE", NFD_ERR_UNSUPPORTED: "NFD_ERR_UNSUPPORTED",
    NFD_ERR_CAPACITY: "NFD_ERR_CAPACITY", NFD_ERR_HIP: "NFD_ERR_HIP", NFD_ERR_ALLOC: "NFD_ERR_ALLOC",
}

EXPORTS = (
    "nfd_attn_create", "nfd_block_causal_attn_fwd", "nfd_kvcache_append", "nfd_attn_destroy",
    "nfd_last_error", "nfd_attn_check_args", "nfd_attn_plan", "nfd_attn_visible_pairs",
    "nfd_rope_kvcache_append", "nfd_rope_check_args",
    "nfd_block_causal_attn_fwd_lse", "nfd_block_causal_attn_bwd",
    "nfd_kvcache_shift", "nfd_spec_init", "nfd_spec_next", "nfd_spec_accept", "nfd_attn_work_item",
    "nfd_block_causal_attn_fwd_noalloc", "nfd_kvcache_append_attn_fwd",
    "nfd_attn_q_tile_rows",
    "nfd_fp8_cache_bytes", "nfd_kvcache_append_fp8", "nfd_block_causal_attn_fwd_fp8kv", "nfd_kvcache_shift_fp8", "nfd_rope_kvcache_append_fp8",
)


class NfdError(RuntimeError):
    def __init__(self, code, where, detail=""):
        self.code = code
        super().__init__("%s failed with %s (%d)%s" % (where, _ERR_NAMES.get(code, "?"), code,
                                                      ": " + detail if detail else ""))


class Plan(ctypes.Structure):
    _fields_ = [
        ("kernel", ctypes.c_int), ("block_m", ctypes.c_int), ("block_n", ctypes.c_int),
        ("n_q_tiles", ctypes.c_int), ("n_splits", ctypes.c_int), ("n_workgroups", ctypes.c_int),
        ("key_tiles_visited", ctypes.c_int64), ("key_tiles_dense", ctypes.c_int64),
        ("workspace_bytes", ctypes.c_size_t),
    ]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Spec(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("capacity", "window", "n_spec", "total", "done", "cached", "t_offset")]


class SpecStep(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("n_drop", "frame_pos", "n_frames", "kv_frames", "q_frames", "t_offset")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


_lib = None


def lib():
    """Load the shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2506_01380_amd.build` "
                "(there is no CPU or PyTorch fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        L.nfd_attn_create.argtypes = [ctypes.POINTER(vp), ci, ci, ctypes.c_size_t]
        L.nfd_attn_create.restype = ci
        L.nfd_block_causal_attn_fwd.argtypes = [vp, vp, vp, vp, vp] + [ci] * 7 + [cf, vp]
        L.nfd_block_causal_attn_fwd.restype = ci
        L.nfd_block_causal_attn_fwd_noalloc.argtypes = [ci, vp, vp, vp, vp] + [ci] * 7 + [cf, vp, ctypes.c_char_p, ctypes.c_size_t]
        L.nfd_block_causal_attn_fwd_noalloc.restype = ci
        L.nfd_kvcache_append_attn_fwd.argtypes = [vp] * 7 + [ci] * 7 + [cf, vp]
        L.nfd_kvcache_append_attn_fwd.restype = ci
        L.nfd_block_causal_attn_fwd_lse.argtypes = [vp] * 6 + [ci] * 7 + [cf, vp]
        L.nfd_block_causal_attn_fwd_lse.restype = ci
        L.nfd_block_causal_attn_bwd.argtypes = [vp] * 10 + [ci] * 7 + [cf, vp]
        L.nfd_block_causal_attn_bwd.restype = ci
        L.nfd_kvcache_append.argtypes = [vp, vp, vp, vp, vp] + [ci] * 7 + [vp]
        L.nfd_kvcache_append.restype = ci
        L.nfd_rope_kvcache_append.argtypes = [vp] * 7 + [ci] * 13 + [cf, vp]
        L.nfd_rope_kvcache_append.restype = ci
        L.nfd_rope_check_args.argtypes = [ci] * 13
        L.nfd_rope_check_args.restype = ci
        L.nfd_kvcache_shift.argtypes = [vp, vp, vp] + [ci] * 7 + [vp]
        L.nfd_kvcache_shift.restype = ci
        L.nfd_spec_init.argtypes = [ctypes.POINTER(Spec)] + [ci] * 5
        L.nfd_spec_init.restype = ci
        L.nfd_spec_next.argtypes = [ctypes.POINTER(Spec), ctypes.POINTER(SpecStep)]
        L.nfd_spec_next.restype = ci
        L.nfd_spec_accept.argtypes = [ctypes.POINTER(Spec), ctypes.POINTER(SpecStep), ctypes.POINTER(ctypes.c_int32), ci,
                                      ctypes.POINTER(ci)]
        L.nfd_spec_accept.restype = ci
        L.nfd_attn_destroy.argtypes = [vp]
        L.nfd_attn_destroy.restype = ci
        L.nfd_last_error.argtypes = [vp]
        L.nfd_last_error.restype = ctypes.c_char_p
        L.nfd_attn_check_args.argtypes = [ci] * 8
        L.nfd_attn_check_args.restype = ci
        L.nfd_attn_plan.argtypes = [ci] * 9 + [ctypes.c_size_t, ctypes.POINTER(Plan)]
        L.nfd_attn_plan.restype = ci
        L.nfd_attn_work_item.argtypes = [ci] * 4 + [ctypes.c_uint] + [ctypes.POINTER(ci)] * 3
        L.nfd_attn_work_item.restype = ci
        L.nfd_attn_q_tile_rows.argtypes = [ci] * 3 + [ctypes.POINTER(ci)] * 2
        L.nfd_attn_q_tile_rows.restype = ci
        L.nfd_fp8_cache_bytes.argtypes = [ci] * 5 + [ctypes.POINTER(ctypes.c_size_t)]
        L.nfd_fp8_cache_bytes.restype = ci
        L.nfd_kvcache_append_fp8.argtypes = [vp] * 7 + [ci] * 7 + [vp]
        L.nfd_kvcache_append_fp8.restype = ci
        L.nfd_rope_kvcache_append_fp8.argtypes = [vp] * 9 + [ci] * 13 + [cf, vp]
        L.nfd_rope_kvcache_append_fp8.restype = ci
        L.nfd_kvcache_shift_fp8.argtypes = [vp, vp, vp] + [ci] * 7 + [vp]
        L.nfd_kvcache_shift_fp8.restype = ci
        L.nfd_block_causal_attn_fwd_fp8kv.argtypes = [vp] * 7 + [ci] * 7 + [cf, vp]
        L.nfd_block_causal_attn_fwd_fp8kv.restype = ci
        L.nfd_attn_visible_pairs.argtypes = [ci] * 3
        L.nfd_attn_visible_pairs.restype = ctypes.c_int64
        _lib = L
    return _lib


def _addr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream
    return int(stream)


def _check(rc, where, h=None):
    if rc != NFD_OK:
        detail = ""
        if h:
            detail = (lib().nfd_last_error(h) or b"").decode()
        raise NfdError(rc, where, detail)


def nfd_attn_create(dtype=NFD_BF16, device=0, workspace_bytes=0):
    h = ctypes.c_void_p()
    _check(lib().nfd_attn_create(ctypes.byref(h), dtype, device, workspace_bytes), "nfd_attn_create")
    return h


def nfd_block_causal_attn_fwd(h, q, k, v, out, B, H, F, T, D, kv_frames, q_frames, scale=0.0, stream=None):
    rc = lib().nfd_block_causal_attn_fwd(h, _addr(q), _addr(k), _addr(v), _addr(out), B, H, F, T, D,
                                         kv_frames, q_frames, scale, _stream(stream))
    _check(rc, "nfd_block_causal_attn_fwd", h)


def nfd_block_causal_attn_fwd_noalloc(dtype, q, k, v, out, B, H, F, T, D, kv_frames, q_frames, scale=0.0, stream=None):
    """The handle-free forward whose scratch is a fixed array inside the library (see the header)."""
    err = ctypes.create_string_buffer(256)
    rc = lib().nfd_block_causal_attn_fwd_noalloc(dtype, _addr(q), _addr(k), _addr(v), _addr(out), B, H, F, T, D,
                                                 kv_frames, q_frames, scale, _stream(stream), err, len(err))
    if rc != NFD_OK:
        raise NfdError(rc, "nfd_block_causal_attn_fwd_noalloc", err.value.decode())


def nfd_kvcache_append_attn_fwd(h, q, k_cache, v_cache, k_new, v_new, out, B, H, F, T, D, kv_frames, q_frames,
                                scale=0.0, stream=None):
    rc = lib().nfd_kvcache_append_attn_fwd(h, _addr(q), _addr(k_cache), _addr(v_cache), _addr(k_new), _addr(v_new),
                                           _addr(out), B, H, F, T, D, kv_frames, q_frames, scale, _stream(stream))
    _check(rc, "nfd_kvcache_append_attn_fwd", h)


def nfd_block_causal_attn_fwd_lse(h, q, k, v, out, lse, B, H, F, T, D, kv_frames, q_frames, scale=0.0, stream=None):
    rc = lib().nfd_block_causal_attn_fwd_lse(h, _addr(q), _addr(k), _addr(v), _addr(out), _addr(lse), B, H, F, T, D,
                                             kv_frames, q_frames, scale, _stream(stream))
    _check(rc, "nfd_block_causal_attn_fwd_lse", h)


def nfd_block_causal_attn_bwd(h, q, k, v, out, dout, lse, dq, dk, dv, B, H, F, T, D, kv_frames, q_frames,
                              scale=0.0, stream=None):
    rc = lib().nfd_block_causal_attn_bwd(h, _addr(q), _addr(k), _addr(v), _addr(out), _addr(dout), _addr(lse),
                                         _addr(dq), _addr(dk), _addr(dv), B, H, F, T, D, kv_frames, q_frames,
                                         scale, _stream(stream))
    _check(rc, "nfd_block_causal_attn_bwd", h)


def nfd_kvcache_append(h, k_cache, v_cache, k_new, v_new, B, H, F, T, D, frame_pos, n_frames, stream=None):
    rc = lib().nfd_kvcache_append(h, _addr(k_cache), _addr(v_cache), _addr(k_new), _addr(v_new), B, H, F, T, D,
                                  frame_pos, n_frames, _stream(stream))
    _check(rc, "nfd_kvcache_append", h)


def nfd_rope_kvcache_append(h, q, q_out, k_cache, v_cache, k_new, v_new, B, H, F, T, D, frame_pos, n_frames,
                            t_offset, grid_h, grid_w, n_t, n_h, n_w, theta=0.0, stream=None):
    rc = lib().nfd_rope_kvcache_append(h, _addr(q), _addr(q_out), _addr(k_cache), _addr(v_cache), _addr(k_new),
                                       _addr(v_new), B, H, F, T, D, frame_pos, n_frames, t_offset, grid_h, grid_w,
                                       n_t, n_h, n_w, theta, _stream(stream))
    _check(rc, "nfd_rope_kvcache_append", h)


def nfd_rope_check_args(dtype, B, H, F, T, D, frame_pos, n_frames, grid_h, grid_w, n_t, n_h, n_w):
    return lib().nfd_rope_check_args(dtype, B, H, F, T, D, frame_pos, n_frames, grid_h, grid_w, n_t, n_h, n_w)


def nfd_kvcache_shift(h, k_cache, v_cache, B, H, F, T, D, kv_frames, n_drop, stream=None):
    rc = lib().nfd_kvcache_shift(h, _addr(k_cache), _addr(v_cache), B, H, F, T, D, kv_frames, n_drop, _stream(stream))
    _check(rc, "nfd_kvcache_shift", h)


def nfd_fp8_cache_bytes(B, H, F, T, D):
    """Bytes of each of the two 8-bit caches (K codes and feature-major V codes)."""
    n = ctypes.c_size_t(0)
    _check(lib().nfd_fp8_cache_bytes(B, H, F, T, D, ctypes.byref(n)), "nfd_fp8_cache_bytes")
    return n.value


def nfd_kvcache_append_fp8(h, k8, v8t, k_scale, v_scale, k_new, v_new, B, H, F, T, D, frame_pos, n_frames, stream=None):
    rc = lib().nfd_kvcache_append_fp8(h, _addr(k8), _addr(v8t), _addr(k_scale), _addr(v_scale), _addr(k_new),
                                      _addr(v_new), B, H, F, T, D, frame_pos, n_frames, _stream(stream))
    _check(rc, "nfd_kvcache_append_fp8", h)


def nfd_rope_kvcache_append_fp8(h, q, q_out, k8, v8t, k_scale, v_scale, k_new, v_new, B, H, F, T, D, frame_pos, n_frames,
                                t_offset, grid_h, grid_w, n_t, n_h, n_w, theta=0.0, stream=None):
    rc = lib().nfd_rope_kvcache_append_fp8(h, _addr(q), _addr(q_out), _addr(k8), _addr(v8t), _addr(k_scale), _addr(v_scale),
                                           _addr(k_new), _addr(v_new), B, H, F, T, D, frame_pos, n_frames, t_offset,
                                           grid_h, grid_w, n_t, n_h, n_w, theta, _stream(stream))
    _check(rc, "nfd_rope_kvcache_append_fp8", h)


def nfd_kvcache_shift_fp8(h, k8, v8t, B, H, F, T, D, kv_frames, n_drop, stream=None):
    rc = lib().nfd_kvcache_shift_fp8(h, _addr(k8), _addr(v8t), B, H, F, T, D, kv_frames, n_drop, _stream(stream))
    _check(rc, "nfd_kvcache_shift_fp8", h)


def nfd_block_causal_attn_fwd_fp8kv(h, q, k8, v8t, k_scale, v_scale, out, B, H, F, T, D, kv_frames, q_frames,
                                    scale=0.0, stream=None):
    rc = lib().nfd_block_causal_attn_fwd_fp8kv(h, _addr(q), _addr(k8), _addr(v8t), _addr(k_scale), _addr(v_scale),
                                               _addr(out), B, H, F, T, D, kv_frames, q_frames, scale, _stream(stream))
    _check(rc, "nfd_block_causal_attn_fwd_fp8kv", h)


def nfd_spec_init(capacity, window, n_spec, n_prompt, total):
    s = Spec()
    _check(lib().nfd_spec_init(ctypes.byref(s), capacity, window, n_spec, n_prompt, total), "nfd_spec_init")
    return s


def nfd_spec_next(s):
    """Returns the next step (SpecStep) or None when all frames are done."""
    st = SpecStep()
    rc = lib().nfd_spec_next(ctypes.byref(s), ctypes.byref(st))
    if rc < 0:
        _check(rc, "nfd_spec_next")
    return st if rc == 1 else None


def nfd_spec_accept(s, step, actions):
    """actions: C-contiguous int32 numpy array [total, action_dim] on the host.  Returns the frames kept."""
    import numpy as np
    a = np.ascontiguousarray(actions, dtype=np.int32)
    n = ctypes.c_int(0)
    _check(lib().nfd_spec_accept(ctypes.byref(s), ctypes.byref(step), a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 a.shape[1], ctypes.byref(n)), "nfd_spec_accept")
    return n.value


def nfd_attn_destroy(h):
    _check(lib().nfd_attn_destroy(h), "nfd_attn_destroy")


def nfd_attn_check_args(dtype, B, H, F, T, D, kv_frames, q_frames):
    return lib().nfd_attn_check_args(dtype, B, H, F, T, D, kv_frames, q_frames)


def nfd_attn_plan(dtype, B, H, F, T, D, kv_frames, q_frames, num_cus=0, workspace_limit=0):
    pl = Plan()
    _check(lib().nfd_attn_plan(dtype, B, H, F, T, D, kv_frames, q_frames, num_cus, workspace_limit,
                               ctypes.byref(pl)), "nfd_attn_plan")
    return pl.as_dict()


def nfd_attn_work_item(BH, n_q_tiles, n_splits, group_q_tiles, block):
    """(bh, q_tile, split) of workgroup ``block``, or None past the end of the launch."""
    bh, qt, sp = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = lib().nfd_attn_work_item(BH, n_q_tiles, n_splits, int(group_q_tiles), block, ctypes.byref(bh), ctypes.byref(qt),
                                  ctypes.byref(sp))
    return (bh.value, qt.value, sp.value) if rc == NFD_OK else None


def nfd_attn_q_tile_rows(rows, n_q_tiles, q_tile):
    """(first_row, n_rows) of a query tile of the matrix-core forward, or None for arguments out of range."""
    r0, n = ctypes.c_int(), ctypes.c_int()
    rc = lib().nfd_attn_q_tile_rows(rows, n_q_tiles, q_tile, ctypes.byref(r0), ctypes.byref(n))
    return (r0.value, n.value) if rc == NFD_OK else None


def nfd_attn_visible_pairs(T, kv_frames, q_frames):
    return lib().nfd_attn_visible_pairs(T, kv_frames, q_frames)


def unmasked_flops(B, H, D, T, kv_frames, q_frames):
    """FLOPs of the visible (query, key) pairs only: 4*D per pair (QK^T and PV)."""
    return 4 * D * nfd_attn_visible_pairs(T, kv_frames, q_frames) * B * H


class Attention:
    """Convenience holder of one handle; shapes are read from the tensors.

    q: [B,H,q_frames*T,D]; k, v: [B,H,F*T,D] (the cache, or the full sequence)."""

    def __init__(self, dtype="bf16", device=0, workspace_bytes=0):
        self.dtype = {"bf16": NFD_BF16, "fp32": NFD_FP32}[dtype]
        self.h = nfd_attn_create(self.dtype, device, workspace_bytes)

    def _want(self):
        import torch
        return torch.bfloat16 if self.dtype == NFD_BF16 else torch.float32

    def _tensors(self, *ts):
        """Every tensor handed to the library: on the GPU, dense, of the handle's dtype."""
        want = self._want()
        for t in ts:
            if t.dtype != want or not t.is_contiguous() or not t.is_cuda or t.dim() != 4:
                raise ValueError("tensors must be contiguous 4-D CUDA tensors of the handle's dtype")

    def _geometry(self, q, k, v, T, kv_frames, q_frames):
        """Checks q [B,H,q_frames*T,D] against k, v [B,H,F*T,D]; returns (B, H, F, D, kv_frames, q_frames)."""
        self._tensors(q, k, v)
        B, H, Sq, D = q.shape
        if T < 1 or Sq % T or k.shape[2] % T:
            raise ValueError("sequence lengths must be multiples of T")
        F = k.shape[2] // T
        q_frames = Sq // T if q_frames is None else q_frames
        kv_frames = F if kv_frames is None else kv_frames
        if Sq != q_frames * T or k.shape != v.shape or tuple(k.shape[:2]) != (B, H) or k.shape[3] != D:
            raise ValueError("shape mismatch between q and k, v")
        return B, H, F, D, kv_frames, q_frames

    def _new_frames(self, k_cache, v_cache, k_new, v_new, T, *like_new):
        """Checks the caches [B,H,F*T,D] against the new frames [B,H,n*T,D]; returns (B, H, F, D, n_frames)."""
        self._tensors(k_cache, v_cache, k_new, v_new, *like_new)
        B, H, Sc, D = k_cache.shape
        if T < 1 or Sc % T or k_new.shape[2] % T:
            raise ValueError("sequence lengths must be multiples of T")
        if v_cache.shape != k_cache.shape or v_new.shape != k_new.shape or tuple(k_new.shape[:2]) != (B, H) or k_new.shape[3] != D:
            raise ValueError("shape mismatch between the caches and the new frames")
        for t in like_new:
            if t.shape != k_new.shape:
                raise ValueError("shape mismatch between q and the new frames")
        return B, H, Sc // T, D, k_new.shape[2] // T

    def forward(self, q, k, v, T, kv_frames=None, q_frames=None, out=None, scale=0.0, stream=None):
        import torch
        B, H, F, D, kv_frames, q_frames = self._geometry(q, k, v, T, kv_frames, q_frames)
        if out is None:
            out = torch.empty_like(q)
        else:
            self._tensors(out)
            if out.shape != q.shape:
                raise ValueError("out must have the shape of q")
        nfd_block_causal_attn_fwd(self.h, q, k, v, out, B, H, F, T, D, kv_frames, q_frames, scale, stream)
        return out

    def forward_lse(self, q, k, v, T, kv_frames=None, q_frames=None, scale=0.0, stream=None):
        """Forward that also returns the per-row log-sum-exp (fp32) for the backward call."""
        import torch
        B, H, F, D, kv_frames, q_frames = self._geometry(q, k, v, T, kv_frames, q_frames)
        out = torch.empty_like(q)
        lse = torch.empty((B, H, q.shape[2]), dtype=torch.float32, device=q.device)
        nfd_block_causal_attn_fwd_lse(self.h, q, k, v, out, lse, B, H, F, T, D, kv_frames, q_frames, scale, stream)
        return out, lse

    def backward(self, q, k, v, out, dout, lse, T, kv_frames=None, q_frames=None, scale=0.0, stream=None):
        """Gradients (dq, dk, dv); dk, dv have the shape of k, v (rows past kv_frames*T are zero)."""
        import torch
        B, H, F, D, kv_frames, q_frames = self._geometry(q, k, v, T, kv_frames, q_frames)
        self._tensors(out, dout)
        if out.shape != q.shape or dout.shape != q.shape:
            raise ValueError("out and dout must have the shape of q")
        if lse.dtype != torch.float32 or not lse.is_cuda or not lse.is_contiguous() or tuple(lse.shape) != (B, H, q.shape[2]):
            raise ValueError("lse must be a contiguous fp32 CUDA tensor [B, H, q_frames*T]")
        dq = torch.empty_like(q)
        dk, dv = torch.zeros_like(k), torch.zeros_like(v)
        nfd_block_causal_attn_bwd(self.h, q, k, v, out, dout, lse, dq, dk, dv, B, H, F, T, D, kv_frames, q_frames,
                                  scale, stream)
        return dq, dk, dv

    def append(self, k_cache, v_cache, k_new, v_new, T, frame_pos, stream=None):
        B, H, F, D, n_frames = self._new_frames(k_cache, v_cache, k_new, v_new, T)
        nfd_kvcache_append(self.h, k_cache, v_cache, k_new, v_new, B, H, F, T, D, frame_pos, n_frames, stream)

    def rope_append(self, q, k_cache, v_cache, k_new, v_new, T, frame_pos, grid, sections, theta=0.0,
                    t_offset=0, q_out=None, stream=None):
        """Rotate q and k_new (3D rotary embedding), write rotated keys and values into the caches.
        Returns the rotated queries (q itself when q_out is q)."""
        import torch
        B, H, F, D, n_frames = self._new_frames(k_cache, v_cache, k_new, v_new, T, q)
        if q_out is None:
            q_out = torch.empty_like(q)
        else:
            self._tensors(q_out)
            if q_out.shape != q.shape:
                raise ValueError("q_out must have the shape of q")
        nfd_rope_kvcache_append(self.h, q, q_out, k_cache, v_cache, k_new, v_new, B, H, F, T, D, frame_pos,
                                n_frames, t_offset, grid[0], grid[1], sections[0], sections[1], sections[2], theta,
                                stream)
        return q_out

    def close(self):
        if self.h is not None:
            nfd_attn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
