"""ctypes front-end of the fp64 CPU oracle in ``nfd_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  It holds no
arithmetic of its own: it widens the inputs to fp64 (exact for bf16 and fp32
values), calls the C routine and returns fp64.

The C source is compiled with gcc on first use (``build()``); the shared
object sits next to the source.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nfd_oracle.c")
_LIB = os.path.join(_HERE, "libnfd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.nfd_oracle_block_causal_attn.argtypes = [dp, dp, dp, dp] + [ctypes.c_int] * 7 + [
            ctypes.c_double, ip, ctypes.c_int64]
        lib.nfd_oracle_block_causal_attn.restype = ctypes.c_int
        lib.nfd_oracle_block_causal_attn_bwd.argtypes = [dp] * 8 + [ctypes.c_int] * 7 + [ctypes.c_double]
        lib.nfd_oracle_block_causal_attn_bwd.restype = ctypes.c_int
        lib.nfd_oracle_kvcache_append.argtypes = [dp, dp] + [ctypes.c_int] * 7
        lib.nfd_oracle_kvcache_append.restype = ctypes.c_int
        lib.nfd_oracle_rope_kvcache_append.argtypes = [dp] * 6 + [ctypes.c_int] * 13 + [ctypes.c_double]
        lib.nfd_oracle_rope_kvcache_append.restype = ctypes.c_int
        lib.nfd_oracle_visible_pairs.argtypes = [ctypes.c_int] * 3
        lib.nfd_oracle_visible_pairs.restype = ctypes.c_int64
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def block_causal_attn(q, k, v, T, kv_frames=None, q_frames=None, scale=None, rows=None):
    """Block-wise causal attention (Sec. 3.1), fp64.

    q: [B,H,q_frames*T,D]; k, v: [B,H,F*T,D] with the first kv_frames*T rows valid.
    rows: optional 1-D int array of query-row indices; then only those rows are
    computed and the result is [B,H,len(rows),D].
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, Sq, D = q.shape
    if k.shape != v.shape or k.shape[:2] != (B, H) or k.shape[3] != D:
        raise ValueError("k/v shape mismatch")
    if Sq % T or k.shape[2] % T:
        raise ValueError("sequence lengths must be multiples of T")
    F = k.shape[2] // T
    if q_frames is None:
        q_frames = Sq // T
    if kv_frames is None:
        kv_frames = F
    if q_frames * T != Sq:
        raise ValueError("q rows != q_frames*T")
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    if rows is not None:
        rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        n_rows = rows.shape[0]
        rp = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        out = np.empty((B, H, n_rows, D), dtype=np.float64)
    else:
        n_rows, rp = 0, None
        out = np.empty((B, H, Sq, D), dtype=np.float64)
    rc = _load().nfd_oracle_block_causal_attn(
        _ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, F, T, D, kv_frames, q_frames,
        float(scale), rp, n_rows)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return out


def block_causal_attn_bwd(q, k, v, dout, T, kv_frames=None, q_frames=None, scale=None):
    """Gradients (dq, dk, dv) of the block-wise causal attention for the upstream gradient ``dout``,
    plus the per-row log of the softmax denominator: returns (dq, dk, dv, lse), all fp64.
    dk, dv have the shape of k, v; rows past kv_frames*T are zero."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, Sq, D = q.shape
    Scap = k.shape[2]
    q_frames = Sq // T if q_frames is None else q_frames
    kv_frames = Scap // T if kv_frames is None else kv_frames
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    lse = np.empty((B, H, Sq), dtype=np.float64)
    rc = _load().nfd_oracle_block_causal_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk),
                                                  _ptr(dv), _ptr(lse), B, H, Scap // T, T, D, kv_frames,
                                                  q_frames, scale)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return dq, dk, dv, lse


def kvcache_append(cache, fresh, T, frame_pos):
    """Write the frames of ``fresh`` into ``cache`` at frame ``frame_pos`` (Appendix B).
    Returns a new fp64 array; the input cache is not modified."""
    cache, fresh = _f64(cache).copy(), _f64(fresh)
    B, H, Sc, D = cache.shape
    n_frames = fresh.shape[2] // T
    rc = _load().nfd_oracle_kvcache_append(_ptr(cache), _ptr(fresh), B, H, Sc // T, T, D,
                                           frame_pos, n_frames)
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return cache


def rope_kvcache_append(q, k_cache, v_cache, k_new, v_new, T, frame_pos, grid, sections,
                        theta=10000.0, t_offset=0):
    """3D rotary embedding of q and k_new, rotated keys and values written into the caches at
    frame ``frame_pos`` (Sec. 3.1 "3D Positional Embedding", Appendix B).  ``grid`` = (grid_h,
    grid_w) with grid_h * grid_w == T; ``sections`` = (n_t, n_h, n_w) summing to D.
    Returns (q_rotated, k_cache, v_cache) as new fp64 arrays; the inputs are not modified."""
    q, k_new, v_new = _f64(q), _f64(k_new), _f64(v_new)
    k_cache, v_cache = _f64(k_cache).copy(), _f64(v_cache).copy()
    B, H, Sc, D = k_cache.shape
    n_frames = k_new.shape[2] // T
    q_out = np.empty_like(q)
    rc = _load().nfd_oracle_rope_kvcache_append(
        _ptr(q), _ptr(q_out), _ptr(k_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new), B, H, Sc // T, T, D,
        frame_pos, n_frames, t_offset, grid[0], grid[1], sections[0], sections[1], sections[2], float(theta))
    if rc != 0:
        raise ValueError("oracle rejected the arguments (rc=%d)" % rc)
    return q_out, k_cache, v_cache


def visible_pairs(T, kv_frames, q_frames):
    """Count of visible (query, key) pairs per head, by enumeration of the mask."""
    return int(_load().nfd_oracle_visible_pairs(T, kv_frames, q_frames))
