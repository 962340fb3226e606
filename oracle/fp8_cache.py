"""CPU oracle of the 8-bit KV cache (the cache of Appendix B, "KV caching", held in 8-bit floating
point: the post-training quantisation the paper names as an acceleration it leaves out, Sec. 6).

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` and never by the product package.

The paper fixes no format, so the reading taken here is the plainest one that a matrix-core kernel
can consume without changing the attention arithmetic:

* codes are OCP 8-bit floating point E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits;
  no infinities, the all-ones magnitude 0x7F is NaN, largest finite value 448, subnormals m * 2^-9);
* one scale per (batch, head) and tensor, chosen by the caller:  stored code = E4M3(x / scale),
  value read back = decode(code) * scale;
* quantisation rounds to nearest, ties to the even code, and saturates at +-448; the quotient
  x / scale is formed in fp32 as x * (1 / scale) with both operations correctly rounded - this is the
  precision in which the decision is taken, on both sides;
* attention then runs on the values read back, exactly as on an unquantised cache.

Layouts: the K cache is [B, H, S, D] codes; the V cache is stored feature-major, [B, H, D, S]
(S = cache capacity in keys), because the second product consumes V transposed.
"""
from __future__ import annotations

import numpy as np

from . import nfd_oracle as orc

E4M3_MAX = 448.0


def _magnitudes() -> np.ndarray:
    """The 127 finite non-negative E4M3 values in code order (code 0x00 .. 0x7E), from the definition."""
    vals = []
    for code in range(0x7F):
        e, m = code >> 3, code & 7
        vals.append(m * 2.0 ** -9 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return np.asarray(vals, dtype=np.float64)


_MAG = _magnitudes()


def e4m3_decode(codes) -> np.ndarray:
    """fp64 value of every code (NaN for 0x7F / 0xFF)."""
    codes = np.asarray(codes, dtype=np.uint8)
    mag = np.append(_MAG, np.nan)[codes & 0x7F]
    return np.where(codes & 0x80, -mag, mag)


def e4m3_encode(x) -> np.ndarray:
    """Nearest code of every fp32 value: ties to the even code, saturating at +-448; -0 and negative
    values that round to zero keep their sign bit."""
    x = np.asarray(x, dtype=np.float32)
    a = np.minimum(np.abs(x).astype(np.float64), E4M3_MAX)
    hi = np.searchsorted(_MAG, a, side="left")          # first code whose value is >= a
    hi = np.minimum(hi, len(_MAG) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - _MAG[lo], _MAG[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return code | (np.signbit(x).astype(np.uint8) << 7)


def quantize(x, scale) -> np.ndarray:
    """Codes of x / scale; scale broadcasts against x.  The quotient is x * (1 / scale) in fp32."""
    inv = (np.float32(1.0) / np.asarray(scale, dtype=np.float32)).astype(np.float32)
    return e4m3_encode(np.asarray(x, dtype=np.float32) * inv)


def kvcache_append_fp8(k8, v8t, k_new, v_new, T, frame_pos, k_scale, v_scale):
    """Quantise the new frames into the caches in place.  k8 [B,H,S,D], v8t [B,H,D,S] uint8;
    k_new, v_new [B,H,n*T,D]; k_scale, v_scale [B,H]."""
    n = k_new.shape[2]
    j0 = frame_pos * T
    if j0 + n > k8.shape[2]:
        raise ValueError("append exceeds the cache capacity")
    ks = np.asarray(k_scale, dtype=np.float32)[:, :, None, None]
    vs = np.asarray(v_scale, dtype=np.float32)[:, :, None, None]
    k8[:, :, j0:j0 + n, :] = quantize(k_new, ks)
    v8t[:, :, :, j0:j0 + n] = np.swapaxes(quantize(v_new, vs), 2, 3)


def dequantize(k8, v8t, k_scale, v_scale):
    """fp64 K and V ([B,H,S,D] both) as the attention reads them."""
    k = e4m3_decode(k8) * np.asarray(k_scale, dtype=np.float64)[:, :, None, None]
    v = np.swapaxes(e4m3_decode(v8t), 2, 3) * np.asarray(v_scale, dtype=np.float64)[:, :, None, None]
    return k, v


def block_causal_attn_fp8kv(q, k8, v8t, k_scale, v_scale, T, kv_frames, q_frames, scale=None, rows=None):
    """Block-wise causal attention (Sec. 3.1) over the first kv_frames frames of an 8-bit cache."""
    Sk = kv_frames * T
    k, v = dequantize(k8[:, :, :Sk], v8t[:, :, :, :Sk], k_scale, v_scale)
    return orc.block_causal_attn(q, k, v, T, kv_frames=kv_frames, q_frames=q_frames, scale=scale, rows=rows)
