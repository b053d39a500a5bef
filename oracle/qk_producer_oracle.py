"""CPU oracle for the producer of Q and K next to the hot path: RMSNorm followed by rotary
position embedding, written head-major in the layout mask selection and attention read.

TEST INFRASTRUCTURE ONLY (same rules as ``hsa_oracle``: only ``tests/``, ``smoke()`` and the
benchmark's ``cpu_baseline`` leg may import it; it shares no code with the GPU library).

The paper names these operators only as deployment kernels ("Efficient Deployment": RoPE,
RMSNorm and a fused scale/shift) and defines none of them, so the oracle is the textbook
definition of each, in binary64:

* RMSNorm of a vector x of length N with weight g:  y_c = x_c / sqrt(mean_c(x_c^2) + eps) * g_c.
  N is one head's channels (per-head norm) or all H*d channels of the token (``across_heads``):
  both conventions occur in video transformers, the caller says which.
* Rotary embedding with a per-token angle table theta[l, i], i < d/2 (the caller builds it: one
  position index for text, three for the temporal/height/width sections of a video token; the
  same table serves every head): channel pair (a, b) of a head is rotated by theta,
      a' = a cos(theta) - b sin(theta),   b' = a sin(theta) + b cos(theta).
  Pairing "interleaved": pair i is channels (2i, 2i+1); "half": pair i is (i, i + d/2).
  The table is passed as cos and sin (float32), as a kernel would take it.
* Output layout: y[h, l, :] -- head-major, d contiguous -- from a token-major input
  x[l, h*d:(h+1)*d] (what the projection's matrix product leaves).

Reading: the scale/shift modulation named beside them acts on the block's input before the
projections, not on Q or K, so it is not part of this producer.
"""
from __future__ import annotations

import numpy as np


def rms_norm(x: np.ndarray, g: np.ndarray, eps: float, heads: int, across_heads: bool) -> np.ndarray:
    """x [L, H*d] -> normalised [L, H*d] in binary64; g [H*d]."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    L, N = x.shape
    d = N // heads
    y = np.empty_like(x)
    for l in range(L):
        if across_heads:
            ms = 0.0
            for c in range(N):
                ms += x[l, c] * x[l, c]
            ms /= N
            y[l] = x[l] / np.sqrt(ms + eps) * g
        else:
            for h in range(heads):
                seg = x[l, h * d:(h + 1) * d]
                ms = 0.0
                for c in range(d):
                    ms += seg[c] * seg[c]
                ms /= d
                y[l, h * d:(h + 1) * d] = seg / np.sqrt(ms + eps) * g[h * d:(h + 1) * d]
    return y


def rope(y: np.ndarray, cos: np.ndarray, sin: np.ndarray, heads: int, pairing: str) -> np.ndarray:
    """Rotate the channel pairs of every head of y [L, H*d] by the token's angles (cos, sin [L, d/2])."""
    y = np.asarray(y, dtype=np.float64)
    cos = np.asarray(cos, dtype=np.float64)
    sin = np.asarray(sin, dtype=np.float64)
    L, N = y.shape
    d = N // heads
    out = np.empty_like(y)
    for h in range(heads):
        for i in range(d // 2):
            ia, ib = (2 * i, 2 * i + 1) if pairing == "interleaved" else (i, i + d // 2)
            a, b = y[:, h * d + ia], y[:, h * d + ib]
            out[:, h * d + ia] = a * cos[:, i] - b * sin[:, i]
            out[:, h * d + ib] = a * sin[:, i] + b * cos[:, i]
    return out


def qk_norm_rope(x: np.ndarray, g: np.ndarray, cos: np.ndarray, sin: np.ndarray, heads: int,
                 eps: float = 1e-6, across_heads: bool = False,
                 pairing: str = "interleaved") -> np.ndarray:
    """x float32 [L, H*d] (bfloat16 values widened) -> binary64 [H, L, d]."""
    L, N = x.shape
    d = N // heads
    y = rope(rms_norm(x, g, eps, heads, across_heads), cos, sin, heads, pairing)
    return np.ascontiguousarray(y.reshape(L, heads, d).transpose(1, 0, 2))
