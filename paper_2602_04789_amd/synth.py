"""Seeded synthetic Q/K/V for the Hierarchical Sparse Attention hot path.

This module only *draws inputs*: it holds none of the method's arithmetic (no
pooling, scoring, selection, softmax or budget formula), so both the CPU
oracle's tests and the GPU path's tests may import it.  Needs numpy only.

What the tensors stand in for: the per-head query / key / value activations of
one self-attention layer of a Wan-1.3B-shaped autoregressive video diffusion
transformer (12 heads x 128, 30x52 = 1560 latent tokens per frame, 3-frame
chunks) while it generates chunk i against the KV cache of chunks < i
(Sec. 4.2, first paragraph of the formal description).  Trained weights and
evaluation prompts are not available, so the statistics below are synthetic:

* every element ~ N(0, 1);
* K gets a per-(head, frame) bias vector added to all tokens of the frame, so
  that frame-level mean pooling carries signal (frame top-k is non-trivial);
  with ``decay`` the bias std shrinks by 0.9 per frame of age;
* with ``sink`` the earliest cached frame has its K doubled (the attention-sink
  pattern the paper's logit visualisation describes);
* Q gets a per-(head, query frame) bias, and with ``q_follow`` each query block
  additionally gets 0.25x the K-bias of one pseudo-randomly chosen history
  frame, so different query blocks prefer different frames (the "diagonal"
  pattern of the same figure);
* everything is rounded to bfloat16 (round-to-nearest-even); values with
  magnitude below 2**-30 are flushed to zero so that a block sum of 64 tokens
  is exact in binary64 (see the arithmetic contract in the oracle header).

Every frame is drawn from its own counter-based stream
``default_rng([seed, kind, chunk, step, frame])`` so a rollout (growing cache,
several denoising steps per chunk) re-creates identical history frames in
every call without storing them.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

import numpy as np

# ratio_of / mode constants mirror the C header's enums (interface constants,
# not arithmetic).
SCHED_FIXED, SCHED_LINEAR, SCHED_CAG = 0, 1, 2
OF_CANDIDATES, OF_HISTORY, OF_ALL = 0, 1, 2

_CLEAN_STEP = 0xFFFF  # stream id of a chunk's committed (clean) frames
_KIND_Q, _KIND_K, _KIND_V, _KIND_KBIAS, _KIND_QBIAS, _KIND_FOLLOW = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Schedule:
    """Plain-data mirror of the C ``lf_schedule`` struct (field meaning there)."""
    mode: int = SCHED_FIXED
    n_chunks: int = 7
    frames_per_chunk: int = 3
    frame_len: int = 1560
    block: int = 64
    n_sink: int = 1
    n_win: int = 2
    k_frames: int = 3
    ratio_of: int = OF_HISTORY
    current_mandatory: int = 1
    first_chunk_dense: int = 0
    keep_fixed: float = 1.0
    keep_first: float = 1.0
    keep_last: float = 1.0
    s_base: float = 0.98
    s_target: float = 0.88


@dataclass(frozen=True)
class Workload:
    """One call of the hot path: shapes, the chunk it belongs to, the recipe."""
    name: str
    heads: int
    head_dim: int
    frame_len: int          # n: tokens per frame
    frames_per_chunk: int   # f
    chunk_idx: int          # i (1-based); history = (i-1)*f frames
    schedule: Schedule
    seed: int
    block: int = 64
    step: int = 0           # denoising step (only changes the current chunk's draw)
    bias_std: float = 0.5
    decay: bool = False
    sink: bool = False
    q_bias: bool = True
    q_follow: bool = False

    @property
    def hist_frames(self) -> int:
        return (self.chunk_idx - 1) * self.frames_per_chunk

    @property
    def frames(self) -> int:
        return self.chunk_idx * self.frames_per_chunk

    @property
    def q_len(self) -> int:
        return self.frames_per_chunk * self.frame_len

    @property
    def kv_len(self) -> int:
        return self.frames * self.frame_len

    @property
    def blocks_per_frame(self) -> int:
        return -(-self.frame_len // self.block)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _round_bf16(x: np.ndarray) -> np.ndarray:
    bits = f32_to_bf16_bits(x)
    back = bf16_bits_to_f32(bits)
    tiny = np.abs(back) < np.float32(2.0 ** -30)
    if tiny.any():
        bits = bits.copy()
        bits[tiny] = 0
    return bits


def _rng(seed: int, kind: int, chunk: int, step: int, frame: int) -> np.random.Generator:
    return np.random.default_rng([seed, kind, chunk, step, frame])


def _k_bias(w: Workload, frame: int) -> np.ndarray:
    """Per-(head, frame) K bias vector, [H, d] float32 (not yet scaled by age)."""
    return _rng(w.seed, _KIND_KBIAS, 0, 0, frame).standard_normal(
        (w.heads, w.head_dim), dtype=np.float32)


def _bias_std(w: Workload, frame: int) -> float:
    if not w.decay:
        return w.bias_std
    age = max(w.hist_frames - 1 - frame, 0)  # current-chunk frames have age 0
    return w.bias_std * (0.9 ** age)


def _frame_owner(w: Workload, frame: int) -> Tuple[int, int]:
    """(chunk, step) whose draw defines this cache frame: history frames are the
    clean frames committed by their own chunk (step = -1 stream); frames of the
    current chunk are redrawn at every denoising step."""
    chunk = frame // w.frames_per_chunk + 1
    if chunk == w.chunk_idx:
        return chunk, w.step
    return chunk, _CLEAN_STEP


def make_inputs(w: Workload) -> Dict[str, np.ndarray]:
    """Draw Q [H, L_q, d], K and V [H, L_k, d] as bfloat16 bit patterns (uint16).

    The current chunk's K/V are the last ``f`` frames of the cache.
    """
    H, d, n, f = w.heads, w.head_dim, w.frame_len, w.frames_per_chunk
    F = w.frames
    K = np.empty((H, F * n, d), dtype=np.uint16)
    V = np.empty((H, F * n, d), dtype=np.uint16)
    Q = np.empty((H, f * n, d), dtype=np.uint16)
    for tau in range(F):
        chunk, step = _frame_owner(w, tau)
        k = _rng(w.seed, _KIND_K, chunk, step, tau).standard_normal((H, n, d), dtype=np.float32)
        k += (np.float32(_bias_std(w, tau)) * _k_bias(w, tau))[:, None, :]
        if w.sink and tau == 0 and w.hist_frames > 0:
            k *= np.float32(2.0)
        K[:, tau * n:(tau + 1) * n, :] = _round_bf16(k)
        v = _rng(w.seed, _KIND_V, chunk, step, tau).standard_normal((H, n, d), dtype=np.float32)
        V[:, tau * n:(tau + 1) * n, :] = _round_bf16(v)
    nb = w.blocks_per_frame
    for qf in range(f):
        tau = w.hist_frames + qf
        q = _rng(w.seed, _KIND_Q, w.chunk_idx, w.step, tau).standard_normal((H, n, d), dtype=np.float32)
        if w.q_bias:
            qb = _rng(w.seed, _KIND_QBIAS, w.chunk_idx, w.step, tau).standard_normal(
                (H, d), dtype=np.float32)
            q += (np.float32(w.bias_std) * qb)[:, None, :]
        if w.q_follow and w.hist_frames > 0:
            pick = _rng(w.seed, _KIND_FOLLOW, w.chunk_idx, w.step, tau).integers(
                0, w.hist_frames, size=(H, nb))
            for j in range(nb):
                lo, hi = j * w.block, min((j + 1) * w.block, n)
                for h in range(H):
                    t = int(pick[h, j])
                    q[h, lo:hi, :] += np.float32(0.25 * _bias_std(w, t)) * _k_bias(w, t)[h]
        Q[:, qf * n:(qf + 1) * n, :] = _round_bf16(q)
    return {"Q": Q, "K": K, "V": V}


# ---------------------------------------------------------------------------
# The named workloads (the five benchmark configurations plus test shapes).
# ---------------------------------------------------------------------------

def _sched(**kw) -> Schedule:
    return Schedule(**kw)


def cfg_tiny() -> Workload:
    """Oracle-scale case: 2 heads x 64, frame 256, 4 cached frames + 1-frame chunk,
    keep 2 frames and 50% of their blocks, current chunk always kept."""
    s = _sched(mode=SCHED_FIXED, n_chunks=5, frames_per_chunk=1, frame_len=256, block=64,
               n_sink=0, n_win=0, k_frames=2, ratio_of=OF_CANDIDATES, current_mandatory=1,
               keep_fixed=0.5)
    return Workload("tiny", 2, 64, 256, 1, 5, s, seed=0, q_bias=False)


def cfg_first_chunk() -> Workload:
    """First chunk, no history: the 75 current blocks compete, 60% kept."""
    s = _sched(mode=SCHED_FIXED, n_chunks=7, n_sink=1, n_win=2, k_frames=3,
               ratio_of=OF_CANDIDATES, current_mandatory=0, keep_fixed=0.6)
    return Workload("first_chunk", 12, 128, 1560, 3, 1, s, seed=1)


def cfg_mid_rollout() -> Workload:
    """Chunk 4 of 7: 9 history frames, 40% of history blocks + full current chunk."""
    s = _sched(mode=SCHED_FIXED, n_chunks=7, n_sink=1, n_win=2, k_frames=3,
               ratio_of=OF_HISTORY, current_mandatory=1, keep_fixed=0.40)
    return Workload("mid_rollout", 12, 128, 1560, 3, 4, s, seed=2,
                    decay=True, sink=True, q_follow=True)


def cfg_last_chunk() -> Workload:
    """Chunk 7 of 7: 18 history frames, 25% of history blocks + full current chunk."""
    s = _sched(mode=SCHED_FIXED, n_chunks=7, n_sink=1, n_win=2, k_frames=3,
               ratio_of=OF_HISTORY, current_mandatory=1, keep_fixed=0.25)
    return Workload("last_chunk", 12, 128, 1560, 3, 7, s, seed=3,
                    decay=True, sink=True, q_follow=True)


def cfg_rollout(chunk_idx: int, step: int, heads: int = 40) -> Workload:
    """One (chunk, step) call of the 7-chunk, 4-step, 40-head rollout with keep
    ratios falling linearly from 80% to 25%."""
    s = _sched(mode=SCHED_LINEAR, n_chunks=7, n_sink=1, n_win=2, k_frames=3,
               ratio_of=OF_HISTORY, current_mandatory=1, keep_first=0.80, keep_last=0.25)
    return Workload(f"rollout_c{chunk_idx}_s{step}", heads, 128, 1560, 3, chunk_idx, s,
                    seed=4, step=step, decay=True, sink=True, q_follow=True)


def cfg_paper_5s(chunk_idx: int, heads: int = 12) -> Workload:
    """The paper's own operating point (Experimental Details; hyper-parameter table):
    512x768 -> 1536 tokens/frame (24 blocks), Chunk-Aware Growth with s_target 0.88 /
    s_base 0.98, 6 retained past frames of which 1 sink + 2 window, first chunk dense,
    budget counted over all KV blocks with the current chunk competing."""
    s = _sched(mode=SCHED_CAG, n_chunks=7, frame_len=1536, n_sink=1, n_win=2, k_frames=3,
               ratio_of=OF_ALL, current_mandatory=0, first_chunk_dense=1,
               s_base=0.98, s_target=0.88)
    return Workload(f"paper5s_c{chunk_idx}", heads, 128, 1536, 3, chunk_idx, s, seed=5,
                    decay=True, sink=True, q_follow=True)


def cfg_paper_15s(chunk_idx: int, heads: int = 12) -> Workload:
    """The paper's 15-second setting (hyper-parameter table): 21 chunks, s_target 0.85 /
    s_base 0.95, 3 retained past frames of which 1 sink + 1 window, otherwise as the
    5-second operating point."""
    s = _sched(mode=SCHED_CAG, n_chunks=21, frame_len=1536, n_sink=1, n_win=1, k_frames=1,
               ratio_of=OF_ALL, current_mandatory=0, first_chunk_dense=1,
               s_base=0.95, s_target=0.85)
    return Workload(f"paper15s_c{chunk_idx}", heads, 128, 1536, 3, chunk_idx, s, seed=6,
                    decay=True, sink=True, q_follow=True)


def scaled(w: Workload, **kw) -> Workload:
    """A copy of ``w`` with fields replaced (schedule fields via ``schedule=``)."""
    return replace(w, **kw)


def small_ragged(seed: int = 11, heads: int = 3, head_dim: int = 128, frame_len: int = 200,
                 chunk_idx: int = 4, frames_per_chunk: int = 2, **sched_kw) -> Workload:
    """A test shape the oracle finishes in seconds that still spans several blocks
    per frame and a ragged tail block (200 = 3*64 + 8)."""
    base = dict(mode=SCHED_FIXED, n_chunks=8, frames_per_chunk=frames_per_chunk,
                frame_len=frame_len, n_sink=1, n_win=1, k_frames=2, ratio_of=OF_HISTORY,
                current_mandatory=1, keep_fixed=0.4)
    base.update(sched_kw)
    s = _sched(**base)
    return Workload(f"ragged_{frame_len}_{chunk_idx}", heads, head_dim, frame_len,
                    frames_per_chunk, chunk_idx, s, seed=seed, decay=True, sink=True,
                    q_follow=True)


# ---------------------------------------------------------------------------
# Inputs of the Q/K producer (RMSNorm + rotary embedding)
# ---------------------------------------------------------------------------

def make_upstream_grad(w: Workload, seed: int = 5) -> np.ndarray:
    """Upstream gradient dO of the attention output, bfloat16 bits [H, q_len, d]: independent
    standard normal entries (what a loss hands back through an output projection has no
    structure the backward pass could exploit)."""
    rng = np.random.default_rng([seed, 91, w.chunk_idx, w.heads, w.head_dim])
    return _round_bf16(rng.standard_normal((w.heads, w.q_len, w.head_dim), dtype=np.float32))


def make_producer_inputs(tokens: int, heads: int, head_dim: int, seed: int,
                         grid_hw: Tuple[int, int] = (30, 52), x_pad: int = 0) -> Dict[str, np.ndarray]:
    """Token-major activations X [tokens, heads*head_dim + x_pad] (bfloat16 bits; what a
    projection layer leaves, with a per-channel gain so channels differ in scale), an RMSNorm
    weight g (float32, around 1) and a rotary angle table theta [tokens, head_dim/2] for video
    tokens laid out frame by frame on a grid of grid_hw patches: the channel pairs are split into
    three sections that rotate with the token's frame index, row and column, each section with
    geometrically spaced frequencies (a generic three-axis rotary construction; the values only
    have to be plausible angles)."""
    rng = np.random.default_rng([seed, 77, tokens, heads, head_dim])
    n = heads * head_dim
    gain = np.exp(0.5 * rng.standard_normal(n)).astype(np.float32)
    x = rng.standard_normal((tokens, n), dtype=np.float32) * gain[None, :]
    X = np.zeros((tokens, n + x_pad), dtype=np.uint16)
    X[:, :n] = _round_bf16(x)
    g = (1.0 + 0.1 * rng.standard_normal(n)).astype(np.float32)
    half = head_dim // 2
    sec = [half - 2 * (half // 3), half // 3, half // 3]
    gh, gw = grid_hw
    l = np.arange(tokens)
    pos = [l // (gh * gw), (l // gw) % gh, l % gw]
    cols = []
    for size, p in zip(sec, pos):
        freq = 10000.0 ** (-np.arange(size, dtype=np.float64) / max(size, 1))
        cols.append(p[:, None].astype(np.float64) * freq[None, :])
    theta = np.concatenate(cols, axis=1)
    return {"X": X, "g": g, "cos": np.cos(theta).astype(np.float32),
            "sin": np.sin(theta).astype(np.float32)}
