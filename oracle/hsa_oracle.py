"""CPU oracle for Light Forcing's per-chunk Hierarchical Sparse Attention (HSA).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow numpy implementation of what the
hot path computes, written from the paper's equations.  Only ``tests/``, the
``smoke()`` check and the benchmark's ``cpu_baseline`` leg may import it; the GPU
library never does, and the two share no code.

Notation (Sec. 4.2): H heads, d head dim, n tokens per frame, f frames per chunk,
b block size (b_q = b_kv), nb = ceil(n / b) blocks per frame, F_h history frames,
F = F_h + f frames in the cache (the current chunk's K/V are the LAST f frames),
n_q = f * nb query blocks, n_k = F * nb KV blocks.  KV block c = tau * nb + j is
block j of cache frame tau and covers tokens [tau*n + j*b, tau*n + min((j+1)*b, n)).

The method is a heuristic pipeline, so the oracle takes its steps in the paper's
order: token compression (Eq. 7), frame-level scores (Eq. 8), frame selection
(Eq. 9), block-level scores (Eq. 10), block selection (Eq. 11), block mask
(Eq. 12, kept as sorted index lists), blockwise sparse attention (Eq. 13 / Eq. 3),
and the Chunk-Aware Growth sparsity allocation (Eq. 5-6).

Arithmetic contract (the paper fixes no precision; selected index lists must be
reproducible bit for bit, so the order of every rounding is stated here):

* inputs are float32 arrays (bfloat16 values widened exactly);
* block sum: binary64 accumulation over the block's tokens in ascending order.
  For bfloat16-representable inputs with 2^-30 <= |x| < 2^8 (or x = 0) the sum of
  up to 64 tokens is exact in binary64, hence independent of the order;
  block mean = float32(sum / count) with count = number of valid tokens;
* frame mean: binary64 sum of the nb float32 block means in ascending j,
  divided by nb, rounded to float32;
* score: acc = 0.0; for t ascending over d: acc += float64(q[t]) * float64(k[t])
  (the product of two float32 is exact in binary64); score = float32(acc);
* top-k: larger float32 score first, equal scores (including -0.0 == +0.0) by lower
  index;
* attention: binary64 throughout, softmax over exactly the valid tokens of the
  kept blocks.

Readings of points the paper leaves open are listed next to the code that takes
them and in the design document.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

SCHED_FIXED, SCHED_LINEAR, SCHED_CAG = 0, 1, 2
OF_CANDIDATES, OF_HISTORY, OF_ALL = 0, 1, 2


@dataclass(frozen=True)
class Budget:
    """Integer keep-counts for one chunk (what mask selection needs)."""
    n_hist_frames: int      # F_h
    frames_per_chunk: int   # f
    n_sink: int             # clamped to the history
    n_win: int              # clamped to what the sink leaves
    k_frames: int           # frames retrieved by top-k from the candidate set M
    k_blocks: int           # blocks retrieved by top-k from the candidate set B_r
    current_mandatory: int  # 1: all current-chunk blocks kept, outside the top-k
    list_len: int           # kept KV blocks per (head, query block)
    keep_ratio: float = 1.0  # the ratio the counts were derived from (informational)


# ---------------------------------------------------------------------------
# Chunk-Aware Growth (Sec. 4.1, Eq. 5 and Eq. 6)
# ---------------------------------------------------------------------------

def cag_beta(n_chunks: int, s_base: float, s_target: float) -> float:
    """Solve the FLOPs equality (Eq. 6) for beta.

    Chunk i has l^q_i = f*n query tokens and l^k_i = i*f*n key tokens, so the weight
    l^q_i l^k_i d of chunk i is proportional to i.  alpha_i, the noise level reached
    by chunk i, scales as one over the square root of the number of denoising steps
    the chunk has effectively received; chunk i continues from chunk i-1's level for
    T further steps, so that number is i*T and alpha_i = 1/sqrt(i) up to a constant
    that beta absorbs.  With w_i = i, Eq. 6 reads
        (1 - s_target) * sum w_i = sum (1 - s_base + alpha_i * beta) * w_i ,  i = 2..n
    which gives beta = (s_base - s_target) * sum w_i / sum(alpha_i * w_i).
    """
    if n_chunks < 2:
        return 0.0
    num = 0.0
    den = 0.0
    for i in range(2, n_chunks + 1):
        num += float(i)
        den += float(i) / math.sqrt(float(i))
    return (s_base - s_target) * num / den


def cag_sparsity(i: int, n_chunks: int, s_base: float, s_target: float) -> float:
    """s_i = s_base - alpha_i * beta for chunk i > 1 (Eq. 5); the first chunk is dense."""
    if i <= 1:
        return 0.0
    return s_base - cag_beta(n_chunks, s_base, s_target) / math.sqrt(float(i))


def keep_ratio(chunk_idx: int, sched) -> float:
    """Fraction of blocks kept for this chunk under the schedule's mode."""
    if sched.first_chunk_dense and chunk_idx == 1:
        return 1.0
    if sched.mode == SCHED_FIXED:
        return float(sched.keep_fixed)
    if sched.mode == SCHED_LINEAR:
        if sched.n_chunks <= 1:
            return float(sched.keep_first)
        t = float(chunk_idx - 1) / float(sched.n_chunks - 1)
        return float(sched.keep_first) + (float(sched.keep_last) - float(sched.keep_first)) * t
    if sched.mode == SCHED_CAG:
        if chunk_idx == 1:
            return 1.0  # Eq. 5 is stated for i > 1; chunk 1 keeps everything
        return 1.0 - cag_sparsity(chunk_idx, sched.n_chunks, sched.s_base, sched.s_target)
    raise ValueError("unknown schedule mode")


def _ceil_count(ratio: float, total: int) -> int:
    # ceiling with a guard so that e.g. 0.4 * 225 = 90.00000000000001 stays 90
    return int(math.ceil(ratio * float(total) - 1e-9))


def chunk_budget(chunk_idx: int, sched) -> Budget:
    """Turn the chunk's keep ratio into integer counts.

    Frame sets (footnote to Eq. 7; text after Eq. 9; appendix, implementation
    details of Light Forcing): the n_sink earliest and the n_win nearest history
    frames and the f current frames are always selected; the candidate set M is the
    rest of the history, m = F_h - n_sink - n_win.  The window takes what the sink
    leaves when the history is short.  Frame retrieval is active only when M holds
    more than k_frames frames; otherwise all of M is kept.

    Reading: with no history at all the current chunk's blocks are the only
    candidates, so they compete in the block top-k whatever ``current_mandatory``
    says.
    """
    f = int(sched.frames_per_chunk)
    nb = -(-int(sched.frame_len) // int(sched.block))
    F_h = (chunk_idx - 1) * f
    n_sink = min(int(sched.n_sink), F_h)
    n_win = min(int(sched.n_win), F_h - n_sink)
    m = F_h - n_sink - n_win
    k_frames = min(int(sched.k_frames), m)
    cur_mand = 1 if (sched.current_mandatory and F_h > 0) else 0
    n_tf = n_sink + n_win + k_frames                # selected history frames
    n_cand = n_tf * nb + (0 if cur_mand else f * nb)  # |B_r|
    rho = keep_ratio(chunk_idx, sched)
    if not (0.0 <= rho <= 1.0):
        # Reading: s_i of Eq. 5 is a sparsity *ratio*; parameters that push it outside [0, 1]
        # (e.g. s_base 0.5, s_target 0.1 over 7 chunks gives s_2 < 0) define no schedule of the
        # method, and the paper gives no rule for them, so they are rejected, not altered.
        raise ValueError(f"keep ratio {rho} of chunk {chunk_idx} is outside [0, 1]")
    if sched.ratio_of == OF_CANDIDATES:
        k_blocks = _ceil_count(rho, n_cand)
    elif sched.ratio_of == OF_HISTORY:
        k_blocks = _ceil_count(rho, F_h * nb if F_h > 0 else n_cand)
    elif sched.ratio_of == OF_ALL:
        k_blocks = _ceil_count(rho, (F_h + f) * nb) - (f * nb if cur_mand else 0)
    else:
        raise ValueError("unknown ratio_of")
    k_blocks = max(min(k_blocks, n_cand), min(1, n_cand))
    list_len = k_blocks + (f * nb if cur_mand else 0)
    return Budget(F_h, f, n_sink, n_win, k_frames, k_blocks, cur_mand, list_len, rho)


# ---------------------------------------------------------------------------
# Token compression (Eq. 7)
# ---------------------------------------------------------------------------

def block_mean_pool(x: np.ndarray, frame_len: int, block: int) -> np.ndarray:
    """phi(x, b): mean over each block of b sequential tokens, blocks cut per frame.

    x: float32 [H, frames*frame_len, d].  Returns float32 [H, frames*nb, d].
    Reading: the shapes stated after Eq. 7 count ceil(n/b) blocks per frame, so
    blocks never straddle a frame; the last block of a frame holds n - (nb-1)*b
    tokens and its mean divides by that count.
    """
    x = np.asarray(x, dtype=np.float32)
    H, L, d = x.shape
    assert L % frame_len == 0
    frames = L // frame_len
    nb = -(-frame_len // block)
    out = np.empty((H, frames * nb, d), dtype=np.float32)
    for tau in range(frames):
        for j in range(nb):
            lo = tau * frame_len + j * block
            hi = tau * frame_len + min((j + 1) * block, frame_len)
            acc = np.zeros((H, d), dtype=np.float64)
            for t in range(lo, hi):                      # ascending token order
                acc += x[:, t, :].astype(np.float64)
            out[:, tau * nb + j, :] = (acc / float(hi - lo)).astype(np.float32)
    return out


def frame_mean_pool(k_tilde: np.ndarray, nb: int, frames: Sequence[int]) -> np.ndarray:
    """k_hat: phi(k_tilde^M, ceil(n/b_kv)) -- the mean of a frame's nb block summaries.

    k_tilde: float32 [H, F*nb, d]; frames: the candidate frame ids M.
    Returns float32 [H, len(frames), d].
    """
    H, _, d = k_tilde.shape
    out = np.empty((H, len(frames), d), dtype=np.float32)
    for a, tau in enumerate(frames):
        acc = np.zeros((H, d), dtype=np.float64)
        for j in range(nb):                              # ascending block order
            acc += k_tilde[:, tau * nb + j, :].astype(np.float64)
        out[:, a, :] = (acc / float(nb)).astype(np.float32)
    return out


# ---------------------------------------------------------------------------
# Scores (Eq. 8, Eq. 10) and TopK_idx (Eq. 9, Eq. 11)
# ---------------------------------------------------------------------------

def inner_products(q_tilde: np.ndarray, keys: np.ndarray) -> np.ndarray:
    """<q_tilde_r, key_c> for all r, c: raw inner product, no scaling, no softmax.

    q_tilde float32 [H, n_q, d], keys float32 [H, n_c, d] -> float32 [H, n_q, n_c].
    Accumulated in binary64 over t = 0..d-1 in ascending order, then rounded once.
    """
    H, n_q, d = q_tilde.shape
    n_c = keys.shape[1]
    acc = np.zeros((H, n_q, n_c), dtype=np.float64)
    q64 = q_tilde.astype(np.float64)
    k64 = keys.astype(np.float64)
    for t in range(d):
        acc += q64[:, :, t, None] * k64[:, None, :, t]
    return acc.astype(np.float32)


def topk_idx(scores: np.ndarray, k: int) -> np.ndarray:
    """Positions of the k largest float32 scores; ties go to the lower position."""
    s = np.asarray(scores, dtype=np.float32)
    order = np.argsort(-s, kind="stable")   # -0.0 and +0.0 compare equal -> stable keeps the lower
    return order[:k]


def frame_sets(b: Budget) -> Tuple[List[int], List[int], List[int], List[int]]:
    """(sink S, window W, current C, candidates M) as ascending frame ids."""
    F_h, f = b.n_hist_frames, b.frames_per_chunk
    S = list(range(0, b.n_sink))
    W = list(range(F_h - b.n_win, F_h))
    C = list(range(F_h, F_h + f))
    M = [t for t in range(F_h) if t not in S and t not in W]
    return S, W, C, M


# ---------------------------------------------------------------------------
# Mask selection (Eq. 7 - Eq. 12)
# ---------------------------------------------------------------------------

def select_mask(Q: np.ndarray, K: np.ndarray, frame_len: int, block: int, b: Budget,
                return_intermediates: bool = False):
    """Sorted KV-block index lists, int32 [H, n_q, list_len] (Eq. 12 as lists).

    Q float32 [H, f*n, d]; K float32 [H, F*n, d] with the current chunk last.
    Selection is per head and per query block, recomputed at every call.
    """
    Q = np.asarray(Q, dtype=np.float32)
    K = np.asarray(K, dtype=np.float32)
    H = Q.shape[0]
    nb = -(-frame_len // block)
    f, F_h = b.frames_per_chunk, b.n_hist_frames
    assert Q.shape[1] == f * frame_len and K.shape[1] == (F_h + f) * frame_len
    n_q = f * nb

    q_tilde = block_mean_pool(Q, frame_len, block)          # Eq. 7, blockwise
    k_tilde = block_mean_pool(K, frame_len, block)
    S, W, C, M = frame_sets(b)
    k_hat = frame_mean_pool(k_tilde, nb, M)                 # Eq. 7, framewise
    p = inner_products(q_tilde, k_hat) if M else np.zeros((H, n_q, 0), np.float32)  # Eq. 8
    o = inner_products(q_tilde, k_tilde)                    # Eq. 10 (all blocks; only B_r is read)

    lists = np.empty((H, n_q, b.list_len), dtype=np.int32)
    frames_sel = np.empty((H, n_q, b.k_frames), dtype=np.int32)
    for h in range(H):
        for r in range(n_q):
            top = [M[a] for a in topk_idx(p[h, r], b.k_frames)]       # Eq. 9
            frames_sel[h, r] = sorted(top)
            T_hist = sorted(set(top) | set(S) | set(W))
            cand_frames = T_hist if b.current_mandatory else T_hist + C
            cand = [tau * nb + j for tau in cand_frames for j in range(nb)]   # B_r
            sc = o[h, r, cand]
            kept = [cand[a] for a in topk_idx(sc, b.k_blocks)]        # Eq. 11
            if b.current_mandatory:
                kept += [tau * nb + j for tau in C for j in range(nb)]
            kept = sorted(kept)
            assert len(kept) == b.list_len and len(set(kept)) == b.list_len
            lists[h, r] = kept
    if return_intermediates:
        return lists, dict(q_tilde=q_tilde, k_tilde=k_tilde, k_hat=k_hat, p=p, o=o,
                           frames_sel=frames_sel, M=M)
    return lists


# ---------------------------------------------------------------------------
# Blockwise sparse attention (Eq. 13, i.e. Eq. 3 with the mask of Eq. 12)
# ---------------------------------------------------------------------------

def block_token_range(c: int, frame_len: int, block: int) -> Tuple[int, int]:
    nb = -(-frame_len // block)
    tau, j = divmod(int(c), nb)
    return tau * frame_len + j * block, tau * frame_len + min((j + 1) * block, frame_len)


def sparse_attention_block(Qh: np.ndarray, Kh: np.ndarray, Vh: np.ndarray, r: int,
                           kept: Sequence[int], frame_len: int, block: int,
                           scale: Optional[float] = None, return_probs: bool = False):
    """Eq. 13 for one head and one query block r.

    Reading: entries of the element mask M(B) that are zero remove the column from
    the softmax (their tiles are skipped); they do not contribute a logit of zero.
    Qh [f*n, d], Kh/Vh [F*n, d] float32; returns float64 [rows_r, d].
    """
    d = Qh.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(float(d))
    qlo, qhi = block_token_range(r, frame_len, block)
    cols: List[int] = []
    for c in kept:
        lo, hi = block_token_range(c, frame_len, block)
        cols.extend(range(lo, hi))
    cols_a = np.asarray(cols, dtype=np.int64)
    q = Qh[qlo:qhi].astype(np.float64)
    k = Kh[cols_a].astype(np.float64)
    v = Vh[cols_a].astype(np.float64)
    s = (q @ k.T) * scale
    s -= s.max(axis=1, keepdims=True)
    e = np.exp(s)
    P = e / e.sum(axis=1, keepdims=True)
    O = P @ v
    if return_probs:
        return O, P, cols_a
    return O


def sparse_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, lists: np.ndarray,
                     frame_len: int, block: int, scale: Optional[float] = None,
                     heads: Optional[Sequence[int]] = None,
                     qblocks: Optional[Sequence[int]] = None) -> np.ndarray:
    """O float64 [H, f*n, d]; rows of (head, query block) pairs not requested stay NaN."""
    H, Lq, d = Q.shape
    nb = -(-frame_len // block)
    n_q = (Lq // frame_len) * nb
    O = np.full((H, Lq, d), np.nan, dtype=np.float64)
    for h in (range(H) if heads is None else heads):
        for r in (range(n_q) if qblocks is None else qblocks):
            qlo, qhi = block_token_range(r, frame_len, block)
            O[h, qlo:qhi] = sparse_attention_block(Q[h], K[h], V[h], r, lists[h, r],
                                                   frame_len, block, scale)
    return O


def sparse_attention_backward(Q: np.ndarray, K: np.ndarray, V: np.ndarray, dO: np.ndarray,
                              lists: np.ndarray, frame_len: int, block: int,
                              scale: Optional[float] = None):
    """Gradients of Eq. 13 with respect to Q, K and V for an upstream gradient dO of O
    (the paper finetunes with the sparse mask in place, which needs exactly this).

    For a query row x of block r with kept columns Y_r, s_xy = scale q_x.k_y,
    p = softmax_y(s), o_x = sum_y p_xy v_y.  By the chain rule
        dV_y  = sum_x p_xy dO_x
        dp_xy = dO_x . v_y,   delta_x = sum_y p_xy dp_xy  (= dO_x . o_x)
        ds_xy = p_xy (dp_xy - delta_x)
        dQ_x  = scale sum_y ds_xy k_y,   dK_y = scale sum_x ds_xy q_x
    summed over every (x, y) pair the lists keep; an id listed twice counts twice, as in the
    forward pass.  All in binary64.  Returns (dQ [H, L_q, d], dK [H, L_k, d], dV [H, L_k, d]).
    """
    H, Lq, d = Q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(float(d))
    nb = -(-frame_len // block)
    n_q = (Lq // frame_len) * nb
    dQ = np.zeros((H, Lq, d), dtype=np.float64)
    dK = np.zeros((H, K.shape[1], d), dtype=np.float64)
    dV = np.zeros((H, K.shape[1], d), dtype=np.float64)
    for h in range(H):
        for r in range(n_q):
            qlo, qhi = block_token_range(r, frame_len, block)
            cols: List[int] = []
            for c in lists[h, r]:
                lo, hi = block_token_range(c, frame_len, block)
                cols.extend(range(lo, hi))
            cols_a = np.asarray(cols, dtype=np.int64)
            q = Q[h, qlo:qhi].astype(np.float64)
            k = K[h][cols_a].astype(np.float64)
            v = V[h][cols_a].astype(np.float64)
            do = dO[h, qlo:qhi].astype(np.float64)
            s = (q @ k.T) * scale
            s -= s.max(axis=1, keepdims=True)
            e = np.exp(s)
            p = e / e.sum(axis=1, keepdims=True)
            dp = do @ v.T
            delta = (p * dp).sum(axis=1, keepdims=True)
            ds = p * (dp - delta)
            dQ[h, qlo:qhi] += scale * (ds @ k)
            np.add.at(dK[h], cols_a, scale * (ds.T @ q))     # add.at: a column may be listed twice
            np.add.at(dV[h], cols_a, p.T @ do)
    return dQ, dK, dV


def full_lists(heads: int, frame_len: int, block: int, f: int, F: int) -> np.ndarray:
    """The all-ones block mask as index lists (full budget)."""
    nb = -(-frame_len // block)
    return np.broadcast_to(np.arange(F * nb, dtype=np.int32), (heads, f * nb, F * nb)).copy()
