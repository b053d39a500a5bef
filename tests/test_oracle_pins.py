"""Pins for the CPU oracle: each check ties one oracle function to something that is not
the oracle itself -- the paper's own equations evaluated another way, brute force on tiny
inputs, integer arithmetic, or a library routine on a special case.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import hsa_oracle as O
from paper_2602_04789_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


def _inputs(w):
    x = synth.make_inputs(w)
    return tuple(synth.bf16_bits_to_f32(x[k]) for k in "QKV")


# ----------------------------------------------------------------------------- CAG (Eq. 5-6)

@pytest.mark.parametrize("row", _rows("lf_hyperparams.txt"), ids=lambda r: r[0])
def test_cag_satisfies_flops_equality(row):
    """Eq. 6 evaluated directly with explicit sequence lengths (not the closed form)."""
    _, s_target, s_base, _, _, _, n_chunks = row
    s_target, s_base, n_chunks = float(s_target), float(s_base), int(n_chunks)
    f, n, d = 3, 1536, 128
    lhs = rhs = 0.0
    s = []
    for i in range(2, n_chunks + 1):
        lq, lk = f * n, i * f * n
        s_i = O.cag_sparsity(i, n_chunks, s_base, s_target)
        s.append(s_i)
        lhs += (1.0 - s_target) * lq * lk * d
        rhs += (1.0 - s_i) * lq * lk * d
    assert abs(lhs - rhs) <= 1e-12 * lhs
    assert all(a < b for a, b in zip(s, s[1:])), "later chunks must be sparser"
    assert all(x < s_base for x in s)
    assert s[0] < s_target < s[-1]
    assert O.cag_sparsity(1, n_chunks, s_base, s_target) == 0.0  # first chunk dense


def test_cag_beta_matches_numeric_root():
    """beta from a root finder on the residual of Eq. 6, independent of the algebra."""
    from scipy.optimize import brentq
    for s_target, s_base, n_chunks in ((0.88, 0.98, 7), (0.85, 0.95, 21), (0.5, 0.9, 4)):
        def resid(beta):
            tot = 0.0
            for i in range(2, n_chunks + 1):
                w = float(i)
                tot += (1.0 - s_target) * w - (1.0 - s_base + beta / math.sqrt(i)) * w
            return tot
        root = brentq(resid, 0.0, 10.0, xtol=1e-15, rtol=1e-15)
        assert abs(root - O.cag_beta(n_chunks, s_base, s_target)) < 1e-12


def test_cag_special_cases():
    # one sparse chunk only: the equality forces s_2 = s_target
    assert abs(O.cag_sparsity(2, 2, 0.98, 0.88) - 0.88) < 1e-15
    # s_base == s_target: beta = 0 and every chunk sits at the target
    for i in range(2, 8):
        assert O.cag_sparsity(i, 7, 0.9, 0.9) == 0.9


def test_linear_schedule_endpoints_and_monotone():
    sch = synth.cfg_rollout(1, 0).schedule
    ks = [O.keep_ratio(i, sch) for i in range(1, 8)]
    assert ks[0] == 0.80 and abs(ks[-1] - 0.25) < 1e-15
    assert all(a > b for a, b in zip(ks, ks[1:]))
    assert np.allclose(np.diff(ks), (0.25 - 0.80) / 6)


# ----------------------------------------------------------------------------- budgets

@pytest.mark.parametrize("row", _rows("baseline_configs.txt"), ids=lambda r: f"{r[0]}-{r[1]}")
def test_budget_counts_of_benchmark_configs(row):
    name, chunk, k_blocks, list_len = row[0], int(row[1]), int(row[2]), int(row[3])
    w = {"first_chunk": synth.cfg_first_chunk, "mid_rollout": synth.cfg_mid_rollout,
         "last_chunk": synth.cfg_last_chunk}.get(name, lambda: synth.cfg_rollout(chunk, 0))()
    assert w.chunk_idx == chunk
    b = O.chunk_budget(chunk, w.schedule)
    assert (b.k_blocks, b.list_len) == (k_blocks, list_len)


@pytest.mark.parametrize("row", _rows("lf_hyperparams.txt"), ids=lambda r: r[0])
def test_candidate_count_and_activation_rule(row):
    """m = (i-1) f - n_sink - n_win (footnote to Eq. 7); retrieval is active only when the
    history is longer than n_past_keep, else every history frame is kept (appendix)."""
    _, s_target, s_base, n_keep, n_sink, n_win, n_chunks = row
    n_keep, n_sink, n_win, n_chunks = int(n_keep), int(n_sink), int(n_win), int(n_chunks)
    f = 3
    sch = synth.Schedule(mode=synth.SCHED_CAG, n_chunks=n_chunks, frames_per_chunk=f,
                         frame_len=1536, n_sink=n_sink, n_win=n_win,
                         k_frames=n_keep - n_sink - n_win, ratio_of=synth.OF_ALL,
                         current_mandatory=0, first_chunk_dense=1,
                         s_base=float(s_base), s_target=float(s_target))
    for i in range(1, n_chunks + 1):
        b = O.chunk_budget(i, sch)
        F_h = (i - 1) * f
        S, W, C, M = O.frame_sets(b)
        assert len(C) == f and C == list(range(F_h, F_h + f))
        assert set(S).isdisjoint(W) and set(S) | set(W) | set(M) == set(range(F_h))
        if F_h >= n_sink + n_win:
            assert len(M) == F_h - n_sink - n_win
        kept_hist = b.n_sink + b.n_win + b.k_frames
        if F_h <= n_keep:
            assert kept_hist == F_h            # all history frames preserved
        else:
            assert kept_hist == n_keep
        if i == 1:
            assert b.list_len == f * 24        # dense first chunk
        else:
            # overall keep count follows ceil((1 - s_i) * n_k), clamped to the candidates
            want = math.ceil((1.0 - O.cag_sparsity(i, n_chunks, float(s_base), float(s_target)))
                             * i * f * 24 - 1e-9)
            assert b.list_len == min(want, (kept_hist + f) * 24)


@pytest.mark.parametrize("row", _rows("cag_list_len.txt"), ids=lambda r: f"{r[0]}-{r[1]}")
def test_budget_counts_of_the_papers_operating_points(row):
    """Keep-counts worked out by hand from Eq. 5-6 and the appendix table (golden file)."""
    setting, chunk, k_blocks = row[0], int(row[1]), int(row[2])
    w = (synth.cfg_paper_5s if setting == "5s" else synth.cfg_paper_15s)(chunk)
    b = O.chunk_budget(chunk, w.schedule)
    assert (b.k_blocks, b.list_len, b.current_mandatory) == (k_blocks, k_blocks, 0)


def test_schedule_leaving_the_unit_interval_is_rejected():
    """Eq. 5 with s_base 0.5 / s_target 0.1 over 7 chunks: beta = 0.4 * 27 / 12.4776 = 0.8655,
    s_2 = 0.5 - 0.8655 / sqrt(2) = -0.112 -- not a sparsity ratio.  In-range chunks of the same
    schedule (s_7 = 0.173) are still served."""
    sch = synth.Schedule(mode=synth.SCHED_CAG, n_chunks=7, frame_len=1536, ratio_of=synth.OF_ALL,
                         current_mandatory=0, first_chunk_dense=1, s_base=0.5, s_target=0.1)
    assert O.cag_sparsity(2, 7, 0.5, 0.1) < 0.0 < O.cag_sparsity(7, 7, 0.5, 0.1)
    with pytest.raises(ValueError):
        O.chunk_budget(2, sch)
    b = O.chunk_budget(7, sch)
    assert b.k_blocks == min(math.ceil((1 - (0.5 - 0.8655369 / math.sqrt(7))) * 7 * 72), 216)


# ----------------------------------------------------------------------------- pooling (Eq. 7)

def test_block_sums_are_exact_integer_arithmetic():
    """For bf16 inputs in range, the binary64 block sum equals the exact sum: check with
    integers (values scaled by 2^37 are integers below 2^45)."""
    w = synth.small_ragged()
    _, K, _ = _inputs(w)
    n, b = w.frame_len, w.block
    pooled = O.block_mean_pool(K, n, b)
    nb = w.blocks_per_frame
    scaled = np.ldexp(K.astype(np.float64), 37)
    ints = scaled.astype(np.int64)
    assert np.array_equal(ints.astype(np.float64), scaled)
    for tau in range(w.frames):
        for j in range(nb):
            lo, hi = tau * n + j * b, tau * n + min((j + 1) * b, n)
            exact = ints[:, lo:hi, :].sum(axis=1)                      # exact integer sum
            want = (np.ldexp(exact.astype(np.float64), -37) / (hi - lo)).astype(np.float32)
            assert np.array_equal(exact.astype(np.float64).astype(np.int64), exact)
            assert np.array_equal(pooled[:, tau * nb + j, :], want)


def test_pooling_tail_block_uses_only_its_own_tokens():
    n, b, d = 100, 64, 8           # blocks of 64 and 36 tokens
    x = np.zeros((1, 2 * n, d), np.float32)
    x[0, :64] = 1.0
    x[0, 64:100] = 3.0
    x[0, 100:] = 1000.0            # next frame must not leak into frame 0's tail block
    p = O.block_mean_pool(x, n, b)
    assert p.shape == (1, 4, d)
    assert np.all(p[0, 0] == 1.0) and np.all(p[0, 1] == 3.0) and np.all(p[0, 2:] == 1000.0)


def test_pooling_shapes_match_paper():
    """q_tilde in R^{(f ceil(n/b)) x d}, k_tilde in R^{(i f ceil(n/b)) x d}, k_hat in R^{m x d}."""
    w = synth.small_ragged(frame_len=200, chunk_idx=4, frames_per_chunk=2)
    Q, K, _ = _inputs(w)
    b = O.chunk_budget(w.chunk_idx, w.schedule)
    nb = math.ceil(200 / 64)
    _, I = O.select_mask(Q, K, w.frame_len, w.block, b, return_intermediates=True)
    assert I["q_tilde"].shape == (w.heads, 2 * nb, w.head_dim)
    assert I["k_tilde"].shape == (w.heads, 4 * 2 * nb, w.head_dim)
    m = (4 - 1) * 2 - w.schedule.n_sink - w.schedule.n_win
    assert I["k_hat"].shape == (w.heads, m, w.head_dim)
    assert I["p"].shape == (w.heads, 2 * nb, m)


def test_frame_mean_equals_token_mean_when_blocks_align():
    """n % b == 0: the mean of block means is the mean over the frame's tokens."""
    rng = np.random.default_rng(3)
    n, b, F = 256, 64, 3
    K = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(rng.standard_normal((2, F * n, 16), dtype=np.float32)))
    kt = O.block_mean_pool(K, n, b)
    kh = O.frame_mean_pool(kt, n // b, [0, 2])
    want = K.astype(np.float64).reshape(2, F, n, 16).mean(axis=2)[:, [0, 2]]
    assert np.allclose(kh, want, rtol=0, atol=1e-6)


def test_pooling_flat_and_per_frame_blocks_agree_when_aligned():
    """Reading check: for n % b == 0 cutting blocks over the flat sequence (Preliminaries)
    and per frame (shapes after Eq. 7) is the same partition."""
    rng = np.random.default_rng(4)
    n, F = 192, 4
    K = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(rng.standard_normal((2, F * n, 8), dtype=np.float32)))
    assert np.array_equal(O.block_mean_pool(K, n, 64), O.block_mean_pool(K, F * n, 64))


# ----------------------------------------------------------------------------- scores

def test_inner_products_against_library_and_exact_on_integers():
    rng = np.random.default_rng(5)
    q = rng.standard_normal((2, 5, 32), dtype=np.float32)
    k = rng.standard_normal((2, 7, 32), dtype=np.float32)
    got = O.inner_products(q, k)
    assert got.shape == (2, 5, 7) and got.dtype == np.float32
    want = np.einsum("hrd,hcd->hrc", q.astype(np.float64), k.astype(np.float64))
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    qi = rng.integers(-8, 9, size=(1, 4, 16)).astype(np.float32)
    ki = rng.integers(-8, 9, size=(1, 6, 16)).astype(np.float32)
    assert np.array_equal(O.inner_products(qi, ki),
                          np.einsum("hrd,hcd->hrc", qi.astype(np.int64), ki.astype(np.int64)).astype(np.float32))


# ----------------------------------------------------------------------------- TopK_idx

def _brute_topk(scores, k):
    """Among all k-subsets: maximal score sum; among those the lexicographically smallest."""
    best, best_set = None, None
    for comb in itertools.combinations(range(len(scores)), k):
        tot = sum(float(scores[i]) for i in comb)
        if best is None or tot > best or (tot == best and comb < best_set):
            best, best_set = tot, comb
    return set(best_set)


def test_topk_brute_force_and_ties():
    rng = np.random.default_rng(6)
    for trial in range(50):
        n = int(rng.integers(1, 9))
        k = int(rng.integers(0, n + 1))
        # few distinct values (exactly representable, so subset sums are exact) -> many ties
        s = rng.integers(-2, 3, size=n).astype(np.float32) * np.float32(0.5)
        got = O.topk_idx(s, k)
        assert len(got) == k
        if k:
            assert set(int(i) for i in got) == _brute_topk(s, k)
    s = np.array([1.0, 2.0, 2.0, 0.0, 2.0], np.float32)
    assert list(O.topk_idx(s, 2)) == [1, 2]
    z = np.array([-0.0, 0.0, -1.0], np.float32)
    assert list(O.topk_idx(z, 1)) == [0]      # -0.0 ties with +0.0; lower index wins
    z = np.array([0.0, -0.0, -1.0], np.float32)
    assert list(O.topk_idx(z, 1)) == [0]


# ----------------------------------------------------------------------------- mask selection

def test_select_mask_brute_force_tiny():
    """Tiny configuration: C(4,2) frame subsets and C(8,4) block subsets enumerated."""
    w = synth.cfg_tiny()
    Q, K, _ = _inputs(w)
    b = O.chunk_budget(w.chunk_idx, w.schedule)
    assert (b.k_frames, b.k_blocks, b.list_len) == (2, 4, 8)
    lists, I = O.select_mask(Q, K, w.frame_len, w.block, b, return_intermediates=True)
    nb = w.blocks_per_frame
    # scores recomputed with library routines on plain means
    qt = Q.astype(np.float64).reshape(w.heads, -1, 64, w.head_dim).mean(axis=2)
    kt = K.astype(np.float64).reshape(w.heads, -1, 64, w.head_dim).mean(axis=2)
    kh = kt.reshape(w.heads, w.frames, nb, w.head_dim).mean(axis=2)[:, :w.hist_frames]
    p = np.einsum("hrd,hcd->hrc", qt, kh)
    o = np.einsum("hrd,hcd->hrc", qt, kt)
    assert np.allclose(I["p"], p, atol=1e-5) and np.allclose(I["o"], o, atol=1e-5)
    cur = set(range(w.hist_frames * nb, w.frames * nb))
    for h in range(w.heads):
        for r in range(lists.shape[1]):
            frames = _brute_topk(p[h, r], 2)
            cand = sorted(t * nb + j for t in frames for j in range(nb))
            pick = _brute_topk(o[h, r, cand], 4)
            want = sorted({cand[i] for i in pick} | cur)
            assert list(lists[h, r]) == want


def test_select_mask_planted_structure():
    """Hand-built K: one history frame and one block inside it point along q, so the
    expected selection is known without computing any score."""
    H, d, n, f, F_h, bsz = 1, 16, 128, 1, 6, 64
    nb = 2
    rng = np.random.default_rng(8)
    Q = np.zeros((H, f * n, d), np.float32)
    Q[..., 0] = 1.0                                    # every q_tilde = e_0
    K = 0.01 * rng.standard_normal((H, (F_h + f) * n, d)).astype(np.float32)
    K[..., 0] = 0.0
    K[0, 3 * n:4 * n, 0] = 1.0                         # frame 3: strong, uniform
    K[0, 4 * n + 64:5 * n, 0] = 1.5                    # frame 4 block 1: mean 0.75 over the frame
    K[0, 0 * n:1 * n, 0] = -5.0                        # sink frame: terrible score, still mandatory
    K[0, 5 * n:6 * n, 0] = -4.0                        # window frame: same
    sch = synth.Schedule(frames_per_chunk=f, frame_len=n, block=bsz, n_sink=1, n_win=1, k_frames=2,
                         ratio_of=synth.OF_CANDIDATES, current_mandatory=1, keep_fixed=0.375)
    b = O.chunk_budget(F_h // f + 1, sch)
    assert (b.n_sink, b.n_win, b.k_frames) == (1, 1, 2) and b.k_blocks == 3   # 0.375 * 8
    lists, I = O.select_mask(Q, K, n, bsz, b, return_intermediates=True)
    assert I["M"] == [1, 2, 3, 4]
    for r in range(nb):
        assert list(I["frames_sel"][0, r]) == [3, 4]
        # candidates: frames 0, 3, 4, 5 -> blocks 0,1,6,7,8,9,10,11; top-3: 9 (1.5), 6, 7 (1.0)
        assert list(lists[0, r]) == [6, 7, 9, 12, 13]


def test_select_mask_tie_prefers_lower_frame_and_block():
    H, d, n, f, F_h = 1, 8, 64, 1, 4
    Q = np.ones((H, n, d), np.float32)
    K = np.zeros((H, (F_h + f) * n, d), np.float32)
    K[0, 1 * n:2 * n] = 0.5
    K[0, 2 * n:3 * n] = 0.5                            # frames 1 and 2 identical -> equal scores
    K[0, 3 * n:4 * n] = 0.25
    sch = synth.Schedule(frames_per_chunk=1, frame_len=n, block=64, n_sink=0, n_win=0, k_frames=1,
                         ratio_of=synth.OF_CANDIDATES, current_mandatory=1, keep_fixed=1.0)
    b = O.chunk_budget(5, sch)
    lists, I = O.select_mask(Q, K, n, 64, b, return_intermediates=True)
    assert I["p"][0, 0, 1] == I["p"][0, 0, 2]
    assert list(I["frames_sel"][0, 0]) == [1]
    assert list(lists[0, 0]) == [1, 4]


@pytest.mark.parametrize("chunk", [1, 2, 3, 5])
def test_select_mask_structure(chunk):
    """Lists ascending and unique, ids in range, every kept block lies in a selected frame,
    mandatory frames present, current blocks present when mandatory; when the history is
    short all of it is a candidate."""
    w = synth.small_ragged(chunk_idx=chunk)
    Q, K, _ = _inputs(w)
    b = O.chunk_budget(chunk, w.schedule)
    lists, I = O.select_mask(Q, K, w.frame_len, w.block, b, return_intermediates=True)
    nb, F_h, f = w.blocks_per_frame, w.hist_frames, w.frames_per_chunk
    S, W, C, M = O.frame_sets(b)
    assert lists.shape == (w.heads, f * nb, b.list_len)
    assert np.all(np.diff(lists, axis=-1) > 0)
    assert lists.min() >= 0 and lists.max() < (F_h + f) * nb
    for h in range(w.heads):
        for r in range(f * nb):
            T = set(I["frames_sel"][h, r]) | set(S) | set(W) | set(C)
            assert {int(c) // nb for c in lists[h, r]} <= T
            if b.current_mandatory:
                assert set(range(F_h * nb, (F_h + f) * nb)) <= set(int(c) for c in lists[h, r])
    if len(M) <= w.schedule.k_frames:
        assert b.k_frames == len(M)


def test_select_mask_full_budget_keeps_everything():
    w = synth.small_ragged(chunk_idx=3, ratio_of=synth.OF_CANDIDATES, keep_fixed=1.0,
                           k_frames=99, current_mandatory=0)
    Q, K, _ = _inputs(w)
    b = O.chunk_budget(3, w.schedule)
    lists = O.select_mask(Q, K, w.frame_len, w.block, b)
    assert np.array_equal(lists, O.full_lists(w.heads, w.frame_len, w.block, w.frames_per_chunk, w.frames))


# ----------------------------------------------------------------------------- attention (Eq. 13)

def _sdpa(Q, K, V, mask=None):
    q, k, v = (torch.from_numpy(np.ascontiguousarray(a)).double()[None] for a in (Q, K, V))
    m = None if mask is None else torch.from_numpy(mask)[None]
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m)[0].numpy()


def test_full_budget_equals_dense_attention():
    """All-ones block mask: Eq. 3 reduces to softmax(q k^T / sqrt(d)) v (library routine)."""
    w = synth.small_ragged(chunk_idx=2)
    Q, K, V = _inputs(w)
    lists = O.full_lists(w.heads, w.frame_len, w.block, w.frames_per_chunk, w.frames)
    got = O.sparse_attention(Q, K, V, lists, w.frame_len, w.block)
    assert np.allclose(got, _sdpa(Q, K, V), rtol=0, atol=1e-12)


def test_sparse_attention_equals_masked_dense_with_ragged_tail():
    """Eq. 3 literally: expand the block mask to the element mask M(B), exclude masked
    columns, run the library's dense masked attention."""
    w = synth.small_ragged(chunk_idx=4)
    Q, K, V = _inputs(w)
    b = O.chunk_budget(w.chunk_idx, w.schedule)
    lists = O.select_mask(Q, K, w.frame_len, w.block, b)
    n, bs, nb = w.frame_len, w.block, w.blocks_per_frame
    tok_block = np.concatenate([np.minimum(np.arange(n) // bs, nb - 1) + t * nb for t in range(w.frames)])
    q_block = tok_block[:w.q_len]
    mask = np.zeros((w.heads, w.q_len, w.kv_len), dtype=bool)
    for h in range(w.heads):
        Bm = np.zeros((w.frames_per_chunk * nb, w.frames * nb), dtype=bool)
        for r in range(Bm.shape[0]):
            Bm[r, lists[h, r]] = True
        mask[h] = Bm[q_block][:, tok_block]
    got = O.sparse_attention(Q, K, V, lists, n, bs)
    assert not np.isnan(got).any()
    assert np.allclose(got, _sdpa(Q, K, V, mask), rtol=0, atol=1e-12)


def test_attention_probabilities():
    w = synth.cfg_tiny()
    Q, K, V = _inputs(w)
    b = O.chunk_budget(w.chunk_idx, w.schedule)
    lists = O.select_mask(Q, K, w.frame_len, w.block, b)
    for h in range(w.heads):
        for r in range(lists.shape[1]):
            Ob, P, cols = O.sparse_attention_block(Q[h], K[h], V[h], r, lists[h, r], w.frame_len,
                                                   w.block, return_probs=True)
            assert P.shape == (64, 8 * 64) and np.all(P >= 0)
            assert np.allclose(P.sum(axis=1), 1.0, atol=1e-13)
            assert set(cols // 64) == set(int(c) for c in lists[h, r])
            # order of the kept blocks is irrelevant
            perm = np.random.default_rng(r).permutation(lists[h, r])
            Op = O.sparse_attention_block(Q[h], K[h], V[h], r, perm, w.frame_len, w.block)
            assert np.allclose(Ob, Op, atol=1e-12)


def test_attention_single_block_constant_values():
    rng = np.random.default_rng(9)
    n, d = 100, 16
    Q = rng.standard_normal((1, n, d), dtype=np.float32)
    K = rng.standard_normal((1, 3 * n, d), dtype=np.float32)
    V = rng.standard_normal((1, 3 * n, d), dtype=np.float32)
    row = V[0, n + 64].copy()
    V[0, n + 64:2 * n] = row                           # tail block (36 tokens) of frame 1
    Ob = O.sparse_attention_block(Q[0], K[0], V[0], 0, [3], n, 64)
    assert np.allclose(Ob, row[None].astype(np.float64), atol=1e-13)


def test_attention_scale_is_inverse_sqrt_d():
    """One query, two keys: closed form sigmoid of the scaled logit difference."""
    d = 4
    Q = np.zeros((1, 1, d), np.float32); Q[0, 0, 0] = 2.0
    K = np.zeros((1, 2, d), np.float32); K[0, 0, 0] = 1.0; K[0, 1, 0] = -1.0
    V = np.zeros((1, 2, d), np.float32); V[0, 0, 0] = 1.0
    Ob = O.sparse_attention_block(Q[0], K[0], V[0], 0, [0, 1], 1, 64)
    want = 1.0 / (1.0 + math.exp(-(2.0 - (-2.0)) / math.sqrt(d)))
    assert abs(Ob[0, 0] - want) < 1e-15


# ----------------------------------------------------------------------------- backward of Eq. 13

def _bwd_case(seed=0, heads=2, frame_len=40, block=16, f=1, F=3, d=8, keep=3):
    rng = np.random.default_rng(seed)
    Lq, Lk = f * frame_len, F * frame_len
    Q = rng.standard_normal((heads, Lq, d))
    K = rng.standard_normal((heads, Lk, d))
    V = rng.standard_normal((heads, Lk, d))
    dO = rng.standard_normal((heads, Lq, d))
    nb = -(-frame_len // block)
    lists = np.stack([np.stack([np.sort(rng.choice(F * nb, size=keep, replace=False))
                                for _ in range(f * nb)]) for _ in range(heads)]).astype(np.int32)
    return Q, K, V, dO, lists, frame_len, block


def _dense_mask(lists, frame_len, block, Lq, Lk):
    H, n_q, _ = lists.shape
    M = np.zeros((H, Lq, Lk), dtype=bool)
    for h in range(H):
        for r in range(n_q):
            qlo, qhi = O.block_token_range(r, frame_len, block)
            for c in lists[h, r]:
                lo, hi = O.block_token_range(c, frame_len, block)
                M[h, qlo:qhi, lo:hi] = True
    return M


def test_backward_matches_library_autodiff_of_masked_dense_attention():
    """torch autograd (binary64) through softmax(QK^T scale + mask) V, an independent derivation."""
    Q, K, V, dO, lists, n, b = _bwd_case()
    M = torch.from_numpy(_dense_mask(lists, n, b, Q.shape[1], K.shape[1]))
    q, k, v = (torch.tensor(t, dtype=torch.float64, requires_grad=True) for t in (Q, K, V))
    scale = 1.0 / math.sqrt(Q.shape[2])
    s = (q @ k.transpose(1, 2)) * scale
    s = s.masked_fill(~M, float("-inf"))
    o = torch.softmax(s, dim=-1) @ v
    o.backward(torch.from_numpy(dO))
    dQ, dK, dV = O.sparse_attention_backward(Q, K, V, dO, lists, n, b)
    assert np.allclose(dQ, q.grad.numpy(), atol=1e-12)
    assert np.allclose(dK, k.grad.numpy(), atol=1e-12)
    assert np.allclose(dV, v.grad.numpy(), atol=1e-12)


def test_backward_matches_finite_differences_of_the_forward_oracle():
    Q, K, V, dO, lists, n, b = _bwd_case(seed=3, heads=1, frame_len=20, block=8, F=2, d=4, keep=2)
    dQ, dK, dV = O.sparse_attention_backward(Q, K, V, dO, lists, n, b)
    loss = lambda q, k, v: float((O.sparse_attention(q, k, v, lists, n, b) * dO).sum())
    rng = np.random.default_rng(0)
    eps = 1e-6
    for name, T, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(6):
            idx = tuple(int(rng.integers(s)) for s in T.shape)
            Tp, Tm = T.copy(), T.copy()
            Tp[idx] += eps
            Tm[idx] -= eps
            args = {"Q": (Tp, K, V), "K": (Q, Tp, V), "V": (Q, K, Tp)}[name]
            argm = {"Q": (Tm, K, V), "K": (Q, Tm, V), "V": (Q, K, Tm)}[name]
            fd = (loss(*args) - loss(*argm)) / (2 * eps)
            assert abs(fd - G[idx]) < 1e-6, (name, idx, fd, G[idx])


def test_backward_invariants_and_duplicates():
    Q, K, V, dO, lists, n, b = _bwd_case(seed=5)
    dQ, dK, dV = O.sparse_attention_backward(Q, K, V, dO, lists, n, b)
    # softmax rows sum to one: the V gradients add up to the upstream gradients ...
    assert np.allclose(dV.sum(axis=1), dO.sum(axis=1), atol=1e-12)
    # ... and a common shift of all keys changes nothing: the K gradients add up to zero
    assert np.allclose(dK.sum(axis=1), 0.0, atol=1e-12)
    # keys no list mentions get no gradient
    M = _dense_mask(lists, n, b, Q.shape[1], K.shape[1])
    unused = ~M.any(axis=1)
    assert np.all(dK[unused] == 0.0) and np.all(dV[unused] == 0.0) and unused.any()
    # an id listed twice counts twice, as in the forward pass: its tokens appear twice among the columns
    twice = lists.copy()
    twice[:, :, 1] = twice[:, :, 0]
    dQ2, dK2, dV2 = O.sparse_attention_backward(Q, K, V, dO, twice, n, b)
    out2 = O.sparse_attention(Q, K, V, twice, n, b)
    eps = 1e-6
    Vp = V.copy(); Vp[0, O.block_token_range(twice[0, 0, 0], n, b)[0], 0] += eps
    fd = ((O.sparse_attention(Q, K, Vp, twice, n, b) - out2) * dO).sum() / eps
    assert abs(fd - dV2[0, O.block_token_range(twice[0, 0, 0], n, b)[0], 0]) < 1e-5
