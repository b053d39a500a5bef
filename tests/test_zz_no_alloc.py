"""The allocation-free entry point (lf_select_mask_static: intermediates in the library's own
static device array) against lf_select_mask on a caller-provided workspace: index lists equal
bit for bit, on two calls in a row of which the second is smaller (the shared array keeps the
first call's contents), and again after a larger one."""
import ctypes as C

import numpy as np
import pytest

from paper_2602_04789_amd import synth

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_matches_workspace_entry():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_04789_amd import lf
    lib = lf.load()
    lf.lf_init()
    assert lf.lf_static_scratch_bytes() == 16 << 20
    big = synth.scaled(synth.cfg_last_chunk(), heads=4)            # 21 frames of 1560 tokens
    small = synth.small_ragged(chunk_idx=4)                        # 8 frames of 200 tokens
    mid = synth.scaled(synth.cfg_mid_rollout(), heads=2)
    for w in (big, small, mid, small):
        print(f"static-scratch case {w.name}: H={w.heads} n={w.frame_len} F={w.frames}", flush=True)
        x = synth.make_inputs(w)
        Q, K = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QK")
        b = lf.lf_chunk_budget(w.chunk_idx, w.schedule)
        n_q = w.frames_per_chunk * w.blocks_per_frame
        want = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
        got = torch.full((w.heads, n_q, b.list_len), -7, dtype=torch.int32, device="cuda")
        lf.lf_select_mask_static(Q, K, w.frame_len, w.block, b, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), w.name
    # a shape that needs more than the static array is refused before anything is enqueued
    w = synth.cfg_rollout(7, 0, heads=64)
    sh = lf.lf_shape()
    sh.heads, sh.head_dim, sh.frame_len, sh.block = w.heads, w.head_dim, w.frame_len, 64
    sh.q_len, sh.kv_len, sh.dtype = w.q_len, w.kv_len, 0
    for t, L in (("q", w.q_len), ("k", w.kv_len), ("v", w.kv_len), ("o", w.q_len)):
        setattr(sh, f"{t}_stride_tok", w.head_dim)
        setattr(sh, f"{t}_stride_head", w.head_dim * L)
    b = lf.lf_chunk_budget(w.chunk_idx, w.schedule)
    assert lf.lf_workspace_bytes(sh, b) > lf.lf_static_scratch_bytes()
    fake = 0x10000
    assert lib.lf_select_mask_static(fake, fake, C.byref(sh), C.byref(b), fake, None) == -6
