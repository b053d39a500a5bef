"""The seeded input generators (host only)."""
import numpy as np
import torch

from paper_2602_04789_amd import synth


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096, dtype=np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 255.0], np.float32)])
    bits = synth.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_inputs_are_deterministic_and_in_contract_range():
    w = synth.small_ragged()
    a, b = synth.make_inputs(w), synth.make_inputs(w)
    for k in "QKV":
        assert np.array_equal(a[k], b[k])
        v = np.abs(synth.bf16_bits_to_f32(a[k]))
        assert v.max() < 256.0 and (v[v > 0].min() >= 2.0 ** -30)
    assert a["Q"].shape == (w.heads, w.q_len, w.head_dim)
    assert a["K"].shape == a["V"].shape == (w.heads, w.kv_len, w.head_dim)
    c = synth.make_inputs(synth.scaled(w, seed=w.seed + 1))
    assert not np.array_equal(a["K"], c["K"])


def test_history_values_persist_across_rollout_calls():
    """Committed history frames are re-created identically for later chunks and steps; the
    current chunk is redrawn at every step."""
    a = synth.make_inputs(synth.scaled(synth.cfg_rollout(2, 0, heads=1), frame_len=70))
    b = synth.make_inputs(synth.scaled(synth.cfg_rollout(3, 2, heads=1), frame_len=70))
    assert np.array_equal(a["V"][:, :3 * 70], b["V"][:, :3 * 70])
    c = synth.make_inputs(synth.scaled(synth.cfg_rollout(3, 3, heads=1), frame_len=70))
    assert np.array_equal(b["V"][:, :6 * 70], c["V"][:, :6 * 70])
    assert not np.array_equal(b["V"][:, 6 * 70:], c["V"][:, 6 * 70:])
    assert not np.array_equal(b["Q"], c["Q"])


def test_benchmark_shapes():
    w = synth.cfg_last_chunk()
    assert (w.heads, w.head_dim, w.q_len, w.kv_len, w.blocks_per_frame) == (12, 128, 4680, 32760, 25)
    w = synth.cfg_mid_rollout()
    assert (w.q_len, w.kv_len) == (4680, 18720)
    w = synth.cfg_first_chunk()
    assert (w.q_len, w.kv_len) == (4680, 4680)
    w = synth.cfg_rollout(7, 3)
    assert (w.heads, w.kv_len) == (40, 32760)
    w = synth.cfg_tiny()
    assert (w.heads, w.head_dim, w.q_len, w.kv_len) == (2, 64, 256, 1280)
