"""Pins for the producer oracle (RMSNorm + rotary embedding): library routines, the complex-number
form of the rotation, and the invariants the two operators are defined by.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import qk_producer_oracle as P


def _case(L=7, H=3, d=16, seed=0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((L, H * d)).astype(np.float32)
    g = (1.0 + 0.1 * rng.standard_normal(H * d)).astype(np.float32)
    theta = rng.uniform(-3.0, 3.0, size=(L, d // 2))
    return x, g, np.cos(theta).astype(np.float32), np.sin(theta).astype(np.float32), theta


@pytest.mark.parametrize("across", [False, True])
def test_rms_norm_matches_library(across):
    x, g, *_ = _case()
    H, d = 3, 16
    got = P.rms_norm(x, g, 1e-6, H, across)
    xt, gt = torch.from_numpy(x).double(), torch.from_numpy(g).double()
    if across:
        want = torch.nn.functional.rms_norm(xt, (H * d,), gt, 1e-6)
    else:
        want = torch.nn.functional.rms_norm(xt.view(-1, H, d), (d,), None, 1e-6).reshape(-1, H * d) * gt
    assert np.allclose(got, want.numpy(), rtol=1e-13, atol=1e-15)


def test_rms_norm_output_has_unit_rms_and_is_scale_invariant():
    x, g, *_ = _case()
    ones = np.ones_like(g)
    for across in (False, True):
        y = P.rms_norm(x, ones, 0.0, 3, across)
        seg = y if across else y.reshape(-1, 3, 16)
        assert np.allclose(np.sqrt((seg ** 2).mean(axis=-1)), 1.0, atol=1e-13)
        assert np.allclose(P.rms_norm(4.0 * x, ones, 0.0, 3, across), y, atol=1e-13)
    # eps matters only for tiny inputs: a zero vector stays zero instead of dividing by zero
    assert np.all(P.rms_norm(np.zeros((2, 48), np.float32), ones, 1e-6, 3, False) == 0.0)


@pytest.mark.parametrize("pairing", ["interleaved", "half"])
def test_rope_is_complex_multiplication(pairing):
    """Pair (a, b) as the complex number a + ib times exp(i theta)."""
    x, g, cos, sin, theta = _case()
    H, d = 3, 16
    y = x.astype(np.float64)
    got = P.rope(y, cos, sin, H, pairing).reshape(-1, H, d)
    yh = y.reshape(-1, H, d)
    z = (yh[..., 0::2] + 1j * yh[..., 1::2]) if pairing == "interleaved" else (yh[..., :d // 2] + 1j * yh[..., d // 2:])
    rot = z * (cos.astype(np.float64) + 1j * sin.astype(np.float64))[:, None, :]
    if pairing == "interleaved":
        assert np.allclose(got[..., 0::2], rot.real, atol=1e-13) and np.allclose(got[..., 1::2], rot.imag, atol=1e-13)
    else:
        assert np.allclose(got[..., :d // 2], rot.real, atol=1e-13) and np.allclose(got[..., d // 2:], rot.imag, atol=1e-13)


def test_rope_invariants():
    x, g, cos, sin, theta = _case()
    H, d = 3, 16
    y = x.astype(np.float64)
    for pairing in ("interleaved", "half"):
        r = P.rope(y, cos, sin, H, pairing)
        # a rotation keeps the norm of every pair, hence of every head vector
        assert np.allclose((r.reshape(-1, H, d) ** 2).sum(-1), (y.reshape(-1, H, d) ** 2).sum(-1), rtol=1e-6)
        # angle zero is the identity
        assert np.array_equal(P.rope(y, np.ones_like(cos), np.zeros_like(sin), H, pairing), y)
        # rotating by theta then by -theta gives the input back
        back = P.rope(r, cos, -sin, H, pairing)
        assert np.allclose(back, y, atol=1e-6)
    # the two pairings are the same map up to the channel permutation that carries pairs to pairs
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])      # interleaved -> half order
    yh = y.reshape(-1, H, d)[..., perm].reshape(-1, H * d)
    a = P.rope(y, cos, sin, H, "interleaved").reshape(-1, H, d)[..., perm]
    b = P.rope(yh, cos, sin, H, "half").reshape(-1, H, d)
    assert np.allclose(a, b, atol=1e-15)


def test_rope_scores_depend_on_relative_position_only():
    """Textbook property: with angles position * frequency, <rope(q, m), rope(k, n)> is a function
    of m - n."""
    rng = np.random.default_rng(3)
    d = 32
    q, k = rng.standard_normal((1, d)), rng.standard_normal((1, d))
    freq = 10000.0 ** (-np.arange(d // 2) / (d // 2))
    def at(v, pos):
        th = (pos * freq)[None, :]
        return P.rope(v, np.cos(th), np.sin(th), 1, "interleaved")[0]
    s1 = at(q, 5) @ at(k, 2)
    s2 = at(q, 105) @ at(k, 102)
    s3 = at(q, 5) @ at(k, 3)
    assert abs(s1 - s2) < 1e-9 and abs(s1 - s3) > 1e-6


def test_layout_and_composition():
    x, g, cos, sin, _ = _case()
    H, d = 3, 16
    out = P.qk_norm_rope(x, g, cos, sin, H, eps=1e-6, across_heads=False, pairing="interleaved")
    assert out.shape == (H, x.shape[0], d) and out.dtype == np.float64
    step = P.rope(P.rms_norm(x, g, 1e-6, H, False), cos, sin, H, "interleaved")
    for h in range(H):
        assert np.array_equal(out[h], step[:, h * d:(h + 1) * d])
