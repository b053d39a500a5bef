"""Parity of the backward pass of the blockwise sparse attention with the CPU oracle.

Bars (derived from the arithmetic: bfloat16 inputs, probabilities and score gradients rounded
to bfloat16 before the accumulating products, float32 accumulation, bfloat16 outputs): for each
of dQ, dK, dV, max |got - ref| <= 2e-2 * max(1, max |ref|) and mean |got - ref| <= 2e-3 *
max(1, rms(ref))."""
import numpy as np
import pytest

from oracle import hsa_oracle as O
from paper_2602_04789_amd import synth

pytestmark = pytest.mark.gpu

MAX_REL, MEAN_REL = 2e-2, 2e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_04789_amd import lf
    lf.load()
    return torch, lf


def _dev(torch, bits):
    return torch.from_numpy(bits).view(torch.bfloat16).cuda()


def _f32(bits):
    return synth.bf16_bits_to_f32(bits)


def _close(name, got, ref):
    err = np.abs(got - ref)
    bar_max = MAX_REL * max(1.0, float(np.abs(ref).max()))
    bar_mean = MEAN_REL * max(1.0, float(np.sqrt((ref ** 2).mean())))
    print(f"  {name}: max err {err.max():.3e} (bar {bar_max:.3e}), mean err {err.mean():.3e} "
          f"(bar {bar_mean:.3e}), max |ref| {np.abs(ref).max():.3f}", flush=True)
    assert np.isfinite(got).all()
    assert err.max() <= bar_max and err.mean() <= bar_mean, (name, err.max(), err.mean())


def _run(torch, lf, w, x, lists, scale=0.0):
    Q, K, V = (_dev(torch, x[k]) for k in "QKV")
    dO = _dev(torch, x["dO"])
    idx = torch.from_numpy(np.ascontiguousarray(lists, dtype=np.int32)).cuda()
    out, lse2 = lf.lf_sparse_attn_fwd(Q, K, V, idx, w.frame_len, w.block, softmax_scale=scale)
    ref_out = lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, softmax_scale=scale)
    dQ, dK, dV = lf.lf_sparse_attn_bwd(Q, K, V, out, dO, lse2, idx, w.frame_len, w.block,
                                       softmax_scale=scale)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out)      # the training forward is the inference forward
    return [t.float().cpu().numpy().astype(np.float64) for t in (dQ, dK, dV)], lse2.cpu().numpy()


def _oracle_lists(w, x):
    ob = O.chunk_budget(w.chunk_idx, w.schedule)
    return O.select_mask(_f32(x["Q"]), _f32(x["K"]), w.frame_len, w.block, ob)


SMALL = {
    "tiny": lambda: synth.cfg_tiny(),
    "ragged_c2": lambda: synth.small_ragged(chunk_idx=2),
    "ragged_c4": lambda: synth.small_ragged(chunk_idx=4),
    "ragged_c6_d64": lambda: synth.small_ragged(chunk_idx=6, head_dim=64, heads=2),
    "ragged_compete": lambda: synth.small_ragged(chunk_idx=4, current_mandatory=0,
                                                 ratio_of=synth.OF_ALL, keep_fixed=0.3),
    "one_token_tail": lambda: synth.small_ragged(frame_len=129, chunk_idx=3, heads=2),
    "short_frame": lambda: synth.small_ragged(frame_len=40, chunk_idx=5, heads=2, k_frames=1),
    "tail_31": lambda: synth.small_ragged(frame_len=95, chunk_idx=3, heads=2),
    "tail_33_d64": lambda: synth.small_ragged(frame_len=97, chunk_idx=3, heads=2, head_dim=64),
    # 260 one-block frames per chunk: lists of 266 entries and transposed lists of 260, both past
    # the 256 entries the kernels decode per pass
    "many_query_blocks": lambda: synth.small_ragged(frame_len=64, chunk_idx=2, frames_per_chunk=260, heads=1,
                                                    head_dim=64, k_frames=3, n_sink=1, n_win=2),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_cases_match_oracle_everywhere(gpu, name):
    torch, lf = gpu
    w = SMALL[name]()
    x = synth.make_inputs(w)
    x["dO"] = synth.make_upstream_grad(w)
    print(f"case {name}: H={w.heads} d={w.head_dim} n={w.frame_len} F={w.frames}", flush=True)
    lists = _oracle_lists(w, x)
    (dQ, dK, dV), lse2 = _run(torch, lf, w, x, lists)
    rQ, rK, rV = O.sparse_attention_backward(_f32(x["Q"]), _f32(x["K"]), _f32(x["V"]), _f32(x["dO"]),
                                             lists, w.frame_len, w.block)
    _close("dQ", dQ, rQ)
    _close("dK", dK, rK)
    _close("dV", dV, rV)
    # the log-sum-exp the forward left: log2 of the sum of exp(s) over the row's kept columns.
    # The kernel's row sum adds the probabilities as rounded to bfloat16 (the values its second
    # product uses), each within 2^-9 of the exact one, so log2 of the sum is within
    # log2(1 + 2^-9) = 2.8e-3; float32 accumulation adds little to that.
    Qf, Kf = _f32(x["Q"]).astype(np.float64), _f32(x["K"]).astype(np.float64)
    scale = 1.0 / np.sqrt(w.head_dim)
    nq = lists.shape[1]
    for h, r in {(0, 0), (w.heads - 1, nq - 1), (w.heads // 2, nq // 2)}:
        lo, hi = O.block_token_range(r, w.frame_len, w.block)
        cols = np.concatenate([np.arange(*O.block_token_range(c, w.frame_len, w.block)) for c in lists[h, r]])
        sc = (Qf[h, lo:hi] @ Kf[h][cols].T) * scale
        m = sc.max(axis=1)
        want = (m + np.log(np.exp(sc - m[:, None]).sum(axis=1))) / np.log(2.0)
        err = np.abs(lse2[h, lo:hi] - want).max()
        assert err <= 3.5e-3, (h, r, err)


def test_full_lists_match_library_autodiff_of_dense_attention(gpu):
    """With every block listed the gradients are those of dense attention: compared with the
    framework's autodiff of its own dense attention in float32 on the GPU (an independent
    implementation of the same derivative)."""
    torch, lf = gpu
    w = synth.small_ragged(chunk_idx=3, heads=2)
    x = synth.make_inputs(w)
    x["dO"] = synth.make_upstream_grad(w)
    lists = O.full_lists(w.heads, w.frame_len, w.block, w.frames_per_chunk, w.frames)
    (dQ, dK, dV), _ = _run(torch, lf, w, x, lists)
    Q, K, V = (_dev(torch, x[k]).float().requires_grad_(True) for k in "QKV")
    out = torch.nn.functional.scaled_dot_product_attention(Q, K, V)
    out.backward(_dev(torch, x["dO"]).float())
    for name, got, ref in (("dQ", dQ, Q.grad), ("dK", dK, K.grad), ("dV", dV, V.grad)):
        _close(name, got, ref.cpu().numpy().astype(np.float64))


def test_list_edge_cases_and_strided_tensors(gpu):
    """Out-of-range ids skipped; a query block whose list holds no valid id (zero dQ rows, +inf
    log-sum-exp, no contribution to dK and dV); KV blocks that no list keeps (zero dK and dV
    rows); explicit softmax scale; tensors carved out of larger buffers."""
    torch, lf = gpu
    w = synth.small_ragged(chunk_idx=3, heads=2)
    x = synth.make_inputs(w)
    x["dO"] = synth.make_upstream_grad(w)
    nb = w.blocks_per_frame
    n_q, n_k = w.frames_per_chunk * nb, w.frames * nb
    rng = np.random.default_rng(3)
    L = 6
    lists = np.empty((w.heads, n_q, L), dtype=np.int32)
    for h in range(w.heads):
        for r in range(n_q):
            keep = np.sort(rng.choice(n_k - 2, size=L - 2, replace=False)).astype(np.int32)
            lists[h, r] = np.concatenate([[-3], keep, [n_k + 5]])       # ascending, ends invalid
    lists[1, 2] = np.array([-5, -4, -3, n_k, n_k + 1, n_k + 2])         # no valid id at all
    assert not (lists == n_k - 1).any() and not (lists == n_k - 2).any()  # two blocks nobody keeps
    scale = 0.11

    def strided(bits, pad_tok, pad_ch):
        H, Lx, d = bits.shape
        buf = torch.zeros((H, Lx + pad_tok, d + pad_ch), dtype=torch.bfloat16, device="cuda")
        view = buf[:, 1:1 + Lx, :d]
        view.copy_(_dev(torch, bits))
        return view
    Q, K, V = strided(x["Q"], 3, 8), strided(x["K"], 5, 16), strided(x["V"], 2, 24)
    dO = strided(x["dO"], 4, 8)
    Oview = torch.zeros((w.heads, w.q_len + 4, w.head_dim + 8), dtype=torch.bfloat16,
                        device="cuda")[:, 1:1 + w.q_len, :w.head_dim]
    idx = torch.from_numpy(lists).cuda()
    out, lse2 = lf.lf_sparse_attn_fwd(Q, K, V, idx, w.frame_len, w.block, softmax_scale=scale, O=Oview)
    dQ, dK, dV = lf.lf_sparse_attn_bwd(Q, K, V, out, dO, lse2, idx, w.frame_len, w.block,
                                       softmax_scale=scale)
    torch.cuda.synchronize()
    assert dQ.stride() == Q.stride() and dK.stride() == K.stride() and dV.stride() == V.stride()

    valid = [[[c for c in lists[h, r] if 0 <= c < n_k] for r in range(n_q)] for h in range(w.heads)]
    Qf, Kf, Vf, dOf = (_f32(x[k]) for k in ("Q", "K", "V", "dO"))
    rQ = np.zeros(Qf.shape)
    rK, rV = np.zeros(Kf.shape), np.zeros(Vf.shape)
    for h in range(w.heads):          # the oracle takes rectangular lists: call it per query block
        for r in range(n_q):
            if not valid[h][r]:
                continue
            lo, hi = O.block_token_range(r, w.frame_len, w.block)
            one = np.zeros((1, n_q, len(valid[h][r])), dtype=np.int32)
            one[0, r] = valid[h][r]
            mask_dO = np.zeros_like(dOf[h:h + 1])
            mask_dO[0, lo:hi] = dOf[h, lo:hi]
            # other query blocks get list [0...] with a zero upstream gradient: no contribution
            a, b, c = O.sparse_attention_backward(Qf[h:h + 1], Kf[h:h + 1], Vf[h:h + 1], mask_dO, one,
                                                  w.frame_len, w.block, scale=scale)
            rQ[h, lo:hi] = a[0, lo:hi]
            rK[h] += b[0]
            rV[h] += c[0]
    g = [t.float().cpu().numpy().astype(np.float64) for t in (dQ, dK, dV)]
    _close("dQ", g[0], rQ)
    _close("dK", g[1], rK)
    _close("dV", g[2], rV)
    lo, hi = O.block_token_range(2, w.frame_len, w.block)
    assert (g[0][1, lo:hi] == 0).all() and np.isposinf(lse2[1, lo:hi].cpu().numpy()).all()
    klo, _ = O.block_token_range(n_k - 2, w.frame_len, w.block)
    assert (g[1][:, klo:] == 0).all() and (g[2][:, klo:] == 0).all()


def test_full_size_last_chunk_one_head_against_oracle(gpu):
    """The paper's 480p last chunk at full size (12 heads on the GPU, the launch the benchmark
    times); the oracle recomputes heads 0 and 7 completely."""
    torch, lf = gpu
    w = synth.cfg_last_chunk()
    x = synth.make_inputs(w)
    x["dO"] = synth.make_upstream_grad(w)
    Q, K = _dev(torch, x["Q"]), _dev(torch, x["K"])
    b = lf.lf_chunk_budget(w.chunk_idx, w.schedule)
    idx = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
    torch.cuda.synchronize()
    lists = idx.cpu().numpy()
    print(f"full size: H={w.heads} n={w.frame_len} F={w.frames} list_len={lists.shape[-1]}", flush=True)
    (dQ, dK, dV), _ = _run(torch, lf, w, x, lists)
    # every head: what holds at any size.  The rows of P sum to one, so the token sums of dV
    # equal those of dO; the rows of dS sum to zero (delta is the P-weighted mean of dP), so the
    # token sums of dK vanish.  Sums of 32 760 bfloat16-rounded terms: absolute slack below.
    dOf = _f32(x["dO"]).astype(np.float64)
    dv_err = np.abs(dV.sum(axis=1) - dOf.sum(axis=1)).max()
    dk_err = np.abs(dK.sum(axis=1)).max()
    print(f" all heads: |sum dV - sum dO| {dv_err:.3f}, |sum dK| {dk_err:.3f}", flush=True)
    assert dv_err <= 0.5 and dk_err <= 0.5
    for h in (0, 7):
        sl = slice(h, h + 1)
        rQ, rK, rV = O.sparse_attention_backward(_f32(x["Q"][sl]), _f32(x["K"][sl]), _f32(x["V"][sl]),
                                                 _f32(x["dO"][sl]), lists[sl], w.frame_len, w.block)
        print(f" head {h}", flush=True)
        _close("dQ", dQ[sl], rQ)
        _close("dK", dK[sl], rK)
        _close("dV", dV[sl], rV)


def test_rollout_call_40_heads(gpu):
    """One call of the 40-head rollout (chunk 4, the shape of the model's full attention layer):
    the token-sum properties on every head, the oracle on the first and the last head."""
    torch, lf = gpu
    w = synth.cfg_rollout(4, 1)
    x = synth.make_inputs(w)
    x["dO"] = synth.make_upstream_grad(w)
    Q, K = _dev(torch, x["Q"]), _dev(torch, x["K"])
    b = lf.lf_chunk_budget(w.chunk_idx, w.schedule)
    lists = lf.lf_select_mask(Q, K, w.frame_len, w.block, b).cpu().numpy()
    del Q, K
    print(f"rollout call: H={w.heads} n={w.frame_len} F={w.frames} list_len={lists.shape[-1]}", flush=True)
    (dQ, dK, dV), _ = _run(torch, lf, w, x, lists)
    dOf = _f32(x["dO"]).astype(np.float64)
    dv_err = np.abs(dV.sum(axis=1) - dOf.sum(axis=1)).max()
    dk_err = np.abs(dK.sum(axis=1)).max()
    print(f" all heads: |sum dV - sum dO| {dv_err:.3f}, |sum dK| {dk_err:.3f}", flush=True)
    assert dv_err <= 0.5 and dk_err <= 0.5
    for h in (0, w.heads - 1):
        sl = slice(h, h + 1)
        rQ, rK, rV = O.sparse_attention_backward(_f32(x["Q"][sl]), _f32(x["K"][sl]), _f32(x["V"][sl]),
                                                 _f32(x["dO"][sl]), lists[sl], w.frame_len, w.block)
        print(f" head {h}", flush=True)
        _close("dQ", dQ[sl], rQ)
        _close("dK", dK[sl], rK)
        _close("dV", dV[sl], rV)


def test_backward_is_reproducible(gpu):
    """No atomics, fixed summation order: two calls give the same bits."""
    torch, lf = gpu
    w = synth.small_ragged(chunk_idx=4)
    x = synth.make_inputs(w)
    x["dO"] = synth.make_upstream_grad(w)
    lists = _oracle_lists(w, x)
    Q, K, V, dO = (_dev(torch, x[k]) for k in ("Q", "K", "V", "dO"))
    idx = torch.from_numpy(lists).cuda()
    out, lse2 = lf.lf_sparse_attn_fwd(Q, K, V, idx, w.frame_len, w.block)
    a = lf.lf_sparse_attn_bwd(Q, K, V, out, dO, lse2, idx, w.frame_len, w.block)
    b = lf.lf_sparse_attn_bwd(Q, K, V, out, dO, lse2, idx, w.frame_len, w.block)
    torch.cuda.synchronize()
    for s, t in zip(a, b):
        assert torch.equal(s, t)


def test_training_step_replays_from_a_captured_graph(gpu):
    """Selection, training forward and backward captured once into a HIP graph (the library
    allocates, clears and synchronises nothing) and replayed on new inputs written into the same
    buffers, with eager work and synchronisations between the replays; every replay must equal
    the eager result bit for bit."""
    torch, lf = gpu
    w = synth.small_ragged(chunk_idx=4)
    b = lf.lf_chunk_budget(w.chunk_idx, w.schedule)
    xs = []
    for s in (11, 12, 13):
        ws_ = synth.small_ragged(chunk_idx=4, seed=s)
        x = synth.make_inputs(ws_)
        x["dO"] = synth.make_upstream_grad(ws_, seed=s)
        xs.append(x)
    Q, K, V, dO = (_dev(torch, xs[0][k]).clone() for k in ("Q", "K", "V", "dO"))
    sh = lf.make_shape(Q, K, V, Q, frame_len=w.frame_len, block=w.block)
    ws = torch.empty(lf.lf_workspace_bytes(sh, b), dtype=torch.uint8, device="cuda")
    bws = torch.empty(lf.lf_attn_bwd_workspace_bytes(sh), dtype=torch.uint8, device="cuda")
    nq = w.frames_per_chunk * w.blocks_per_frame
    idx = torch.empty((w.heads, nq, b.list_len), dtype=torch.int32, device="cuda")
    out = torch.empty_like(Q)
    lse2 = torch.empty((w.heads, w.q_len), dtype=torch.float32, device="cuda")
    grads = (torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V))

    def step():
        lf.lf_select_mask(Q, K, w.frame_len, w.block, b, indices=idx, workspace=ws)
        lf.lf_sparse_attn_fwd(Q, K, V, idx, w.frame_len, w.block, O=out, lse2=lse2)
        lf.lf_sparse_attn_bwd(Q, K, V, out, dO, lse2, idx, w.frame_len, w.block, workspace=bws, grads=grads)

    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for x in xs[1:] + xs[:1] + xs[1:2]:
        for t, k in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
            t.copy_(_dev(torch, x[k]))
        for t in grads:
            t.fill_(7.0)
        bws.fill_(255)
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in grads]
        want_idx = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
        want_out, want_lse = lf.lf_sparse_attn_fwd(Q, K, V, want_idx, w.frame_len, w.block)
        want = lf.lf_sparse_attn_bwd(Q, K, V, want_out, dO, want_lse, want_idx, w.frame_len, w.block)
        torch.cuda.synchronize()
        for a, e in zip(got, want):
            assert torch.equal(a.view(torch.int16), e.view(torch.int16))
