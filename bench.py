#!/usr/bin/env python3
"""Benchmark of the per-chunk Hierarchical Sparse Attention hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic chunk already resident in HBM:
lf_chunk_budget (host) -> lf_select_mask -> lf_sparse_attn.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload last_chunk]

    python bench.py --workload rollout     # 7 chunks x 4 steps, 40 heads: 28 calls per step

value        effective TFLOP/s on kept blocks over the whole step (select + attention):
             4 d sum_{kept (r,c)} rows_r cols_c valid-token FLOPs / wall time per step.
roofline     dominant kernel (block-sparse attention, bf16 MFMA): the same FLOPs over the
             kernel's own duration, HIP events on the launch stream inside the timed region.
select       mask selection as an HBM-bound stage: one read of Q and K (bf16) per call.
cpu_baseline the numpy oracle on the host cores, on a bounded sample of the same workload.
measured     what this GPU reaches on two micro-benchmarks of this repository (a streaming
             16-byte read and a register-only MFMA loop): ceilings measured in the same run,
             beside the published peaks the roofline fractions are taken against.
per_config   the same select / attention figures for the other benchmark configurations and
             the paper's own operating points, each with its index lists checked against the
             oracle (--no-per-config skips them).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E

PROFILE_COUNTERS = os.path.join(ROOT, "profiles", "last_chunk_pmc_counters.txt")


def measured_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE / WRITE_SIZE
    runs, scaled by the copy calibration stated there): the line
    'traffic_bytes attn=<bytes> select=<bytes> commit=<hash>' of profiles/last_chunk_pmc_counters.txt.
    Returns ({}, None) when the file or the line is missing."""
    try:
        for line in open(PROFILE_COUNTERS):
            if line.startswith("traffic_bytes "):
                kv = dict(tok.split("=", 1) for tok in line.split()[1:])
                return ({"attn": float(kv["attn"]), "select": float(kv["select"])}, kv.get("commit"))
    except (OSError, KeyError, ValueError):
        pass
    return {}, None


def _workloads():
    from paper_2602_04789_amd import synth
    return {"first_chunk": synth.cfg_first_chunk, "mid_rollout": synth.cfg_mid_rollout,
            "last_chunk": synth.cfg_last_chunk, "tiny": synth.cfg_tiny,
            # the paper's own operating point (1536 tokens per frame, Chunk-Aware Growth,
            # current chunk competing) at its fourth and its last chunk
            "paper5s_mid": lambda: synth.cfg_paper_5s(4), "paper5s_last": lambda: synth.cfg_paper_5s(7),
            # the 15-second setting: 21 chunks, at chunk 20 the cache holds 57 history frames
            "paper15s_late": lambda: synth.cfg_paper_15s(20)}


def kept_flops(lists: np.ndarray, w) -> float:
    """4 d sum over kept (query block, KV block) pairs of valid rows x valid columns."""
    nb, n, b = w.blocks_per_frame, w.frame_len, w.block
    sizes = np.minimum(b, n - (np.arange(nb) * b))            # tokens per block within a frame
    cols = sizes[lists % nb].sum(axis=-1)                     # [H, n_q] valid columns
    rows = sizes[np.arange(lists.shape[1]) % nb]              # [n_q]
    return float(4.0 * w.head_dim * (cols * rows[None, :]).sum())


def cpu_baseline(w, x, lists_gpu, out_gpu, budget_s: float = 15.0):
    """Time the oracle (as it stands) on a bounded sample: full mask selection, then attention
    for (head, query block) pairs until the time budget is used."""
    from oracle import hsa_oracle as O
    from paper_2602_04789_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    Qf, Kf, Vf = (synth.bf16_bits_to_f32(x[k]) for k in "QKV")
    ob = O.chunk_budget(w.chunk_idx, w.schedule)
    t0 = time.perf_counter()
    lists = O.select_mask(Qf, Kf, w.frame_len, w.block, ob)
    t_sel = time.perf_counter() - t0
    lists_match = bool(np.array_equal(lists, lists_gpu))
    n_q = lists.shape[1]
    rng = np.random.default_rng(0)
    order = rng.permutation(w.heads * n_q)
    t_attn, flops, done, worst, err_sum, err_cnt = 0.0, 0.0, 0, 0.0, 0.0, 0
    nb = w.blocks_per_frame
    sizes = np.minimum(w.block, w.frame_len - np.arange(nb) * w.block)
    for flat in order:
        h, r = divmod(int(flat), n_q)
        t1 = time.perf_counter()
        ref = O.sparse_attention_block(Qf[h], Kf[h], Vf[h], r, lists[h, r], w.frame_len, w.block)
        t_attn += time.perf_counter() - t1
        lo, hi = O.block_token_range(r, w.frame_len, w.block)
        err = np.abs(out_gpu[h, lo:hi] - ref)
        worst = max(worst, float(err.max()))
        err_sum += float(err.sum())
        err_cnt += err.size
        flops += 4.0 * w.head_dim * float(sizes[r % nb]) * float(sizes[lists[h, r] % nb].sum())
        done += 1
        if t_sel + t_attn > budget_s:
            break
    frac = done / float(w.heads * n_q)
    # whole-step time = full selection + attention extrapolated from the sampled pairs
    est_step_s = t_sel + t_attn / frac
    total_flops = flops / frac
    return {
        "value": total_flops / est_step_s / 1e12, "unit": "TFLOP/s", "cores": int(cores),
        "kind": "oracle",
        "sample": (f"full mask selection ({t_sel:.2f} s) + attention for {done} of "
                   f"{w.heads * n_q} (head, query block) pairs ({t_attn:.2f} s), extrapolated "
                   f"to the whole chunk: {est_step_s:.1f} s per step"),
        "lists_match_gpu": lists_match, "sample_max_abs_err_gpu_vs_oracle": worst,
        "sample_mean_abs_err_gpu_vs_oracle": err_sum / max(err_cnt, 1),
    }


def measured_peaks(torch, select_bytes: int):
    """Ceilings measured with this repository's own micro-benchmarks (liblf_bench.so): a streaming
    16-byte read of as many bytes as mask selection reads, the same over 1 GiB, and a loop of
    back-to-back bf16 MFMAs on register operands."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2602_04789_amd", "liblf_bench.so")
    if not os.path.exists(path):
        return {"error": "liblf_bench.so not built"}
    lib = C.CDLL(path)
    lib.lfb_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.lfb_mfma_loop.argtypes = [C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def timed(fn, n):
        for _ in range(3):
            assert fn() == 0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    out = {}
    for name, nbytes in (("stream_read_select_bytes_gbps", select_bytes // 16 * 16),
                         ("stream_read_1gib_gbps", 1 << 30)):
        buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
        t = timed(lambda: lib.lfb_stream_read(buf.data_ptr(), nbytes, sink.data_ptr(), st), 20)
        out[name] = nbytes / t / 1e9
        del buf
    flop = C.c_double()
    for name, rnd in (("mfma_bf16_loop_constant_operands_tflops", 0), ("mfma_bf16_loop_random_operands_tflops", 1)):
        t = timed(lambda: lib.lfb_mfma_loop(4000, rnd, sink.data_ptr(), C.byref(flop), st), 5)
        out[name] = flop.value / t / 1e12
    # the attention step's instruction mix without memory: matrix instructions alone, the vector
    # work of the softmax alone, both in every wavefront (microseconds per launch of 2000 steps)
    lib.lfb_issue_mix.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    for wps in (2, 4):   # wavefronts per SIMD
        mix = {}
        for name, what in (("mfma_only_us", 1), ("softmax_valu_only_us", 2), ("both_us", 3)):
            mix[name] = timed(lambda: lib.lfb_issue_mix(what, 2000, wps, sink.data_ptr(), st), 5) * 1e6
        mix["overlap"] = (mix["mfma_only_us"] + mix["softmax_valu_only_us"] - mix["both_us"]) / \
            min(mix["mfma_only_us"], mix["softmax_valu_only_us"])
        # 16 matrix instructions of 2*32*32*16 FLOP per wavefront and step
        mix["both_tflops"] = 256 * 4 * wps * 2000 * 16 * 2.0 * 32 * 32 * 16 / (mix["both_us"] * 1e-6) / 1e12
        out[f"issue_mix_16_mfma_plus_softmax_step_{wps}_waves_per_simd"] = mix
    return out


def run_select_phases(torch, lf, synth, workload):
    """Where the selection kernel's time goes: the probe build of the library notes the wall clock
    (100 MHz) at the kernel's phase boundaries in every workgroup; lists are those of the product."""
    import ctypes
    from paper_2602_04789_amd import build as B
    path = B.probe_lib("stamps")
    if not os.path.exists(path):
        sys.exit(f"bench.py: {path} not built")
    w = _workloads()[workload]()
    x = synth.make_inputs(w)
    Q, K = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QK")
    b = lf.lf_chunk_budget(w.chunk_idx, lf.make_schedule(w.schedule))
    ref = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
    lf._lib, lf._LIB_PATH = None, path
    lf.load()
    raw = ctypes.CDLL(path)
    for _ in range(5):
        idx = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
    torch.cuda.synchronize()
    out = np.zeros(4096 * 8, dtype=np.uint64)
    rc = raw.lf_probe_select_stamps(ctypes.c_void_p(out.ctypes.data))
    if rc != 0:
        sys.exit(f"bench.py: lf_probe_select_stamps failed ({rc})")
    n_wg = min(4096, w.heads * w.frames_per_chunk * w.blocks_per_frame)
    st = out.reshape(4096, 8)[:n_wg, :7].astype(np.int64)
    names = ["load q_tilde", "frame scores (+ scores of the known candidates)", "frame ranking and list",
             "block scores of the retrieved frames", "block ranking", "compaction and store"]
    phases = []
    for i, name in enumerate(names):
        d = (st[:, i + 1] - st[:, i]) * 10.0
        phases.append({"phase": name, "mean_ns": float(d.mean()), "median_ns": float(np.median(d)),
                       "p90_ns": float(np.percentile(d, 90)), "max_ns": float(d.max())})
    tot = (st[:, 6] - st[:, 0]) * 10.0
    t0 = st[:, 0].min()
    print(json.dumps({"select_phases": phases, "workload": w.name, "workgroups": int(n_wg),
                      "workgroup_ns": {"mean": float(tot.mean()), "max": float(tot.max())},
                      "start_spread_ns": {"median": float(np.median(st[:, 0] - t0) * 10.0),
                                          "max": float((st[:, 0] - t0).max() * 10.0)},
                      "first_start_to_last_end_ns": float((st[:, 6].max() - t0) * 10.0),
                      "lists_equal_product": bool(torch.equal(idx, ref)),
                      "what": "probe build (LF_PROBE_STAMPS): wall clock of 10 ns ticks read by thread 0 of every "
                              "workgroup at the phase boundaries; last of 5 launches"}))


def run_fill_scan(torch, lf, synth, workload):
    """The attention kernel on the same shapes with 3 .. 28 heads, i.e. from fewer workgroups than
    compute units to four per unit: how its time grows with the fill of the chip."""
    from dataclasses import replace
    base = _workloads()[workload]()
    rows = []
    for heads in (3, 6, 7, 9, 10, 12, 13, 14, 16, 20, 24, 27, 28):
        w = replace(base, heads=heads)
        x = synth.make_inputs(w)
        Q, K, V = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QKV")
        b = lf.lf_chunk_budget(w.chunk_idx, lf.make_schedule(w.schedule))
        idx = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
        out = torch.empty_like(Q)
        flops = kept_flops(idx.cpu().numpy(), w)
        ts = []
        for _ in range(3):
            for _ in range(5):
                lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / 20)
        n_wg = (heads * w.frames_per_chunk * w.blocks_per_frame + 1) // 2
        rows.append({"heads": heads, "workgroups": n_wg, "ms": min(ts), "us_per_head": min(ts) * 1e3 / heads,
                     "tflops": flops / (min(ts) * 1e-3) / 1e12})
        del Q, K, V, out, idx
    print(json.dumps({"fill_scan": rows, "workload": base.name,
                      "what": "lf_sparse_attn alone, 20 launches back to back, minimum of 3 rounds; two query "
                              "blocks per workgroup, two workgroups per compute unit at a time"}))


def run_sensitivity(torch, lf, synth, workload):
    """How much the attention kernel lengthens when one unit gets more work per step: probe builds
    of the library (same kernel plus redundant work for one unit, results discarded, output
    unchanged) are timed against the product build, interleaved, on the same inputs."""
    from paper_2602_04789_amd import build as B
    w = _workloads()[workload]()
    x = synth.make_inputs(w)
    Q, K, V = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QKV")
    b = lf.lf_chunk_budget(w.chunk_idx, lf.make_schedule(w.schedule))
    idx = lf.lf_select_mask(Q, K, w.frame_len, w.block, b)
    ref = lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block)
    flops = kept_flops(idx.cpu().numpy(), w)
    # per step a wavefront does 16 transposing V reads, 8 K fragment reads, 16 MFMAs, 16 exp2
    cases = [("product", None, "nothing extra"),
             ("v_reads_x2", "tr", "+16 ds_read_b64_tr_b16 per step (+100 %)"),
             ("k_reads_x2", "k", "+8 ds_read_b128 per step (+100 %)"),
             ("mfma_x1.5", "mfma", "+8 v_mfma_f32_32x32x16_bf16 per step (+50 %)"),
             ("exp_x2", "exp", "+16 v_exp_f32 per step (+100 %)")]
    handles = []
    product = lf.load()
    for name, tag, desc in cases:
        if tag is None:
            handles.append(product)
            continue
        if not os.path.exists(B.probe_lib(tag)):
            sys.exit(f"bench.py: {B.probe_lib(tag)} not built")
        lf._lib, lf._LIB_PATH = None, B.probe_lib(tag)
        handles.append(lf.load())
    out = torch.empty_like(Q)
    res = [{"case": n, "extra": d, "ms": []} for n, _, d in cases]
    for rep in range(4):
        for i, h in enumerate(handles):
            lf._lib = h
            for _ in range(3):
                lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(20):
                lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
            e1.record()
            torch.cuda.synchronize()
            res[i]["ms"].append(e0.elapsed_time(e1) / 20)
            res[i]["output_equals_product"] = bool(torch.equal(out.view(torch.int16), ref.view(torch.int16)))
    lf._lib = product
    base = min(res[0]["ms"])
    for r in res:
        r["ms_min"] = min(r["ms"])
        r["slowdown"] = r["ms_min"] / base
    print(json.dumps({"sensitivity": res, "workload": w.name, "kept_gflop": flops / 1e9,
                      "baseline_tflops": flops / (base * 1e-3) / 1e12}))


def time_config(torch, lf, synth, w, steps, warmup, check_lists=True, train=True):
    """select / attention times of one workload (HIP events on the launch stream), its kept FLOPs,
    and whether every index list equals the oracle's."""
    from oracle import hsa_oracle as O
    x = synth.make_inputs(w)
    Q, K, V = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QKV")
    sched = lf.make_schedule(w.schedule)
    b = lf.lf_chunk_budget(w.chunk_idx, sched)
    sh = lf.make_shape(Q, K, frame_len=w.frame_len, block=w.block)
    ws = torch.empty(lf.lf_workspace_bytes(sh, b), dtype=torch.uint8, device="cuda")
    aws = torch.empty(lf.lf_attn_workspace_bytes(sh), dtype=torch.uint8, device="cuda")
    idx = torch.empty((w.heads, w.frames_per_chunk * w.blocks_per_frame, b.list_len), dtype=torch.int32,
                      device="cuda")
    out = torch.empty_like(Q)

    def timed(fn):
        for _ in range(warmup):
            fn()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
        torch.cuda.synchronize()
        for e in ev:
            e[0].record()
            fn()
            e[1].record()
        torch.cuda.synchronize()
        return float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))

    sel_ms = timed(lambda: lf.lf_select_mask(Q, K, w.frame_len, w.block, b, indices=idx, workspace=ws))
    one_pass = lambda: lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
    split = lambda: lf.lf_sparse_attn_split(Q, K, V, idx, w.frame_len, w.block, b, O=out, workspace=aws)
    # the two attention calls are timed in alternating rounds, so that neither gets the cooler chip
    rounds = [[], []]
    for _ in range(3 if b.current_mandatory else 1):
        rounds[0].append(timed(one_pass))
        if b.current_mandatory:
            rounds[1].append(timed(split))
    attn_ms = float(np.mean(rounds[0]))
    lists = idx.cpu().numpy()
    flops = kept_flops(lists, w)
    sel_bytes = float((w.q_len + w.kv_len) * w.heads * w.head_dim * 2)
    res = {"workload": w.name, "heads": w.heads, "q_len": w.q_len, "kv_len": w.kv_len,
           "list_len": int(b.list_len), "kv_blocks": w.frames * w.blocks_per_frame,
           "select_ms": sel_ms, "attn_ms": attn_ms, "kept_gflop": flops / 1e9,
           "attn_tflops": flops / (attn_ms * 1e-3) / 1e12,
           "attn_frac_of_bf16_peak": flops / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "select_gbps": sel_bytes / (sel_ms * 1e-3) / 1e9,
           "select_frac_of_hbm_peak": sel_bytes / (sel_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS}
    if b.current_mandatory:
        res["attn_split_ms"] = float(np.mean(rounds[1]))
    if train:
        one_pass()
        tr = time_training(torch, lf, synth, w, Q, K, V, idx, out, flops, n=max(3, steps // 2))
        res["bwd_ms"], res["bwd_tflops"] = tr["bwd_ms"], tr["bwd_achieved"]
    if check_lists:
        ob = O.chunk_budget(w.chunk_idx, w.schedule)
        want = O.select_mask(synth.bf16_bits_to_f32(x["Q"]), synth.bf16_bits_to_f32(x["K"]),
                             w.frame_len, w.block, ob)
        res["lists_match_oracle"] = bool(np.array_equal(want, lists))
    return res


def time_training(torch, lf, synth, w, Q, K, V, idx, out, flops, n=20):
    """Training pair (the paper finetunes with the sparse mask in place): the forward call that
    also leaves the rows' log-sum-exp, and the backward call (delta, transposed lists, dQ, dK and
    dV launches).  Algorithmic work of the backward: five products per kept tile (dV, dP, dQ, dK
    and the recomputed scores), 2.5 x the forward's."""
    dO = torch.from_numpy(synth.make_upstream_grad(w)).view(torch.bfloat16).cuda()
    lse2 = torch.empty((w.heads, w.q_len), dtype=torch.float32, device="cuda")
    sh = lf.make_shape(Q, K, V, out, frame_len=w.frame_len, block=w.block)
    bws = torch.empty(lf.lf_attn_bwd_workspace_bytes(sh), dtype=torch.uint8, device="cuda")
    fwd = lambda: lf.lf_sparse_attn_fwd(Q, K, V, idx, w.frame_len, w.block, O=out, lse2=lse2)
    bwd = lambda: lf.lf_sparse_attn_bwd(Q, K, V, out, dO, lse2, idx, w.frame_len, w.block, workspace=bws)
    t_ms = []
    for fn in (fwd, bwd):
        # untimed calls, then the timed ones right behind them (no idle gap in between: after one
        # the first launches run at a lower clock for a few milliseconds); the median
        te = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]
        for _ in range(10):
            fn()
        for e in te:
            e[0].record()
            fn()
            e[1].record()
        torch.cuda.synchronize()
        t_ms.append(float(np.median([e[0].elapsed_time(e[1]) for e in te])))
    tf = 2.5 * flops / (t_ms[1] * 1e-3) / 1e12
    return {"what": "lf_sparse_attn_fwd (O and log-sum-exp) and lf_sparse_attn_bwd (dQ, dK, dV) on the same "
                    "lists; backward work counted as 2.5 x the forward's kept flops",
            "fwd_ms": t_ms[0], "bwd_ms": t_ms[1], "bwd_achieved": tf, "unit": "TFLOP/s",
            "bwd_frac": tf / PEAK_BF16_TFLOPS}


def run_rollout(args, torch, lf, synth):
    """One step = the 28 calls of a 7-chunk, 4-denoising-step rollout at 40 heads: the cache
    grows by one chunk per chunk index, the keep ratio follows the schedule, history K/V stay
    fixed over the four steps of a chunk and the current chunk is redrawn per step."""
    calls = []
    total_flops = 0.0
    for chunk in range(1, 8):
        for step_i in range(4):
            w = synth.cfg_rollout(chunk, step_i)
            print(f"rollout: generating chunk {chunk} step {step_i}", file=sys.stderr, flush=True)
            x = synth.make_inputs(w)
            Q, K, V = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QKV")
            sched = lf.make_schedule(w.schedule)
            b = lf.lf_chunk_budget(w.chunk_idx, sched)
            sh = lf.make_shape(Q, K, frame_len=w.frame_len, block=w.block)
            ws = torch.empty(lf.lf_workspace_bytes(sh, b), dtype=torch.uint8, device="cuda")
            idx = torch.empty((w.heads, w.frames_per_chunk * w.blocks_per_frame, b.list_len),
                              dtype=torch.int32, device="cuda")
            out = torch.empty_like(Q)
            calls.append((w, sched, Q, K, V, b, ws, idx, out))

    def step():
        for (w, sched, Q, K, V, b, ws, idx, out) in calls:
            bb = lf.lf_chunk_budget(w.chunk_idx, sched)
            lf.lf_select_mask(Q, K, w.frame_len, w.block, bb, indices=idx, workspace=ws)
            lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_chunk = []
    for (w, sched, Q, K, V, b, ws, idx, out) in calls:
        total_flops += kept_flops(idx.cpu().numpy(), w)
    # per-chunk times: the four steps of each chunk, timed on their own
    for c in range(7):
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for (w, sched, Q, K, V, b, ws, idx, out) in calls[4 * c:4 * c + 4]:
            bb = lf.lf_chunk_budget(w.chunk_idx, sched)
            lf.lf_select_mask(Q, K, w.frame_len, w.block, bb, indices=idx, workspace=ws)
            lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
        torch.cuda.synchronize()
        per_chunk.append((time.perf_counter() - t1) * 1e3)
    ms_step = wall * 1e3 / args.steps
    w0 = calls[0][0]
    print(json.dumps({
        "metric": "effective TFLOP/s on kept blocks, whole step (mask selection + block-sparse attention)",
        "value": total_flops / (ms_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"rollout: {w0.heads} heads x {w0.head_dim}, 7 chunks x 4 steps = 28 calls, "
                               f"Q {w0.q_len}, KV {w0.q_len}..{calls[-1][0].kv_len}, keep ratio by the linear schedule",
                   "heads": w0.heads, "head_dim": w0.head_dim, "calls": len(calls),
                   "list_len_per_chunk": [int(calls[4 * c][5].list_len) for c in range(7)]},
        "ms_per_chunk_4_steps": per_chunk, "kept_gflop": total_flops / 1e9,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="last_chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the micro-benchmarks (streaming read, MFMA loop)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per_config list (other benchmark configurations, the paper's own "
                         "operating points, one call per chunk of the 40-head rollout)")
    ap.add_argument("--no-training", action="store_true",
                    help="skip the timing of the training pair (forward with log-sum-exp, backward)")
    ap.add_argument("--training-only", action="store_true",
                    help="one selection, then only the training pair (for kernel traces of the backward)")
    ap.add_argument("--no-cached-select", action="store_true",
                    help="skip the pooled-key-cache variant of the selection (keeps profiles to the "
                         "four kernels of the main path)")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip timing the step as one captured HIP graph")
    ap.add_argument("--attn", choices=("one_pass", "split"), default="one_pass",
                    help="attention call of the timed step: lf_sparse_attn (one list-driven kernel) or "
                         "lf_sparse_attn_split (dense kernel over the current chunk + list-driven kernel)")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the timed step: no cached selection, graph replay, pooling-only and split "
                         "timings, per_config list, micro-benchmarks or CPU baseline (for profiler runs)")
    ap.add_argument("--sensitivity", action="store_true",
                    help="time the probe build of the attention kernel with extra work per unit "
                         "(prints its own JSON line and exits)")
    ap.add_argument("--select-phases", action="store_true",
                    help="phase times of the selection kernel from its probe build (prints its own JSON line and exits)")
    ap.add_argument("--fill-scan", action="store_true",
                    help="time the attention kernel alone at 3 .. 28 heads (prints its own JSON line and exits)")
    ap.add_argument("--micro-only", action="store_true",
                    help="run only the micro-benchmarks (streaming read, MFMA loop) and exit")
    ap.add_argument("--cold", action="store_true",
                    help="also time one step right after streaming a 1 GiB buffer through the caches")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE scaling)")
    args = ap.parse_args()
    if args.headline_only:
        args.no_cached_select = args.no_graph = args.no_per_config = True
        args.no_measured_peaks = args.no_cpu_baseline = True
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (heads would shard across GPUs "
                 "without communication; no multi-GPU figure is produced). Use --gpus 1.")

    import torch
    from paper_2602_04789_amd import lf, synth
    lf.load()   # raises if the HIP library is not built: there is no fallback path
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.micro_only:
        print(json.dumps({"measured": measured_peaks(torch, 115015680)}))
        return
    if args.sensitivity:
        return run_sensitivity(torch, lf, synth, args.workload)
    if args.fill_scan:
        return run_fill_scan(torch, lf, synth, args.workload)
    if args.select_phases:
        return run_select_phases(torch, lf, synth, args.workload)
    if args.workload == "rollout":
        if args.steps == 100 and args.warmup == 20:   # the defaults are sized for one chunk
            args.steps, args.warmup = 5, 1
        return run_rollout(args, torch, lf, synth)
    w = _workloads()[args.workload]()
    x = synth.make_inputs(w)
    Q, K, V = (torch.from_numpy(x[k]).view(torch.bfloat16).cuda() for k in "QKV")
    sched = lf.make_schedule(w.schedule)
    b = lf.lf_chunk_budget(w.chunk_idx, sched)
    sh = lf.make_shape(Q, K, frame_len=w.frame_len, block=w.block)
    ws = torch.empty(lf.lf_workspace_bytes(sh, b), dtype=torch.uint8, device="cuda")
    nb = w.blocks_per_frame
    idx = torch.empty((w.heads, w.frames_per_chunk * nb, b.list_len), dtype=torch.int32, device="cuda")
    out = torch.empty_like(Q)
    use_split = args.attn == "split" and bool(b.current_mandatory)
    aws0 = torch.empty(lf.lf_attn_workspace_bytes(sh), dtype=torch.uint8, device="cuda") if use_split else None

    def attend(bb):
        if use_split:
            lf.lf_sparse_attn_split(Q, K, V, idx, w.frame_len, w.block, bb, O=out, workspace=aws0)
        else:
            lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)

    def step():
        bb = lf.lf_chunk_budget(w.chunk_idx, sched)
        lf.lf_select_mask(Q, K, w.frame_len, w.block, bb, indices=idx, workspace=ws)
        attend(bb)

    if args.training_only:
        step()
        torch.cuda.synchronize()
        print(json.dumps({"workload": w.name,
                          "training": time_training(torch, lf, synth, w, Q, K, V, idx, out,
                                                    kept_flops(idx.cpu().numpy(), w), n=args.steps)}))
        return
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # one copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        bb = lf.lf_chunk_budget(w.chunk_idx, sched)
        ev[i][0].record()
        lf.lf_select_mask(Q, K, w.frame_len, w.block, bb, indices=idx, workspace=ws)
        ev[i][1].record()
        attend(bb)
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    sel_all = np.array([e[0].elapsed_time(e[1]) for e in ev])
    attn_all = np.array([e[1].elapsed_time(e[2]) for e in ev])
    sel_ms, attn_ms = float(sel_all.mean()), float(attn_all.mean())
    cold = None
    if args.cold:
        big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        big.fill_(3)                 # 1 GiB through L2 and the memory-side cache
        torch.cuda.synchronize()
        c = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        c[0].record()
        lf.lf_select_mask(Q, K, w.frame_len, w.block, b, indices=idx, workspace=ws)
        c[1].record()
        lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)
        c[2].record()
        torch.cuda.synchronize()
        cold = {"select_ms": c[0].elapsed_time(c[1]), "attn_ms": c[1].elapsed_time(c[2])}
        del big
    traffic, traffic_commit = measured_traffic()
    lists = idx.cpu().numpy()
    flops = kept_flops(lists, w)
    tile_flops = 4.0 * 64 * 64 * w.head_dim * lists.size
    sel_bytes = float((w.q_len + w.kv_len) * w.heads * w.head_dim * 2)
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12
    sel_gbps = sel_bytes / (sel_ms * 1e-3) / 1e9

    res = {
        "metric": "effective TFLOP/s on kept blocks, whole step (mask selection + block-sparse attention)",
        "value": flops / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.heads} heads x {w.head_dim}, Q {w.q_len}, KV {w.kv_len} "
                               f"({w.frames} frames x {w.frame_len}), block 64, "
                               f"{b.list_len} of {w.frames * nb} KV blocks kept per query block",
                   "heads": w.heads, "head_dim": w.head_dim, "q_len": w.q_len, "kv_len": w.kv_len,
                   "list_len": int(b.list_len), "k_blocks": int(b.k_blocks), "k_frames": int(b.k_frames)},
        "ms_per_chunk": ms_step, "select_ms": sel_ms, "attn_ms": attn_ms,
        "select_ms_median_min": [float(np.median(sel_all)), float(sel_all.min())],
        "attn_ms_median_min": [float(np.median(attn_all)), float(attn_all.min())],
        "kept_gflop": flops / 1e9, "tile_gflop": tile_flops / 1e9,
        "roofline": {"kernel": "lf_attn_kernel (list-driven)" if not use_split else
                               "lf_sparse_attn_split: dense + list-driven lf_attn_kernel launches together",
                     "bound": "mfma", "achieved": attn_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / PEAK_BF16_TFLOPS,
                     "traffic": traffic.get("attn") if args.workload == "last_chunk" and not use_split else None},
        "select": {"bound": "hbm", "achieved": sel_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                   "frac": sel_gbps / PEAK_HBM_GBPS, "bytes": sel_bytes,
                   "traffic": traffic.get("select") if args.workload == "last_chunk" else None},
        "traffic_source": {"file": "profiles/last_chunk_pmc_counters.txt", "profile_commit": traffic_commit},
    }
    # the pooling pass alone (block and frame means of the whole cache, no Q, no scoring): the
    # HBM-bound part of mask selection on its own bytes
    if args.headline_only:
        print(json.dumps(res))
        return
    kc_all = torch.empty(lf.lf_kcache_bytes(sh, w.frames), dtype=torch.uint8, device="cuda")
    pe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(30)]
    for _ in range(5):
        lf.lf_kcache_update(K, w.frame_len, w.block, 0, w.frames, w.frames, kc_all)
    torch.cuda.synchronize()
    for e in pe:
        e[0].record()
        lf.lf_kcache_update(K, w.frame_len, w.block, 0, w.frames, w.frames, kc_all)
        e[1].record()
    torch.cuda.synchronize()
    p_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in pe]))
    p_bytes = float(w.kv_len * w.heads * w.head_dim * 2)
    res["pool_only"] = {"what": "lf_kcache_update over the whole cache: pooling kernel + frame means, K only",
                        "ms": p_ms, "bytes": p_bytes, "achieved": p_bytes / (p_ms * 1e-3) / 1e9, "unit": "GB/s",
                        "frac": p_bytes / (p_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS}
    del kc_all
    if b.current_mandatory and not args.headline_only and not use_split:
        aws = torch.empty(lf.lf_attn_workspace_bytes(sh), dtype=torch.uint8, device="cuda")
        # 20 untimed calls, then 30 timed ones right behind them (no idle gap in between: after
        # one the first launches run at a lower clock for a few milliseconds); the median
        se = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(30)]
        for _ in range(20):
            lf.lf_sparse_attn_split(Q, K, V, idx, w.frame_len, w.block, b, O=out, workspace=aws)
        for e in se:
            e[0].record()
            lf.lf_sparse_attn_split(Q, K, V, idx, w.frame_len, w.block, b, O=out, workspace=aws)
            e[1].record()
        torch.cuda.synchronize()
        s_ms = float(np.median([e[0].elapsed_time(e[1]) for e in se]))
        res["attn_split"] = {"what": "lf_sparse_attn_split: dense kernel over the current chunk + list-driven kernel "
                                     "over the retrieved blocks", "ms": s_ms,
                             "achieved": flops / (s_ms * 1e-3) / 1e12, "unit": "TFLOP/s"}
        lf.lf_sparse_attn(Q, K, V, idx, w.frame_len, w.block, O=out)   # `out` again holds the one-pass result
    if not args.no_training:
        res["training"] = time_training(torch, lf, synth, w, Q, K, V, idx, out, flops)
    if not args.no_cached_select:
        # Selection with the pooled-key cache: the history frames were pooled when their chunk was
        # generated (not timed: it happened in earlier calls of the rollout); a call pools only Q
        # and the chunk being denoised.
        max_frames = w.frames
        kc = torch.empty(lf.lf_kcache_bytes(sh, max_frames), dtype=torch.uint8, device="cuda")
        lf.lf_kcache_update(K, w.frame_len, w.block, 0, w.hist_frames, max_frames, kc)
        idx_c = torch.empty_like(idx)

        def cached():
            lf.lf_select_mask_cached(Q, kc, max_frames, w.kv_len, w.frame_len, w.block, b, Kcache=K,
                                     indices=idx_c, workspace=ws)

        for _ in range(5):
            cached()
        ce = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(50)]
        torch.cuda.synchronize()
        for e in ce:
            e[0].record()
            cached()
            e[1].record()
        torch.cuda.synchronize()
        c_ms = np.array([e[0].elapsed_time(e[1]) for e in ce])
        c_bytes = float((w.q_len + w.q_len) * w.heads * w.head_dim * 2)   # Q and the current chunk's K
        res["select_cached"] = {"ms": float(c_ms.mean()), "ms_median_min": [float(np.median(c_ms)), float(c_ms.min())],
                                "bytes": c_bytes, "achieved": c_bytes / (c_ms.mean() * 1e-3) / 1e9,
                                "unit": "GB/s", "lists_equal_uncached": bool(torch.equal(idx_c, idx))}
    if not args.no_graph:
        # The same step (budget on the host, four kernels) captured once and replayed: what a
        # caller that fixes its buffers pays without the per-launch host work.
        try:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step()
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            res["graph_replay"] = {"ms_per_step": (time.perf_counter() - t0) * 1e3 / args.steps}
        except RuntimeError as exc:   # an extra: the headline numbers above do not depend on it
            res["graph_replay"] = {"ms_per_step": None, "error": str(exc)[:200]}
    if cold is not None:
        res["cold_after_1gib_stream"] = cold
    if not args.no_measured_peaks:
        res["measured"] = m = measured_peaks(torch, int(sel_bytes))
        # the same two fractions against what this chip reached in this run: the register-only
        # matrix loop on pseudo-random operands, and the plain streaming read of the same bytes
        res["roofline"]["frac_of_measured_mfma_loop_random_operands"] = \
            res["roofline"]["achieved"] / m["mfma_bf16_loop_random_operands_tflops"]
        res["select"]["frac_of_measured_stream_read"] = res["select"]["achieved"] / m["stream_read_select_bytes_gbps"]
    if not args.no_per_config:
        per = []
        names = [n for n in ("first_chunk", "mid_rollout", "last_chunk", "paper5s_last", "paper15s_late")
                 if n != args.workload]
        for n in names:
            print(f"per_config: {n}", file=sys.stderr, flush=True)
            per.append(time_config(torch, lf, synth, _workloads()[n](), 20, 5, train=not args.no_training))
        for chunk in range(1, 8):
            print(f"per_config: rollout chunk {chunk} (40 heads)", file=sys.stderr, flush=True)
            per.append(time_config(torch, lf, synth, synth.cfg_rollout(chunk, 0), 10, 3, train=not args.no_training))
        res["per_config"] = per
        ro = [p for p in per if p["workload"].startswith("rollout_")]
        # a 5-second video's 7 chunks x 4 denoising steps, one layer: each chunk's call four times
        res["rollout_28_calls_est"] = {"ms": 4.0 * sum(p["select_ms"] + p["attn_ms"] for p in ro),
                                       "kept_gflop": 4.0 * sum(p["kept_gflop"] for p in ro),
                                       "how": "4 x the sum of the seven 40-head calls above (step 0 of each chunk); "
                                              "--workload rollout times all 28 calls"}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, x, lists, out.float().cpu().numpy().astype(np.float64))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
