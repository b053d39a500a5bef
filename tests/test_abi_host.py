"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, lf_chunk_budget agrees with the oracle's budget on every schedule tried, and
every argument error is reported before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

from oracle import hsa_oracle as O
from paper_2602_04789_amd import lf, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lf.library_path()):
        from paper_2602_04789_amd import build
        build.build()
    return lf.load()


def test_library_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "lf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(lf_[a-z_]+)\s*\(", text))
    assert {"lf_chunk_budget", "lf_select_mask", "lf_sparse_attn", "lf_workspace_bytes",
            "lf_workspace_layout", "lf_strerror", "lf_version", "lf_kcache_bytes",
            "lf_kcache_update", "lf_select_mask_cached", "lf_sparse_attn_split",
            "lf_attn_workspace_bytes", "lf_select_mask_static", "lf_init", "lf_qk_norm_rope",
            "lf_sparse_attn_fwd", "lf_sparse_attn_bwd", "lf_attn_bwd_workspace_bytes"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert lf.lf_version() >= 100
    assert lf.lf_strerror(0) == "ok" and "NULL" in lf.lf_strerror(-1)


def test_probe_and_benchmark_libraries_load(lib):
    """The probe builds (product library with one redundant-work variant of the attention kernel)
    and the micro-benchmark library resolve all their symbols."""
    from paper_2602_04789_amd import build
    for tag in build.PROBES:
        probe = C.CDLL(build.probe_lib(tag))
        assert hasattr(probe, "lf_sparse_attn") and hasattr(probe, "lf_sparse_attn_bwd")
    stamps = C.CDLL(build.probe_lib("stamps"))   # selection kernel with phase stamps
    assert hasattr(stamps, "lf_select_mask") and hasattr(stamps, "lf_probe_select_stamps")
    assert not hasattr(lib, "lf_probe_select_stamps")   # the product build carries no stamps
    assert hasattr(C.CDLL(build.BENCH_LIB), "lfb_stream_read")


def test_struct_sizes_match_header(lib):
    # 12 int32 + 5 double; 8 int32 + double; 8 int32 + 8 int64
    assert C.sizeof(lf.lf_schedule) == 12 * 4 + 5 * 8
    assert C.sizeof(lf.lf_budget) == 8 * 4 + 8
    assert C.sizeof(lf.lf_shape) == 8 * 4 + 8 * 8


def _all_schedules():
    yield synth.cfg_tiny().schedule, range(1, 8)
    yield synth.cfg_first_chunk().schedule, range(1, 8)
    yield synth.cfg_mid_rollout().schedule, range(1, 8)
    yield synth.cfg_last_chunk().schedule, range(1, 8)
    yield synth.cfg_rollout(1, 0).schedule, range(1, 8)
    yield synth.cfg_paper_5s(1).schedule, range(1, 8)
    yield synth.cfg_paper_15s(1).schedule, range(1, 22)
    for mode in (0, 1, 2):
        for ratio_of in (0, 1, 2):
            for cm in (0, 1):
                for fcd in (0, 1):
                    for (ns, nw, kf) in ((0, 0, 0), (1, 2, 3), (2, 1, 1), (1, 1, 40)):
                        for n, nch in ((1560, 7), (1536, 21), (200, 5), (64, 3)):
                            yield synth.Schedule(mode=mode, n_chunks=nch, frames_per_chunk=3,
                                                 frame_len=n, n_sink=ns, n_win=nw, k_frames=kf,
                                                 ratio_of=ratio_of, current_mandatory=cm,
                                                 first_chunk_dense=fcd, keep_fixed=0.37,
                                                 keep_first=0.9, keep_last=0.15, s_base=0.95,
                                                 s_target=0.85), range(1, nch + 1)


def test_chunk_budget_matches_oracle(lib):
    count = 0
    for sch, chunks in _all_schedules():
        for i in chunks:
            got = lf.lf_chunk_budget(i, sch)
            want = O.chunk_budget(i, sch)
            for name in ("n_hist_frames", "frames_per_chunk", "n_sink", "n_win", "k_frames",
                         "k_blocks", "current_mandatory", "list_len"):
                assert getattr(got, name) == getattr(want, name), (sch, i, name)
            # the two sides evaluate Eq. 5-6 with differently arranged sums
            assert abs(got.keep_ratio - want.keep_ratio) <= 1e-14, (sch, i)
            count += 1
    assert count > 3000


def _golden(name):
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


def test_chunk_budget_matches_hand_computed_counts(lib):
    """The C call against the golden tables (hand arithmetic from the benchmark wording and
    from Eq. 5-6 with the appendix table), not against the oracle."""
    for name, chunk, k_blocks, list_len in _golden("baseline_configs.txt"):
        chunk = int(chunk)
        w = {"first_chunk": synth.cfg_first_chunk, "mid_rollout": synth.cfg_mid_rollout,
             "last_chunk": synth.cfg_last_chunk}.get(name, lambda: synth.cfg_rollout(chunk, 0))()
        b = lf.lf_chunk_budget(chunk, w.schedule)
        assert (b.k_blocks, b.list_len) == (int(k_blocks), int(list_len)), (name, chunk)
    for setting, chunk, k_blocks in _golden("cag_list_len.txt"):
        w = (synth.cfg_paper_5s if setting == "5s" else synth.cfg_paper_15s)(int(chunk))
        b = lf.lf_chunk_budget(int(chunk), w.schedule)
        assert (b.k_blocks, b.list_len, b.current_mandatory) == (int(k_blocks), int(k_blocks), 0)


def test_chunk_budget_rejects_a_schedule_that_leaves_the_unit_interval(lib):
    """s_base 0.5 / s_target 0.1 over 7 chunks: s_2 = -0.112 (not a ratio), s_7 = 0.173."""
    sch = lf.make_schedule(synth.Schedule(mode=synth.SCHED_CAG, n_chunks=7, frame_len=1536,
                                          ratio_of=synth.OF_ALL, current_mandatory=0,
                                          first_chunk_dense=1, s_base=0.5, s_target=0.1))
    out = lf.lf_budget()
    assert lib.lf_chunk_budget(2, C.byref(sch), C.byref(out)) == -8
    assert lib.lf_chunk_budget(3, C.byref(sch), C.byref(out)) == 0   # s_3 = 0.0003
    assert lib.lf_chunk_budget(7, C.byref(sch), C.byref(out)) == 0 and out.k_blocks == 216
    with pytest.raises(ValueError):
        O.chunk_budget(2, synth.Schedule(mode=synth.SCHED_CAG, n_chunks=7, frame_len=1536,
                                         ratio_of=synth.OF_ALL, current_mandatory=0,
                                         first_chunk_dense=1, s_base=0.5, s_target=0.1))


def test_chunk_budget_errors(lib):
    s = lf.make_schedule(synth.cfg_last_chunk().schedule)
    out = lf.lf_budget()
    assert lib.lf_chunk_budget(1, None, C.byref(out)) == -1
    assert lib.lf_chunk_budget(1, C.byref(s), None) == -1
    assert lib.lf_chunk_budget(0, C.byref(s), C.byref(out)) == -8
    for field, bad in (("mode", 7), ("ratio_of", -1), ("frames_per_chunk", 0), ("frame_len", 0),
                       ("block", 0), ("n_sink", -1), ("k_frames", -2), ("keep_fixed", 1.5)):
        t = lf.make_schedule(synth.cfg_last_chunk().schedule)
        setattr(t, field, bad)
        assert lib.lf_chunk_budget(2, C.byref(t), C.byref(out)) == -8, field


def _good():
    w = synth.cfg_last_chunk()
    sh = lf.lf_shape()
    sh.heads, sh.head_dim, sh.frame_len, sh.block = w.heads, w.head_dim, w.frame_len, 64
    sh.q_len, sh.kv_len, sh.dtype = w.q_len, w.kv_len, 0
    for t, L in (("q", w.q_len), ("k", w.kv_len), ("v", w.kv_len), ("o", w.q_len)):
        setattr(sh, f"{t}_stride_tok", w.head_dim)
        setattr(sh, f"{t}_stride_head", w.head_dim * L)
    return w, sh, lf.lf_chunk_budget(w.chunk_idx, w.schedule)


FAKE = 0x10000  # a non-NULL, 256-byte aligned address that is never dereferenced on error paths


def test_workspace_size_and_layout(lib):
    w, sh, b = _good()
    need = lf.lf_workspace_bytes(sh, b)
    nb = 25
    assert need >= 4 * w.heads * w.head_dim * (3 * nb + 21 * nb + 15)
    o = lf.lf_workspace_layout(sh, b)
    assert o[0] == 0 and o[0] < o[1] < o[2] < need and all(x % 256 == 0 for x in o)
    b.k_blocks += 1                      # list_len no longer consistent
    assert lf.lf_workspace_bytes(sh, b) == 0


def test_select_mask_argument_errors_enqueue_nothing(lib):
    w, sh, b = _good()
    need = lf.lf_workspace_bytes(sh, b)
    call = lambda Q=FAKE, K=FAKE, s=sh, bb=b, idx=FAKE, ws=FAKE, nbytes=need: lib.lf_select_mask(
        Q, K, C.byref(s) if s is not None else None, C.byref(bb) if bb is not None else None,
        idx, ws, nbytes, None)
    assert call(Q=None) == -1 and call(K=None) == -1 and call(idx=None) == -1
    assert call(s=None) == -1 and call(bb=None) == -1
    assert call(ws=None) == -6 and call(nbytes=need - 1) == -6
    assert call(Q=FAKE + 2) == -5 and call(ws=FAKE + 16) == -5
    for field, bad, code in (("block", 32, -2), ("head_dim", 96, -2), ("dtype", 1, -4),
                             ("q_len", w.q_len + 1, -2), ("kv_len", w.frame_len, -2),
                             ("heads", 0, -2), ("k_stride_tok", 129, -5), ("k_stride_tok", 64, -2)):
        _, s2, _ = _good()
        setattr(s2, field, bad)
        assert call(s=s2) == code, field
    for field, bad in (("k_blocks", 151), ("k_blocks", -1), ("k_frames", 16), ("n_sink", 17),
                       ("list_len", 187), ("n_hist_frames", 17), ("current_mandatory", 2)):
        _, _, b2 = _good()
        setattr(b2, field, bad)
        assert call(bb=b2) == -3, field


def test_kcache_size_and_argument_errors_enqueue_nothing(lib):
    w, sh, b = _good()           # last chunk: 21 frames of 25 blocks, 12 heads x 128
    need = lf.lf_kcache_bytes(sh, 21)
    assert need == 12 * (21 * 25 + 21) * 128 * 4
    assert lf.lf_kcache_bytes(sh, 24) > need
    assert lf.lf_kcache_bytes(sh, 0) == 0 and lf.lf_kcache_bytes(sh, 1 << 20) == 0
    _, bad, _ = _good()
    bad.head_dim = 96
    assert lf.lf_kcache_bytes(bad, 21) == 0
    upd = lambda K=FAKE, s=sh, f0=0, f1=21, mf=21, kc=FAKE, nbytes=need: lib.lf_kcache_update(
        K, C.byref(s) if s is not None else None, f0, f1, mf, kc, nbytes, None)
    assert upd(K=None) == -1 and upd(s=None) == -1
    assert upd(f0=-1) == -2 and upd(f0=5, f1=4) == -2 and upd(f1=22) == -2 and upd(mf=20) == -2
    assert upd(kc=None) == -6 and upd(nbytes=need - 1) == -6
    assert upd(K=FAKE + 4) == -5 and upd(kc=FAKE + 64) == -5
    assert upd(f0=7, f1=7) == 0          # empty range: nothing to do, nothing enqueued
    qbytes = 12 * 75 * 128 * 4
    sel = lambda Q=FAKE, K=None, kc=FAKE, nbytes=need, mf=21, s=sh, bb=b, idx=FAKE, ws=FAKE, wsb=qbytes: \
        lib.lf_select_mask_cached(Q, K, kc, nbytes, mf, C.byref(s) if s is not None else None,
                                  C.byref(bb) if bb is not None else None, idx, ws, wsb, None)
    assert sel(Q=None) == -1 and sel(idx=None) == -1 and sel(s=None) == -1 and sel(bb=None) == -1
    assert sel(kc=None) == -6 and sel(nbytes=need - 1) == -6
    assert sel(ws=None) == -6 and sel(wsb=qbytes - 1) == -6
    assert sel(mf=20) == -2
    assert sel(Q=FAKE + 2) == -5 and sel(kc=FAKE + 16) == -5 and sel(K=FAKE + 8) == -5
    _, _, b2 = _good()
    b2.k_blocks += 1
    assert sel(bb=b2) == -3


def test_sparse_attn_argument_errors_enqueue_nothing(lib):
    w, sh, b = _good()
    call = lambda Q=FAKE, K=FAKE, V=FAKE, s=sh, idx=FAKE, ll=188, sc=0.0, Out=FAKE: \
        lib.lf_sparse_attn(Q, K, V, C.byref(s) if s is not None else None, idx, ll, sc, Out, None)
    assert call(Q=None) == -1 and call(K=None) == -1 and call(V=None) == -1
    assert call(idx=None) == -1 and call(Out=None) == -1 and call(s=None) == -1
    assert call(ll=0) == -3
    assert call(sc=-1.0) == -2 and call(sc=float("nan")) == -2
    assert call(V=FAKE + 8) == -5
    _, s2, _ = _good()
    s2.head_dim = 256
    assert call(s=s2) == -2


def test_sparse_attn_split_argument_errors_enqueue_nothing(lib):
    w, sh, b = _good()
    need = lf.lf_attn_workspace_bytes(sh)
    assert need >= w.heads * w.q_len * (w.head_dim + 2) * 4
    call = lambda Q=FAKE, K=FAKE, V=FAKE, s=sh, bb=b, idx=FAKE, sc=0.0, Out=FAKE, ws=FAKE, nbytes=need: \
        lib.lf_sparse_attn_split(Q, K, V, C.byref(s) if s is not None else None,
                                 C.byref(bb) if bb is not None else None, idx, sc, Out, ws, nbytes, None)
    assert call(Q=None) == -1 and call(V=None) == -1 and call(bb=None) == -1 and call(Out=None) == -1
    assert call(ws=None) == -6 and call(nbytes=need - 1) == -6 and call(ws=FAKE + 16) == -5
    assert call(sc=-1.0) == -2 and call(K=FAKE + 8) == -5
    _, _, b2 = _good()
    b2.list_len -= 1
    assert call(bb=b2) == -3
    _, s2, _ = _good()
    s2.head_dim = 96
    assert lf.lf_attn_workspace_bytes(s2) == 0 and call(s=s2) == -2


def test_sparse_attn_training_pair_argument_errors_enqueue_nothing(lib):
    w, sh, b = _good()
    fwd = lambda Q=FAKE, K=FAKE, V=FAKE, s=sh, idx=FAKE, ll=188, sc=0.0, Out=FAKE, lse=FAKE: \
        lib.lf_sparse_attn_fwd(Q, K, V, C.byref(s) if s is not None else None, idx, ll, sc, Out, lse, None)
    assert fwd(Q=None) == -1 and fwd(lse=None) == -1 and fwd(Out=None) == -1 and fwd(s=None) == -1
    assert fwd(ll=0) == -3 and fwd(sc=-1.0) == -2 and fwd(lse=FAKE + 2) == -5 and fwd(K=FAKE + 8) == -5
    need = lf.lf_attn_bwd_workspace_bytes(sh)
    nb = -(-w.frame_len // w.block)
    n_q, n_k = w.frames_per_chunk * nb, w.frames * nb
    assert need >= w.heads * (w.q_len * 4 + n_k * n_q * 4 + n_k * 4)
    bwd = lambda Q=FAKE, K=FAKE, V=FAKE, Out=FAKE, dO=FAKE, lse=FAKE, s=sh, idx=FAKE, ll=188, sc=0.0, \
        dQ=FAKE, dK=FAKE, dV=FAKE, ws=FAKE, nbytes=need: \
        lib.lf_sparse_attn_bwd(Q, K, V, Out, dO, lse, C.byref(s) if s is not None else None, idx, ll, sc,
                               dQ, dK, dV, ws, nbytes, None)
    for kw in (dict(Q=None), dict(K=None), dict(V=None), dict(Out=None), dict(dO=None), dict(lse=None),
               dict(s=None), dict(idx=None), dict(dQ=None), dict(dK=None), dict(dV=None)):
        assert bwd(**kw) == -1, kw
    assert bwd(ll=0) == -3 and bwd(sc=float("inf")) == -2
    assert bwd(ws=None) == -6 and bwd(nbytes=need - 1) == -6 and bwd(ws=FAKE + 16) == -5
    assert bwd(dO=FAKE + 8) == -5 and bwd(dK=FAKE + 4) == -5 and bwd(lse=FAKE + 1) == -5
    _, s2, _ = _good()
    s2.head_dim = 96
    assert lf.lf_attn_bwd_workspace_bytes(s2) == 0 and bwd(s=s2) == -2 and fwd(s=s2) == -2


def test_qk_norm_rope_argument_errors_enqueue_nothing(lib):
    def shape(**kw):
        p = lf.lf_producer_shape()
        p.heads, p.head_dim, p.tokens, p.across_heads, p.pairing, p.eps = 12, 128, 4680, 0, 0, 1e-6
        p.x_stride_tok, p.y_stride_tok, p.y_stride_head = 1536, 128, 128 * 4680
        for k, v in kw.items():
            setattr(p, k, v)
        return p
    call = lambda X=FAKE, g=FAKE, c=FAKE, s=FAKE, p=None, Y=FAKE: lib.lf_qk_norm_rope(
        X, g, c, s, C.byref(p if p is not None else shape()), Y, None)
    assert lib.lf_qk_norm_rope(FAKE, FAKE, FAKE, FAKE, None, FAKE, None) == -1
    assert call(X=None) == -1 and call(g=None) == -1 and call(c=None) == -1 and call(Y=None) == -1
    for kw in (dict(head_dim=96), dict(heads=0), dict(tokens=0), dict(across_heads=2), dict(pairing=-1),
               dict(eps=-1.0), dict(eps=float("inf")), dict(x_stride_tok=1528), dict(y_stride_tok=64)):
        assert call(p=shape(**kw)) == -2, kw
    assert call(p=shape(x_stride_tok=1540)) == -5 and call(p=shape(y_stride_head=12)) == -5
    assert call(X=FAKE + 2) == -5 and call(c=FAKE + 4) == -5


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(lf, "_lib", None)
    monkeypatch.setattr(lf, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        lf.lf_chunk_budget(1, synth.cfg_tiny().schedule)


def test_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """lf_host.cpp built for the CPU with -fsanitize=address,undefined and driven through every
    budget mode and every argument-error path by tests/host_sanitize_driver.cpp."""
    import subprocess
    from paper_2602_04789_amd import build
    exe = build.build_sanitized_host(str(tmp_path))
    # the environment is passed on as it is; a preloaded library may come before the sanitizer
    # runtime, which the link-order check would otherwise refuse
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert res.returncode == 0 and "ALL OK" in res.stdout, res.stdout[-3000:]
