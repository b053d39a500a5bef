// Host-only driver for the sanitizer build of the C ABI's host side (argument validation,
// Chunk-Aware Growth budgets, workspace sizes).  lf_host.cpp is compiled for the CPU with
// -fsanitize=address,undefined together with this file, which stands in for the kernel
// launchers: every launcher counts its calls, so the driver can also check that a rejected call
// enqueues nothing.  Pointers handed to the entry points are never dereferenced on these paths.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "lf_common.h"

static int g_launches = 0;
int lf_launch_select(const void*, const void*, const lf_shape*, const lf_budget*, const lf_dims*, int32_t*,
                     void*, void*) { ++g_launches; return LF_OK; }
int lf_launch_kcache_update(const void*, const lf_shape*, const lf_dims*, int, int, int, void*, void*) {
  ++g_launches; return LF_OK;
}
int lf_launch_select_cached(const void*, const void*, void*, int, const lf_shape*, const lf_budget*,
                            const lf_dims*, int32_t*, void*, void*) { ++g_launches; return LF_OK; }
int lf_launch_attn(const void*, const void*, const void*, const lf_shape*, const lf_dims*, const int32_t*,
                   int32_t, int32_t, float, void*, const float*, const float*, float*, void*) {
  ++g_launches; return LF_OK;
}
int lf_launch_attn_bwd(const void*, const void*, const void*, const void*, const void*, const float*,
                       const lf_shape*, const lf_dims*, const int32_t*, int32_t, float, void*, void*, void*,
                       float*, int32_t*, int32_t*, int32_t*, void*) { ++g_launches; return LF_OK; }
int lf_launch_attn_dense(const void*, const void*, const void*, const lf_shape*, const lf_dims*, int, int,
                         float, float*, float*, void*) { ++g_launches; return LF_OK; }
int lf_launch_qk_norm_rope(const void*, const float*, const float*, const float*, const lf_producer_shape*,
                           void*, void*) { ++g_launches; return LF_OK; }
int lf_static_scratch(void** p) { *p = (void*)0x20000; return LF_OK; }

static int g_fail = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++g_fail; } } while (0)

static lf_schedule schedule() {
  lf_schedule s;
  memset(&s, 0, sizeof(s));
  s.mode = LF_SCHED_FIXED; s.n_chunks = 7; s.frames_per_chunk = 3; s.frame_len = 1560; s.block = 64;
  s.n_sink = 1; s.n_win = 2; s.k_frames = 3; s.ratio_of = LF_OF_HISTORY; s.current_mandatory = 1;
  s.keep_fixed = 0.25; s.keep_first = 0.8; s.keep_last = 0.25; s.s_base = 0.98; s.s_target = 0.88;
  return s;
}

static lf_shape shape(int frames) {
  lf_shape h;
  memset(&h, 0, sizeof(h));
  h.heads = 12; h.head_dim = 128; h.frame_len = 1560; h.block = 64; h.q_len = 3 * 1560;
  h.kv_len = frames * 1560; h.dtype = LF_BF16;
  h.q_stride_tok = h.k_stride_tok = h.v_stride_tok = h.o_stride_tok = 128;
  h.q_stride_head = h.o_stride_head = 128LL * h.q_len;
  h.k_stride_head = h.v_stride_head = 128LL * h.kv_len;
  return h;
}

int main() {
  void* const P = (void*)0x10000;   // non-NULL, 256-byte aligned, never dereferenced
  lf_budget b;
  lf_schedule s = schedule();

  // budgets: every mode / denominator / chunk, including schedules that must be rejected
  for (int mode = 0; mode <= 2; ++mode)
    for (int of = 0; of <= 2; ++of)
      for (int cm = 0; cm <= 1; ++cm)
        for (int chunk = 1; chunk <= 21; ++chunk) {
          lf_schedule t = s;
          t.mode = mode; t.ratio_of = of; t.current_mandatory = cm; t.n_chunks = 21;
          const int rc = lf_chunk_budget(chunk, &t, &b);
          EXPECT(rc == LF_OK);
          EXPECT(b.list_len >= 1 && b.k_blocks >= 0 && b.keep_ratio >= 0.0 && b.keep_ratio <= 1.0);
        }
  EXPECT(lf_chunk_budget(7, &s, &b) == LF_OK && b.k_blocks == 113 && b.list_len == 188);
  EXPECT(lf_chunk_budget(0, &s, &b) == LF_ERR_SCHEDULE);
  EXPECT(lf_chunk_budget(1, nullptr, &b) == LF_ERR_NULL && lf_chunk_budget(1, &s, nullptr) == LF_ERR_NULL);
  { lf_schedule t = s; t.mode = LF_SCHED_CAG; t.s_base = 0.5; t.s_target = 0.1; t.ratio_of = LF_OF_ALL;
    EXPECT(lf_chunk_budget(2, &t, &b) == LF_ERR_SCHEDULE); EXPECT(lf_chunk_budget(7, &t, &b) == LF_OK); }
  { lf_schedule t = s; t.frames_per_chunk = 1 << 20; EXPECT(lf_chunk_budget(1 << 10, &t, &b) == LF_ERR_SCHEDULE); }
  { lf_schedule t = s; t.keep_fixed = NAN; EXPECT(lf_chunk_budget(2, &t, &b) == LF_ERR_SCHEDULE); }

  // selection, attention, caches: accepted once, then every rejection, which must launch nothing
  lf_shape h = shape(21);
  EXPECT(lf_chunk_budget(7, &s, &b) == LF_OK);
  const size_t ws = lf_workspace_bytes(&h, &b), aws = lf_attn_workspace_bytes(&h), kcb = lf_kcache_bytes(&h, 21);
  EXPECT(ws > 0 && aws > 0 && kcb > 0);
  size_t off[3];
  EXPECT(lf_workspace_layout(&h, &b, off) == LF_OK && off[0] < off[1] && off[1] < off[2] && off[2] < ws);
  EXPECT(lf_select_mask(P, P, &h, &b, (int32_t*)P, P, ws, nullptr) == LF_OK);
  EXPECT(lf_select_mask_static(P, P, &h, &b, (int32_t*)P, nullptr) == LF_OK);
  EXPECT(lf_sparse_attn(P, P, P, &h, (const int32_t*)P, 188, 0.0f, P, nullptr) == LF_OK);
  EXPECT(lf_sparse_attn_split(P, P, P, &h, &b, (const int32_t*)P, 0.0f, P, P, aws, nullptr) == LF_OK);
  EXPECT(lf_kcache_update(P, &h, 0, 21, 21, P, kcb, nullptr) == LF_OK);
  EXPECT(lf_select_mask_cached(P, P, P, kcb, 21, &h, &b, (int32_t*)P, P, ws, nullptr) == LF_OK);
  const size_t bws = lf_attn_bwd_workspace_bytes(&h);
  EXPECT(bws > 0);
  EXPECT(lf_sparse_attn_fwd(P, P, P, &h, (const int32_t*)P, 188, 0.0f, P, (float*)P, nullptr) == LF_OK);
  EXPECT(lf_sparse_attn_bwd(P, P, P, P, P, (const float*)P, &h, (const int32_t*)P, 188, 0.0f, P, P, P, P, bws,
                            nullptr) == LF_OK);
  const int accepted = g_launches;
  EXPECT(accepted == 9);   // the split call launches two kernels; the backward stub counts once

  EXPECT(lf_select_mask(nullptr, P, &h, &b, (int32_t*)P, P, ws, nullptr) == LF_ERR_NULL);
  EXPECT(lf_select_mask(P, P, &h, &b, (int32_t*)P, P, ws - 1, nullptr) == LF_ERR_WORKSPACE);
  EXPECT(lf_select_mask(P, P, &h, &b, (int32_t*)P, (char*)P + 16, ws, nullptr) == LF_ERR_ALIGN);
  EXPECT(lf_sparse_attn(P, P, P, &h, (const int32_t*)P, 0, 0.0f, P, nullptr) == LF_ERR_BUDGET);
  EXPECT(lf_sparse_attn(P, P, P, &h, (const int32_t*)P, 188, -1.0f, P, nullptr) == LF_ERR_SHAPE);
  EXPECT(lf_sparse_attn_split(P, P, P, &h, &b, (const int32_t*)P, 0.0f, P, P, aws - 1, nullptr) == LF_ERR_WORKSPACE);
  EXPECT(lf_sparse_attn_fwd(P, P, P, &h, (const int32_t*)P, 188, 0.0f, P, nullptr, nullptr) == LF_ERR_NULL);
  EXPECT(lf_sparse_attn_bwd(P, P, P, P, P, (const float*)P, &h, (const int32_t*)P, 188, 0.0f, P, P, P, P, bws - 1,
                            nullptr) == LF_ERR_WORKSPACE);
  EXPECT(lf_sparse_attn_bwd(P, P, P, P, nullptr, (const float*)P, &h, (const int32_t*)P, 188, 0.0f, P, P, P, P,
                            bws, nullptr) == LF_ERR_NULL);
  EXPECT(lf_kcache_update(P, &h, 5, 4, 21, P, kcb, nullptr) == LF_ERR_SHAPE);
  EXPECT(lf_kcache_update(P, &h, 0, 21, 21, P, kcb - 1, nullptr) == LF_ERR_WORKSPACE);
  EXPECT(lf_select_mask_cached(P, P, P, kcb, 20, &h, &b, (int32_t*)P, P, ws, nullptr) == LF_ERR_SHAPE);
  for (int field = 0; field < 9; ++field) {
    lf_shape t = h;
    int want = LF_ERR_SHAPE;
    switch (field) {
      case 0: t.block = 32; break;
      case 1: t.head_dim = 96; break;
      case 2: t.dtype = 1; want = LF_ERR_DTYPE; break;
      case 3: t.q_len += 1; break;
      case 4: t.kv_len = t.frame_len; break;
      case 5: t.heads = 0; break;
      case 6: t.k_stride_tok = 129; want = LF_ERR_ALIGN; break;
      case 7: t.k_stride_tok = 64; break;
      case 8: t.v_stride_tok = (1LL << 40); break;   // a head of V would span more than 2 GiB
    }
    EXPECT(lf_select_mask(P, P, &t, &b, (int32_t*)P, P, ws, nullptr) == want);
    EXPECT(lf_sparse_attn(P, P, P, &t, (const int32_t*)P, 188, 0.0f, P, nullptr) == want);
    EXPECT(lf_workspace_bytes(&t, &b) == 0);
  }
  for (int field = 0; field < 7; ++field) {
    lf_budget t = b;
    switch (field) {
      case 0: t.k_blocks = 151; break;
      case 1: t.k_blocks = -1; break;
      case 2: t.k_frames = 16; break;
      case 3: t.n_sink = 17; break;
      case 4: t.list_len = 187; break;
      case 5: t.n_hist_frames = 17; break;
      case 6: t.current_mandatory = 2; break;
    }
    EXPECT(lf_select_mask(P, P, &h, &t, (int32_t*)P, P, ws, nullptr) == LF_ERR_BUDGET);
    EXPECT(lf_sparse_attn_split(P, P, P, &h, &t, (const int32_t*)P, 0.0f, P, P, aws, nullptr) == LF_ERR_BUDGET);
  }
  { lf_shape big = shape(21); big.heads = 64; big.q_stride_head *= 1; lf_budget bb = b;
    EXPECT(lf_workspace_bytes(&big, &bb) > lf_static_scratch_bytes());
    EXPECT(lf_select_mask_static(P, P, &big, &bb, (int32_t*)P, nullptr) == LF_ERR_WORKSPACE); }
  { lf_producer_shape p; memset(&p, 0, sizeof(p));
    p.heads = 12; p.head_dim = 128; p.tokens = 4680; p.eps = 1e-6f; p.x_stride_tok = 1536; p.y_stride_tok = 128;
    p.y_stride_head = 128LL * 4680;
    EXPECT(lf_qk_norm_rope(P, (const float*)P, (const float*)P, (const float*)P, &p, P, nullptr) == LF_OK);
    --g_launches;   // the one accepted call
    p.head_dim = 96; EXPECT(lf_qk_norm_rope(P, (const float*)P, (const float*)P, (const float*)P, &p, P, nullptr) == LF_ERR_SHAPE);
    p.head_dim = 128; p.eps = NAN; EXPECT(lf_qk_norm_rope(P, (const float*)P, (const float*)P, (const float*)P, &p, P, nullptr) == LF_ERR_SHAPE); }
  EXPECT(g_launches == accepted);   // none of the rejected calls reached a launcher
  for (int st = -9; st <= 1; ++st) EXPECT(lf_strerror(st) != nullptr && strlen(lf_strerror(st)) > 0);
  EXPECT(lf_version() >= 100);

  if (g_fail) { printf("%d check(s) failed\n", g_fail); return 1; }
  printf("ALL OK\n");
  return 0;
}
