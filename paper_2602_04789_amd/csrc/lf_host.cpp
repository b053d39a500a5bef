// Host side of the C ABI: Chunk-Aware Growth budgets (Sec. 4.1, Eq. 5-6), argument
// validation, workspace layout.  No GPU code here.  Compiled with -ffp-contract=off so the
// binary64 expressions below round exactly as written.
#include <math.h>
#include <string.h>

#include "lf_common.h"

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// How the history of F_h frames splits for one chunk (footnote to Eq. 7, text after Eq. 9):
// the earliest frames are the sink, the nearest ones the window (it takes what the sink
// leaves), the rest is the candidate set M, of which top-k retrieves `pick` frames.
struct HistorySplit {
  int sink, window, candidates, pick;
  int kept() const { return sink + window + pick; }
};

HistorySplit split_history(int F_h, const lf_schedule& sc) {
  HistorySplit h;
  h.sink = sc.n_sink > F_h ? F_h : sc.n_sink;
  const int rest = F_h - h.sink;
  h.window = sc.n_win > rest ? rest : sc.n_win;
  h.candidates = rest - h.window;
  h.pick = sc.k_frames > h.candidates ? h.candidates : sc.k_frames;
  return h;
}

// Fraction of blocks chunk i keeps.  Chunk-Aware Growth (Eq. 5): s_i = s_base - beta alpha_i
// with alpha_i = i^(-1/2); Eq. 6 with chunk weights proportional to i fixes
//   beta = (s_base - s_target) * W / A,  W = sum_{i=2..n} i = n(n+1)/2 - 1,
//   A = sum_{i=2..n} i^(1/2).
// Returns false when the fraction is not a ratio (outside [0, 1]).
bool keep_fraction(int i, const lf_schedule& sc, double* out) {
  double keep = 1.0;
  const bool dense = i == 1 && (sc.first_chunk_dense || sc.mode == LF_SCHED_CAG);
  if (!dense) {
    if (sc.mode == LF_SCHED_FIXED) {
      keep = sc.keep_fixed;
    } else if (sc.mode == LF_SCHED_LINEAR) {
      const double span = sc.n_chunks > 1 ? (double)(i - 1) / (double)(sc.n_chunks - 1) : 0.0;
      keep = sc.keep_first + span * (sc.keep_last - sc.keep_first);
    } else {
      const double n = (double)sc.n_chunks;
      const double W = 0.5 * n * (n + 1.0) - 1.0;
      double A = 0.0;
      for (int j = 2; j <= sc.n_chunks; ++j) A += sqrt((double)j);
      const double beta = sc.n_chunks >= 2 ? (sc.s_base - sc.s_target) * W / A : 0.0;
      keep = 1.0 - (sc.s_base - beta / sqrt((double)i));
    }
  }
  *out = keep;
  return keep >= 0.0 && keep <= 1.0;
}

// Smallest integer count that is not below ratio * total, where products within 1e-9 of an
// integer count as that integer (0.4 * 225 must give 90, not 91).
inline int64_t blocks_for(double ratio, int64_t total) {
  const double x = ratio * (double)total;
  int64_t k = (int64_t)x;
  if (x - (double)k > 1e-9) ++k;
  return k;
}

inline bool ratio_ok(double r) { return r >= 0.0 && r <= 1.0; }

}  // namespace

extern "C" int lf_chunk_budget(int32_t chunk_idx, const lf_schedule* s, lf_budget* out) {
  if (!s || !out) return LF_ERR_NULL;
  if (chunk_idx < 1 || s->n_chunks < 1 || s->frames_per_chunk < 1 || s->frame_len < 1 ||
      s->block < 1 || s->n_sink < 0 || s->n_win < 0 || s->k_frames < 0)
    return LF_ERR_SCHEDULE;
  if (s->mode < LF_SCHED_FIXED || s->mode > LF_SCHED_CAG) return LF_ERR_SCHEDULE;
  if (s->ratio_of < LF_OF_CANDIDATES || s->ratio_of > LF_OF_ALL) return LF_ERR_SCHEDULE;
  if (s->mode == LF_SCHED_FIXED && !ratio_ok(s->keep_fixed)) return LF_ERR_SCHEDULE;
  if (s->mode == LF_SCHED_LINEAR && !(ratio_ok(s->keep_first) && ratio_ok(s->keep_last)))
    return LF_ERR_SCHEDULE;
  if (s->mode == LF_SCHED_CAG &&
      !(ratio_ok(s->s_base) && ratio_ok(s->s_target) && s->s_target <= s->s_base))
    return LF_ERR_SCHEDULE;
  if ((int64_t)(chunk_idx) * s->frames_per_chunk > (int64_t)1 << 24) return LF_ERR_SCHEDULE;

  const int64_t f = s->frames_per_chunk;
  const int64_t nb = ceil_div(s->frame_len, s->block);
  const int F_h = (chunk_idx - 1) * (int)f;
  const HistorySplit hs = split_history(F_h, *s);
  // With no history the current blocks are the only candidates, whatever the flag says.
  const bool current_outside_topk = s->current_mandatory && F_h > 0;
  const int64_t current_blocks = f * nb;
  const int64_t candidates = hs.kept() * nb + (current_outside_topk ? 0 : current_blocks);
  if (candidates > (int64_t)1 << 30 || (F_h + f) * nb > (int64_t)1 << 30) return LF_ERR_SCHEDULE;

  // Sec. 4.1: s_i is a sparsity ratio; a schedule whose Eq. 5 leaves [0, 1] at this chunk is
  // rejected rather than altered.
  double keep;
  if (!keep_fraction(chunk_idx, *s, &keep)) return LF_ERR_SCHEDULE;

  // The ratio is a fraction of the candidates, of the history blocks (of the candidates when
  // there is no history), or of all KV blocks; in the last case the current blocks, when they
  // are kept outside the top-k, come off the count.
  int64_t k;
  if (s->ratio_of == LF_OF_ALL)
    k = blocks_for(keep, (F_h + f) * nb) - (current_outside_topk ? current_blocks : 0);
  else if (s->ratio_of == LF_OF_HISTORY && F_h > 0)
    k = blocks_for(keep, F_h * nb);
  else
    k = blocks_for(keep, candidates);
  if (k < 1) k = 1;                     // never attend to nothing ...
  if (k > candidates) k = candidates;   // ... nor to more than there is

  memset(out, 0, sizeof(*out));
  out->n_hist_frames = F_h;
  out->frames_per_chunk = (int32_t)f;
  out->n_sink = hs.sink;
  out->n_win = hs.window;
  out->k_frames = hs.pick;
  out->k_blocks = (int32_t)k;
  out->current_mandatory = current_outside_topk ? 1 : 0;
  out->list_len = (int32_t)(k + (current_outside_topk ? current_blocks : 0));
  out->keep_ratio = keep;
  return LF_OK;
}

static bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

int lf_derive(const lf_shape* s, const lf_budget* b, lf_dims* o) {
  if (!s || !o) return LF_ERR_NULL;
  if (s->dtype != LF_BF16) return LF_ERR_DTYPE;
  if (s->heads < 1 || s->frame_len < 1 || s->q_len < 1 || s->kv_len < 1) return LF_ERR_SHAPE;
  if (s->block != 64) return LF_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return LF_ERR_SHAPE;
  if (s->q_len % s->frame_len || s->kv_len % s->frame_len || s->kv_len < s->q_len)
    return LF_ERR_SHAPE;
  const int64_t strides[8] = {s->q_stride_tok, s->q_stride_head, s->k_stride_tok,
                              s->k_stride_head, s->v_stride_tok, s->v_stride_head,
                              s->o_stride_tok, s->o_stride_head};
  for (int i = 0; i < 8; ++i) {
    if (strides[i] < 0) return LF_ERR_SHAPE;
    if (strides[i] % 8) return LF_ERR_ALIGN;
  }
  if (s->q_stride_tok < s->head_dim || s->k_stride_tok < s->head_dim ||
      s->v_stride_tok < s->head_dim || s->o_stride_tok < s->head_dim)
    return LF_ERR_SHAPE;
  // one head's K and V must each span less than 2 GiB (32-bit buffer offsets in the kernels)
  const int64_t lim = ((int64_t)1 << 31) - 1;
  if (((int64_t)s->kv_len - 1) * s->k_stride_tok * 2 + s->head_dim * 2 > lim ||
      ((int64_t)s->kv_len - 1) * s->v_stride_tok * 2 + s->head_dim * 2 > lim)
    return LF_ERR_SHAPE;
  memset(o, 0, sizeof(*o));
  o->H = s->heads;
  o->d = s->head_dim;
  o->n = s->frame_len;
  o->f = s->q_len / s->frame_len;
  o->F = s->kv_len / s->frame_len;
  o->F_h = o->F - o->f;
  o->nb = ceil_div(s->frame_len, s->block);
  if ((int64_t)o->F * o->nb > (int64_t)1 << 30 || (int64_t)s->heads * o->F * o->nb > (int64_t)1 << 31)
    return LF_ERR_SHAPE;
  o->n_q = o->f * o->nb;
  o->n_k = o->F * o->nb;
  if (!b) return LF_OK;

  if (b->n_hist_frames != o->F_h || b->frames_per_chunk != o->f) return LF_ERR_BUDGET;
  if (b->n_sink < 0 || b->n_win < 0 || b->k_frames < 0 || b->k_blocks < 0) return LF_ERR_BUDGET;
  if ((int64_t)b->n_sink + b->n_win > o->F_h) return LF_ERR_BUDGET;
  o->m = o->F_h - b->n_sink - b->n_win;
  if (b->k_frames > o->m) return LF_ERR_BUDGET;
  if (b->current_mandatory != 0 && b->current_mandatory != 1) return LF_ERR_BUDGET;
  if (o->F_h > LF_MAX_HIST_FRAMES || o->m > LF_MAX_CAND_FRAMES || o->f > LF_MAX_CHUNK_FRAMES)
    return LF_ERR_BUDGET;
  o->n_tf = b->n_sink + b->n_win + b->k_frames;
  const int64_t n_cand = (int64_t)o->n_tf * o->nb + (b->current_mandatory ? 0 : (int64_t)o->f * o->nb);
  if (n_cand > LF_MAX_CAND_BLOCKS) return LF_ERR_BUDGET;
  o->n_cand = (int)n_cand;
  if (b->k_blocks > o->n_cand) return LF_ERR_BUDGET;
  const int want_len = b->k_blocks + (b->current_mandatory ? o->f * o->nb : 0);
  if (b->list_len != want_len || want_len < 1) return LF_ERR_BUDGET;

  size_t off = 0;
  o->off_qt = off;
  off = align_up(off + (size_t)o->H * o->n_q * o->d * sizeof(float), 256);
  o->off_kt = off;
  off = align_up(off + (size_t)o->H * o->n_k * o->d * sizeof(float), 256);
  o->off_kh = off;
  off = align_up(off + (size_t)o->H * (o->m > 0 ? o->m : 1) * o->d * sizeof(float), 256);
  o->ws_bytes = off;
  return LF_OK;
}

extern "C" size_t lf_workspace_bytes(const lf_shape* s, const lf_budget* b) {
  lf_dims dm;
  if (!b || lf_derive(s, b, &dm) != LF_OK) return 0;
  return dm.ws_bytes;
}

extern "C" int lf_workspace_layout(const lf_shape* s, const lf_budget* b, size_t off[3]) {
  if (!b || !off) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, b, &dm);
  if (rc != LF_OK) return rc;
  off[0] = dm.off_qt;
  off[1] = dm.off_kt;
  off[2] = dm.off_kh;
  return LF_OK;
}

extern "C" int lf_select_mask(const void* Q, const void* K, const lf_shape* s, const lf_budget* b,
                              int32_t* indices, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!Q || !K || !s || !b || !indices) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, b, &dm);
  if (rc != LF_OK) return rc;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(indices, 4)) return LF_ERR_ALIGN;
  if (!workspace || workspace_bytes < dm.ws_bytes) return LF_ERR_WORKSPACE;
  if (misaligned(workspace, 256)) return LF_ERR_ALIGN;
  return lf_launch_select(Q, K, s, b, &dm, indices, workspace, stream);
}

extern "C" int lf_init(void) {
  void* p;
  return lf_static_scratch(&p);
}

extern "C" size_t lf_static_scratch_bytes(void) { return LF_STATIC_SCRATCH_BYTES; }

extern "C" int lf_select_mask_static(const void* Q, const void* K, const lf_shape* s,
                                     const lf_budget* b, int32_t* indices, void* stream) {
  if (!Q || !K || !s || !b || !indices) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, b, &dm);
  if (rc != LF_OK) return rc;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(indices, 4)) return LF_ERR_ALIGN;
  if (dm.ws_bytes > LF_STATIC_SCRATCH_BYTES) return LF_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = lf_static_scratch(&ws);
  if (rc != LF_OK) return rc;
  return lf_launch_select(Q, K, s, b, &dm, indices, ws, stream);
}

// Bytes of the pooled-key cache; 0 when the sizes are unusable.
static size_t kcache_bytes(const lf_dims& dm, int32_t max_frames) {
  if (max_frames < 1 || max_frames > LF_MAX_HIST_FRAMES + 64) return 0;
  const size_t rows = (size_t)max_frames * dm.nb + (size_t)max_frames;
  return align_up((size_t)dm.H * rows * dm.d * sizeof(float), 256);
}

extern "C" size_t lf_kcache_bytes(const lf_shape* s, int32_t max_frames) {
  if (!s) return 0;
  // only heads, head_dim, frame_len and block matter here: check them on a one-frame shape
  lf_shape one = *s;
  one.q_len = one.kv_len = s->frame_len;
  one.q_stride_tok = one.k_stride_tok = one.v_stride_tok = one.o_stride_tok = 128;
  one.q_stride_head = one.k_stride_head = one.v_stride_head = one.o_stride_head = 0;
  lf_dims dm;
  if (lf_derive(&one, nullptr, &dm) != LF_OK) return 0;
  return kcache_bytes(dm, max_frames);
}

extern "C" int lf_kcache_update(const void* K, const lf_shape* s, int32_t frame_begin,
                                int32_t frame_end, int32_t max_frames, void* kcache,
                                size_t kcache_bytes_given, void* stream) {
  if (!K || !s) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, nullptr, &dm);
  if (rc != LF_OK) return rc;
  if (frame_begin < 0 || frame_end < frame_begin || frame_end > dm.F || dm.F > max_frames)
    return LF_ERR_SHAPE;
  const size_t need = kcache_bytes(dm, max_frames);
  if (need == 0) return LF_ERR_SHAPE;
  if (!kcache || kcache_bytes_given < need) return LF_ERR_WORKSPACE;
  if (misaligned(K, 16) || misaligned(kcache, 256)) return LF_ERR_ALIGN;
  if (frame_end == frame_begin) return LF_OK;
  return lf_launch_kcache_update(K, s, &dm, frame_begin, frame_end, max_frames, kcache, stream);
}

extern "C" int lf_select_mask_cached(const void* Q, const void* Kcache, void* kcache,
                                     size_t kcache_bytes_given, int32_t max_frames,
                                     const lf_shape* s, const lf_budget* b,
                                     int32_t* indices, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  if (!Q || !s || !b || !indices) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, b, &dm);
  if (rc != LF_OK) return rc;
  if (dm.F > max_frames) return LF_ERR_SHAPE;
  const size_t need = kcache_bytes(dm, max_frames);
  if (need == 0) return LF_ERR_SHAPE;
  if (!kcache || kcache_bytes_given < need) return LF_ERR_WORKSPACE;
  if (!workspace || workspace_bytes < (size_t)dm.H * dm.n_q * dm.d * sizeof(float))
    return LF_ERR_WORKSPACE;
  if (misaligned(Q, 16) || misaligned(Kcache, 16) || misaligned(indices, 4) ||
      misaligned(kcache, 256) || misaligned(workspace, 256))
    return LF_ERR_ALIGN;
  return lf_launch_select_cached(Q, Kcache, kcache, max_frames, s, b, &dm, indices, workspace, stream);
}

extern "C" int lf_sparse_attn(const void* Q, const void* K, const void* V, const lf_shape* s,
                              const int32_t* indices, int32_t list_len, float softmax_scale,
                              void* O, void* stream) {
  if (!Q || !K || !V || !s || !indices || !O) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, nullptr, &dm);
  if (rc != LF_OK) return rc;
  if (list_len < 1) return LF_ERR_BUDGET;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return LF_ERR_SHAPE;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(O, 16) ||
      misaligned(indices, 4))
    return LF_ERR_ALIGN;
  float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)dm.d);
  return lf_launch_attn(Q, K, V, s, &dm, indices, list_len, list_len, scale, O, nullptr, nullptr, nullptr,
                        stream);
}

// Scratch of lf_sparse_attn_split: O state float32 [H][q_len][d], then (m, l) float32 [H][q_len][2].
static size_t attn_state_bytes(const lf_dims& dm, size_t* off_ml) {
  const size_t rows = (size_t)dm.H * dm.f * dm.n;
  const size_t o = align_up(rows * dm.d * sizeof(float), 256);
  if (off_ml) *off_ml = o;
  return o + align_up(rows * 2 * sizeof(float), 256);
}

extern "C" size_t lf_attn_workspace_bytes(const lf_shape* s) {
  lf_dims dm;
  if (lf_derive(s, nullptr, &dm) != LF_OK) return 0;
  return attn_state_bytes(dm, nullptr);
}

extern "C" int lf_sparse_attn_split(const void* Q, const void* K, const void* V, const lf_shape* s,
                                    const lf_budget* b, const int32_t* indices, float softmax_scale,
                                    void* O, void* workspace, size_t workspace_bytes, void* stream) {
  if (!Q || !K || !V || !s || !b || !indices || !O) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, b, &dm);
  if (rc != LF_OK) return rc;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return LF_ERR_SHAPE;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(O, 16) ||
      misaligned(indices, 4))
    return LF_ERR_ALIGN;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)dm.d);
  if (!b->current_mandatory)   // nothing is common to all query blocks: one list-driven pass
    return lf_launch_attn(Q, K, V, s, &dm, indices, b->list_len, b->list_len, scale, O, nullptr,
                          nullptr, nullptr, stream);
  size_t off_ml = 0;
  const size_t need = attn_state_bytes(dm, &off_ml);
  if (!workspace || workspace_bytes < need) return LF_ERR_WORKSPACE;
  if (misaligned(workspace, 256)) return LF_ERR_ALIGN;
  float* state_o = (float*)workspace;
  float* state_ml = (float*)((char*)workspace + off_ml);
  rc = lf_launch_attn_dense(Q, K, V, s, &dm, dm.F_h * dm.n, dm.F * dm.n, scale, state_o, state_ml, stream);
  if (rc != LF_OK) return rc;
  return lf_launch_attn(Q, K, V, s, &dm, indices, b->k_blocks, b->list_len, scale, O, state_o,
                        state_ml, nullptr, stream);
}

extern "C" int lf_sparse_attn_fwd(const void* Q, const void* K, const void* V, const lf_shape* s,
                                  const int32_t* indices, int32_t list_len, float softmax_scale,
                                  void* O, float* lse2, void* stream) {
  if (!Q || !K || !V || !s || !indices || !O || !lse2) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, nullptr, &dm);
  if (rc != LF_OK) return rc;
  if (list_len < 1) return LF_ERR_BUDGET;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return LF_ERR_SHAPE;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(O, 16) ||
      misaligned(indices, 4) || misaligned(lse2, 4))
    return LF_ERR_ALIGN;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)dm.d);
  return lf_launch_attn(Q, K, V, s, &dm, indices, list_len, list_len, scale, O, nullptr, nullptr, lse2,
                        stream);
}

// Scratch of lf_sparse_attn_bwd: (lse2, delta) float32 [H][q_len][2], the transposed lists int32
// [H][n_k][n_q], their lengths int32 [H][n_k] and the launch order int32 [H][n_k].
static size_t attn_bwd_bytes(const lf_dims& dm, size_t* off_tlist, size_t* off_tcnt, size_t* off_order) {
  const size_t rows = (size_t)dm.H * dm.f * dm.n;
  const size_t o1 = align_up(rows * 2 * sizeof(float), 256);
  const size_t o2 = o1 + align_up((size_t)dm.H * dm.n_k * dm.n_q * sizeof(int32_t), 256);
  const size_t o3 = o2 + align_up((size_t)dm.H * dm.n_k * sizeof(int32_t), 256);
  if (off_tlist) *off_tlist = o1;
  if (off_tcnt) *off_tcnt = o2;
  if (off_order) *off_order = o3;
  return o3 + align_up((size_t)dm.H * dm.n_k * sizeof(int32_t), 256);
}

extern "C" size_t lf_attn_bwd_workspace_bytes(const lf_shape* s) {
  lf_dims dm;
  if (lf_derive(s, nullptr, &dm) != LF_OK) return 0;
  return attn_bwd_bytes(dm, nullptr, nullptr, nullptr);
}

extern "C" int lf_sparse_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                                  const void* dO, const float* lse2, const lf_shape* s,
                                  const int32_t* indices, int32_t list_len, float softmax_scale,
                                  void* dQ, void* dK, void* dV, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  if (!Q || !K || !V || !O || !dO || !lse2 || !s || !indices || !dQ || !dK || !dV) return LF_ERR_NULL;
  lf_dims dm;
  int rc = lf_derive(s, nullptr, &dm);
  if (rc != LF_OK) return rc;
  if (list_len < 1) return LF_ERR_BUDGET;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return LF_ERR_SHAPE;
  size_t off_tlist = 0, off_tcnt = 0, off_order = 0;
  const size_t need = attn_bwd_bytes(dm, &off_tlist, &off_tcnt, &off_order);
  if (!workspace || workspace_bytes < need) return LF_ERR_WORKSPACE;
  if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(O, 16) ||
      misaligned(dO, 16) || misaligned(dQ, 16) || misaligned(dK, 16) || misaligned(dV, 16) ||
      misaligned(indices, 4) || misaligned(lse2, 4) || misaligned(workspace, 256))
    return LF_ERR_ALIGN;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)dm.d);
  return lf_launch_attn_bwd(Q, K, V, O, dO, lse2, s, &dm, indices, list_len, scale, dQ, dK, dV,
                            (float*)workspace, (int32_t*)((char*)workspace + off_tlist),
                            (int32_t*)((char*)workspace + off_tcnt),
                            (int32_t*)((char*)workspace + off_order), stream);
}

extern "C" int lf_qk_norm_rope(const void* X, const float* g, const float* cos_table,
                               const float* sin_table, const lf_producer_shape* p, void* Y,
                               void* stream) {
  if (!X || !g || !cos_table || !sin_table || !p || !Y) return LF_ERR_NULL;
  if (p->head_dim != 64 && p->head_dim != 128) return LF_ERR_SHAPE;
  if (p->heads < 1 || p->tokens < 1 || p->heads > (1 << 16)) return LF_ERR_SHAPE;
  if ((p->across_heads != 0 && p->across_heads != 1) || (p->pairing != 0 && p->pairing != 1))
    return LF_ERR_SHAPE;
  if (!(p->eps >= 0.0f) || isinf(p->eps)) return LF_ERR_SHAPE;
  if (p->x_stride_tok < (int64_t)p->heads * p->head_dim || p->y_stride_tok < p->head_dim ||
      p->y_stride_head < 0)
    return LF_ERR_SHAPE;
  if (p->x_stride_tok % 8 || p->y_stride_tok % 8 || p->y_stride_head % 8) return LF_ERR_ALIGN;
  if (misaligned(X, 16) || misaligned(Y, 16) || misaligned(g, 16) || misaligned(cos_table, 16) ||
      misaligned(sin_table, 16))
    return LF_ERR_ALIGN;
  return lf_launch_qk_norm_rope(X, g, cos_table, sin_table, p, Y, stream);
}

extern "C" const char* lf_strerror(int status) {
  switch (status) {
    case LF_OK: return "ok";
    case LF_ERR_NULL: return "a required pointer is NULL";
    case LF_ERR_SHAPE: return "shape inconsistent or unsupported";
    case LF_ERR_BUDGET: return "budget inconsistent with the shape or beyond kernel limits";
    case LF_ERR_DTYPE: return "unsupported dtype (bfloat16 only)";
    case LF_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
    case LF_ERR_WORKSPACE: return "workspace missing or too small";
    case LF_ERR_HIP: return "HIP kernel launch failed";
    case LF_ERR_SCHEDULE: return "schedule fields out of range";
    default: return "unknown lf_status";
  }
}

extern "C" int lf_version(void) { return 200; }
