// Host side of the C ABI: Chunk-Aware Growth budgets (Sec. 4.1, Eq. 5-6), argument
// validation, workspace layout.  No GPU code here.  Compiled with -ffp-contract=off so the
// binary64 expressions below round exactly as written.
#include <math.h>
#include <string.h>

#include "lf_common.h"

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// beta of Eq. 6 with alpha_i = 1/sqrt(i) and chunk weights l^q_i l^k_i d proportional to i.
double cag_beta(int n_chunks, double s_base, double s_target) {
  if (n_chunks < 2) return 0.0;
  double num = 0.0, den = 0.0;
  for (int i = 2; i <= n_chunks; ++i) {
    num += (double)i;
    den += (double)i / sqrt((double)i);
  }
  return (s_base - s_target) * num / den;
}

double keep_ratio(int i, const lf_schedule* s) {
  if (s->first_chunk_dense && i == 1) return 1.0;
  switch (s->mode) {
    case LF_SCHED_FIXED:
      return s->keep_fixed;
    case LF_SCHED_LINEAR: {
      if (s->n_chunks <= 1) return s->keep_first;
      double t = (double)(i - 1) / (double)(s->n_chunks - 1);
      return s->keep_first + (s->keep_last - s->keep_first) * t;
    }
    default: {  // LF_SCHED_CAG; Eq. 5 is stated for i > 1
      if (i == 1) return 1.0;
      double s_i = s->s_base - cag_beta(s->n_chunks, s->s_base, s->s_target) / sqrt((double)i);
      return 1.0 - s_i;
    }
  }
}

inline int ceil_count(double ratio, int total) {
  return (int)ceil(ratio * (double)total - 1e-9);
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

  const int f = s->frames_per_chunk;
  const int nb = ceil_div(s->frame_len, s->block);
  const int F_h = (chunk_idx - 1) * f;
  const int n_sink = s->n_sink < F_h ? s->n_sink : F_h;
  const int n_win = s->n_win < F_h - n_sink ? s->n_win : F_h - n_sink;
  const int m = F_h - n_sink - n_win;
  const int k_frames = s->k_frames < m ? s->k_frames : m;
  const int cur_mand = (s->current_mandatory && F_h > 0) ? 1 : 0;
  const int64_t n_tf = (int64_t)n_sink + n_win + k_frames;
  const int64_t n_cand64 = n_tf * nb + (cur_mand ? 0 : (int64_t)f * nb);
  if (n_cand64 > (int64_t)1 << 30 || (int64_t)(F_h + f) * nb > (int64_t)1 << 30)
    return LF_ERR_SCHEDULE;
  const int n_cand = (int)n_cand64;
  double rho = keep_ratio(chunk_idx, s);
  if (rho < 0.0) rho = 0.0;  // CAG with extreme parameters
  if (rho > 1.0) rho = 1.0;
  int k_blocks;
  if (s->ratio_of == LF_OF_CANDIDATES)
    k_blocks = ceil_count(rho, n_cand);
  else if (s->ratio_of == LF_OF_HISTORY)
    k_blocks = ceil_count(rho, F_h > 0 ? F_h * nb : n_cand);
  else
    k_blocks = ceil_count(rho, (F_h + f) * nb) - (cur_mand ? f * nb : 0);
  if (k_blocks > n_cand) k_blocks = n_cand;
  const int lo = n_cand < 1 ? n_cand : 1;
  if (k_blocks < lo) k_blocks = lo;

  memset(out, 0, sizeof(*out));
  out->n_hist_frames = F_h;
  out->frames_per_chunk = f;
  out->n_sink = n_sink;
  out->n_win = n_win;
  out->k_frames = k_frames;
  out->k_blocks = k_blocks;
  out->current_mandatory = cur_mand;
  out->list_len = k_blocks + (cur_mand ? f * nb : 0);
  out->keep_ratio = rho;
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
  if (o->F_h > LF_MAX_HIST_FRAMES || o->m > LF_MAX_CAND_FRAMES) return LF_ERR_BUDGET;
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
  return lf_launch_attn(Q, K, V, s, &dm, indices, list_len, scale, O, stream);
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
