// Mask selection kernels for gfx950 (Sec. 4.2, Eq. 7 - Eq. 12).
//
//   lf_pool_kernel        block mean pooling of Q and K (Eq. 7, blockwise): the one pass
//                         over the bf16 inputs, HBM-bound.
//   lf_frame_mean_kernel  frame means of the candidate frames (Eq. 7, framewise).
//   lf_select_kernel      per (head, query block): frame scores (Eq. 8), frame top-k
//                         (Eq. 9), block scores (Eq. 10), block top-k by a bitonic sort in
//                         LDS (Eq. 11), ascending index list (Eq. 12).
//
// Arithmetic contract (see lf.h): block sums in binary64 (exact for in-range bf16 inputs,
// so the reduction tree is free), means rounded to float32; scores are binary64 sums over
// the head dimension in ascending order, one thread per score, rounded to float32.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "lf_common.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

struct PoolArgs {
  const uint16_t* Q;
  const uint16_t* K;
  float* qt;
  float* kt;
  int64_t q_stride_tok, q_stride_head, k_stride_tok, k_stride_head;
  int n, nb, n_q, n_k;
};

// One workgroup per block of <= 64 tokens.  Thread t owns 8 consecutive channels
// (one 16-byte load per token) of every (256/CH)-th token.
template <int D>
__global__ __launch_bounds__(kThreads) void lf_pool_kernel(PoolArgs a) {
  constexpr int CH = D / 8;          // 16-byte chunks per token row
  constexpr int RG = kThreads / CH;  // token rows in flight per pass
  __shared__ double red[RG][D];

  const int per_head = a.n_q + a.n_k;
  const int h = blockIdx.x / per_head;
  const int u = blockIdx.x % per_head;
  const bool is_q = u < a.n_q;
  const int c = is_q ? u : u - a.n_q;
  const int tau = c / a.nb, j = c % a.nb;
  const int tok0 = tau * a.n + j * 64;
  const int cnt = min(64, a.n - j * 64);
  const uint16_t* src = is_q ? a.Q + (int64_t)h * a.q_stride_head
                             : a.K + (int64_t)h * a.k_stride_head;
  const int64_t stride = is_q ? a.q_stride_tok : a.k_stride_tok;
  const int ch = threadIdx.x % CH, rg = threadIdx.x / CH;

  double acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0;
#pragma unroll
  for (int row = rg; row < 64; row += RG) {
    if (row < cnt) {
      const uint4 v = *reinterpret_cast<const uint4*>(src + (int64_t)(tok0 + row) * stride + ch * 8);
      acc[0] += (double)bf16lo(v.x);
      acc[1] += (double)bf16hi(v.x);
      acc[2] += (double)bf16lo(v.y);
      acc[3] += (double)bf16hi(v.y);
      acc[4] += (double)bf16lo(v.z);
      acc[5] += (double)bf16hi(v.z);
      acc[6] += (double)bf16lo(v.w);
      acc[7] += (double)bf16hi(v.w);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[rg][ch * 8 + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < D) {
    double s = 0.0;
#pragma unroll
    for (int g = 0; g < RG; ++g) s += red[g][threadIdx.x];
    float* dst = is_q ? a.qt + ((int64_t)h * a.n_q + c) * D : a.kt + ((int64_t)h * a.n_k + c) * D;
    dst[threadIdx.x] = (float)(s / (double)cnt);
  }
}

// k_hat[h][a][:] for candidate frame tau = n_sink + a: binary64 sum of the frame's nb block
// means in ascending block order, / nb, rounded to float32.
__global__ void lf_frame_mean_kernel(const float* __restrict__ kt, float* __restrict__ kh,
                                     int d, int nb, int n_k, int m, int n_sink) {
  const int h = blockIdx.x / m, a = blockIdx.x % m;
  const int tau = n_sink + a;
  const float* src = kt + ((int64_t)h * n_k + (int64_t)tau * nb) * d;
  for (int t = threadIdx.x; t < d; t += blockDim.x) {
    double s = 0.0;
    for (int j = 0; j < nb; ++j) s += (double)src[(int64_t)j * d + t];
    kh[((int64_t)h * m + a) * d + t] = (float)(s / (double)nb);
  }
}

struct SelectArgs {
  const float* qt;
  const float* kt;
  const float* kh;
  int32_t* indices;
  int d, nb, n_q, n_k, F_h, f, m;
  int n_sink, n_win, k_frames, k_blocks, current_mandatory, list_len;
  int n_cand, n_cand_pow2;
};

// <q, k> over the head dimension, ascending, binary64 accumulate (products are exact).
template <int D>
__device__ __forceinline__ float dot_seq(const double* __restrict__ qd, const float* __restrict__ k) {
  double acc = 0.0;
#pragma unroll 8
  for (int t = 0; t < D; t += 4) {
    const float4 kv = *reinterpret_cast<const float4*>(k + t);
    acc += qd[t + 0] * (double)kv.x;
    acc += qd[t + 1] * (double)kv.y;
    acc += qd[t + 2] * (double)kv.z;
    acc += qd[t + 3] * (double)kv.w;
  }
  return (float)acc;
}

// a ranks before b: larger score first, equal scores by lower position.
__device__ __forceinline__ bool ranks_before(float sa, int ia, float sb, int ib) {
  return sa > sb || (sa == sb && ia < ib);
}

// Ascending compaction of the set positions of flag[0..count) by one wavefront.
// emit(pos, i) is called for the pos-th set flag at position i.
template <typename Emit>
__device__ __forceinline__ void wave_compact(const unsigned char* flag, int count, Emit emit) {
  const int lane = threadIdx.x & 63;
  int base_out = 0;
  for (int base = 0; base < count; base += 64) {
    const int i = base + lane;
    const bool on = i < count && flag[i];
    const unsigned long long mask = __ballot(on);
    if (on) emit(base_out + __popcll(mask & ((1ull << lane) - 1ull)), i);
    base_out += __popcll(mask);
  }
}

template <int D>
__global__ __launch_bounds__(kThreads) void lf_select_kernel(SelectArgs a) {
  __shared__ double qd[D];
  __shared__ float fscore[LF_MAX_CAND_FRAMES];
  __shared__ unsigned char fflag[LF_MAX_HIST_FRAMES];
  __shared__ int flist[LF_MAX_CAND_BLOCKS];
  __shared__ float skey[LF_MAX_CAND_BLOCKS];
  __shared__ int spos[LF_MAX_CAND_BLOCKS];
  __shared__ unsigned char sel[LF_MAX_CAND_BLOCKS];

  const int tid = threadIdx.x;
  const int h = blockIdx.x / a.n_q, r = blockIdx.x % a.n_q;
  const float* qrow = a.qt + ((int64_t)h * a.n_q + r) * D;
  if (tid < D) qd[tid] = (double)qrow[tid];
  __syncthreads();

  // Eq. 8: frame-level scores against the candidate frames M = [n_sink, F_h - n_win).
  const bool retrieve = a.k_frames < a.m;
  if (retrieve) {
    for (int c = tid; c < a.m; c += kThreads)
      fscore[c] = dot_seq<D>(qd, a.kh + ((int64_t)h * a.m + c) * D);
  }
  __syncthreads();

  // Eq. 9: T_r = top-k frames U sink U window (U current, appended below).
  for (int t = tid; t < a.F_h; t += kThreads) {
    bool on = true;
    if (t >= a.n_sink && t < a.F_h - a.n_win && retrieve) {
      const int c = t - a.n_sink;
      const float sc = fscore[c];
      int rank = 0;
      for (int o = 0; o < a.m; ++o) rank += ranks_before(fscore[o], o, sc, c) ? 1 : 0;
      on = rank < a.k_frames;
    }
    fflag[t] = on ? 1 : 0;
  }
  __syncthreads();
  if (tid < 64) wave_compact(fflag, a.F_h, [&](int pos, int i) { flist[pos] = i; });
  const int n_tf = a.n_sink + a.n_win + a.k_frames;
  if (!a.current_mandatory)
    for (int t = tid; t < a.f; t += kThreads) flist[n_tf + t] = a.F_h + t;
  __syncthreads();

  // Eq. 10: block-level scores over B_r, candidates in ascending block id.
  for (int i = tid; i < a.n_cand_pow2; i += kThreads) {
    float sc = -INFINITY;
    int pos = 0x7fffffff;
    if (i < a.n_cand) {
      const int c = flist[i / a.nb] * a.nb + i % a.nb;
      sc = dot_seq<D>(qd, a.kt + ((int64_t)h * a.n_k + c) * D);
      pos = i;
    }
    skey[i] = sc;
    spos[i] = pos;
    if (i < a.n_cand) sel[i] = 0;
  }
  __syncthreads();

  // Eq. 11: top-k blocks.  Bitonic sort of (score, position) so that ranks_before holds
  // along the array; the first k_blocks entries are J_r.
  if (a.k_blocks < a.n_cand) {
    for (int k = 2; k <= a.n_cand_pow2; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int i = tid; i < a.n_cand_pow2; i += kThreads) {
          const int p = i ^ j;
          if (p > i) {
            const float s0 = skey[i], s1 = skey[p];
            const int p0 = spos[i], p1 = spos[p];
            const bool first_half = (i & k) == 0;
            const bool swap = first_half ? ranks_before(s1, p1, s0, p0) : ranks_before(s0, p0, s1, p1);
            if (swap) {
              skey[i] = s1; skey[p] = s0;
              spos[i] = p1; spos[p] = p0;
            }
          }
        }
        __syncthreads();
      }
    }
    for (int i = tid; i < a.k_blocks; i += kThreads) sel[spos[i]] = 1;
  } else {
    for (int i = tid; i < a.n_cand; i += kThreads) sel[i] = 1;
  }
  __syncthreads();

  // Eq. 12 as a sorted list: kept candidates in ascending id, then the mandatory current blocks.
  int32_t* out = a.indices + ((int64_t)h * a.n_q + r) * a.list_len;
  if (tid < 64)
    wave_compact(sel, a.n_cand, [&](int pos, int i) { out[pos] = flist[i / a.nb] * a.nb + i % a.nb; });
  if (a.current_mandatory)
    for (int i = tid; i < a.f * a.nb; i += kThreads) out[a.k_blocks + i] = a.F_h * a.nb + i;
}

}  // namespace

int lf_launch_select(const void* Q, const void* K, const lf_shape* s, const lf_budget* b,
                     const lf_dims* dm, int32_t* indices, void* workspace, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* qt = (float*)(ws + dm->off_qt);
  float* kt = (float*)(ws + dm->off_kt);
  float* kh = (float*)(ws + dm->off_kh);

  PoolArgs pa;
  pa.Q = (const uint16_t*)Q;
  pa.K = (const uint16_t*)K;
  pa.qt = qt;
  pa.kt = kt;
  pa.q_stride_tok = s->q_stride_tok;
  pa.q_stride_head = s->q_stride_head;
  pa.k_stride_tok = s->k_stride_tok;
  pa.k_stride_head = s->k_stride_head;
  pa.n = dm->n;
  pa.nb = dm->nb;
  pa.n_q = dm->n_q;
  pa.n_k = dm->n_k;
  const unsigned pool_grid = (unsigned)(dm->H * (dm->n_q + dm->n_k));
  if (dm->d == 128)
    hipLaunchKernelGGL(lf_pool_kernel<128>, dim3(pool_grid), dim3(kThreads), 0, st, pa);
  else
    hipLaunchKernelGGL(lf_pool_kernel<64>, dim3(pool_grid), dim3(kThreads), 0, st, pa);

  const bool retrieve = b->k_frames < dm->m;
  if (retrieve)
    hipLaunchKernelGGL(lf_frame_mean_kernel, dim3((unsigned)(dm->H * dm->m)), dim3(dm->d), 0, st,
                       kt, kh, dm->d, dm->nb, dm->n_k, dm->m, b->n_sink);

  SelectArgs sa;
  sa.qt = qt;
  sa.kt = kt;
  sa.kh = kh;
  sa.indices = indices;
  sa.d = dm->d;
  sa.nb = dm->nb;
  sa.n_q = dm->n_q;
  sa.n_k = dm->n_k;
  sa.F_h = dm->F_h;
  sa.f = dm->f;
  sa.m = dm->m;
  sa.n_sink = b->n_sink;
  sa.n_win = b->n_win;
  sa.k_frames = b->k_frames;
  sa.k_blocks = b->k_blocks;
  sa.current_mandatory = b->current_mandatory;
  sa.list_len = b->list_len;
  sa.n_cand = dm->n_cand;
  int p2 = 1;
  while (p2 < dm->n_cand) p2 <<= 1;
  sa.n_cand_pow2 = p2;
  const unsigned sel_grid = (unsigned)(dm->H * dm->n_q);
  if (dm->d == 128)
    hipLaunchKernelGGL(lf_select_kernel<128>, dim3(sel_grid), dim3(kThreads), 0, st, sa);
  else
    hipLaunchKernelGGL(lf_select_kernel<64>, dim3(sel_grid), dim3(kThreads), 0, st, sa);
  return hipGetLastError() == hipSuccess ? LF_OK : LF_ERR_HIP;
}
