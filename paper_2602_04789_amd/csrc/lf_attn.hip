// Blockwise sparse attention for gfx950 (Eq. 13; Eq. 3 and the paragraph after it: only
// listed tiles are computed, the element mask is never materialised).
//
// One workgroup (4 wavefronts) per (head, query block of 64 rows).  For each listed KV
// block the 64 x d K and V tiles are staged in LDS; wavefront (rh, kh) owns query rows
// [32 rh, 32 rh + 32) and KV rows [32 kh, 32 kh + 32) of every tile and keeps its own
// online-softmax state (m, l, O), so no data crosses wavefronts inside the loop; the two
// KV halves are merged once at the end.
//
// The products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
// v_mfma_f32_32x32x16_bf16: in the 32x32 accumulator layout a lane then holds one query
// column and 16 KV rows, which is exactly the B-operand layout the second product wants,
// so P never moves between lanes.  Softmax is float32, in the exp2 domain.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "lf_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

struct AttnArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* O;
  const int32_t* idx;
  int64_t q_stride_tok, q_stride_head, k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head, o_stride_tok, o_stride_head;
  int n, nb, n_q, n_k, list_len;
  int total_wg, wg_per_xcd;
  float c;  // softmax_scale * log2(e)
};

union Frag {
  uint4 u;
  bf16x8 v;
  uint16_t h[8];
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void lf_attn_kernel(AttnArgs a) {
  constexpr int CH = D / 8;             // 16-byte chunks per token row
  constexpr int KS = D / 16;            // k-steps of S^T = K Q^T
  constexpr int MB = D / 32;            // 32-row blocks of O^T
  constexpr int LPT = 64 * CH / kThreads;  // 16-byte loads per thread, per tile, per tensor
  constexpr int RPP = kThreads / CH;    // tile rows covered per load pass

  __shared__ uint4 smem[2 * 64 * CH];   // K tile | V tile; reused for the final merge
  __shared__ float ml[2][2][64];
  uint4* Ks = smem;
  uint4* Vs = smem + 64 * CH;

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // (head, query block) pairs so that neighbours sharing KV blocks share an L2.
  const int w = (blockIdx.x & 7) * a.wg_per_xcd + (blockIdx.x >> 3);
  if (w >= a.total_wg) return;
  const int h = w / a.n_q, r = w % a.n_q;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rh = wave & 1, kh = wave >> 1;
  const int ln = lane & 31, kg = lane >> 5;

  const int qtok0 = (r / a.nb) * a.n + (r % a.nb) * 64;
  const int q_cnt = min(64, a.n - (r % a.nb) * 64);
  const int qrow = 32 * rh + ln;

  // Q^T fragments (B operand): lane (column q = ln, k-group kg) holds 8 consecutive channels.
  Frag qf[KS];
  {
    const uint16_t* qp = a.Q + (int64_t)h * a.q_stride_head + (int64_t)(qtok0 + qrow) * a.q_stride_tok;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (qrow < q_cnt)
        qf[s].u = *reinterpret_cast<const uint4*>(qp + s * 16 + kg * 8);
      else
        qf[s].u = make_uint4(0, 0, 0, 0);
    }
  }

  const int32_t* list = a.idx + ((int64_t)h * a.n_q + r) * a.list_len;
  const uint16_t* Kh = a.K + (int64_t)h * a.k_stride_head;
  const uint16_t* Vh = a.V + (int64_t)h * a.v_stride_head;
  const int ld_row = tid / CH, ld_ch = tid % CH;

  uint4 kreg[LPT], vreg[LPT];
  auto fetch = [&](int t) -> int {
    const int c = list[t];
    const bool ok = (unsigned)c < (unsigned)a.n_k;
    const int tau = ok ? c / a.nb : 0, j = ok ? c % a.nb : 0;
    const int tok0 = tau * a.n + j * 64;
    const int cnt = ok ? min(64, a.n - j * 64) : 0;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int row = ld_row + RPP * i;
      if (row < cnt) {
        kreg[i] = *reinterpret_cast<const uint4*>(Kh + (int64_t)(tok0 + row) * a.k_stride_tok + ld_ch * 8);
        vreg[i] = *reinterpret_cast<const uint4*>(Vh + (int64_t)(tok0 + row) * a.v_stride_tok + ld_ch * 8);
      } else {
        kreg[i] = make_uint4(0, 0, 0, 0);
        vreg[i] = make_uint4(0, 0, 0, 0);
      }
    }
    return cnt;
  };

  f32x16 oacc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[mb][i] = 0.0f;
  float m_run = -1.0e30f, l_run = 0.0f;

  int cnt_next = fetch(0);
  for (int t = 0; t < a.list_len; ++t) {
    const int cnt = cnt_next;
    __syncthreads();  // every wavefront has finished reading the previous tile
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int row = ld_row + RPP * i;
      Ks[row * CH + (ld_ch ^ (row & (CH - 1)))] = kreg[i];
      Vs[row * CH + (ld_ch ^ (((row >> 2) & 1) << 2))] = vreg[i];
    }
    __syncthreads();
    if (t + 1 < a.list_len) cnt_next = fetch(t + 1);

    // S^T[kv, q] for this wavefront's 32 KV rows x 32 query rows.
    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.0f;
    {
      const int row = 32 * kh + ln;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        Frag kf;
        kf.u = Ks[row * CH + ((2 * s + kg) ^ (row & (CH - 1)))];
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[s].v, sacc, 0, 0, 0);
      }
    }
    // accumulator i of a lane: KV row 32 kh + 8 (i/4) + 4 kg + i%4, query column ln
    if (cnt < 64) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kv = 32 * kh + 8 * (i >> 2) + 4 * kg + (i & 3);
        if (kv >= cnt) sacc[i] = -INFINITY;
      }
    }
    float mx = sacc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sacc[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx * a.c);
    if (__ballot(m_new > m_run) != 0ull) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[mb][i] *= alpha;
      m_run = m_new;
    }
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      p[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], a.c, -m_run));
      l_run += p[i];
    }

    // O^T[d, q] += V^T[d, kv] P^T[kv, q]; k-step u takes accumulators 8u .. 8u+7, i.e.
    // KV rows 16u + 4kg + {0..3} and 16u + 8 + 4kg + {0..3} of this wavefront's half.
    const uint16_t* Vs16 = reinterpret_cast<const uint16_t*>(Vs);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      Frag pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) pf.h[e] = f32_to_bf16_rne(p[8 * u + e]);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int col = 32 * mb + ln;
        Frag vf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int row = 32 * kh + 16 * u + 8 * (e >> 2) + 4 * kg + (e & 3);
          const int chunk = (col >> 3) ^ (((row >> 2) & 1) << 2);
          vf.h[e] = Vs16[(row * CH + chunk) * 8 + (col & 7)];
        }
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, oacc[mb], 0, 0, 0);
      }
    }
  }

  // Merge the two KV halves: wavefronts with kh = 1 publish (m, l, O^T), kh = 0 combine.
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();
  float* mbuf = reinterpret_cast<float*>(smem);  // [rh][MB*16][64]
  if (kh == 1) {
    ml[rh][0][lane] = m_run;
    ml[rh][1][lane] = l_run;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mbuf[(rh * MB * 16 + mb * 16 + i) * 64 + lane] = oacc[mb][i];
  }
  __syncthreads();
  if (kh == 0) {
    const float m2 = ml[rh][0][lane], l2 = ml[rh][1][lane];
    const float m = fmaxf(m_run, m2);
    const float a1 = __builtin_amdgcn_exp2f(m_run - m), a2 = __builtin_amdgcn_exp2f(m2 - m);
    const float inv = 1.0f / (l_run * a1 + l2 * a2);
    if (qrow < q_cnt) {
      uint16_t* op = a.O + (int64_t)h * a.o_stride_head + (int64_t)(qtok0 + qrow) * a.o_stride_tok;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint16_t o4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * g + e;
            const float o2 = mbuf[(rh * MB * 16 + mb * 16 + i) * 64 + lane];
            o4[e] = f32_to_bf16_rne((oacc[mb][i] * a1 + o2 * a2) * inv);
          }
          uint2 pk;
          pk.x = (uint32_t)o4[0] | ((uint32_t)o4[1] << 16);
          pk.y = (uint32_t)o4[2] | ((uint32_t)o4[3] << 16);
          *reinterpret_cast<uint2*>(op + 32 * mb + 8 * g + 4 * kg) = pk;
        }
      }
    }
  }
}

}  // namespace

int lf_launch_attn(const void* Q, const void* K, const void* V, const lf_shape* s,
                   const lf_dims* dm, const int32_t* indices, int32_t list_len, float scale,
                   void* O, void* stream) {
  AttnArgs a;
  a.Q = (const uint16_t*)Q;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
  a.O = (uint16_t*)O;
  a.idx = indices;
  a.q_stride_tok = s->q_stride_tok;
  a.q_stride_head = s->q_stride_head;
  a.k_stride_tok = s->k_stride_tok;
  a.k_stride_head = s->k_stride_head;
  a.v_stride_tok = s->v_stride_tok;
  a.v_stride_head = s->v_stride_head;
  a.o_stride_tok = s->o_stride_tok;
  a.o_stride_head = s->o_stride_head;
  a.n = dm->n;
  a.nb = dm->nb;
  a.n_q = dm->n_q;
  a.n_k = dm->n_k;
  a.list_len = list_len;
  a.total_wg = dm->H * dm->n_q;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  a.c = scale * 1.4426950408889634f;
  const unsigned grid = (unsigned)(a.wg_per_xcd * 8);
  hipStream_t st = (hipStream_t)stream;
  if (dm->d == 128)
    hipLaunchKernelGGL(lf_attn_kernel<128>, dim3(grid), dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL(lf_attn_kernel<64>, dim3(grid), dim3(kThreads), 0, st, a);
  return hipGetLastError() == hipSuccess ? LF_OK : LF_ERR_HIP;
}
