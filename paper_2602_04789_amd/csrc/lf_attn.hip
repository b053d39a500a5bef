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
constexpr int kMaxEnt = 512;  // list entries decoded per pass (power of two)

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
};

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// 16-byte chunk swizzles of the LDS tiles (row = token within the tile, ch = 8-channel chunk).
// K is read row-wise, 16 bytes per lane, 16 consecutive rows at one logical chunk: XOR with
// the row spreads them over all banks.  V is read with the transposing 8-byte LDS read, four
// consecutive rows x 64 bytes at a time: XOR moves each of the four rows to its own 64 bytes.
template <int CH> __device__ __forceinline__ int k_swz(int row, int ch) { return ch ^ (row & (CH - 1)); }
template <int CH> __device__ __forceinline__ int v_swz(int row, int ch) {
  return ch ^ ((row & (CH / 4 - 1)) << 2);
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void lf_attn_kernel(AttnArgs a) {
  constexpr int CH = D / 8;                 // 16-byte chunks per token row
  constexpr int KS = D / 16;                // k-steps of S^T = K Q^T
  constexpr int MB = D / 32;                // 32-row blocks of O^T
  constexpr int RPI = 64 / CH;              // tile rows one wavefront load instruction covers
  constexpr int LPW = 64 / (RPI * 4);       // load instructions per wavefront, per tile, per tensor
  constexpr int TILE = 64 * CH;             // uint4 per tile

  // Two tile buffers (K | V each) as separate LDS objects, so that the compiler can tell
  // the asynchronous fill of one from the reads of the other; lds0 is reused for the merge.
  __shared__ uint4 lds0[2 * TILE];
  __shared__ uint4 lds1[2 * TILE];
  __shared__ float ml[2][2][64];
  __shared__ int2 ent[kMaxEnt];            // (first token, token count) per list entry

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
  const char* Kh = reinterpret_cast<const char*>(a.K + (int64_t)h * a.k_stride_head);
  const char* Vh = reinterpret_cast<const char*>(a.V + (int64_t)h * a.v_stride_head);
  const int64_t k_row_bytes = a.k_stride_tok * 2, v_row_bytes = a.v_stride_tok * 2;

  // Tile load, global -> LDS without passing through registers: load instruction i of
  // wavefront `wave` fills tile rows [RPI*(LPW*wave+i), +RPI); lane l lands at byte 16*l
  // of that 1 KiB stripe, so it fetches the chunk the swizzle assigns to that place.  Rows
  // past the block's token count re-read its last token (finite data that the mask removes).
  // Per-lane byte offsets inside a full tile are loop invariants.
  const int ld_r = lane / CH, ld_p = lane % CH;
  uint32_t koff[LPW], voff[LPW], kswz[LPW], vswz[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = RPI * (LPW * wave + i) + ld_r;
    kswz[i] = (uint32_t)k_swz<CH>(row, ld_p) * 16u;
    vswz[i] = (uint32_t)v_swz<CH>(row, ld_p) * 16u;
    koff[i] = (uint32_t)row * (uint32_t)k_row_bytes + kswz[i];
    voff[i] = (uint32_t)row * (uint32_t)v_row_bytes + vswz[i];
  }
  // (first token, token count) of list entry t, wavefront-uniform.
  auto entry = [&](int t) -> int2 {
    const int2 e = ent[t & (kMaxEnt - 1)];
    return make_int2(__builtin_amdgcn_readfirstlane(e.x), __builtin_amdgcn_readfirstlane(e.y));
  };
  auto fetch = [&](int2 e, uint4* kb) {
    const char* kbase = Kh + (int64_t)e.x * k_row_bytes;
    const char* vbase = Vh + (int64_t)e.x * v_row_bytes;
    uint4* vb = kb + TILE;
    if (e.y == 64) {
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int row0 = RPI * (LPW * wave + i);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(kbase + koff[i]), LDS_PTR(void, kb + row0 * CH), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(vbase + voff[i]), LDS_PTR(void, vb + row0 * CH), 16, 0, 0);
      }
    } else {
      const int last = max(e.y - 1, 0);
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int row0 = RPI * (LPW * wave + i);
        const uint32_t srow = (uint32_t)min(row0 + ld_r, last);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(kbase + (srow * (uint32_t)k_row_bytes + kswz[i])),
                                         LDS_PTR(void, kb + row0 * CH), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(vbase + (srow * (uint32_t)v_row_bytes + vswz[i])),
                                         LDS_PTR(void, vb + row0 * CH), 16, 0, 0);
      }
    }
  };

  f32x16 oacc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[mb][i] = 0.0f;
  float m_run = -1.0e30f, l_run = 0.0f;

  // Lists are decoded kMaxEnt entries at a time into LDS: block id -> (first token, count);
  // an id outside [0, n_k) becomes an empty block (count 0).
  for (int t0 = 0; t0 < a.list_len; t0 += kMaxEnt) {
  const int t1 = min(a.list_len, t0 + kMaxEnt);
  __syncthreads();
  for (int i = t0 + tid; i < t1; i += kThreads) {
    const int c = list[i];
    const bool ok = (unsigned)c < (unsigned)a.n_k;
    const int tau = ok ? c / a.nb : 0, j = ok ? c % a.nb : 0;
    ent[i - t0] = make_int2(tau * a.n + j * 64, ok ? min(64, a.n - j * 64) : 0);
  }
  __syncthreads();
  int2 e_cur = entry(t0);
  fetch(e_cur, lds0);
  int2 e_next = entry(min(t0 + 1, t1 - 1));
  // One tile: wait for it, start the next tile's fill into the other buffer, compute.
  auto tile = [&](int t, const uint4* Ks, uint4* other) __attribute__((always_inline)) {
    const int cnt = e_cur.y;
    __builtin_amdgcn_s_waitcnt(0);  // this wavefront's part of tile t has landed in LDS
    __syncthreads();                // ... and everyone's; the other buffer is no longer being read
    if (t + 1 < t1) fetch(e_next, other);
    e_cur = e_next;
    e_next = entry(min(t + 2, t1 - 1));
    const uint4* Vs = Ks + TILE;

    // S^T[kv, q] for this wavefront's 32 KV rows x 32 query rows.
    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.0f;
    {
      const int row = 32 * kh + ln;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        Frag kf;
        kf.u = Ks[row * CH + k_swz<CH>(row, 2 * s + kg)];
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
    // The A operand (V^T) comes from the row-major V tile through the transposing LDS
    // read: within each group of 16 lanes, lane 4e+g supplies the address of row e,
    // columns 4g..4g+3, and lane i receives column i of the four rows.
    const uint16_t* Vs16 = reinterpret_cast<const uint16_t*>(Vs);
    const int i16 = lane & 15;
    const int tr_row = 32 * kh + 4 * kg + (i16 >> 2);
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      bf16x8 pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) pf[e] = (__bf16)p[8 * u + e];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int col = 32 * mb + tr_col;
        const int r0 = tr_row + 16 * u, r1 = r0 + 8;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            LDS_PTR(bf16x4, Vs16 + (r0 * CH + v_swz<CH>(r0, col >> 3)) * 8 + (col & 7)));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            LDS_PTR(bf16x4, Vs16 + (r1 * CH + v_swz<CH>(r1, col >> 3)) * 8 + (col & 7)));
        const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[mb], 0, 0, 0);
      }
    }
  };
  for (int t = t0; t < t1; t += 2) {
    tile(t, lds0, lds1);
    if (t + 1 < t1) tile(t + 1, lds1, lds0);
  }
  }

  // Merge the two KV halves: wavefronts with kh = 1 publish (m, l, O^T), kh = 0 combine.
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();
  float* mbuf = reinterpret_cast<float*>(lds0);  // [rh][MB*16][64]
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
          bf16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * g + e;
            const float o2 = mbuf[(rh * MB * 16 + mb * 16 + i) * 64 + lane];
            o4[e] = (__bf16)((oacc[mb][i] * a1 + o2 * a2) * inv);
          }
          *reinterpret_cast<bf16x4*>(op + 32 * mb + 8 * g + 4 * kg) = o4;
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
