// Mask selection kernels for gfx950 (Sec. 4.2, Eq. 7 - Eq. 12).
//
//   lf_pool_kernel        block mean pooling of Q and K (Eq. 7, blockwise): the one pass
//                         over the bf16 inputs, HBM-bound.
//   lf_frame_mean_kernel  frame means of the candidate frames (Eq. 7, framewise); the block
//                         means of Q ride along in the same launch.
//   lf_select_kernel      per (head, query block): frame scores (Eq. 8), frame top-k
//                         (Eq. 9), block scores (Eq. 10), block top-k (Eq. 11: by counting
//                         the keys that rank before each candidate when there are at most
//                         256 of them, by a bitonic sort over lane shuffles and LDS beyond
//                         that), ascending index list (Eq. 12).
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
  int n, nb, n_q;
  int k_block0, n_kp;   // KV blocks pooled by this launch: [k_block0, k_block0 + n_kp)
  int kt_rows;          // rows of the quad-major pooled-key matrix (KV blocks it has room for)
};

// Pooled keys are stored "channel-quad major": element (row c, channel t) of a [rows][d]
// matrix lives at ((t/4) * rows + c) * 4 + t%4.  A thread that walks one row's channels in
// order then reads 16 bytes per step, and neighbouring rows (= neighbouring threads) are
// contiguous, so the score loops below read straight from global memory with coalesced
// 16-byte loads and need no staging.
__device__ __forceinline__ int64_t quad_major(int rows, int c, int t) {
  return ((int64_t)(t >> 2) * rows + c) * 4 + (t & 3);
}

// One workgroup per block of <= 64 tokens.  Thread t owns 8 consecutive channels
// (one 16-byte load per token) of every (256/CH)-th token.
template <int D>
__device__ __forceinline__ void pool_block(const PoolArgs& a, int h, int u, double* lds) {
  constexpr int CH = D / 8;          // 16-byte chunks per token row
  constexpr int RG = kThreads / CH;  // token rows in flight per pass
  double (*red)[D] = reinterpret_cast<double (*)[D]>(lds);   // [RG][D]

  const bool is_q = u < a.n_q;
  const int c = is_q ? u : a.k_block0 + u - a.n_q;
  const int tau = c / a.nb, j = c % a.nb;
  const int tok0 = tau * a.n + j * 64;
  const int cnt = min(64, a.n - j * 64);
  const uint16_t* src = is_q ? a.Q + (int64_t)h * a.q_stride_head
                             : a.K + (int64_t)h * a.k_stride_head;
  const int64_t stride = is_q ? a.q_stride_tok : a.k_stride_tok;
  const int ch = threadIdx.x % CH, rg = threadIdx.x / CH;

  uint4 v[64 / RG];
#pragma unroll
  for (int i = 0; i < 64 / RG; ++i) {
    const int row = rg + RG * i;
    v[i] = row < cnt ? *reinterpret_cast<const uint4*>(src + (int64_t)(tok0 + row) * stride + ch * 8)
                     : make_uint4(0, 0, 0, 0);
  }
  double acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0;
#pragma unroll
  for (int i = 0; i < 64 / RG; ++i) {
    acc[0] += (double)bf16lo(v[i].x);
    acc[1] += (double)bf16hi(v[i].x);
    acc[2] += (double)bf16lo(v[i].y);
    acc[3] += (double)bf16hi(v[i].y);
    acc[4] += (double)bf16lo(v[i].z);
    acc[5] += (double)bf16hi(v[i].z);
    acc[6] += (double)bf16lo(v[i].w);
    acc[7] += (double)bf16hi(v[i].w);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[rg][ch * 8 + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < D) {
    double s = 0.0;
#pragma unroll
    for (int g = 0; g < RG; ++g) s += red[g][threadIdx.x];
    const float mean = (float)(s / (double)cnt);
    if (is_q)
      a.qt[((int64_t)h * a.n_q + c) * D + threadIdx.x] = mean;
    else
      a.kt[(int64_t)h * a.kt_rows * D + quad_major(a.kt_rows, c, threadIdx.x)] = mean;
  }
}

// Bytes of LDS pool_block<D> needs: 16 KB for either head dimension.
template <int D> constexpr int pool_lds_doubles() { return (kThreads / (D / 8)) * D; }

template <int D>
__global__ __launch_bounds__(kThreads) void lf_pool_kernel(PoolArgs a) {
  __shared__ double red[pool_lds_doubles<D>()];
  const int per_head = a.n_q + a.n_kp;
  pool_block<D>(a, blockIdx.x / per_head, blockIdx.x % per_head, red);
}

// k_hat of frames tau0 .. tau0 + count - 1 of every head, written to rows out0 .. of the
// quad-major matrix kh (kh_rows rows per head): binary64 sum of the frame's nb block means in
// ascending block order, / nb, rounded to float32.  One workgroup per (head, frame), one thread
// per channel quad.  The workgroups after the first H * count pool query blocks instead (the
// block means of Q are not needed before the selection kernel, so they travel with this small
// launch rather than lengthen the pass over K): workgroup H * count + i is unit i of `qp`.
struct FrameMeanArgs {
  const float* kt;
  float* kh;
  int nb, kt_rows, kh_rows, tau0, out0, count, H;
};

template <int D>
__global__ __launch_bounds__(kThreads) void lf_frame_mean_kernel(FrameMeanArgs f, PoolArgs qp) {
  __shared__ double red[pool_lds_doubles<D>()];
  const int n_fm = f.H * f.count;
  if ((int)blockIdx.x >= n_fm) {
    const int u = blockIdx.x - n_fm, per_head = qp.n_q + qp.n_kp;
    pool_block<D>(qp, u / per_head, u % per_head, red);
    return;
  }
  const int h = blockIdx.x / f.count, a = blockIdx.x % f.count;
  const int tau = f.tau0 + a;
  const int q = threadIdx.x;
  if (q >= D / 4) return;
  const float4* src = reinterpret_cast<const float4*>(f.kt + (int64_t)h * f.kt_rows * D) +
                      ((int64_t)q * f.kt_rows + (int64_t)tau * f.nb);
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  int j = 0;
  for (; j + 8 <= f.nb; j += 8) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[j + u];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      s0 += (double)v[u].x; s1 += (double)v[u].y; s2 += (double)v[u].z; s3 += (double)v[u].w;
    }
  }
  for (; j < f.nb; ++j) {
    const float4 v = src[j];
    s0 += (double)v.x; s1 += (double)v.y; s2 += (double)v.z; s3 += (double)v.w;
  }
  float4 o;
  o.x = (float)(s0 / (double)f.nb); o.y = (float)(s1 / (double)f.nb);
  o.z = (float)(s2 / (double)f.nb); o.w = (float)(s3 / (double)f.nb);
  reinterpret_cast<float4*>(f.kh + (int64_t)h * f.kh_rows * D)[(int64_t)q * f.kh_rows + f.out0 + a] = o;
}

struct SelectArgs {
  const float* qt;
  const float* kt;
  const float* kh;
  int32_t* indices;
  int d, nb, n_q, n_k, F_h, f, m;
  int n_sink, n_win, k_frames, k_blocks, current_mandatory, list_len;
  int n_cand, n_tf;
  int kt_rows, kh_rows;  // rows per head of the quad-major matrices kt and kh
  int kh_row0;           // row of kh that holds candidate frame 0 (frame n_sink)
};

// Dynamic LDS of lf_select_kernel<D, E>; must mirror the carving at the top of the kernel.
inline size_t select_lds_bytes(const SelectArgs& a, int e) {
  size_t b = (size_t)a.d * sizeof(double);
  b += (size_t)kThreads * e * (sizeof(float) + sizeof(int));   // exchange arrays of the sort
  b += (size_t)a.m * sizeof(float);
  b += (size_t)(a.n_tf + a.f) * sizeof(int);
  b += (size_t)((a.F_h + 3) & ~3) + (size_t)((a.n_cand + 3) & ~3);
  return b;
}

// <q_tilde, row c> over the head dimension in ascending order, binary64 accumulate (the product
// of two float32 is exact in binary64, so only the order matters), rounded to float32 once.
// `base` points at row 0, channel quad 0 of a quad-major matrix with `rows` rows and is the
// same for the whole workgroup, so the quad's address is a scalar base plus the lane's 16 c.
// Sixteen of the row's channel quads are in flight at any time: four groups of four, each
// group requested again as soon as it has been used, so that the load latency is paid once.
template <int D>
__device__ __forceinline__ float dot_quad_major(const double* __restrict__ qd,
                                                const float4* __restrict__ base, uint32_t c, int rows) {
  constexpr int G = 4, NG = D / 4 / G;
  static_assert(NG >= 4, "the ring holds four groups");
  float4 v[4][G];
  double acc = 0.0;
  // q_tilde is read through an offset the compiler cannot see through (always 0): called from
  // a loop, its 2 d registers' worth of reads would otherwise be hoisted out of the loop
  int z = 0;
  asm volatile("" : "+v"(z));
  const double* __restrict__ q = qd + z;
  auto fetch = [&](float4 (&x)[G], int g, uint32_t cc) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < G; ++u) x[u] = (base + (int64_t)(g * G + u) * rows)[cc];
  };
  auto use = [&](const float4 (&x)[G], int g) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int t = 4 * (g * G + u);
      acc += q[t + 0] * (double)x[u].x;
      acc += q[t + 1] * (double)x[u].y;
      acc += q[t + 2] * (double)x[u].z;
      acc += q[t + 3] * (double)x[u].w;
    }
  };
#pragma unroll
  for (int i = 0; i < 4; ++i) fetch(v[i], i, c);
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    use(v[g & 3], g);
    // An empty statement that takes the sum so far and hands back the row index: the sum cannot
    // sink below it and the next request cannot rise above it, which keeps the ring as written
    // (left to itself the compiler gathers all loads first and spills).
    uint32_t cc = c;
    asm volatile("" : "+v"(acc), "+v"(cc));
    if (g + 4 < NG) fetch(v[g & 3], g + 4, cc);
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

// Bitonic sort of 256*E (score, position) pairs held E per thread, element e of thread t
// being index e*256 + t, into ranks_before order along the index.  Partners at distance
// < 64 are reached with lane shuffles, at distance 64 and 128 through the LDS arrays xs/xp
// (one barrier pair per such step), at distance >= 256 inside the thread.
template <int E>
__device__ __forceinline__ void bitonic_sort(float (&s)[E], int (&p)[E], float* xs, int* xp) {
  const int tid = threadIdx.x;
#pragma unroll 1
  for (int k = 2; k <= kThreads * E; k <<= 1) {
#pragma unroll 1
    for (int j = k >> 1; j > 0; j >>= 1) {
      if (j >= kThreads) {
        const int de = j / kThreads;
#pragma unroll
        for (int e = 0; e < E; ++e) {
          if ((e & de) == 0 && (e | de) < E) {
            const int e2 = e | de, i = e * kThreads + tid;
            const bool up = (i & k) == 0;
            const bool first_is_lo = ranks_before(s[e], p[e], s[e2], p[e2]);
            if (first_is_lo != up) {
              const float ts = s[e]; s[e] = s[e2]; s[e2] = ts;
              const int tp = p[e]; p[e] = p[e2]; p[e2] = tp;
            }
          }
        }
      } else {
        float os[E];
        int op[E];
        if (j >= 64) {
          __syncthreads();
#pragma unroll
          for (int e = 0; e < E; ++e) { xs[e * kThreads + tid] = s[e]; xp[e * kThreads + tid] = p[e]; }
          __syncthreads();
#pragma unroll
          for (int e = 0; e < E; ++e) { os[e] = xs[e * kThreads + (tid ^ j)]; op[e] = xp[e * kThreads + (tid ^ j)]; }
        } else {
#pragma unroll
          for (int e = 0; e < E; ++e) { os[e] = __shfl_xor(s[e], j); op[e] = __shfl_xor(p[e], j); }
        }
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const int i = e * kThreads + tid;
          const bool want_first = ((i & j) == 0) == ((i & k) == 0);
          const bool mine_first = ranks_before(s[e], p[e], os[e], op[e]);
          const bool other_first = ranks_before(os[e], op[e], s[e], p[e]);
          if (want_first ? other_first : mine_first) { s[e] = os[e]; p[e] = op[e]; }
        }
      }
    }
  }
}

// 32-bit key whose unsigned order is the score order: float32 bits made monotonic, -0.0
// folded onto +0.0 so that the two tie (ties go to the lower position, see ranks_before).
__device__ __forceinline__ uint32_t rank_key32(float score) {
  const uint32_t u = __float_as_uint(score + 0.0f);
  return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

// Probe build only (liblf_hsa_probe_stamps.so, for `bench.py --select-phases`): thread 0 of the
// first 4096 workgroups notes the 100 MHz wall clock at the phase boundaries of the kernel, to
// see where its time goes.  The lists are unchanged; the product build has none of this.
#ifdef LF_PROBE_STAMPS
__device__ unsigned long long g_stamps[4096 * 8];
#define LF_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 4096) g_stamps[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#define LF_STAMP_SYNC() __syncthreads()
#else
#define LF_STAMP(i)
#define LF_STAMP_SYNC()
#endif

template <int D, int E>
__global__ __launch_bounds__(kThreads, (E <= 2 ? 4 : 2)) void lf_select_kernel(SelectArgs a) {
  LF_STAMP(0);
  // LDS carved from one dynamic allocation sized for this call (see select_lds_bytes()).
  extern __shared__ double lds_raw[];
  double* qd = lds_raw;                                         // [D]
  float* xs = reinterpret_cast<float*>(qd + D);                 // [256*E]
  int* xp = reinterpret_cast<int*>(xs + kThreads * E);          // [256*E]
  float* fscore = reinterpret_cast<float*>(xp + kThreads * E);  // [m]
  int* flist = reinterpret_cast<int*>(fscore + a.m);            // [n_tf + f]
  unsigned char* fflag = reinterpret_cast<unsigned char*>(flist + a.n_tf + a.f);  // [F_h]
  unsigned char* sel = fflag + ((a.F_h + 3) & ~3);              // [n_cand]

  const int tid = threadIdx.x;
  const int h = blockIdx.x / a.n_q, r = blockIdx.x % a.n_q;
  const float* qrow = a.qt + ((int64_t)h * a.n_q + r) * D;
  if (tid < D) qd[tid] = (double)qrow[tid];
  __syncthreads();
  LF_STAMP(1);   // q_tilde is in LDS

  const bool retrieve = a.k_frames < a.m;
  const float4* kth = reinterpret_cast<const float4*>(a.kt + (int64_t)h * a.kt_rows * D);

  // With one candidate per thread (E == 1), Eq. 10 is taken in two parts.  The candidates of
  // the sink, window and (when they compete) current frames are known before any frame score
  // is: there are n_cand - k_frames nb of them, position (= rank by block id among the
  // candidates) below n_sink nb or from (n_sink + k_frames) nb on, and in list slot i >= n_sink
  // + k_frames sits frame F_h - n_tf + i.  They are scored now, by the threads counted down
  // from the last one, i.e. by the wavefronts that have nothing to do while the first one
  // scores the frames; the candidates of the retrieved frames follow below, on the threads
  // counted up from the first.  The two sets of threads are disjoint (n_cand <= 256).
  const int ret_b = (E == 1 && retrieve) ? a.k_frames * a.nb : 0;
  const bool need_scores = a.k_blocks < a.n_cand;
  float s1 = -INFINITY;   // E == 1: this thread's score and its candidate's position
  int p1 = -1;
  if (E == 1) {
    uint32_t* keys = reinterpret_cast<uint32_t*>(xs);
    keys[tid] = 0u;       // pads must hold 0 (see the ranking below)
    if (tid < a.n_cand) sel[tid] = 0;
    const int slot = kThreads - 1 - tid, sink_b = a.n_sink * a.nb;
    if (need_scores && slot < a.n_cand - ret_b) {
      p1 = slot < sink_b ? slot : slot + ret_b;
      const int i = p1 / a.nb;
      const int frame = i < a.n_sink ? i : a.F_h - a.n_tf + i;
      s1 = dot_quad_major<D>(qd, kth, (uint32_t)(frame * a.nb + p1 % a.nb), a.kt_rows);
    }
  }

  // Eq. 8: frame-level scores against the candidate frames M = [n_sink, F_h - n_win).
  if (retrieve) {
    const float4* khh = reinterpret_cast<const float4*>(a.kh + (int64_t)h * a.kh_rows * D) + a.kh_row0;
    for (int c = tid; c < a.m; c += kThreads) fscore[c] = dot_quad_major<D>(qd, khh, (uint32_t)c, a.kh_rows);
  }
  __syncthreads();
  LF_STAMP(2);   // frame scores (and, with one candidate per thread, the scores of the known candidates)

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
  if (!a.current_mandatory)
    for (int t = tid; t < a.f; t += kThreads) flist[a.n_tf + t] = a.F_h + t;
  __syncthreads();
  LF_STAMP(3);   // frame ranking and frame list

  // Eq. 10: block-level scores over B_r, candidates in ascending block id; candidate
  // e*256 + tid is element e of this thread (E > 1; for E == 1 see above).
  float s[E];
  int p[E];
  if (E == 1) {
    if (need_scores && tid < ret_b) {
      p1 = a.n_sink * a.nb + tid;
      s1 = dot_quad_major<D>(qd, kth, (uint32_t)(flist[p1 / a.nb] * a.nb + p1 % a.nb), a.kt_rows);
    }
    s[0] = s1;
    p[0] = p1;
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int i = e * kThreads + tid;
      s[e] = -INFINITY;
      p[e] = 0x7fffffff;
      if (i < a.n_cand) {
        const int c = flist[i / a.nb] * a.nb + i % a.nb;
        s[e] = dot_quad_major<D>(qd, kth, (uint32_t)c, a.kt_rows);
        p[e] = i;
        sel[i] = 0;
      }
    }
  }

  LF_STAMP_SYNC();
  LF_STAMP(4);   // block scores
  // Eq. 11: top-k blocks, J_r = the candidates of rank < k_blocks.  With at most one
  // candidate per thread the rank is counted directly (how many keys are larger, keys read
  // as LDS broadcasts); larger candidate sets are sorted, after which index = rank.
  if (a.k_blocks < a.n_cand && E == 1) {
    // 32-bit keys in position order.  A candidate's rank = earlier positions with a key >= its
    // own + later positions with a key > its own; for a wavefront the positions before its
    // first lane are all earlier and those after its last lane all later, so only the 64
    // positions of its own lanes need the position compared.  Pads hold 0, which no key is below.
    uint32_t* keys = reinterpret_cast<uint32_t*>(xs);   // [256], 16-byte aligned, zeroed above
    if (p[0] >= 0) keys[p[0]] = rank_key32(s[0]);
    __syncthreads();
    const uint32_t mine = keys[tid];
    const int w0 = __builtin_amdgcn_readfirstlane(tid & ~63);
    if (w0 < a.n_cand) {
      // four counters, so that a compare and the add that takes its carry need not be neighbours
      int r0 = 0, r1 = 0, r2 = 0, r3 = 0;
#pragma unroll 4
      for (int j = 0; j < w0; j += 4) {
        const uint4 kk = *reinterpret_cast<const uint4*>(keys + j);
        r0 += kk.x >= mine ? 1 : 0; r1 += kk.y >= mine ? 1 : 0;
        r2 += kk.z >= mine ? 1 : 0; r3 += kk.w >= mine ? 1 : 0;
      }
      const int lane = tid & 63;
#pragma unroll 4
      for (int j = 0; j < 64; j += 4) {
        const uint4 kk = *reinterpret_cast<const uint4*>(keys + w0 + j);
        r0 += (kk.x > mine || (kk.x == mine && j + 0 < lane)) ? 1 : 0;
        r1 += (kk.y > mine || (kk.y == mine && j + 1 < lane)) ? 1 : 0;
        r2 += (kk.z > mine || (kk.z == mine && j + 2 < lane)) ? 1 : 0;
        r3 += (kk.w > mine || (kk.w == mine && j + 3 < lane)) ? 1 : 0;
      }
#pragma unroll 4
      for (int j = w0 + 64; j < a.n_cand; j += 4) {
        const uint4 kk = *reinterpret_cast<const uint4*>(keys + j);
        r0 += kk.x > mine ? 1 : 0; r1 += kk.y > mine ? 1 : 0;
        r2 += kk.z > mine ? 1 : 0; r3 += kk.w > mine ? 1 : 0;
      }
      const int rank = (r0 + r1) + (r2 + r3);
      if (tid < a.n_cand && rank < a.k_blocks) sel[tid] = 1;
    }
  } else if (a.k_blocks < a.n_cand) {
    bitonic_sort<E>(s, p, xs, xp);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (e * kThreads + tid < a.k_blocks) sel[p[e]] = 1;
  } else {
    __syncthreads();
    for (int i = tid; i < a.n_cand; i += kThreads) sel[i] = 1;
  }
  __syncthreads();
  LF_STAMP(5);   // block ranking

  // Eq. 12 as a sorted list: kept candidates in ascending id, then the mandatory current blocks.
  int32_t* out = a.indices + ((int64_t)h * a.n_q + r) * a.list_len;
  if (tid < 64)
    wave_compact(sel, a.n_cand, [&](int pos, int i) { out[pos] = flist[i / a.nb] * a.nb + i % a.nb; });
  if (a.current_mandatory)
    for (int i = tid; i < a.f * a.nb; i += kThreads) out[a.k_blocks + i] = a.F_h * a.nb + i;
  LF_STAMP_SYNC();
  LF_STAMP(6);   // compaction and store
}

}  // namespace

// Arguments for pooling the query blocks (when Q is given) and the KV blocks of frames
// [frame0, frame1) into qt / the quad-major matrix kt with kt_rows rows per head.
static PoolArgs pool_args(const void* Q, const void* K, const lf_shape* s, const lf_dims* dm, float* qt,
                          float* kt, int kt_rows, int frame0, int frame1) {
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
  pa.n_q = Q ? dm->n_q : 0;
  pa.k_block0 = frame0 * dm->nb;
  pa.n_kp = (frame1 - frame0) * dm->nb;
  pa.kt_rows = kt_rows;
  return pa;
}

static hipError_t launch_pool(const void* Q, const void* K, const lf_shape* s, const lf_dims* dm, float* qt,
                        float* kt, int kt_rows, int frame0, int frame1, hipStream_t st) {
  const PoolArgs pa = pool_args(Q, K, s, dm, qt, kt, kt_rows, frame0, frame1);
  const unsigned pool_grid = (unsigned)(dm->H * (pa.n_q + pa.n_kp));
  if (pool_grid == 0) return hipSuccess;
  return dm->d == 128 ? lf_launch(lf_pool_kernel<128>, dim3(pool_grid), dim3(kThreads), 0, st, pa)
                      : lf_launch(lf_pool_kernel<64>, dim3(pool_grid), dim3(kThreads), 0, st, pa);
}

// Frame means of frames [tau0, tau0 + count) of every head, to rows out0 .. of kh; after them,
// in the same launch, the units of `qp` are pooled (qp.n_q = qp.n_kp = 0: none).
static hipError_t launch_frame_means(const lf_dims* dm, const float* kt, float* kh, int kt_rows, int kh_rows,
                                     int tau0, int out0, int count, const PoolArgs& qp, hipStream_t st) {
  FrameMeanArgs f;
  f.kt = kt;
  f.kh = kh;
  f.nb = dm->nb;
  f.kt_rows = kt_rows;
  f.kh_rows = kh_rows;
  f.tau0 = tau0;
  f.out0 = out0;
  f.count = count;
  f.H = dm->H;
  const unsigned grid = (unsigned)(dm->H * count + dm->H * (qp.n_q + qp.n_kp));
  if (grid == 0) return hipSuccess;
  return dm->d == 128 ? lf_launch(lf_frame_mean_kernel<128>, dim3(grid), dim3(kThreads), 0, st, f, qp)
                      : lf_launch(lf_frame_mean_kernel<64>, dim3(grid), dim3(kThreads), 0, st, f, qp);
}

static hipError_t launch_select(const lf_budget* b, const lf_dims* dm, const float* qt, const float* kt,
                          const float* kh, int kt_rows, int kh_rows, int kh_row0, int32_t* indices,
                          hipStream_t st) {
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
  sa.n_tf = dm->n_tf;
  sa.kt_rows = kt_rows;
  sa.kh_rows = kh_rows;
  sa.kh_row0 = kh_row0;
  // E = candidate pairs per thread in the sort: 256*E >= n_cand, E a power of two
  int e = 1;
  while (kThreads * e < dm->n_cand) e <<= 1;
  const unsigned sel_grid = (unsigned)(dm->H * dm->n_q);
  const size_t lds = select_lds_bytes(sa, e);
#define LF_LAUNCH_SELECT(DD, EE) \
  lf_launch(lf_select_kernel<DD, EE>, dim3(sel_grid), dim3(kThreads), lds, st, sa)
  if (dm->d == 128) {
    if (e == 1) return LF_LAUNCH_SELECT(128, 1);
    if (e == 2) return LF_LAUNCH_SELECT(128, 2);
    if (e == 4) return LF_LAUNCH_SELECT(128, 4);
    return LF_LAUNCH_SELECT(128, 8);
  }
  if (e == 1) return LF_LAUNCH_SELECT(64, 1);
  if (e == 2) return LF_LAUNCH_SELECT(64, 2);
  if (e == 4) return LF_LAUNCH_SELECT(64, 4);
  return LF_LAUNCH_SELECT(64, 8);
#undef LF_LAUNCH_SELECT
}

int lf_launch_select(const void* Q, const void* K, const lf_shape* s, const lf_budget* b,
                     const lf_dims* dm, int32_t* indices, void* workspace, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* qt = (float*)(ws + dm->off_qt);
  float* kt = (float*)(ws + dm->off_kt);
  float* kh = (float*)(ws + dm->off_kh);
  // With frames to retrieve there are three launches: the pass over K; the frame means, with the
  // pooling of Q riding along (nothing needs q_tilde before the third); the selection.
  const bool retrieve = b->k_frames < dm->m;
  if (launch_pool(retrieve ? nullptr : Q, K, s, dm, qt, kt, dm->n_k, 0, dm->F, st) != hipSuccess) return LF_ERR_HIP;
  if (retrieve &&
      launch_frame_means(dm, kt, kh, dm->n_k, dm->m, b->n_sink, 0, dm->m,
                         pool_args(Q, nullptr, s, dm, qt, nullptr, 1, 0, 0), st) != hipSuccess)
    return LF_ERR_HIP;
  return launch_select(b, dm, qt, kt, kh, dm->n_k, dm->m > 0 ? dm->m : 1, 0, indices, st) == hipSuccess
             ? LF_OK : LF_ERR_HIP;
}

// Pooled-key cache: kt for max_frames * nb blocks, then kh for max_frames frames (all frames,
// row = absolute frame index), both quad-major per head.
int lf_launch_kcache_update(const void* K, const lf_shape* s, const lf_dims* dm, int frame0, int frame1,
                            int max_frames, void* kcache, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  float* kt = (float*)kcache;
  float* kh = kt + (size_t)dm->H * max_frames * dm->nb * dm->d;
  if (launch_pool(nullptr, K, s, dm, nullptr, kt, max_frames * dm->nb, frame0, frame1, st) != hipSuccess)
    return LF_ERR_HIP;
  return launch_frame_means(dm, kt, kh, max_frames * dm->nb, max_frames, frame0, frame0, frame1 - frame0,
                            pool_args(nullptr, nullptr, s, dm, nullptr, nullptr, 1, 0, 0), st) == hipSuccess
             ? LF_OK : LF_ERR_HIP;
}

int lf_launch_select_cached(const void* Q, const void* Kcur, void* kcache, int max_frames,
                            const lf_shape* s, const lf_budget* b, const lf_dims* dm, int32_t* indices,
                            void* workspace, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  float* qt = (float*)workspace;
  float* kt = (float*)kcache;
  const float* kh = kt + (size_t)dm->H * max_frames * dm->nb * dm->d;
  // one launch pools Q and, when the keys are given, the block means of the current chunk
  // (its frame means are not needed while it is current: the candidate frames are history)
  const hipError_t rc = Kcur ? launch_pool(Q, Kcur, s, dm, qt, kt, max_frames * dm->nb, dm->F_h, dm->F, st)
                             : launch_pool(Q, nullptr, s, dm, qt, nullptr, 1, 0, 0, st);
  if (rc != hipSuccess) return LF_ERR_HIP;
  return launch_select(b, dm, qt, kt, kh, max_frames * dm->nb, max_frames, b->n_sink, indices, st) == hipSuccess
             ? LF_OK : LF_ERR_HIP;
}

// ---------------------------------------------------------------------------------------------
// Scratch owned by the library, for callers that cannot allocate: one file-scope device array
// per GPU (every device the library's code object is loaded on holds its own copy, at its own
// address, until the process ends).  The array's name is a host-side handle, not a device
// address: its address is looked up once per device and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[LF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // zero-initialised; written once per device (same value if raced)
}

#ifdef LF_PROBE_STAMPS
// Copies the stamps of the last selection launch to host memory: [4096][8] uint64, entries 0..6 of
// a workgroup as noted above.  Returns 0 or a hipError_t.
extern "C" int lf_probe_select_stamps(void* host_out) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_stamps), sizeof(unsigned long long) * 4096 * 8);
}
#endif

int lf_static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LF_ERR_HIP;
  void* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LF_ERR_HIP;
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
  }
  *out = p;
  return LF_OK;
}
