// Blockwise sparse attention for gfx950 (Eq. 13; Eq. 3 and the paragraph after it: only
// listed tiles are computed, the element mask is never materialised).
//
// Two wavefronts per (head, query block of 64 rows), wavefront rh owning query rows
// [32 rh, 32 rh + 32) with its own online-softmax state (m, l, O): nothing crosses
// wavefronts, and there is no merge at the end.  A workgroup holds two such query blocks and two
// workgroups share a compute unit, so every SIMD holds two wavefronts, free to be in different
// parts of their step (the matrix core of one beside the vector ALU of the other).  Each listed
// KV block is taken as half tiles of 32 KV rows (two, or one when the block has at most 32
// tokens): the 32 x d K and V half tiles are brought into a double-buffered LDS
// stage by asynchronous global->LDS loads, a wavefront's share of a half tile in one group
// (V of the next step right after the barrier, K of the step after that after the first
// half of the score product).
//
// The products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
// v_mfma_f32_32x32x16_bf16: in the 32x32 accumulator layout a lane then holds one query
// column and 16 KV rows, which is exactly the B-operand layout the second product wants,
// so P never moves between lanes.  Softmax is float32, in the exp2 domain, against a lazy
// reference: P = exp2(s*c - m) with a per-row m that is moved (and O, l rescaled) only when a
// row sum shows that it has fallen too far behind the scores; the common path takes no row
// maximum.  The result is the same softmax: the reference cancels in O / l.
//
// The same per-wavefront step serves two kernels.  The list-driven one above, and a dense one
// for KV blocks that every query block of a head keeps (the always-selected current-chunk
// frames of Eq. 9): there a workgroup of 4 wavefronts owns 128 consecutive query rows and
// walks one contiguous KV token range, so a K/V half tile brought into LDS serves 4 x 32 query
// rows instead of 2 x 32 (8 wavefronts per workgroup measured slower: then the two wavefronts
// of a SIMD wait at the same barrier and run their phases in step).  The dense kernel leaves its online-softmax state (reference m, row
// sum l, unnormalised O) per query row in float32, and the list-driven kernel can start from
// such a state instead of from zero: together they compute one softmax over the union.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "lf_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int int32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxEnt = 512;  // half tiles decoded per pass (power of two)

struct AttnArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* O;
  const int32_t* idx;
  int64_t q_stride_tok, q_stride_head, k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head, o_stride_tok, o_stride_head;
  int n, nb, n_q, n_k;
  int list_len;     // entries walked per list
  int list_stride;  // entries between two lists in memory
  int total_wg, wg_per_xcd;
  float c;  // softmax_scale * log2(e)
  // Online-softmax state per query row, float32: O unnormalised [H][q_len][d] and (m, l)
  // [H][q_len].  The dense kernel writes it; the list-driven kernel starts from it when
  // state_o is not null.
  float* state_o;
  float2* state_ml;
  // list-driven kernel, optional: log2 of the row's sum of exp2(s c) over its kept columns,
  // float32 [H][q_len] (+inf for a row without a kept column), for the backward pass
  float* lse2;
  // dense kernel only: query rows per workgroup, workgroups per head, KV token range
  int q_len, rows_per_wg, wg_per_head, kv0, kv1;
};

union Frag {
  uint4 u;
  bf16x8 v;
};

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt immediate (gfx9 encoding) that waits until at most n vector-memory operations
// of this wavefront are outstanding and does not wait on the other counters.
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// 16-byte chunk swizzles of the LDS tiles (row = token within the tile, ch = 8-channel chunk).
// K is read row-wise, 16 bytes per lane, 16 consecutive rows at one logical chunk: XOR with
// the row spreads them over all banks.  V is read with the transposing 8-byte LDS read: half a
// wavefront takes 64 contiguous bytes (four chunks) from each of four consecutive rows, and the
// four rows must land in four different quarters of the 64 banks: for 256-byte rows the row's
// two low bits go to the chunk's two high bits; for 128-byte rows two consecutive rows already
// sit in different halves and the row's second bit picks the quarter.  With these the counter
// of LDS bank-conflict cycles reads zero for the kernel (it was a third of the LDS-active
// cycles with a shift of two chunks per row).  Both are unchanged by +8 and +16 rows, which the
// address arithmetic of the transposing reads relies on.
template <int CH> __device__ __forceinline__ int k_swz(int row, int ch) { return ch ^ (row & (CH - 1)); }
template <int CH> __device__ __forceinline__ int v_swz(int row, int ch) {
  return CH == 16 ? ch ^ ((row & 3) << 2) : ch ^ (((row >> 1) & 1) << 2);
}

// Workgroup barrier that orders LDS accesses only; the global->LDS loads are waited for
// explicitly (s_waitcnt vmcnt) by the wavefront that issued them, just before the barrier.
// The tile loads are inline assembly that writes M0 and LDS, declared as such ("m0", "memory"),
// so the compiler keeps LDS reads on their side of a load that reuses the buffer.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0) only: no LDS read of this wavefront is still in flight
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// WAVES wavefronts of 32 query rows each per workgroup.  DENSE: the workgroup walks the KV
// token range [kv0, kv1) and stores its state, all wavefronts sharing one tile stage.  Otherwise
// it holds WAVES / 2 query blocks of two wavefronts each, every query block with a tile stage of
// its own and walking its own list (two query blocks per workgroup measured 2 % faster than
// one); the barriers are common, the lists being equally long.
template <int D, int WAVES, bool DENSE>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void lf_attn_kernel(AttnArgs a) {
  constexpr int QPW = DENSE ? 1 : WAVES / 2;    // query blocks per workgroup
  constexpr int WPQ = WAVES / QPW;              // wavefronts that share one tile stage
  constexpr int kThreads = 64 * WPQ;            // ... and their threads
  constexpr int CH = D / 8;                 // 16-byte chunks per token row
  constexpr int KS = D / 16;                // k-steps of S^T = K Q^T
  constexpr int MB = D / 32;                // 32-row blocks of O^T
  constexpr int RPI = 64 / CH;              // tile rows one wavefront load instruction covers
  constexpr int LPW = 32 / (RPI * WPQ);     // load instructions per wavefront, per tile, per tensor
  constexpr int TILE = 32 * CH;             // uint4 per half tile (32 KV rows)
  static_assert(LPW >= 1 && LPW * RPI * WPQ == 32, "a half tile must split evenly over the wavefronts");

  __shared__ uint4 buf0_all[QPW][2 * TILE];          // K | V of even tiles
  __shared__ uint4 buf1_all[QPW][2 * TILE];          // K | V of odd tiles
  __shared__ int2 ent_all[QPW][DENSE ? 1 : kMaxEnt];   // (first token, token count <= 32) per half tile of a pass
  __shared__ int nh_all[QPW][WPQ];                      // half tiles the wavefronts decoded in a pass

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // (head, query block) pairs so that neighbours sharing KV blocks share an L2.
  const int wg = (blockIdx.x & 7) * a.wg_per_xcd + (blockIdx.x >> 3);
  const int qb = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) / WPQ;   // query block inside the workgroup
  int w = wg * QPW + qb;
  // A workgroup past the end leaves as a whole.  Inside the last one a query block past the end
  // repeats the last valid one (it has to keep step at the barriers) and stores nothing.
  if (wg * QPW >= a.total_wg) return;
  const bool w_valid = w < a.total_wg;
  w = min(w, a.total_wg - 1);
  const int per_head = DENSE ? a.wg_per_head : a.n_q;
  const int h = w / per_head, r = w % per_head;
  uint4* const buf0 = buf0_all[qb];
  uint4* const buf1 = buf1_all[qb];
  int2* const ent = ent_all[qb];
  int* const nh_mine = nh_all[qb];

  const int tid = threadIdx.x % kThreads, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront inside its query block, in a scalar register
  const int rh = wave;
  const int ln = lane & 31, kg = lane >> 5;

  // first query token and number of query rows of this workgroup: a query block of <= 64
  // tokens, or (dense) an even share of the chunk's rows, which need not follow the blocks
  const int qtok0 = DENSE ? r * a.rows_per_wg : (r / a.nb) * a.n + (r % a.nb) * 64;
  const int q_cnt = DENSE ? min(a.rows_per_wg, a.q_len - qtok0) : min(64, a.n - (r % a.nb) * 64);
  const int qrow = 32 * rh + ln;

  // The list entries of the first pass are requested first, so that they travel together with
  // the Q fragments instead of after them.
  const int32_t* list = DENSE ? nullptr : a.idx + ((int64_t)h * a.n_q + r) * a.list_stride;
  constexpr int EPT = DENSE ? 1 : kMaxEnt / 2 / kThreads;   // list entries per thread and pass (up to two half tiles each)
  int pre[EPT];
  if constexpr (!DENSE) {
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      const int i = EPT * tid + j;
      pre[j] = i < a.list_len ? list[i] : -1;
    }
  }
  // A wavefront whose 32 query rows all lie past the end of a short query block loads its share
  // of the tiles and keeps the barriers, but computes nothing.
  const bool active = DENSE || 32 * rh < q_cnt;

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

  const char* Kh = reinterpret_cast<const char*>(a.K + (int64_t)h * a.k_stride_head);
  const char* Vh = reinterpret_cast<const char*>(a.V + (int64_t)h * a.v_stride_head);
  const int64_t k_row_bytes = a.k_stride_tok * 2, v_row_bytes = a.v_stride_tok * 2;

  // Tile load, global -> LDS without passing through registers: load instruction i of
  // wavefront `wave` fills tile rows [RPI*(LPW*wave+i), +RPI); lane l lands at byte 16*l
  // of that 1 KiB stripe, so it fetches the chunk the swizzle assigns to that place.
  // Per-lane byte offsets inside a tile are loop invariants.
  const int ld_r = lane / CH, ld_p = lane % CH;
  uint32_t koff[LPW], voff[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = RPI * (LPW * wave + i) + ld_r;
    // load i carries the immediate offset 1024 i, which moves its LDS target to the i-th stripe
    // and is taken off the memory offset here (row >= RPI i and a row is at least 1024 / RPI
    // bytes, so the difference is not negative)
    koff[i] = (uint32_t)row * (uint32_t)k_row_bytes + (uint32_t)k_swz<CH>(row, ld_p) * 16u - 1024u * i;
    voff[i] = (uint32_t)row * (uint32_t)v_row_bytes + (uint32_t)v_swz<CH>(row, ld_p) * 16u - 1024u * i;
  }
  // (first token, token count) of half tile i of the pass, wavefront-uniform; past the pass's
  // last half tile an empty one (count 0: its loads touch no memory and its scores are masked).
  int nh_q = 0;   // half tiles of this query block in the current pass
  auto hent_finish = [&](int2 e, int i) -> int2 {
    const bool in = i < nh_q;
    return make_int2(__builtin_amdgcn_readfirstlane(in ? e.x : 0), __builtin_amdgcn_readfirstlane(in ? e.y : 0));
  };
  auto hent = [&](int i) -> int2 { return hent_finish(ent[i & (kMaxEnt - 1)], i); };
  // The loads are raw buffer loads whose resource is the tile itself: base = the block's
  // first token, num_records = its token count x the row pitch.  Rows past a short block's
  // count are then out of range, which touches no memory and writes zeros, so the loads need
  // no per-lane address arithmetic and no branch.  They are issued from inline assembly.
  auto tile_rsrc = [](const char* base, uint32_t row_bytes, int2 e) {
    int32x4 r;
    const uint64_t b = (uint64_t)base + (uint64_t)(uint32_t)e.x * row_bytes;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));  // stride 0: raw buffer
    r[2] = __builtin_amdgcn_readfirstlane((int)((uint32_t)e.y * row_bytes));
    r[3] = 0x00020000;
    return r;
  };
  // One write of M0 (the LDS base of this wavefront's stripes) serves all loads of a tile:
  // every further write of M0 has to wait for the loads before it.
  auto fetch_all = [&](int32x4 rs, uint4* dst, const uint32_t (&off)[LPW]) __attribute__((always_inline)) {
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)LDS_PTR(void, dst + RPI * LPW * wave * CH));
    if constexpr (LPW == 4)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %5, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %5, 0 offen offset:1024 lds\n\t"
                   "buffer_load_dwordx4 %3, %5, 0 offen offset:2048 lds\n\t"
                   "buffer_load_dwordx4 %4, %5, 0 offen offset:3072 lds"
                   :: "s"(lds0), "v"(off[0]), "v"(off[1]), "v"(off[2]), "v"(off[3]), "s"(rs) : "memory", "m0");
    else if constexpr (LPW == 2)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %3, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 lds"
                   :: "s"(lds0), "v"(off[0]), "v"(off[1]), "s"(rs) : "memory", "m0");
    else
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(lds0), "v"(off[0]), "s"(rs) : "memory", "m0");
  };
  auto k_rsrc = [&](int2 e) { return tile_rsrc(Kh, (uint32_t)k_row_bytes, e); };
  auto v_rsrc = [&](int2 e) { return tile_rsrc(Vh, (uint32_t)v_row_bytes, e); };
  auto fetch_k = [&](int32x4 rs, uint4* buf) __attribute__((always_inline)) { fetch_all(rs, buf, koff); };
  auto fetch_v = [&](int32x4 rs, uint4* buf) __attribute__((always_inline)) { fetch_all(rs, buf + TILE, voff); };

  // LDS addresses of this lane's operand fragments inside a tile (loop invariants).
  // K (A operand of S^T): row ln of the half tile, logical chunk 2 s + kg.
  int kaddr[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    const int row = ln;
    kaddr[s] = row * CH + k_swz<CH>(row, 2 * s + kg);
  }
  // V^T (A operand of O^T) through the transposing LDS read: within each group of 16 lanes,
  // lane 4e+g supplies the address of row e, columns 4g..4g+3, and lane i receives column i
  // of the four rows.  vaddr[u][half][mb] is in units of bf16 elements.
  int vbase[MB];
  {
    const int i16 = lane & 15;
    const int tr_row = 4 * kg + (i16 >> 2);
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int col = 32 * mb + tr_col;
      vbase[mb] = (tr_row * CH + v_swz<CH>(tr_row, col >> 3)) * 8 + (col & 7);
    }
  }
  // k-step u, half hf: 16 u + 8 hf rows further, which the swizzle does not notice
  auto vaddr = [&](int u, int hf, int mb) { return vbase[mb] + (16 * u + 8 * hf) * CH * 8; };

  f32x16 oacc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[mb][i] = 0.0f;
  // Online softmax in the exp2 domain with a lazily updated reference m_run: P = exp2(s c -
  // m_run) is formed without looking for the row maximum first, and m_run is checked through
  // the row sum afterwards.  It moves when the sum leaves the range below (a score far above
  // the reference; +inf if exp2 overflowed, which is also how a row's first score announces
  // itself, m_run starting at -1e30).  bfloat16 and float32 share their exponent range, so P,
  // the row sums and O stay finite far beyond that range, and O / l does not depend on m_run.
#ifdef LF_PROBE_MFMA
  // one accumulator for all the extra products: 16 registers, so that the probe build still
  // fits two wavefronts per SIMD without spilling (four accumulators made it spill, and the
  // slowdown then measured the spills)
  f32x16 probe_acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) probe_acc[i] = 0.0f;
#endif
  constexpr float kSumMax = 1.0e30f;
  float m_run = -1.0e30f, l_run = 0.0f;
  // Accumulator i of oacc[mb] is channel 32 mb + 8 (i/4) + 4 kg + i%4 of query row qrow; the
  // stored state uses the same order within a row, so a lane moves float4s.
  float* state_row = nullptr;
  if (a.state_o != nullptr && qrow < q_cnt) {
    const int64_t row = (int64_t)h * a.q_len + qtok0 + qrow;
    state_row = a.state_o + row * D;
    if constexpr (!DENSE) {
      const float2 ml = a.state_ml[row];
      m_run = ml.x;
      l_run = kg == 0 ? ml.y : 0.0f;   // the two lanes of a row each carry part of the sum
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 v = *reinterpret_cast<const float4*>(state_row + 32 * mb + 8 * g + 4 * kg);
          oacc[mb][4 * g + 0] = v.x; oacc[mb][4 * g + 1] = v.y;
          oacc[mb][4 * g + 2] = v.z; oacc[mb][4 * g + 3] = v.w;
        }
    }
  }

  // Lists are decoded kMaxEnt / 2 entries at a time into LDS: block id -> its half tiles of 32
  // KV rows (first token, count), one for a block of at most 32 tokens, two otherwise, none
  // for an id outside [0, n_k); the half tiles of a pass are stored back to back, so a step is
  // never spent on an empty upper half.  The query blocks of a workgroup share the barriers and
  // therefore take the same number of steps: the longer one's, rounded up to an even number,
  // the shorter one ending on empty half tiles.
  // The dense kernel has no list: half tile t is KV tokens [kv0 + 32 t, +32) cut at kv1 (empty
  // beyond it), all in one pass of an even number of steps.
  auto dense_half = [&](int t) {
    const int tok = a.kv0 + 32 * t;
    return make_int2(min(tok, a.kv1), min(max(a.kv1 - tok, 0), 32));
  };
  const int n_entries = DENSE ? (a.kv1 - a.kv0 + 63) / 64 : a.list_len;
  const int pass_len = DENSE ? n_entries : kMaxEnt / 2;
  for (int l0 = 0; l0 < n_entries; l0 += pass_len) {
    const int l1 = min(n_entries, l0 + pass_len);
    int nsteps = 2 * (l1 - l0);   // half-tile steps of this pass
    if constexpr (!DENSE) {
      int htok[EPT], hcnt[EPT], halves = 0;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int i = l0 + EPT * tid + e;
        const int c = i < l1 ? (l0 == 0 ? pre[e] : list[i]) : -1;
        const bool ok = (unsigned)c < (unsigned)a.n_k;
        const int tau = ok ? c / a.nb : 0, j = ok ? c % a.nb : 0;
        htok[e] = tau * a.n + j * 64;
        hcnt[e] = ok ? min(64, a.n - j * 64) : 0;
        halves += hcnt[e] > 32 ? 2 : (hcnt[e] > 0 ? 1 : 0);
      }
      // inclusive prefix of `halves` over the wavefront, then over the wavefronts through LDS
      int incl = halves;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
      }
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __syncthreads();   // the previous pass no longer reads ent / nh_all, its tile loads have landed
      if (lane == 63) nh_mine[wave] = incl;
      __syncthreads();
      int pos = incl - halves;
      nh_q = 0;
#pragma unroll
      for (int w2 = 0; w2 < WPQ; ++w2) {
        const int n = nh_mine[w2];
        if (w2 < wave) pos += n;
        nh_q += n;
      }
      nh_q = __builtin_amdgcn_readfirstlane(nh_q);
      int longest = 0;
#pragma unroll
      for (int q2 = 0; q2 < QPW; ++q2) {
        int n = 0;
#pragma unroll
        for (int w2 = 0; w2 < WPQ; ++w2) n += nh_all[q2][w2];
        longest = max(longest, n);
      }
      nsteps = __builtin_amdgcn_readfirstlane((longest + 1) & ~1);
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        if (hcnt[e] > 0) ent[pos++] = make_int2(htok[e], min(hcnt[e], 32));
        if (hcnt[e] > 32) ent[pos++] = make_int2(htok[e] + 32, hcnt[e] - 32);
      }
      __syncthreads();
      if (nsteps == 0) continue;   // no valid id in this pass, for any query block of the workgroup
    }
    // Software pipeline, one step deep (a step, "tile" below, is one half tile of 32 KV rows):
    // iteration t computes S^T of tile t+1 (matrix core)
    // next to the softmax of tile t (vector ALU), then O^T += V^T P^T of tile t.  In flight
    // while it runs: K of tile t+2 and V of tile t+1.  Buffer t&1 holds K_t and V_t.
    int2 e0, e1, e2;
    if constexpr (DENSE) {
      e0 = dense_half(0); e1 = dense_half(1); e2 = dense_half(2);
    } else {
      e0 = hent(0); e1 = hent(1); e2 = hent(2);
    }
    fetch_k(k_rsrc(e0), buf0);
    fetch_v(v_rsrc(e0), buf0);
    fetch_k(k_rsrc(e1), buf1);

    // S^T[kv, q] of this wavefront's 32 KV rows x 32 query rows, from the K tile in `kt`.
    auto s_half = [&](const uint4* kt, f32x16 acc, int s0) __attribute__((always_inline)) {
      Frag kf[KS / 2];
#pragma unroll
      for (int s = 0; s < KS / 2; ++s) kf[s].u = kt[kaddr[s0 + s]];
#pragma unroll
      for (int s = 0; s < KS / 2; ++s)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s].v, qf[s0 + s].v, acc, 0, 0, 0);
      return acc;
    };

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    lds_barrier();
    f32x16 zero16;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero16[i] = 0.0f;
    f32x16 sacc = s_half(buf0, s_half(buf0, zero16, 0), KS / 2);

    // Past the pass's last half tile the pipeline runs on empty ones: their loads touch no memory
    // and their S^T is unused, which keeps the loop body free of branches.
    auto tile = [&](int t, uint4* cur, uint4* other) __attribute__((always_inline)) {
      const int cnt = e0.y;
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this wavefront's share of K_{t+1}, V_t has landed
      lds_barrier();                             // ... everyone's has; K_t and V_{t-1} are no longer read
      // half tile t+3 is looked up now and made wavefront-uniform at the end of the step
      const int2 e_raw = DENSE ? make_int2(0, 0) : ent[(t + 3) & (kMaxEnt - 1)];
      const int32x4 krs = k_rsrc(e2), vrs = v_rsrc(e1);
      fetch_v(vrs, other);
      // accumulator i of a lane: KV row 8 (i/4) + 4 kg + i%4 of the half tile, query column ln
      if (cnt < 32) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kv = 8 * (i >> 2) + 4 * kg + (i & 3);
          if (kv >= cnt) sacc[i] = -INFINITY;
        }
      }
      f32x16 snext = s_half(other, zero16, 0);
      fetch_k(krs, cur);
      // P^T = exp2(s c - m_run), packed to bfloat16 in the
      // B-operand layout of the second product; row sums from the packed values.
      bf16x8 pf[2];
      float l_new = l_run;
      auto softmax = [&]() __attribute__((always_inline)) {
        l_new = l_run;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
          for (int e = 0; e < 8; ++e) pf[u][e] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[8 * u + e], a.c, -m_run));
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const bf16x2 pr = {pf[u][e], pf[u][e + 1]};
            const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
            l_new = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l_new, false);
          }
        }
      };
      softmax();
      snext = s_half(other, snext, KS / 2);
      // The V^T fragments of the first k-step are requested before the branch below, so that
      // the second product does not start by waiting for LDS.
      const uint16_t* Vs16 = reinterpret_cast<const uint16_t*>(cur + TILE);
      bf16x8 vf0[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, Vs16 + vaddr(0, 0, mb)));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, Vs16 + vaddr(0, 1, mb)));
        vf0[mb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
      // Rare: the row sum says the reference is far too low (or was never set).  Then the
      // maxima are taken, the reference moves up to them and P^T is made again.
      if (__ballot(l_new > kSumMax) != 0ull) {
        float mx = fmaxf(fmaxf(sacc[0], sacc[1]), fmaxf(sacc[2], sacc[3]));
#pragma unroll
        for (int i = 4; i < 16; i += 2) mx = fmaxf(mx, fmaxf(sacc[i], sacc[i + 1]));
        // lanes l and l+32 hold the same query column: exchange through the lane-swap unit
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        const float m_new = fmaxf(m_run, mx * a.c);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[mb][i] *= alpha;
        softmax();
      }
      l_run = l_new;

      // O^T[d, q] += V^T[d, kv] P^T[kv, q]; k-step u takes accumulators 8u .. 8u+7, i.e.
      // KV rows 16u + 4kg + {0..3} and 16u + 8 + 4kg + {0..3} of this wavefront's half.
      // The second product runs at low priority, the score/softmax part at high priority: with
      // two wavefronts per SIMD this helps to keep them in different parts of the step.
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf0[mb], pf[0], oacc[mb], 0, 0, 0);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, Vs16 + vaddr(1, 0, mb)));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, Vs16 + vaddr(1, 1, mb)));
        const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[1], oacc[mb], 0, 0, 0);
      }
      // Probe builds only (liblf_hsa_probe_*.so, for `bench.py --sensitivity`): redundant work added
      // to every step to see how much the step lengthens when one unit gets more to do.  The extra
      // results are discarded (the extra products go to an accumulator of their own), the output
      // is unchanged.
#ifdef LF_PROBE_TR   // +16 transposing V reads (+100 %)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, Vs16 + vaddr(u, 0, mb)));
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, Vs16 + vaddr(u, 1, mb)));
          asm volatile("" :: "v"(lo), "v"(hi));
        }
#endif
#ifdef LF_PROBE_K    // +8 K fragment reads (+100 %)
#pragma unroll
      for (int s2 = 0; s2 < KS; ++s2) {
        const uint4 kk = other[kaddr[s2]];
        asm volatile("" :: "v"(kk.x), "v"(kk.y), "v"(kk.z), "v"(kk.w));
      }
#endif
#ifdef LF_PROBE_MFMA // +8 matrix instructions (+50 %)
#pragma unroll
      for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          probe_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf0[mb], pf[r2], probe_acc, 0, 0, 0);
#endif
#ifdef LF_PROBE_EXP  // +16 exp2 (+100 %)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float ex = __builtin_amdgcn_exp2f(snext[i] * 1.0e-3f);
        asm volatile("" :: "v"(ex));
      }
#endif
      __builtin_amdgcn_s_setprio(3);
      sacc = snext;
      e0 = e1;
      e1 = e2;
      if constexpr (DENSE) e2 = dense_half(t + 3);
      else e2 = hent_finish(e_raw, t + 3);
    };
    // The step of a wavefront without query rows: its share of the loads, and the barrier.
    auto tile_idle = [&](int t, uint4* cur, uint4* other) __attribute__((always_inline)) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      lds_barrier();
      const int2 e_raw = ent[(t + 3) & (kMaxEnt - 1)];
      const int32x4 krs = k_rsrc(e2), vrs = v_rsrc(e1);
      fetch_v(vrs, other);
      fetch_k(krs, cur);
      e0 = e1;
      e1 = e2;
      e2 = hent_finish(e_raw, t + 3);
    };
    if (active) {
      for (int t = 0; t < nsteps; t += 2) {
        tile(t, buf0, buf1);
        tile(t + 1, buf1, buf0);
      }
    } else {
      for (int t = 0; t < nsteps; t += 2) {
        tile_idle(t, buf0, buf1);
        tile_idle(t + 1, buf1, buf0);
      }
    }
  }

#ifdef LF_PROBE_MFMA
  {
    float sd = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) sd += probe_acc[i];
    if (sd == -123.0f) l_run += 1.0f;   // practically never true: keeps the extra products alive
  }
#endif
  // Every wavefront owns its 32 query rows completely.
  l_run += __shfl_xor(l_run, 32);
  if constexpr (DENSE) {
    // leave the state for the list-driven kernel to continue from
    if (state_row != nullptr) {
      if (kg == 0) a.state_ml[(int64_t)h * a.q_len + qtok0 + qrow] = make_float2(m_run, l_run);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(state_row + 32 * mb + 8 * g + 4 * kg) =
              make_float4(oacc[mb][4 * g + 0], oacc[mb][4 * g + 1], oacc[mb][4 * g + 2], oacc[mb][4 * g + 3]);
    }
    return;
  }
  // normalise and store
  const float inv = l_run > 0.0f ? 1.0f / l_run : 0.0f;   // a list without a valid id gives zero rows
  if (qrow < q_cnt && w_valid) {
    if (a.lse2 != nullptr && kg == 0)
      a.lse2[(int64_t)h * a.q_len + qtok0 + qrow] = l_run > 0.0f ? m_run + __builtin_log2f(l_run) : INFINITY;
    uint16_t* op = a.O + (int64_t)h * a.o_stride_head + (int64_t)(qtok0 + qrow) * a.o_stride_tok;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[mb][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(op + 32 * mb + 8 * g + 4 * kg) = o4;
      }
    }
  }
}

}  // namespace

static AttnArgs attn_args(const void* Q, const void* K, const void* V, const lf_shape* s,
                          const lf_dims* dm, float scale) {
  AttnArgs a = {};
  a.Q = (const uint16_t*)Q;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
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
  a.q_len = dm->f * dm->n;
  a.c = scale * 1.4426950408889634f;
  return a;
}

// List-driven kernel: walks the first list_len entries of every list (lists are list_stride
// entries apart); with a state (state_o, state_ml) it continues that online softmax.
int lf_launch_attn(const void* Q, const void* K, const void* V, const lf_shape* s,
                   const lf_dims* dm, const int32_t* indices, int32_t list_len, int32_t list_stride,
                   float scale, void* O, const float* state_o, const float* state_ml, float* lse2,
                   void* stream) {
  AttnArgs a = attn_args(Q, K, V, s, dm, scale);
  a.O = (uint16_t*)O;
  a.lse2 = lse2;
  a.idx = indices;
  a.list_len = list_len;
  a.list_stride = list_stride;
  a.state_o = const_cast<float*>(state_o);
  a.state_ml = reinterpret_cast<float2*>(const_cast<float*>(state_ml));
  a.total_wg = dm->H * dm->n_q;
  constexpr int kListWaves = 4;                  // two query blocks per workgroup
  const int n_wg = (a.total_wg + kListWaves / 2 - 1) / (kListWaves / 2);
  a.wg_per_xcd = (n_wg + 7) / 8;
  const unsigned grid = (unsigned)(a.wg_per_xcd * 8);
  hipStream_t st = (hipStream_t)stream;
  const hipError_t rc = dm->d == 128
      ? lf_launch(lf_attn_kernel<128, kListWaves, false>, dim3(grid), dim3(64 * kListWaves), 0, st, a)
      : lf_launch(lf_attn_kernel<64, kListWaves, false>, dim3(grid), dim3(64 * kListWaves), 0, st, a);
  return rc == hipSuccess ? LF_OK : LF_ERR_HIP;
}

// Dense kernel over KV tokens [kv0, kv1) for every query row of every head; writes the state.
// The rows of a head are dealt evenly to ceil(q_len / (32 WAVES)) workgroups.
int lf_launch_attn_dense(const void* Q, const void* K, const void* V, const lf_shape* s,
                         const lf_dims* dm, int kv0, int kv1, float scale, float* state_o,
                         float* state_ml, void* stream) {
  AttnArgs a = attn_args(Q, K, V, s, dm, scale);
  a.state_o = state_o;
  a.state_ml = reinterpret_cast<float2*>(state_ml);
  a.kv0 = kv0;
  a.kv1 = kv1;
  constexpr int kDenseWaves = 4;            // 128 query rows per workgroup, two workgroups per CU
  const int rows_max = 32 * kDenseWaves;
  a.wg_per_head = (a.q_len + rows_max - 1) / rows_max;
  a.rows_per_wg = (a.q_len + a.wg_per_head - 1) / a.wg_per_head;
  a.total_wg = dm->H * a.wg_per_head;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  const unsigned grid = (unsigned)(a.wg_per_xcd * 8);
  hipStream_t st = (hipStream_t)stream;
  const hipError_t rc = dm->d == 128
      ? lf_launch(lf_attn_kernel<128, kDenseWaves, true>, dim3(grid), dim3(64 * kDenseWaves), 0, st, a)
      : lf_launch(lf_attn_kernel<64, kDenseWaves, true>, dim3(grid), dim3(64 * kDenseWaves), 0, st, a);
  return rc == hipSuccess ? LF_OK : LF_ERR_HIP;
}
