// Backward pass of the blockwise sparse attention (Eq. 13) for gfx950: gradients with respect
// to Q, K and V for an upstream gradient dO, over exactly the tiles the index lists keep
// (the paper finetunes with the sparse mask in place, Sec. 5 "Experimental Details").
//
// With s_xy = scale q_x.k_y, p = softmax over the kept columns, o = p v:
//     dV_y = sum_x p_xy dO_x          dp_xy = dO_x . v_y      delta_x = dO_x . o_x
//     ds_xy = p_xy (dp_xy - delta_x)  dQ_x = scale sum_y ds_xy k_y    dK_y = scale sum_x ds_xy q_x
// p is rebuilt from the row's log-sum-exp, which the training forward call leaves (in the exp2
// domain: lse2_x = log2 sum_y exp2(s_xy log2 e)), so no row maximum or sum is needed here.
//
// No atomics and a fixed summation order: every launch owns its outputs.  The dQ launch is
// query-major (a workgroup owns a query block, walks its list of KV blocks, keeps dQ in
// registers); the dK/dV launch is key-major (a workgroup owns a KV block and walks the list of
// query blocks that keep it -- the transposed lists, made by a small kernel -- and keeps dK and dV
// in registers).  Both recompute the scores of a tile.  The products are arranged as in the
// forward kernel: the "score-like" products S' = A1 X^T and dP' = A2 Y^T take their A operand
// from a 32-row tile in LDS (row reads) and their B operand from registers that hold the owner
// block, which leaves a lane with one owner column and 16 stream rows; P' and dS' are then
// already in the B-operand layout of the accumulating product, whose A operand is the same tile
// read through the transposing LDS read.
//     dQ:      owner = query block (X = Q, Y = dO), stream = KV blocks (A1 = K, A2 = V),
//              dQ^T += K^T dS'
//     dK, dV:  owner = KV block (X = K, Y = V), stream = query blocks (A1 = Q, A2 = dO),
//              dK^T += Q^T dS'  and  dV^T += dO^T P', by two kinds of wavefront that share P'
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "lf_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int int32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 128;    // two wavefronts of 32 owner rows each
constexpr int kPass = 256;       // list entries decoded per pass

struct BwdArgs {
  const uint16_t* X;     // owner-side operand of the scores (Q for dQ, K for dK and dV)
  const uint16_t* Y;     // owner-side operand of dP (dO for dQ, V for dK)
  const uint16_t* A1;    // streamed operand of the scores (K for dQ, Q for dK and dV)
  const uint16_t* A2;    // streamed operand of dP (V for dQ, dO for dK and dV)
  uint16_t* out1;        // dQ or dK: scale * sum of A1^T dS'
  uint16_t* out2;        // dV: sum of A2^T P'
  const float2* stats;   // (lse2, delta) per query row, [H][q_len]
  const int32_t* idx;    // lists: [H][owners][list_stride]
  const int32_t* cnt;    // key-major: entries per transposed list
  const int32_t* order;  // key-major: owner handled by workgroup slot w
  int64_t x_tok, x_head, y_tok, y_head, a1_tok, a1_head, a2_tok, a2_head;
  int64_t o1_tok, o1_head, o2_tok, o2_head;
  int n, nb, owners, streams, list_len, list_stride, q_len;
  int total_wg, wg_per_xcd;
  float c, scale;
};

union Frag {
  uint4 u;
  bf16x8 v;
};

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// One swizzle for both tiles of a step, since each is read both ways.  Row reads: 16 bytes per
// lane, 16 consecutive rows at one logical chunk per quarter wavefront, which must land in 16
// different chunks.  Transposing reads: half a wavefront takes four consecutive chunks from each
// of four consecutive rows (4 k .. 4 k + 3), which must land in four different quarters of the
// banks.  For 256-byte rows: the row's two low bits go to the chunk's two high bits (the four
// rows of a transposing read differ there), the next two row bits to the chunk's two low bits
// (constant within a transposing read, and together a bijection of the 16 rows of a row read).
template <int CH> __device__ __forceinline__ int swz(int row, int ch) {
  return CH == 16 ? ch ^ (((row & 3) << 2) | ((row >> 2) & 3)) : ch ^ ((row & 1) << 2);
}
// The transposing read of rows 8..15 of a 16-row group sees row bit 3, i.e. chunk bit 1, flipped:
// 16 elements aside.
template <int CH> constexpr int kTrHiFlip = CH == 16 ? 16 : 0;

__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// dQ: a workgroup of two wavefronts owns a query block (wavefront rh its rows [32 rh, +32)) and
// walks the block's list of KV blocks in half tiles of 32 KV rows.
template <int D>
__global__ __launch_bounds__(kThreads, 2) void lf_attn_bwd_q_kernel(BwdArgs a) {
  constexpr int CH = D / 8;
  constexpr int KS = D / 16;
  constexpr int MB = D / 32;
  constexpr int RPI = 64 / CH;
  constexpr int LPW = 32 / (RPI * 2);
  constexpr int TILE = 32 * CH;             // uint4 per 32-row tile
  constexpr int NBUF = 2;

  __shared__ uint4 buf[NBUF][2 * TILE];     // [step mod NBUF][A1 tile | A2 tile]
  __shared__ int2 ent[kPass];               // (first token, token count) per list entry of a pass

  const int w = (blockIdx.x & 7) * a.wg_per_xcd + (blockIdx.x >> 3);
  if (w >= a.total_wg) return;
  const int h = w / a.owners, r = w % a.owners;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 31, kg = lane >> 5;

  // owner block: tokens [otok0, otok0 + o_cnt); this lane's owner row (a column of S')
  const int otok0 = (r / a.nb) * a.n + (r % a.nb) * 64;
  const int o_cnt = min(64, a.n - (r % a.nb) * 64);
  const int orow = 32 * wave + ln;
  const bool o_ok = orow < o_cnt;

  const int32_t* list = a.idx + ((int64_t)h * a.owners + r) * a.list_stride;
  const int n_ent = a.list_len;

  // B operands: lane (column ln, k-group kg) holds 8 consecutive channels of its owner row
  Frag xf[KS], yf[KS];
  {
    const uint16_t* xp = a.X + (int64_t)h * a.x_head + (int64_t)(otok0 + orow) * a.x_tok;
    const uint16_t* yp = a.Y + (int64_t)h * a.y_head + (int64_t)(otok0 + orow) * a.y_tok;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      xf[s].u = o_ok ? *reinterpret_cast<const uint4*>(xp + s * 16 + kg * 8) : make_uint4(0, 0, 0, 0);
      yf[s].u = o_ok ? *reinterpret_cast<const uint4*>(yp + s * 16 + kg * 8) : make_uint4(0, 0, 0, 0);
    }
  }
  // dQ: the query row of this lane; its log-sum-exp and delta (a row outside the block gets
  // +inf, which makes all its probabilities zero)
  float2 mine = make_float2(INFINITY, 0.0f);
  if (o_ok) mine = a.stats[(int64_t)h * a.q_len + otok0 + orow];

  const char* A1h = reinterpret_cast<const char*>(a.A1 + (int64_t)h * a.a1_head);
  const char* A2h = reinterpret_cast<const char*>(a.A2 + (int64_t)h * a.a2_head);
  const uint32_t a1_row_bytes = (uint32_t)(a.a1_tok * 2), a2_row_bytes = (uint32_t)(a.a2_tok * 2);

  // tile loads, global -> LDS (see the forward kernel): load i of wavefront `wave` fills rows
  // [RPI (LPW wave + i), +RPI); the buffer resource is the tile itself, so rows past the count
  // read as zeros and ids outside the tensor become empty tiles
  const int ld_r = lane / CH, ld_p = lane % CH;
  uint32_t off1[LPW], off2[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = RPI * (LPW * wave + i) + ld_r;
    off1[i] = (uint32_t)row * a1_row_bytes + (uint32_t)swz<CH>(row, ld_p) * 16u - 1024u * i;
    off2[i] = (uint32_t)row * a2_row_bytes + (uint32_t)swz<CH>(row, ld_p) * 16u - 1024u * i;
  }
  auto rsrc = [](const char* base, uint32_t row_bytes, int2 e) {
    int32x4 rs;
    const uint64_t b = (uint64_t)base + (uint64_t)(uint32_t)e.x * row_bytes;
    rs[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    rs[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
    rs[2] = __builtin_amdgcn_readfirstlane((int)((uint32_t)e.y * row_bytes));
    rs[3] = 0x00020000;
    return rs;
  };
  auto fetch = [&](int32x4 rs, uint4* dst, const uint32_t (&off)[LPW]) __attribute__((always_inline)) {
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)LDS_PTR(void, dst + RPI * LPW * wave * CH));
    if constexpr (LPW == 4)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %5, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %5, 0 offen offset:1024 lds\n\t"
                   "buffer_load_dwordx4 %3, %5, 0 offen offset:2048 lds\n\t"
                   "buffer_load_dwordx4 %4, %5, 0 offen offset:3072 lds"
                   :: "s"(lds0), "v"(off[0]), "v"(off[1]), "v"(off[2]), "v"(off[3]), "s"(rs) : "memory", "m0");
    else
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %3, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 lds"
                   :: "s"(lds0), "v"(off[0]), "v"(off[1]), "s"(rs) : "memory", "m0");
  };
  // half tile t of the pass: list entry t/2, rows [32 (t&1), +32) of its block
  auto half = [&](int t, int n_local) {
    const int2 e = ent[min(t >> 1, n_local - 1)];
    const int2 u = make_int2(__builtin_amdgcn_readfirstlane(e.x), __builtin_amdgcn_readfirstlane(e.y));
    return (t & 1) ? make_int2(u.x + 32, max(u.y - 32, 0)) : make_int2(u.x, min(u.y, 32));
  };
  auto request = [&](int t, int n_local) __attribute__((always_inline)) {
    const int2 e = half(t, n_local);
    fetch(rsrc(A1h, a1_row_bytes, e), buf[t % NBUF], off1);
    fetch(rsrc(A2h, a2_row_bytes, e), buf[t % NBUF] + TILE, off2);
  };

  // LDS addresses of this lane's fragments (loop invariants): row reads of row ln, chunk 2s+kg
  int raddr[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) raddr[s] = ln * CH + swz<CH>(ln, 2 * s + kg);
  // transposing reads (see the forward kernel), in bf16 elements
  int tbase[MB];
  {
    const int i16 = lane & 15;
    const int tr_row = 4 * kg + (i16 >> 2);
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int col = 32 * mb + tr_col;
      tbase[mb] = (tr_row * CH + swz<CH>(tr_row, col >> 3)) * 8 + (col & 7);
    }
  }
  auto tfrag = [&](const uint4* tile, int u, int mb) __attribute__((always_inline)) {
    const uint16_t* p16 = reinterpret_cast<const uint16_t*>(tile);
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p16 + tbase[mb] + (16 * u) * CH * 8));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        LDS_PTR(bf16x4, p16 + (tbase[mb] ^ kTrHiFlip<CH>) + (16 * u + 8) * CH * 8));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;
  f32x16 zero16;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero16[i] = 0.0f;

  // S'[stream row, owner column] = A1 X^T and dP' = A2 Y^T of this wavefront's 32 x 32 tile.
  // The fragment reads are kept KS/2 k-steps ahead of the products that use them (the compiler,
  // left alone, issues each read right before its product and waits for it); the scheduling
  // barriers pin that order.
  auto scores = [&](const uint4* tile, f32x16& sacc, f32x16& pacc) __attribute__((always_inline)) {
    constexpr int HB = KS / 2;
    Frag f1[HB], f2[HB];
    sacc = zero16;
    pacc = zero16;
#pragma unroll
    for (int s = 0; s < HB; ++s) {
      f1[s].u = tile[raddr[s]];
      f2[s].u = tile[TILE + raddr[s]];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < HB; ++s) {
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[s].v, xf[s].v, sacc, 0, 0, 0);
      f1[s].u = tile[raddr[HB + s]];
      pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[s].v, yf[s].v, pacc, 0, 0, 0);
      f2[s].u = tile[TILE + raddr[HB + s]];
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int s = 0; s < HB; ++s) {
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[s].v, xf[HB + s].v, sacc, 0, 0, 0);
      pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[s].v, yf[HB + s].v, pacc, 0, 0, 0);
    }
  };
  // P' = exp2(s c - lse2), dS' = P' (dP' - delta), packed to bfloat16 in the B-operand layout of
  // the accumulating product; accumulator i is stream row 8 (i/4) + 4 kg + i%4
  auto probs = [&](f32x16& sacc, const f32x16& pacc, int cnt, bf16x8 (&dsf)[2]) __attribute__((always_inline)) {
    // stream rows past a short half tile's count were loaded as zeros: their scores become -inf
    // (P' = 0); a full half tile, the common case, skips this
    if (cnt < 32) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (8 * (i >> 2) + 4 * kg + (i & 3) >= cnt) sacc[i] = -INFINITY;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], a.c, -mine.x));
      dsf[i >> 3][i & 7] = (__bf16)(p * (pacc[i] - mine.y));
    }
  };
  // acc += K^T dS'.  The transposed fragments of the first 16
  // stream rows are requested by `first_half` before the exp2 work, which covers their latency;
  // those of the second 16 rows are requested between the products of the first.
  auto first_half = [&](const uint4* tile, bf16x8 (&tf)[MB]) __attribute__((always_inline)) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) tf[mb] = tfrag(tile, 0, mb);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto accumulate = [&](const uint4* tile, bf16x8 (&tf)[MB], const bf16x8 (&dsf)[2]) __attribute__((always_inline)) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[mb], dsf[0], acc[mb], 0, 0, 0);
      tf[mb] = tfrag(tile, 1, mb);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
      acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[mb], dsf[1], acc[mb], 0, 0, 0);
  };

  for (int l0 = 0; l0 < n_ent; l0 += kPass) {
    const int l1 = min(n_ent, l0 + kPass);
    const int n_local = l1 - l0, steps = 2 * n_local;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    for (int i = tid; i < n_local; i += kThreads) {
      const int cidx = list[l0 + i];
      const bool ok = (unsigned)cidx < (unsigned)a.streams;
      const int tau = ok ? cidx / a.nb : 0, j = ok ? cidx % a.nb : 0;
      ent[i] = make_int2(tau * a.n + j * 64, ok ? min(64, a.n - j * 64) : 0);
    }
    __syncthreads();

    // step t uses buf[t & 1]; its tiles are requested one step ahead
    request(0, n_local);
    for (int t = 0; t < steps; ++t) {
      const int cnt = half(t, n_local).y;
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      lds_barrier();
      if (t + 1 < steps) request(t + 1, n_local);
      f32x16 sacc, pacc;
      bf16x8 dsf[2];
      bf16x8 tf[MB];
      scores(buf[t & 1], sacc, pacc);
      first_half(buf[t & 1], tf);
      probs(sacc, pacc, cnt, dsf);
      // the accumulating products run at low priority, scores and exp2 at high priority: with
      // two wavefronts per SIMD this helps to keep them in different parts of the step
      __builtin_amdgcn_s_setprio(0);
      accumulate(buf[t & 1], tf, dsf);
      __builtin_amdgcn_s_setprio(3);
    }
  }

  // accumulator i of acc[mb] is channel 32 mb + 8 (i/4) + 4 kg + i%4 of the owner row
  if (o_ok) {
    uint16_t* op = a.out1 + (int64_t)h * a.o1_head + (int64_t)(otok0 + orow) * a.o1_tok;
    const float factor = a.scale;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc[mb][4 * g + e] * factor);
        *reinterpret_cast<bf16x4*>(op + 32 * mb + 8 * g + 4 * kg) = o4;
      }
  }
}

// dK and dV in one launch without computing the scores twice: a workgroup of four wavefronts
// owns one KV block and walks the query blocks that keep it in half tiles of 32 query rows.
// Wavefront i = (rh, role): rh = owner row half; role 0 computes S' = Q K^T, P' and
// dV^T += dO^T P'; role 1 computes dP' = dO V^T, dS' = P' (dP' - delta) and dK^T += Q^T dS'.
// P' goes from the role-0 wavefront to its role-1 partner (same rh: the same lanes hold the same
// elements) through LDS, and the partner uses it one step later, so the one barrier per step is
// enough; a tile therefore lives for two steps and the stage is triple-buffered.  Each wavefront
// keeps one owner operand and one accumulator set, which fits two wavefronts per SIMD (two
// workgroups per CU, not in step with each other).
constexpr int kKvThreads = 256;
template <int D>
__global__ __launch_bounds__(kKvThreads, 2) void lf_attn_bwd_kv_kernel(BwdArgs a) {
  constexpr int CH = D / 8;
  constexpr int KS = D / 16;
  constexpr int MB = D / 32;
  constexpr int RPI = 64 / CH;              // tile rows one wavefront load instruction covers
  constexpr int LPW = 32 / (RPI * 4);       // load instructions per wavefront, per tensor, per half tile
  constexpr int T32 = 32 * CH;              // uint4 per half tile (32 rows)
  static_assert(LPW == 1 || LPW == 2, "a half tile splits over four wavefronts");

  __shared__ uint4 buf[3][2 * T32];         // [half tile mod 3][Q | dO]
  __shared__ float2 st[3][4][32];           // (lse2, delta) of the 32 streamed rows, one copy per wavefront
  __shared__ uint4 ph[2][2][2][64];         // P' handoff: [step parity][rh][k-step][lane]
  __shared__ int2 ent[kPass];

  const int slot = (blockIdx.x & 7) * a.wg_per_xcd + (blockIdx.x >> 3);
  if (slot >= a.total_wg) return;
  const int w = a.order[slot];
  const int h = w / a.owners, r = w % a.owners;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rh = wave & 1, pair = rh;
  const bool is_ds = wave >= 2;             // role 1: dP', dS', dK
  const int ln = lane & 31, kg = lane >> 5;

  const int otok0 = (r / a.nb) * a.n + (r % a.nb) * 64;
  const int o_cnt = min(64, a.n - (r % a.nb) * 64);
  const int orow = 32 * rh + ln;
  const bool o_ok = orow < o_cnt;
  const int32_t* list = a.idx + ((int64_t)h * a.owners + r) * a.list_stride;
  const int n_ent = a.cnt[(int64_t)h * a.owners + r];

  // owner operand: K rows for role 0 (scores), V rows for role 1 (dP')
  Frag of[KS];
  {
    const uint16_t* op = is_ds ? a.Y + (int64_t)h * a.y_head + (int64_t)(otok0 + orow) * a.y_tok
                               : a.X + (int64_t)h * a.x_head + (int64_t)(otok0 + orow) * a.x_tok;
#pragma unroll
    for (int s = 0; s < KS; ++s)
      of[s].u = o_ok ? *reinterpret_cast<const uint4*>(op + s * 16 + kg * 8) : make_uint4(0, 0, 0, 0);
  }

  const char* A1h = reinterpret_cast<const char*>(a.A1 + (int64_t)h * a.a1_head);
  const char* A2h = reinterpret_cast<const char*>(a.A2 + (int64_t)h * a.a2_head);
  const char* STh = reinterpret_cast<const char*>(a.stats + (int64_t)h * a.q_len);
  const uint32_t a1_row_bytes = (uint32_t)(a.a1_tok * 2), a2_row_bytes = (uint32_t)(a.a2_tok * 2);

  // tile loads: wavefront `wave` fills rows [8 wave, +8) of a half tile with LPW instructions
  const int ld_r = lane / CH, ld_p = lane % CH;
  uint32_t off1[LPW], off2[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = RPI * (LPW * wave + i) + ld_r;
    off1[i] = (uint32_t)row * a1_row_bytes + (uint32_t)swz<CH>(row, ld_p) * 16u - 1024u * i;
    off2[i] = (uint32_t)row * a2_row_bytes + (uint32_t)swz<CH>(row, ld_p) * 16u - 1024u * i;
  }
  const uint32_t st_off = (uint32_t)lane * 4u;
  auto rsrc = [](const char* base, uint32_t row_bytes, int first, int count) {
    int32x4 rs;
    const uint64_t b = (uint64_t)base + (uint64_t)(uint32_t)first * row_bytes;
    rs[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    rs[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
    rs[2] = __builtin_amdgcn_readfirstlane((int)((uint32_t)count * row_bytes));
    rs[3] = 0x00020000;
    return rs;
  };
  auto fetch = [&](int32x4 rs, uint4* dst, const uint32_t (&off)[LPW]) __attribute__((always_inline)) {
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)LDS_PTR(void, dst + RPI * LPW * wave * CH));
    if constexpr (LPW == 2)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %3, 0 offen lds\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 lds"
                   :: "s"(lds0), "v"(off[0]), "v"(off[1]), "s"(rs) : "memory", "m0");
    else
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(lds0), "v"(off[0]), "s"(rs) : "memory", "m0");
  };
  // half tile t of the pass: list entry t/2, rows [32 (t&1), +32) of its block
  auto half = [&](int t) {
    const int2 e = ent[t >> 1];
    const int2 u = make_int2(__builtin_amdgcn_readfirstlane(e.x), __builtin_amdgcn_readfirstlane(e.y));
    return (t & 1) ? make_int2(u.x + 32, max(u.y - 32, 0)) : make_int2(u.x, min(u.y, 32));
  };
  // half tile t -> stage t mod 3: the Q and dO rows and the (lse2, delta) pairs (every wavefront its own copy)
  auto request = [&](int t, int stage) __attribute__((always_inline)) {
    const int2 e = half(t);
    fetch(rsrc(A1h, a1_row_bytes, e.x, e.y), buf[stage], off1);
    fetch(rsrc(A2h, a2_row_bytes, e.x, e.y), buf[stage] + T32, off2);
    const int32x4 rs = rsrc(STh, 8u, e.x, e.y);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(void, st[stage][wave]));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "buffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(lds0), "v"(st_off), "s"(rs) : "memory", "m0");
  };

  int raddr[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) raddr[s] = ln * CH + swz<CH>(ln, 2 * s + kg);
  int tbase[MB];
  {
    const int i16 = lane & 15;
    const int tr_row = 4 * kg + (i16 >> 2);
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int col = 32 * mb + tr_col;
      tbase[mb] = (tr_row * CH + swz<CH>(tr_row, col >> 3)) * 8 + (col & 7);
    }
  }
  auto tfrag = [&](const uint4* tile, int u, int mb) __attribute__((always_inline)) {
    const uint16_t* p16 = reinterpret_cast<const uint16_t*>(tile);
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(LDS_PTR(bf16x4, p16 + tbase[mb] + (16 * u) * CH * 8));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        LDS_PTR(bf16x4, p16 + (tbase[mb] ^ kTrHiFlip<CH>) + (16 * u + 8) * CH * 8));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };

  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;
  f32x16 zero16;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero16[i] = 0.0f;

  // the score-like product of this wavefront's role: rows of `tile` times the owner operand
  auto product = [&](const uint4* tile) __attribute__((always_inline)) {
    constexpr int HB = KS / 2;
    Frag f[HB];
    f32x16 c = zero16;
#pragma unroll
    for (int s = 0; s < HB; ++s) f[s].u = tile[raddr[s]];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < HB; ++s) {
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[s].v, of[s].v, c, 0, 0, 0);
      f[s].u = tile[raddr[HB + s]];
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int s = 0; s < HB; ++s) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[s].v, of[HB + s].v, c, 0, 0, 0);
    return c;
  };
  // acc += tile^T (transposing reads) times b[0], b[1]
  auto accumulate = [&](const uint4* tile, const bf16x8 (&b)[2]) __attribute__((always_inline)) {
    bf16x8 tf[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) tf[mb] = tfrag(tile, 0, mb);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[mb], b[0], acc[mb], 0, 0, 0);
      tf[mb] = tfrag(tile, 1, mb);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
      acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf[mb], b[1], acc[mb], 0, 0, 0);
  };
  // accumulator i of a score tile is streamed row 8 (i/4) + 4 kg + i%4; the (lse2, delta)
  // pairs of rows 8 g + 4 kg .. + 3 are two 16-byte reads
  auto stats4 = [&](const float2* strow, int g, float (&lse)[4], float (&dl)[4]) __attribute__((always_inline)) {
    const float4 sa = *reinterpret_cast<const float4*>(strow + 8 * g + 4 * kg);
    const float4 sb = *reinterpret_cast<const float4*>(strow + 8 * g + 4 * kg + 2);
    lse[0] = sa.x; lse[1] = sa.z; lse[2] = sb.x; lse[3] = sb.z;
    dl[0] = sa.y; dl[1] = sa.w; dl[2] = sb.y; dl[3] = sb.w;
  };

  for (int l0 = 0; l0 < n_ent; l0 += kPass) {
    const int n_local = min(n_ent - l0, kPass);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    for (int i = tid; i < n_local; i += kKvThreads) {
      const int cidx = list[l0 + i];
      const bool ok = (unsigned)cidx < (unsigned)a.streams;
      const int tau = ok ? cidx / a.nb : 0, j = ok ? cidx % a.nb : 0;
      ent[i] = make_int2(tau * a.n + j * 64, ok ? min(64, a.n - j * 64) : 0);
    }
    __syncthreads();

    // Step t: half tile t is in stage t mod 3 (requested a step ago), half tile t-1 still in its
    // stage.  Role 0 works on t; role 1 forms dP' of t and finishes t-1 with the P' its partner
    // left during step t-1.  The first step has nothing to finish and the last one only finishes,
    // so they are peeled off and the loop body has no condition but the role.
    const int steps = 2 * n_local;
    f32x16 dp_prev = zero16;
    int cur = 0, nxt = 1, prv = 2;
    auto rotate = [&]() { const int was = prv; prv = cur; cur = nxt; nxt = was; };
    // role 0 on half tile t (stage cur): S', P' (handed over), dV^T += dO^T P'
    auto p_step = [&](int t) __attribute__((always_inline)) {
      const int cnt = half(t).y;
      f32x16 sacc = product(buf[cur]);
      // stream rows past a short half tile's count were loaded as zeros (scores and statistics
      // alike): their scores become -inf (P' = 0); a full half tile, the common case, skips this
      if (cnt < 32) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (8 * (i >> 2) + 4 * kg + (i & 3) >= cnt) sacc[i] = -INFINITY;
      }
      bf16x8 pf[2];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float lse[4], dl[4];
        stats4(st[cur][wave], g, lse, dl);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * g + e;
          pf[i >> 3][i & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[i], a.c, -lse[e]));
        }
      }
      ph[t & 1][pair][0][lane] = __builtin_bit_cast(uint4, pf[0]);
      ph[t & 1][pair][1][lane] = __builtin_bit_cast(uint4, pf[1]);
      accumulate(buf[cur] + T32, pf);
    };
    // role 1 finishing half tile t (stage prv): dS' = P' (dP' - delta), dK^T += Q^T dS'
    auto ds_finish = [&](int t) __attribute__((always_inline)) {
      bf16x8 pf[2], dsf[2];
      pf[0] = __builtin_bit_cast(bf16x8, ph[t & 1][pair][0][lane]);
      pf[1] = __builtin_bit_cast(bf16x8, ph[t & 1][pair][1][lane]);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float lse[4], dl[4];
        stats4(st[prv][wave], g, lse, dl);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * g + e;
          dsf[i >> 3][i & 7] = (__bf16)((float)pf[i >> 3][i & 7] * (dp_prev[i] - dl[e]));
        }
      }
      accumulate(buf[prv], dsf);
    };
    request(0, 0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    lds_barrier();
    request(1, nxt);                       // steps >= 2: a list entry is two half tiles
    if (!is_ds) p_step(0); else dp_prev = product(buf[cur] + T32);
    rotate();
    for (int t = 1; t < steps; ++t) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      lds_barrier();
      if (t + 1 < steps) request(t + 1, nxt);
      if (!is_ds) {
        p_step(t);
      } else {
        const f32x16 dp_cur = product(buf[cur] + T32);   // dP' of half tile t
        ds_finish(t - 1);
        dp_prev = dp_cur;
      }
      rotate();
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    lds_barrier();
    if (is_ds) ds_finish(steps - 1);
  }

  // accumulator i of acc[mb] is channel 32 mb + 8 (i/4) + 4 kg + i%4 of the owner row
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  if (o_ok) {
    uint16_t* op = is_ds ? a.out1 + (int64_t)h * a.o1_head + (int64_t)(otok0 + orow) * a.o1_tok
                         : a.out2 + (int64_t)h * a.o2_head + (int64_t)(otok0 + orow) * a.o2_tok;
    const float factor = is_ds ? a.scale : 1.0f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc[mb][4 * g + e] * factor);
        *reinterpret_cast<bf16x4*>(op + 32 * mb + 8 * g + 4 * kg) = o4;
      }
  }
}

// delta_x = dO_x . O_x (float32), one group of d/8 lanes per row; written next to the row's
// log-sum-exp, so that the attention kernels fetch both with one load.
template <int D>
__global__ __launch_bounds__(256) void lf_attn_delta_kernel(const uint16_t* __restrict__ O,
                                                            const uint16_t* __restrict__ dO,
                                                            const float* __restrict__ lse2,
                                                            float2* __restrict__ stats, int64_t o_tok,
                                                            int64_t o_head, int q_len, int rows) {
  constexpr int LPR = D / 8;                  // lanes per row
  const int gid = blockIdx.x * 256 + threadIdx.x;
  const int row = gid / LPR, ch = gid % LPR;
  float s = 0.0f;
  if (row < rows) {
    const int h = row / q_len, x = row % q_len;
    const int64_t off = (int64_t)h * o_head + (int64_t)x * o_tok + ch * 8;
    const uint4 u = *reinterpret_cast<const uint4*>(O + off), v = *reinterpret_cast<const uint4*>(dO + off);
    const uint32_t uu[4] = {u.x, u.y, u.z, u.w}, vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s = fmaf(__uint_as_float(uu[i] << 16), __uint_as_float(vv[i] << 16), s);
      s = fmaf(__uint_as_float(uu[i] & 0xffff0000u), __uint_as_float(vv[i] & 0xffff0000u), s);
    }
  }
#pragma unroll
  for (int o = 1; o < LPR; o <<= 1) s += __shfl_xor(s, o);
  if (row < rows && ch == 0) stats[row] = make_float2(lse2[row], s);
}

// Transposed lists: for every (head, KV block c) the query blocks whose list holds c, ascending.
// One wavefront per (head, c): lane i looks c up in the list of query block r0 + i by bisection
// (lists are ascending), and the hits of the 64 lanes are compacted in order through a ballot.
__global__ __launch_bounds__(256) void lf_transpose_lists_kernel(const int32_t* __restrict__ idx,
                                                                 int32_t* __restrict__ tlist,
                                                                 int32_t* __restrict__ tcnt, int heads,
                                                                 int n_q, int n_k, int list_len) {
  const int gid = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (gid >= heads * n_k) return;
  const int lane = threadIdx.x & 63;
  const int h = gid / n_k, c = gid % n_k;
  int32_t* out = tlist + (int64_t)gid * n_q;
  int cnt = 0;
  for (int r0 = 0; r0 < n_q; r0 += 64) {
    const int r = r0 + lane;
    bool hit = false;
    if (r < n_q) {
      const int32_t* l = idx + ((int64_t)h * n_q + r) * list_len;
      int lo = 0, hi = list_len;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (l[mid] < c) lo = mid + 1; else hi = mid;
      }
      hit = lo < list_len && l[lo] == c;
    }
    const uint64_t m = __ballot(hit);
    if (hit) out[cnt + __popcll(m & ((1ull << lane) - 1))] = r;
    cnt += __popcll(m);
  }
  if (lane == 0) tcnt[gid] = cnt;
}

// Launch order of the key-major pass: its workgroups differ in work by the length of their
// transposed list (a sink or current-chunk block is kept by every query block, a block of the
// middle history by few), and workgroups are started in index order, so the long ones go first.
// The workgroup indices are dealt to the eight XCDs in contiguous ranges (see the kernel); one
// block per range sorts it by descending count with a counting sort.  The place of equal counts
// among each other is left to the order the atomics happen to take: any permutation is valid,
// and the gradients do not depend on which workgroup computes a block.
constexpr int kOrderBins = 1024;
__global__ __launch_bounds__(1024) void lf_order_kernel(const int32_t* __restrict__ tcnt,
                                                        int32_t* __restrict__ order, int total,
                                                        int per_xcd) {
  __shared__ int bins[kOrderBins];
  const int w0 = blockIdx.x * per_xcd, w1 = min(total, w0 + per_xcd);
  for (int i = threadIdx.x; i < kOrderBins; i += 1024) bins[i] = 0;
  __syncthreads();
  for (int w = w0 + threadIdx.x; w < w1; w += 1024) atomicAdd(&bins[min(tcnt[w], kOrderBins - 1)], 1);
  __syncthreads();
  // bins[b] <- number of workgroups in bins above b (where bin b starts in the descending order):
  // an inclusive scan over the reversed bins by doubling, minus the bin's own count
  {
    const int b = kOrderBins - 1 - threadIdx.x;   // thread i scans position i of the reversed bins
    const int own = bins[b];
    int run = own;
    for (int d = 1; d < kOrderBins; d <<= 1) {
      const int other = (int)threadIdx.x >= d ? bins[b + d] : 0;
      __syncthreads();
      run += other;
      bins[b] = run;
      __syncthreads();
    }
    bins[b] = run - own;
  }
  __syncthreads();
  for (int w = w0 + threadIdx.x; w < w1; w += 1024)
    order[w0 + atomicAdd(&bins[min(tcnt[w], kOrderBins - 1)], 1)] = w;
}

}  // namespace

int lf_launch_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                       const float* lse2, const lf_shape* s, const lf_dims* dm, const int32_t* indices,
                       int32_t list_len, float scale, void* dQ, void* dK, void* dV, float* stats,
                       int32_t* tlist, int32_t* tcnt, int32_t* order, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int q_len = dm->f * dm->n;
  const int rows = dm->H * q_len;
  {
    const int lanes = rows * (dm->d / 8);
    const unsigned grid = (unsigned)((lanes + 255) / 256);
    const hipError_t rc = dm->d == 128
        ? lf_launch(lf_attn_delta_kernel<128>, dim3(grid), dim3(256), 0, st, (const uint16_t*)O,
                    (const uint16_t*)dO, lse2, (float2*)stats, (int64_t)s->o_stride_tok, (int64_t)s->o_stride_head, q_len, rows)
        : lf_launch(lf_attn_delta_kernel<64>, dim3(grid), dim3(256), 0, st, (const uint16_t*)O,
                    (const uint16_t*)dO, lse2, (float2*)stats, (int64_t)s->o_stride_tok, (int64_t)s->o_stride_head, q_len, rows);
    if (rc != hipSuccess) return LF_ERR_HIP;
  }
  {
    const unsigned grid = (unsigned)((dm->H * dm->n_k + 3) / 4);
    if (lf_launch(lf_transpose_lists_kernel, dim3(grid), dim3(256), 0, st, indices, tlist, tcnt, dm->H,
                  dm->n_q, dm->n_k, (int)list_len) != hipSuccess)
      return LF_ERR_HIP;
  }
  BwdArgs a = {};
  a.stats = (const float2*)stats;
  a.n = dm->n;
  a.nb = dm->nb;
  a.q_len = q_len;
  a.c = scale * 1.4426950408889634f;
  a.scale = scale;
  // dQ
  a.X = (const uint16_t*)Q;   a.x_tok = s->q_stride_tok;  a.x_head = s->q_stride_head;
  a.Y = (const uint16_t*)dO;  a.y_tok = s->o_stride_tok;  a.y_head = s->o_stride_head;
  a.A1 = (const uint16_t*)K;  a.a1_tok = s->k_stride_tok; a.a1_head = s->k_stride_head;
  a.A2 = (const uint16_t*)V;  a.a2_tok = s->v_stride_tok; a.a2_head = s->v_stride_head;
  a.out1 = (uint16_t*)dQ;     a.o1_tok = s->q_stride_tok; a.o1_head = s->q_stride_head;
  a.out2 = nullptr;
  a.idx = indices; a.cnt = nullptr; a.list_len = list_len; a.list_stride = list_len;
  a.owners = dm->n_q; a.streams = dm->n_k;
  a.total_wg = dm->H * dm->n_q;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  hipError_t rc = dm->d == 128
      ? lf_launch(lf_attn_bwd_q_kernel<128>, dim3((unsigned)(a.wg_per_xcd * 8)), dim3(kThreads), 0, st, a)
      : lf_launch(lf_attn_bwd_q_kernel<64>, dim3((unsigned)(a.wg_per_xcd * 8)), dim3(kThreads), 0, st, a);
  if (rc != hipSuccess) return LF_ERR_HIP;
  // dK and dV
  a.X = (const uint16_t*)K;   a.x_tok = s->k_stride_tok;  a.x_head = s->k_stride_head;
  a.Y = (const uint16_t*)V;   a.y_tok = s->v_stride_tok;  a.y_head = s->v_stride_head;
  a.A1 = (const uint16_t*)Q;  a.a1_tok = s->q_stride_tok; a.a1_head = s->q_stride_head;
  a.A2 = (const uint16_t*)dO; a.a2_tok = s->o_stride_tok; a.a2_head = s->o_stride_head;
  a.out1 = (uint16_t*)dK;     a.o1_tok = s->k_stride_tok; a.o1_head = s->k_stride_head;
  a.out2 = (uint16_t*)dV;     a.o2_tok = s->v_stride_tok; a.o2_head = s->v_stride_head;
  a.idx = tlist; a.cnt = tcnt; a.list_len = dm->n_q; a.list_stride = dm->n_q;
  a.owners = dm->n_k; a.streams = dm->n_q;
  a.total_wg = dm->H * dm->n_k;
  a.wg_per_xcd = (a.total_wg + 7) / 8;
  if (lf_launch(lf_order_kernel, dim3(8), dim3(1024), 0, st, (const int32_t*)tcnt, order, a.total_wg,
                a.wg_per_xcd) != hipSuccess)
    return LF_ERR_HIP;
  a.order = order;
  const dim3 grid2((unsigned)(a.wg_per_xcd * 8));
  rc = dm->d == 128 ? lf_launch(lf_attn_bwd_kv_kernel<128>, grid2, dim3(kKvThreads), 0, st, a)
                    : lf_launch(lf_attn_bwd_kv_kernel<64>, grid2, dim3(kKvThreads), 0, st, a);
  return rc == hipSuccess ? LF_OK : LF_ERR_HIP;
}
