// Producer of Q and K next to the hot path: RMSNorm, then rotary position embedding, written
// head-major in the layout mask selection and attention read (the paper's "Efficient
// Deployment" section names fused RoPE and RMSNorm kernels; it defines neither, so these are
// the textbook operators, see lf.h).  HBM-bound: one read of the token-major activations, one
// write of the head-major result, plus the angle table.
//
// One wavefront per token.  A lane owns 16-byte chunks (8 channels) of the token, chunk
// 64 it + lane in iteration it; the CH = d/8 chunks of a head sit in CH neighbouring lanes, so
// the per-head mean of squares is a reduction over CH lanes and the rotation partner of the
// "half" pairing is CH/2 lanes away.  All arithmetic is float32; the result is rounded to
// bfloat16 once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lf_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct ProducerArgs {
  const uint16_t* X;
  const float* g;
  const float* cosv;
  const float* sinv;
  uint16_t* Y;
  int64_t x_stride_tok, y_stride_tok, y_stride_head;
  int H, L, across_heads, pairing;
  float eps;
};

constexpr int kTokensPerWg = 4;

__device__ __forceinline__ void unpack8(const uint4& u, float (&x)[8]) {
  x[0] = __uint_as_float(u.x << 16); x[1] = __uint_as_float(u.x & 0xffff0000u);
  x[2] = __uint_as_float(u.y << 16); x[3] = __uint_as_float(u.y & 0xffff0000u);
  x[4] = __uint_as_float(u.z << 16); x[5] = __uint_as_float(u.z & 0xffff0000u);
  x[6] = __uint_as_float(u.w << 16); x[7] = __uint_as_float(u.w & 0xffff0000u);
}

template <int D>
__global__ __launch_bounds__(64 * kTokensPerWg) void lf_qk_norm_rope_kernel(ProducerArgs a) {
  constexpr int CH = D / 8;
  const int lane = threadIdx.x & 63;
  const int tok = blockIdx.x * kTokensPerWg + (threadIdx.x >> 6);
  if (tok >= a.L) return;                       // whole wavefronts leave; no barrier below
  const int nc = a.H * CH;                      // chunks per token
  const uint16_t* xrow = a.X + (int64_t)tok * a.x_stride_tok;

  float inv_all = 0.0f;
  if (a.across_heads) {
    float ss = 0.0f;
    for (int c = lane; c < nc; c += 64) {
      float x[8];
      unpack8(*reinterpret_cast<const uint4*>(xrow + 8 * c), x);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) ss += __shfl_xor(ss, off);
    inv_all = 1.0f / sqrtf(ss / (float)(a.H * D) + a.eps);
  }

  for (int c0 = 0; c0 < nc; c0 += 64) {
    const int c = c0 + lane;
    const bool on = c < nc;                     // lanes past the last chunk still take part in the exchanges
    const int h = on ? c / CH : 0, cih = c % CH;
    float x[8];
    if (on) {
      unpack8(*reinterpret_cast<const uint4*>(xrow + 8 * c), x);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = 0.0f;
    }
    float inv = inv_all;
    if (!a.across_heads) {
      float ss = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
#pragma unroll
      for (int off = 1; off < CH; off <<= 1) ss += __shfl_xor(ss, off);
      inv = 1.0f / sqrtf(ss / (float)D + a.eps);
    }
    float y[8];
    {
      const float4 g0 = on ? *reinterpret_cast<const float4*>(a.g + 8 * c) : make_float4(0, 0, 0, 0);
      const float4 g1 = on ? *reinterpret_cast<const float4*>(a.g + 8 * c + 4) : make_float4(0, 0, 0, 0);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] = x[e] * inv * gg[e];
    }
    float r[8];
    const float* ct = a.cosv + (int64_t)tok * (D / 2);
    const float* st = a.sinv + (int64_t)tok * (D / 2);
    if (a.pairing == 0) {
      // pairs (2i, 2i+1): this chunk holds pairs 4 cih .. 4 cih + 3
      const float4 cs = *reinterpret_cast<const float4*>(ct + 4 * cih);
      const float4 sn = *reinterpret_cast<const float4*>(st + 4 * cih);
      const float cc[4] = {cs.x, cs.y, cs.z, cs.w}, ss4[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        r[2 * p] = y[2 * p] * cc[p] - y[2 * p + 1] * ss4[p];
        r[2 * p + 1] = y[2 * p] * ss4[p] + y[2 * p + 1] * cc[p];
      }
    } else {
      // pairs (i, i + d/2): the partner chunk is CH/2 lanes away inside the head
      const int i0 = 8 * (cih % (CH / 2));
      const bool first = cih < CH / 2;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float other = __shfl_xor(y[e], CH / 2);
        const float cv = ct[i0 + e], sv = st[i0 + e];
        r[e] = first ? y[e] * cv - other * sv : other * sv + y[e] * cv;
      }
    }
    if (on) {
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (__bf16)r[e];
      *reinterpret_cast<bf16x8*>(a.Y + (int64_t)h * a.y_stride_head + (int64_t)tok * a.y_stride_tok + 8 * cih) = o;
    }
  }
}

}  // namespace

int lf_launch_qk_norm_rope(const void* X, const float* g, const float* cosv, const float* sinv,
                           const lf_producer_shape* p, void* Y, void* stream) {
  ProducerArgs a;
  a.X = (const uint16_t*)X;
  a.g = g;
  a.cosv = cosv;
  a.sinv = sinv;
  a.Y = (uint16_t*)Y;
  a.x_stride_tok = p->x_stride_tok;
  a.y_stride_tok = p->y_stride_tok;
  a.y_stride_head = p->y_stride_head;
  a.H = p->heads;
  a.L = p->tokens;
  a.across_heads = p->across_heads;
  a.pairing = p->pairing;
  a.eps = p->eps;
  const unsigned grid = (unsigned)((p->tokens + kTokensPerWg - 1) / kTokensPerWg);
  hipStream_t st = (hipStream_t)stream;
  const hipError_t rc = p->head_dim == 128
      ? lf_launch(lf_qk_norm_rope_kernel<128>, dim3(grid), dim3(64 * kTokensPerWg), 0, st, a)
      : lf_launch(lf_qk_norm_rope_kernel<64>, dim3(grid), dim3(64 * kTokensPerWg), 0, st, a);
  return rc == hipSuccess ? LF_OK : LF_ERR_HIP;
}
