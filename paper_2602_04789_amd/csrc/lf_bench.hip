// Two micro-benchmarks that put a measured ceiling next to the published peaks the roofline
// fractions are taken against.  They are not part of the hot path and live in a library of
// their own (liblf_bench.so), which only the benchmark script loads.
//
//   lfb_stream_read  streams a buffer once with 16-byte loads (what the pooling pass of mask
//                    selection does with Q and K), nothing else: achievable read bandwidth.
//   lfb_mfma_loop    back-to-back v_mfma_f32_32x32x16_bf16 on register operands, four
//                    independent accumulators per wavefront, two wavefronts per SIMD:
//                    achievable matrix rate at the clock the chip sustains under that load,
//                    with constant operands and with pseudo-random ones.
//   lfb_issue_mix    the attention step's instruction mix without memory: per iteration and
//                    wavefront 16 matrix instructions and / or the vector work of one softmax
//                    step (16 fma, 16 exp2, 8 packs to bfloat16, 8 dot2 row-sum steps), the two
//                    independent of each other: how far matrix and vector instructions of the
//                    wavefronts of a SIMD overlap.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kReadThreads = 256;
constexpr int kInFlight = 8;   // 16-byte loads a thread has outstanding

__global__ __launch_bounds__(kReadThreads) void stream_read_kernel(const uint4* __restrict__ src,
                                                                   size_t n16, uint32_t* sink) {
  // a workgroup walks consecutive spans of kInFlight * 256 * 16 bytes, dealt round-robin
  const size_t span = (size_t)kInFlight * kReadThreads;
  uint32_t acc = 0;
  for (size_t base = (size_t)blockIdx.x * span; base < n16; base += (size_t)gridDim.x * span) {
    uint4 v[kInFlight];
#pragma unroll
    for (int i = 0; i < kInFlight; ++i) {
      const size_t j = base + (size_t)i * kReadThreads + threadIdx.x;
      v[i] = j < n16 ? src[j] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kInFlight; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;   // keeps the loads alive; practically never taken
}

// 32-bit mix (xorshift-multiply) for the pseudo-random operand bits.
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// RANDOM = false: every operand register holds the same small integers (hardly any bit toggles
// between consecutive instructions).  RANDOM = true: four different A and four different B
// operands of pseudo-random bfloat16 values in (-2, 2), cycled through, as activations are: the
// matrix rate the chip sustains depends on the data, because its clock follows the power drawn.
template <bool RANDOM>
__global__ __launch_bounds__(512, 1) void mfma_loop_kernel(float* sink, int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (RANDOM) {
        const uint32_t ha = mix32((blockIdx.x * 512u + threadIdx.x) * 64u + r * 16u + i);
        const uint32_t hb = mix32(ha + 0x9e3779b9u);
        // sign | exponent 0x7c..0x7f (magnitudes 1/8 .. 2) | 7 random mantissa bits
        const uint16_t ua = (uint16_t)(((ha >> 16) & 0x8000u) | ((0x7cu + (ha & 3u)) << 7) | ((ha >> 8) & 0x7fu));
        const uint16_t ub = (uint16_t)(((hb >> 16) & 0x8000u) | ((0x7cu + (hb & 3u)) << 7) | ((hb >> 8) & 0x7fu));
        a[r][i] = __builtin_bit_cast(__bf16, ua);
        b[r][i] = __builtin_bit_cast(__bf16, ub);
      } else {
        a[r][i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[r][i] = (__bf16)(float)((threadIdx.x * 7 + i) & 1);
      }
    }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[(u + 0) & 3], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 1) & 3], b[(u + 2) & 3], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 2) & 3], b[(u + 3) & 3], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 3) & 3], b[(u + 1) & 3], c3, 0, 0, 0);
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 123456.789f) sink[0] = s;   // keeps the products alive; practically never taken
}

// WHAT: 1 = matrix instructions only, 2 = vector work only, 3 = both in every wavefront.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <int WHAT>
__global__ __launch_bounds__(512, 2) void issue_mix_kernel(float* sink, int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t ha = mix32((blockIdx.x * 512u + threadIdx.x) * 64u + r * 16u + i);
      const uint32_t hb = mix32(ha + 0x9e3779b9u);
      a[r][i] = __builtin_bit_cast(__bf16, (uint16_t)(((ha >> 16) & 0x8000u) | ((0x7cu + (ha & 3u)) << 7) | ((ha >> 8) & 0x7fu)));
      b[r][i] = __builtin_bit_cast(__bf16, (uint16_t)(((hb >> 16) & 0x8000u) | ((0x7cu + (hb & 3u)) << 7) | ((hb >> 8) & 0x7fu)));
    }
  f32x16 c0, c1, c2, c3;
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    c0[i] = c1[i] = c2[i] = c3[i] = 0.0f;
    x[i] = -1.0f - 0.001f * (float)((threadIdx.x + i) & 63);
  }
  float l = 0.0f;
  for (int it = 0; it < iters; ++it) {
    if (WHAT & 1) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[(u + 0) & 3], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 1) & 3], b[(u + 2) & 3], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 2) & 3], b[(u + 3) & 3], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 3) & 3], b[(u + 1) & 3], c3, 0, 0, 0);
      }
    }
    if (WHAT & 2) {
      // one softmax step on 16 values: scale and shift, exp2, pack to bfloat16, row sum
      bf16x8 p[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) p[i >> 3][i & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(x[i], 1.0009765625f, -0.5f));
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const bf16x2 pr = {p[i >> 3][i & 7], p[i >> 3][(i & 7) + 1]};
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        l = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l, false);
      }
      // feed the packed values back, so that no iteration's work can be dropped or hoisted
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = -1.0f - (float)p[i >> 3][i & 7];
    }
  }
  float s = l;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i] + x[i];
  if (s == 123456.789f) sink[0] = s;
}

}  // namespace

extern "C" {

// Reads `bytes` (a multiple of 16) of device memory at `buf` once.  Returns 0 or a hipError_t.
int lfb_stream_read(const void* buf, size_t bytes, void* sink, void* hip_stream) {
  if (!buf || !sink || bytes % 16) return (int)hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const size_t span = (size_t)kInFlight * kReadThreads;
  size_t grid = (n16 + span - 1) / span;
  if (grid > 256 * 16) grid = 256 * 16;
  if (grid == 0) return 0;
  void* args[] = {(void*)&buf, (void*)&n16, (void*)&sink};
  return (int)hipLaunchKernel(reinterpret_cast<const void*>(stream_read_kernel), dim3((unsigned)grid),
                              dim3(kReadThreads), args, 0, (hipStream_t)hip_stream);
}

// 256 workgroups of 8 wavefronts, each wavefront issuing 16 * iters matrix instructions of
// 2 * 32 * 32 * 16 FLOP, on constant (random_data = 0) or pseudo-random (1) operands.  *flop
// (host) receives the FLOP count of the launch.
int lfb_mfma_loop(int iters, int random_data, void* sink, double* flop, void* hip_stream) {
  if (!sink || iters < 1) return (int)hipErrorInvalidValue;
  if (flop) *flop = 256.0 * 8.0 * 16.0 * (double)iters * 2.0 * 32.0 * 32.0 * 16.0;
  void* args[] = {(void*)&sink, (void*)&iters};
  const void* fn = random_data ? reinterpret_cast<const void*>(mfma_loop_kernel<true>)
                               : reinterpret_cast<const void*>(mfma_loop_kernel<false>);
  return (int)hipLaunchKernel(fn, dim3(256), dim3(512), args, 0, (hipStream_t)hip_stream);
}

// 256 * waves_per_simd / 2 workgroups of 8 wavefronts (waves_per_simd = 2 or 4 wavefronts per
// SIMD; the kernel needs few registers); what: 1 matrix instructions only (16 per iteration),
// 2 the vector work of one softmax step only, 3 both.
int lfb_issue_mix(int what, int iters, int waves_per_simd, void* sink, void* hip_stream) {
  if (!sink || iters < 1 || what < 1 || what > 3 || (waves_per_simd != 2 && waves_per_simd != 4))
    return (int)hipErrorInvalidValue;
  void* args[] = {(void*)&sink, (void*)&iters};
  const void* fn = what == 1 ? reinterpret_cast<const void*>(issue_mix_kernel<1>)
                 : what == 2 ? reinterpret_cast<const void*>(issue_mix_kernel<2>)
                             : reinterpret_cast<const void*>(issue_mix_kernel<3>);
  return (int)hipLaunchKernel(fn, dim3(128u * (unsigned)waves_per_simd), dim3(512), args, 0, (hipStream_t)hip_stream);
}

}  // extern "C"
