// Internal declarations shared by the host entry points and the gfx950 kernels.
#ifndef LF_COMMON_H
#define LF_COMMON_H

#include <stddef.h>
#include <stdint.h>

#include "lf.h"

#define LF_MAX_CAND_BLOCKS 2048  // |B_r| the selection kernel can rank in LDS
#define LF_MAX_CAND_FRAMES 1024  // |M| the selection kernel can rank in LDS
#define LF_MAX_HIST_FRAMES 4096  // F_h bound (flag array in LDS)
#define LF_MAX_CHUNK_FRAMES 1024 // f bound: with the three above it keeps the selection kernel's
                                 // dynamic LDS below 64 KiB, so the size is known to fit
                                 // before anything is enqueued

// Size of the library-owned device scratch behind lf_select_mask_static (per GPU).
#define LF_STATIC_SCRATCH_BYTES ((size_t)16 << 20)

// Derived sizes of one call; filled by lf_derive() after validation.
struct lf_dims {
  int H, d, n, f, F, F_h, nb, n_q, n_k, m;
  int n_tf;     // selected history frames: n_sink + n_win + k_frames
  int n_cand;   // |B_r|
  size_t off_qt, off_kt, off_kh, ws_bytes;
};

// Validates shape (and budget when non-NULL); returns LF_OK or an lf_status.
int lf_derive(const lf_shape* s, const lf_budget* b, lf_dims* out);

// Kernel launchers (defined in the .hip files); return LF_OK or LF_ERR_HIP.
int lf_launch_select(const void* Q, const void* K, const lf_shape* s, const lf_budget* b,
                     const lf_dims* dm, int32_t* indices, void* workspace, void* stream);
int lf_launch_kcache_update(const void* K, const lf_shape* s, const lf_dims* dm, int frame0, int frame1,
                            int max_frames, void* kcache, void* stream);
int lf_launch_select_cached(const void* Q, const void* Kcur, void* kcache, int max_frames,
                            const lf_shape* s, const lf_budget* b, const lf_dims* dm, int32_t* indices,
                            void* workspace, void* stream);
int lf_launch_qk_norm_rope(const void* X, const float* g, const float* cosv, const float* sinv,
                           const lf_producer_shape* p, void* Y, void* stream);
// Device address of the library's static scratch on the current device (looked up on the first
// call per device); LF_OK or LF_ERR_HIP.
int lf_static_scratch(void** ptr);
int lf_launch_attn(const void* Q, const void* K, const void* V, const lf_shape* s,
                   const lf_dims* dm, const int32_t* indices, int32_t list_len, int32_t list_stride,
                   float scale, void* O, const float* state_o, const float* state_ml, float* lse2,
                   void* stream);
int lf_launch_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                       const float* lse2, const lf_shape* s, const lf_dims* dm, const int32_t* indices,
                       int32_t list_len, float scale, void* dQ, void* dK, void* dV, float* stats,
                       int32_t* tlist, int32_t* tcnt, int32_t* order, void* stream);
int lf_launch_attn_dense(const void* Q, const void* K, const void* V, const lf_shape* s,
                         const lf_dims* dm, int kv0, int kv1, float scale, float* state_o,
                         float* state_ml, void* stream);

#ifdef __HIPCC__
#include <hip/hip_runtime.h>
// Launches a kernel and returns this launch's own status (an error left behind by the caller's
// earlier work is neither reported nor cleared).
template <typename... KArgs, typename... Args>
inline hipError_t lf_launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes,
                            hipStream_t stream, Args... args) {
  void* argv[] = {(void*)&args...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, lds_bytes, stream);
}
#endif

#endif
