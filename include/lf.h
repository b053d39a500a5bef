/*
 * lf.h -- C ABI of the per-chunk Hierarchical Sparse Attention (HSA) hot path of
 * "Light Forcing" for AMD MI355X (gfx950).
 *
 * The three calls follow the paper's statement of the problem (Sec. 4.1, Sec. 4.2):
 *
 *   lf_chunk_budget   Chunk-Aware Growth: chunk index + schedule -> integer keep-counts
 *                     (Eq. 5, Eq. 6; appendix, implementation details of Light Forcing).
 *   lf_select_mask    token compression, frame- and block-level scores and top-k
 *                     (Eq. 7 - Eq. 12) -> sorted KV-block index lists per (head, query block).
 *   lf_sparse_attn    blockwise sparse attention over the listed KV blocks (Eq. 13 / Eq. 3).
 *
 * Conventions
 *   - Plain pointers and sizes only.  Every tensor pointer is DEVICE memory owned by the
 *     caller; the library never allocates, frees or synchronises.  Calls enqueue kernels
 *     on `hip_stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     return at once.
 *   - Return value: LF_OK (0) or a negative lf_status.  On error nothing is enqueued.
 *   - Layout.  H heads (the caller folds batch into heads), d = head_dim, n = frame_len
 *     tokens per frame, f frames per chunk, F_h history frames, F = F_h + f frames in the
 *     cache.  Q is [H][q_len = f*n][d]; Kcache, Vcache are [H][kv_len = F*n][d] with the
 *     current chunk's K/V as the LAST f frames (Sec. 4.2: k^{:i} includes chunk i).  d is
 *     contiguous; token and head strides are given in elements.  Elements are bfloat16.
 *     All base pointers and strides must keep every token row 16-byte aligned.
 *   - Blocks (shapes stated after Eq. 7): every frame is cut into nb = ceil(n / block)
 *     blocks; the last block of a frame holds n - (nb-1)*block tokens.  KV block id
 *     c = tau*nb + j is block j of cache frame tau; query block r likewise within the
 *     chunk.  n_q = f*nb query blocks, n_k = F*nb KV blocks.
 */
#ifndef LF_H
#define LF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LF_OK = 0,
  LF_ERR_NULL = -1,      /* a required pointer is NULL */
  LF_ERR_SHAPE = -2,     /* sizes inconsistent or unsupported (see lf_shape) */
  LF_ERR_BUDGET = -3,    /* budget inconsistent with the shape */
  LF_ERR_DTYPE = -4,     /* dtype other than LF_BF16 */
  LF_ERR_ALIGN = -5,     /* pointer or stride breaks the 16-byte row alignment */
  LF_ERR_WORKSPACE = -6, /* workspace NULL or smaller than lf_workspace_bytes() */
  LF_ERR_HIP = -7,       /* a kernel launch of this call failed */
  LF_ERR_SCHEDULE = -8   /* schedule fields out of range */
} lf_status;

typedef enum { LF_BF16 = 0 } lf_dtype;

/* How the per-chunk keep ratio is chosen. */
typedef enum {
  LF_SCHED_FIXED = 0,  /* keep_fixed for every chunk */
  LF_SCHED_LINEAR = 1, /* keep_first at chunk 1 ... keep_last at chunk n_chunks, linear */
  LF_SCHED_CAG = 2     /* Chunk-Aware Growth: keep = 1 - s_i, s_i = s_base - beta/sqrt(i) (Eq. 5),
                          beta from the FLOPs equality over chunks 2..n_chunks (Eq. 6) */
} lf_sched_mode;

/* What the keep ratio is a fraction of when it is turned into a block count. */
typedef enum {
  LF_OF_CANDIDATES = 0, /* of the candidate blocks B_r (Eq. 11) */
  LF_OF_HISTORY = 1,    /* of all history blocks F_h*nb (clamped to |B_r|) */
  LF_OF_ALL = 2         /* of all KV blocks n_k: the paper's sparsity ratio s_i */
} lf_ratio_of;

/* Everything known before the rollout starts (host memory, plain data). */
typedef struct {
  int32_t mode;              /* lf_sched_mode */
  int32_t n_chunks;          /* chunks in the rollout (7 for a 5 s video) */
  int32_t frames_per_chunk;  /* f (3 in the paper's experiments) */
  int32_t frame_len;         /* n */
  int32_t block;             /* b_q = b_kv (64 in the paper's experiments) */
  int32_t n_sink;            /* earliest history frames always selected */
  int32_t n_win;             /* nearest history frames always selected */
  int32_t k_frames;          /* history frames retrieved by top-k from the candidate set M
                                (= n_past_keep - n_sink - n_win in the appendix's terms) */
  int32_t ratio_of;          /* lf_ratio_of */
  int32_t current_mandatory; /* 1: every current-chunk block is kept and does not compete in
                                the block top-k; 0: current-chunk blocks compete (Eq. 11 as
                                written).  With no history they always compete. */
  int32_t first_chunk_dense; /* 1: chunk 1 keeps every block (Sec. 4.1) */
  int32_t reserved;          /* set to 0 */
  double keep_fixed;         /* LF_SCHED_FIXED */
  double keep_first;         /* LF_SCHED_LINEAR */
  double keep_last;          /* LF_SCHED_LINEAR */
  double s_base;             /* LF_SCHED_CAG (0.98 for 5 s videos) */
  double s_target;           /* LF_SCHED_CAG (0.88 for 5 s videos) */
} lf_schedule;

/* Integer keep-counts of one chunk: all that mask selection needs (host memory). */
typedef struct {
  int32_t n_hist_frames;     /* F_h = (chunk_idx-1)*f */
  int32_t frames_per_chunk;  /* f */
  int32_t n_sink;            /* clamped to F_h */
  int32_t n_win;             /* clamped to F_h - n_sink */
  int32_t k_frames;          /* clamped to m = F_h - n_sink - n_win (footnote to Eq. 7):
                                when m <= k_frames retrieval is inactive and all history
                                frames are kept */
  int32_t k_blocks;          /* size of the block top-k (Eq. 11) */
  int32_t current_mandatory; /* effective value (0 when F_h == 0) */
  int32_t list_len;          /* kept KV blocks per (head, query block)
                                = k_blocks + (current_mandatory ? f*nb : 0) */
  double keep_ratio;         /* the ratio the counts came from (informational) */
} lf_budget;

/* Tensor geometry shared by lf_select_mask and lf_sparse_attn (host memory). */
typedef struct {
  int32_t heads;     /* H >= 1 */
  int32_t head_dim;  /* d: 64 or 128 */
  int32_t frame_len; /* n >= 1 */
  int32_t block;     /* 64 */
  int32_t q_len;     /* f*n */
  int32_t kv_len;    /* F*n, >= q_len, multiple of n */
  int32_t dtype;     /* LF_BF16 */
  int32_t reserved;  /* set to 0 */
  int64_t q_stride_tok, q_stride_head; /* elements; multiples of 8 */
  int64_t k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head;
  int64_t o_stride_tok, o_stride_head;
} lf_shape;

/*
 * Chunk-Aware Growth (Sec. 4.1).  Host only; no GPU work.
 *   chunk_idx  1-based index i of the chunk being generated.
 *   schedule   in.   out: budget.
 * keep ratio rho_i: FIXED / LINEAR as named above; CAG: rho_i = 1 - s_i with
 *   alpha_i = 1/sqrt(i), w_i = l^q_i l^k_i d ~ i, beta = (s_base - s_target) * sum w_i /
 *   sum(alpha_i w_i) over i = 2..n_chunks; chunk 1 keeps everything.
 * counts: n_sink, n_win, k_frames clamped to the history as documented in lf_budget;
 *   |B_r| = (n_sink + n_win + k_frames)*nb (+ f*nb when the current chunk competes);
 *   k_blocks = the smallest integer >= rho_i * N, a product within 1e-9 above an integer
 *   counting as that integer, with N per ratio_of (for LF_OF_ALL with a mandatory current
 *   chunk the f*nb current blocks are subtracted), clamped to [min(1,|B_r|), |B_r|].
 * Errors: LF_ERR_NULL; LF_ERR_SCHEDULE (chunk_idx < 1, non-positive sizes, negative counts,
 *   ratios outside [0, 1], unknown mode / ratio_of, or a Chunk-Aware Growth schedule whose
 *   s_i of Eq. 5 leaves [0, 1] at this chunk: s_i is a sparsity ratio and such parameters are
 *   rejected, not clamped).
 */
int lf_chunk_budget(int32_t chunk_idx, const lf_schedule* schedule, lf_budget* budget);

/* Bytes of device scratch lf_select_mask needs for this shape and budget (0 on bad input). */
size_t lf_workspace_bytes(const lf_shape* shape, const lf_budget* budget);

/*
 * Where lf_select_mask leaves its intermediates inside the workspace, as byte offsets
 * (for tests and profiling; contents are valid once the call's kernels have finished):
 *   off[0]  q_tilde  float32 [H][n_q][d]      block means of Q          (Eq. 7)
 *   off[1]  k_tilde  float32 [H][d/4][n_k][4] block means of K          (Eq. 7)
 *   off[2]  k_hat    float32 [H][d/4][m][4]   frame means of the candidate frames M,
 *                                             ascending frame id        (Eq. 7)
 * k_tilde and k_hat are stored channel-quad major: channel t of row c sits at
 * [t/4][c][t%4], so that the scoring kernel reads 16 bytes per row and step, coalesced
 * over neighbouring rows.
 * Returns LF_OK or the error lf_select_mask would return for the same shape/budget.
 */
int lf_workspace_layout(const lf_shape* shape, const lf_budget* budget, size_t off[3]);

/*
 * Mask selection (Sec. 4.2, Eq. 7 - Eq. 12), per head and per query block r:
 *   q_tilde_r, k_tilde_c  block means (divide by the block's own token count);
 *   k_hat_tau             mean of frame tau's nb block means, tau in M = history frames
 *                         other than the n_sink earliest and the n_win nearest;
 *   p_r[tau] = <q_tilde_r, k_hat_tau>;  T_r = top-k_frames(p_r) U sink U window U current;
 *   B_r = blocks of the frames of T_r (without the current frames when current_mandatory);
 *   o_r[c] = <q_tilde_r, k_tilde_c>;  J_r = top-k_blocks over B_r;
 *   kept = J_r (U all current blocks when current_mandatory).
 * Arithmetic (fixed so that lists are reproducible bit for bit): block sums exact
 *   (binary64; exact for bfloat16 inputs with |x| = 0 or 2^-30 <= |x| < 2^8), means rounded
 *   to float32; frame mean = binary64 sum of the nb float32 block means in ascending j,
 *   divided by nb, rounded to float32; scores = binary64 sum over the head dimension in
 *   ascending order of exact products, rounded to float32; top-k orders by larger score,
 *   then lower index.  Inputs must be finite.
 * Arguments
 *   Q, Kcache     device, bfloat16, layout above (V is not read).
 *   shape, budget host; budget as returned by lf_chunk_budget for this chunk
 *                 (kv_len must equal (n_hist_frames + frames_per_chunk)*frame_len).
 *   indices       device, int32 [H][n_q][list_len], written: ascending KV-block ids.
 *   workspace     device scratch of >= lf_workspace_bytes(), 256-byte aligned.
 * Errors: LF_ERR_NULL, LF_ERR_SHAPE, LF_ERR_DTYPE, LF_ERR_ALIGN, LF_ERR_BUDGET (counts
 *   negative, exceeding their candidate sets, list_len inconsistent, more than 2048
 *   candidate blocks, 1024 candidate frames, 4096 history frames or 1024 frames per chunk),
 *   LF_ERR_WORKSPACE, LF_ERR_HIP.
 */
int lf_select_mask(const void* Q, const void* Kcache, const lf_shape* shape,
                   const lf_budget* budget, int32_t* indices, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/*
 * Blockwise sparse attention (Eq. 13): for every query token x of query block r
 *   O_x = sum_y softmax_y(q_x . k_y * softmax_scale) v_y,
 * y ranging over exactly the tokens of the KV blocks listed for (head, r); unlisted tiles
 * are skipped, never materialised (Eq. 3 and the paragraph after it).  bf16 MFMA products,
 * float32 online softmax and accumulation, bfloat16 output.
 * Arguments
 *   Q, Kcache, Vcache  device, bfloat16, layout above.
 *   indices            device, int32 [H][n_q][list_len]; ids outside [0, n_k) are skipped;
 *                      order is free, duplicates count twice.  list_len >= 1; the rows of a
 *                      query block whose list holds no valid id are written as zeros.
 *   softmax_scale      0 selects 1/sqrt(d).
 *   O                  device, bfloat16 [H][q_len][d] with the o_ strides, written.
 * Errors: LF_ERR_NULL, LF_ERR_SHAPE, LF_ERR_DTYPE, LF_ERR_ALIGN, LF_ERR_BUDGET
 *   (list_len < 1), LF_ERR_HIP.
 */
int lf_sparse_attn(const void* Q, const void* Kcache, const void* Vcache,
                   const lf_shape* shape, const int32_t* indices, int32_t list_len,
                   float softmax_scale, void* O, void* hip_stream);

/*
 * Blockwise sparse attention (Eq. 13) in two phases, for lists written by lf_select_mask with
 * budget->current_mandatory = 1.  The always-selected current-chunk frames of Eq. 9 put the same
 * f*nb KV blocks, one contiguous token range, into every list of a head; that part of every row's
 * softmax is a plain dense attention problem and is computed by a dense kernel (128 query rows
 * per workgroup share each K/V tile), which leaves an online-softmax state per query row
 * (reference m, row sum l, unnormalised O, float32) in `workspace`; the list-driven kernel then
 * continues that state over the first budget->k_blocks entries of each list and writes O.  The
 * result is the softmax over the union, as lf_sparse_attn computes it in one pass.
 * Arguments as lf_sparse_attn, plus
 *   budget     the budget the lists were selected with.  Entries [k_blocks, list_len) of every
 *              list are taken to be the current chunk's blocks F_h*nb .. n_k-1 (what
 *              lf_select_mask writes) and are not read.  With current_mandatory = 0 nothing is
 *              common to all lists and the call is lf_sparse_attn (workspace unused).
 *   workspace  device scratch of >= lf_attn_workspace_bytes(shape), 256-byte aligned; contents
 *              need not be preserved or cleared between calls.
 * Errors: as lf_sparse_attn and LF_ERR_BUDGET as lf_select_mask; LF_ERR_WORKSPACE.
 */
size_t lf_attn_workspace_bytes(const lf_shape* shape);
int lf_sparse_attn_split(const void* Q, const void* Kcache, const void* Vcache,
                         const lf_shape* shape, const lf_budget* budget, const int32_t* indices,
                         float softmax_scale, void* O, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * Training pair for the blockwise sparse attention (Eq. 13; the paper finetunes the generator
 * with the sparse mask in place, Sec. 5 "Experimental Details", which needs the gradient of
 * Eq. 13 through the kept tiles; the lists themselves carry no gradient).
 *
 * lf_sparse_attn_fwd is lf_sparse_attn that also leaves, per query row x,
 *   lse2_x = log2 sum_y exp2(q_x . k_y * softmax_scale * log2 e)   over the row's kept tokens
 * (float32 [H][q_len], contiguous; +inf for a row whose list holds no valid id).
 *
 * lf_sparse_attn_bwd computes, for an upstream gradient dO and with p_xy = exp2(s_xy log2 e -
 * lse2_x), s_xy = softmax_scale q_x . k_y, delta_x = dO_x . O_x:
 *   dV_y = sum_x p_xy dO_x
 *   dQ_x = softmax_scale sum_y p_xy (dO_x . v_y - delta_x) k_y
 *   dK_y = softmax_scale sum_x p_xy (dO_x . v_y - delta_x) q_x
 * the sums running over exactly the (query block, KV block) tiles the lists keep.  bf16 MFMA
 * products (p and p (dp - delta) are rounded to bfloat16 before the accumulating products),
 * float32 accumulation in a fixed order (no atomics: results are reproducible), bfloat16 output.
 * Arguments
 *   Q, Kcache, Vcache, shape, softmax_scale   as in the forward call.
 *   O, dO          device, bfloat16 [H][q_len][d], both with the o_ strides; O as the forward
 *                  call wrote it.
 *   lse2           device, float32 [H][q_len], as the forward call wrote it.
 *   indices        device, int32 [H][n_q][list_len], the forward call's lists.  Every list must
 *                  be strictly ascending as a whole, compared as signed integers (what
 *                  lf_select_mask writes; ids outside [0, n_k) are skipped, so negative ones may
 *                  only lead and ids >= n_k only trail).  This is not checked: the key-major
 *                  launch finds the query blocks that keep a KV block by bisection, and lists
 *                  in another order or with repeated ids give wrong dK and dV.
 *   dQ             device, bfloat16, written, with the q_ strides.
 *   dK, dV         device, bfloat16, written for every KV token (zeros where no list keeps the
 *                  token's block), with the k_ and v_ strides.
 *   workspace      device scratch of >= lf_attn_bwd_workspace_bytes(shape), 256-byte aligned;
 *                  holds delta and the transposed lists during the call.
 * Errors: as lf_sparse_attn; LF_ERR_WORKSPACE.
 */
int lf_sparse_attn_fwd(const void* Q, const void* Kcache, const void* Vcache,
                       const lf_shape* shape, const int32_t* indices, int32_t list_len,
                       float softmax_scale, void* O, float* lse2, void* hip_stream);
size_t lf_attn_bwd_workspace_bytes(const lf_shape* shape);
int lf_sparse_attn_bwd(const void* Q, const void* Kcache, const void* Vcache, const void* O,
                       const void* dO, const float* lse2, const lf_shape* shape,
                       const int32_t* indices, int32_t list_len, float softmax_scale,
                       void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                       void* hip_stream);

/*
 * Pooled-key cache (an extension the paper does not describe; it follows from its setting).
 * The keys of a finished chunk never change again (Sec. 3: the rollout appends each generated
 * chunk's K/V to the cache and later chunks only read it), so their block means and frame means
 * (Eq. 7) need not be recomputed by every call: only Q and the chunk being denoised change
 * between the calls of a rollout.  The cache holds, for up to max_frames frames,
 *   k_tilde  float32 [H][d/4][max_frames*nb][4]   block means, row = KV block id
 *   k_hat    float32 [H][d/4][max_frames][4]      frame means, row = frame id (every frame)
 * in this order, channel-quad major as in lf_workspace_layout.  The caller owns the memory
 * (device, 256-byte aligned, >= lf_kcache_bytes()) and keeps it between calls.
 *
 * lf_kcache_bytes   bytes for `shape` (heads, head_dim, frame_len, block are read) and
 *                   max_frames; 0 on bad input.
 * lf_kcache_update  pools frames [frame_begin, frame_end) of Kcache into the cache, with the
 *                   arithmetic of lf_select_mask.  0 <= frame_begin <= frame_end <= frames of
 *                   Kcache (kv_len / frame_len) <= max_frames; an empty range enqueues nothing.
 * lf_select_mask_cached  lf_select_mask with k_tilde and k_hat taken from the cache.  If
 *                   Kcache is not NULL, the block means of the current chunk's frames
 *                   [n_hist_frames, n_hist_frames + frames_per_chunk) are first refreshed from
 *                   it, in the same launch that pools Q (their frame means are left alone:
 *                   candidate frames are history frames; lf_kcache_update writes them when the
 *                   chunk is committed); with Kcache NULL only Q is read.  Returns the same
 *                   lists as lf_select_mask bit for bit, provided the history frames have been
 *                   updated from the keys the caller would pass to lf_select_mask (and the
 *                   current ones too when Kcache is NULL).  workspace: device scratch,
 *                   256-byte aligned, of >= heads * n_q * head_dim * 4 bytes
 *                   (lf_workspace_bytes() is enough).
 * Errors: as lf_select_mask; LF_ERR_SHAPE for a bad frame range or max_frames;
 *   LF_ERR_WORKSPACE for a cache or workspace that is missing or too small.
 */
size_t lf_kcache_bytes(const lf_shape* shape, int32_t max_frames);
int lf_kcache_update(const void* Kcache, const lf_shape* shape, int32_t frame_begin,
                     int32_t frame_end, int32_t max_frames, void* kcache, size_t kcache_bytes,
                     void* hip_stream);
int lf_select_mask_cached(const void* Q, const void* Kcache, void* kcache, size_t kcache_bytes,
                          int32_t max_frames, const lf_shape* shape, const lf_budget* budget,
                          int32_t* indices, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/*
 * Mask selection for callers that cannot allocate or hand over scratch memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same
 * kernels and same lists as lf_select_mask, but the intermediates (q_tilde, k_tilde, k_hat) live
 * in a device array that is part of the library itself: lf_static_scratch_bytes() = 16 MiB per
 * GPU, held from the moment the library is loaded on that GPU until the process ends.  The call
 * allocates and frees nothing.
 *   lf_init                   looks up the array's address on the CURRENT device (once per
 *                             device; later calls return at once).  lf_select_mask_static does
 *                             this itself on its first call per device; call lf_init beforehand
 *                             where that lookup must not happen inside the call (e.g. before
 *                             starting a graph capture).  Returns LF_OK or LF_ERR_HIP.
 *   lf_select_mask_static     arguments as lf_select_mask, without the workspace.
 * Limits and sharing: shapes whose lf_workspace_bytes() exceeds lf_static_scratch_bytes() are
 * rejected with LF_ERR_WORKSPACE (the last-chunk configuration at 12 heads needs 3.7 MiB, at 40
 * heads 12.3 MiB).  All calls on one GPU share that GPU's array: calls that may overlap on the
 * same GPU (different streams) race; calls on one stream are ordered and safe.  Nothing has to
 * be cleared between calls: every intermediate a call reads it has written first.
 * Errors: as lf_select_mask, with LF_ERR_WORKSPACE as above.
 */
int lf_init(void);
size_t lf_static_scratch_bytes(void);
int lf_select_mask_static(const void* Q, const void* Kcache, const lf_shape* shape,
                          const lf_budget* budget, int32_t* indices, void* hip_stream);

/*
 * Producer of Q and K beside the hot path ("Efficient Deployment": the paper deploys fused
 * RoPE and RMSNorm kernels next to the sparse attention; it defines neither, so these are the
 * textbook operators).  For every token l and head h of a token-major activation X[l][h*d + c]:
 *   RMSNorm   y_c = x_c / sqrt(mean(x^2) + eps) * g_c, the mean taken over the d channels of the
 *             head (across_heads = 0) or over all H*d channels of the token (across_heads = 1);
 *   rotation  channel pair i of the head by the token's angle theta[l][i], given as cos and sin:
 *             (a, b) -> (a cos - b sin, a sin + b cos); pairing 0: pair i = channels (2i, 2i+1),
 *             pairing 1: pair i = channels (i, i + d/2).  One table serves all heads;
 *   output    Y[h][l][c] bfloat16, head-major: with Y pointing into Q or at the first token of
 *             the current chunk inside the K cache, and y_stride_* equal to that tensor's
 *             strides, the result is exactly what lf_select_mask and lf_sparse_attn read.
 * Arithmetic: float32 throughout, one rounding to bfloat16 at the end.
 * Arguments
 *   X     device, bfloat16 [tokens][>= H*d], row stride x_stride_tok elements.
 *   g     device, float32 [H*d] norm weight.   cos, sin  device, float32 [tokens][d/2].
 *   Y     device, bfloat16, written.  All pointers 16-byte aligned, strides multiples of 8.
 * Errors: LF_ERR_NULL, LF_ERR_SHAPE (head_dim not 64 or 128, sizes < 1, strides too small,
 *   flags other than 0 / 1, eps negative or not finite), LF_ERR_ALIGN, LF_ERR_HIP.
 */
typedef struct {
  int32_t heads;        /* H */
  int32_t head_dim;     /* d: 64 or 128 */
  int32_t tokens;       /* L */
  int32_t across_heads; /* 0 / 1 */
  int32_t pairing;      /* 0 interleaved, 1 half */
  float eps;
  int64_t x_stride_tok; /* elements, >= H*d */
  int64_t y_stride_tok, y_stride_head;
} lf_producer_shape;

int lf_qk_norm_rope(const void* X, const float* g, const float* cos_table, const float* sin_table,
                    const lf_producer_shape* shape, void* Y, void* hip_stream);

/* Static, NUL-terminated description of an lf_status value. */
const char* lf_strerror(int status);

/* Library version as major*10000 + minor*100 + patch. */
int lf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LF_H */
