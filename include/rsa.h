/*
 * rsa.h -- C-ABI of librsa.so: rectified block-sparse self-attention of a video DiT
 * (Rectified SpaAttn, arXiv 2511.19835) for one AMD MI355X (gfx950).
 *
 * One attention layer is three calls on one HIP stream, with no host synchronisation
 * in between (paper Alg. 1):
 *
 *   rsa_pool                   steps 1-11   pooling, implicit full attention (IPAR),
 *                                           compensation mask (GAPR)
 *   rsa_select_blocks          steps 13-14, 19   sparse mask, block lists, factor R
 *   rsa_sparse_attn_rectified  steps 16-23  block-sparse attention + rectification
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller. The library never
 *     allocates, frees or synchronises; all work is enqueued on `stream` (a hipStream_t
 *     passed as void*; NULL is the default stream). Outputs are fully overwritten.
 *   - Q, K, V, O are bf16, token order [video | text] (Alg. 1 steps 1-2, 23), addressed as
 *     ptr[b*stride_b + h*stride_h + t*stride_t + c], c < head_dim contiguous. Strides are
 *     in elements and must be multiples of 8 (16-byte rows).
 *   - Blocks (Sec. 3.1): B = B^q = B^k = `block`. Video block m < N covers tokens
 *     [m*B, min((m+1)*B, T_v)); text block N+i covers [T_v + i*B, min(T_v + (i+1)*B, T)).
 *     N = ceil(T_v/B), M = N + ceil(T_t/B). Text always starts a block of its own (isolated
 *     pooling, Sec. 4.1); the last video and last text block may be ragged. Query blocks use
 *     the same partition: blocks n < N are the sparse rows, text query blocks run dense.
 *   - Pooled/score tensors are fp32, contiguous, batch-major then head-major:
 *     [batch][heads][...].  W = ceil(M/32) 32-bit words per bit-mask row, bit (m % 32) of
 *     word (m / 32) is block m; bits at m >= M are zero.
 *   - Return value: RSA_OK or a negative RSA_E_* code. Arguments are validated on the host
 *     before anything is launched: with any code but RSA_E_LAUNCH nothing has been enqueued.
 *     RSA_E_LAUNCH (the HIP runtime refused a kernel launch) may leave the kernels launched
 *     before the refused one enqueued; the outputs are then unspecified. No exceptions, no exit.
 *   - Results are deterministic (no atomics on any output path).
 */
#ifndef RSA_H
#define RSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RSA_OK = 0,
  RSA_E_NULL = -1,        /* a required pointer is NULL */
  RSA_E_SHAPE = -2,       /* non-positive sizes, misaligned strides */
  RSA_E_UNSUPPORTED = -3, /* head_dim or block outside {64,128}, M > RSA_MAX_BLOCKS,
                             block * stride_t * 2 bytes >= 2^31 */
  RSA_E_WORKSPACE = -4,   /* workspace smaller than rsa_workspace_bytes says */
  RSA_E_RANGE = -5,       /* sparsity / p / mode / flags out of range */
  RSA_E_LAUNCH = -6       /* the HIP runtime refused a launch */
};

#define RSA_MAX_BLOCKS 4096 /* largest M = key blocks per (batch, head) */
#define RSA_STATIC_SCRATCH_BYTES (16u << 20) /* scratch held per GPU for rsa_sparse_attn_rectified_static */

/* Problem statement of Alg. 1 ("Require": Q, K, V, T_v, T_t) plus the block size of Sec. 3.1. */
typedef struct rsa_shape {
  int32_t batch;     /* >= 1 */
  int32_t heads;     /* >= 1 */
  int32_t head_dim;  /* d: 64 or 128 */
  int32_t block;     /* B: 64 or 128 */
  int64_t t_video;   /* T_v >= 1 */
  int64_t t_text;    /* T_t >= 0 */
  int64_t stride_b, stride_h, stride_t; /* element strides of Q, K, V and O */
  float scale;       /* softmax scale; 0 selects 1/sqrt(d) (Sec. 3.1) */
} rsa_shape;

/* rsa_sparse_attn_rectified flags */
#define RSA_RECTIFY_CRITICAL 1 /* multiply video rows by R_n      (Alg. 1 step 20) */
#define RSA_COMPENSATE 2       /* add the pooled non-critical term (Alg. 1 steps 21-22) */
#define RSA_DENSE 4            /* ignore lists: every query block attends to all M blocks,
                                  no rectification (full attention, Sec. 3.1) */

/* Host only. N (video blocks), M (all key blocks) and W (mask words per row) for a shape. */
int rsa_block_counts(const rsa_shape* shape, int64_t* n_video_blocks, int64_t* n_blocks,
                     int64_t* mask_words);

/* Host only. Bytes of device scratch rsa_pool and rsa_sparse_attn_rectified need. */
int rsa_workspace_bytes(const rsa_shape* shape, size_t* pool_ws_bytes, size_t* attn_ws_bytes);

/*
 * Alg. 1 steps 1-11.
 *   Qp  [b][h][N][d]  block means of the video queries      (Sec. 3.2 pooled equations)
 *   Kp  [b][h][M][d]  block means of all key blocks; a text block's mean is only used by
 *                     the gain/error gate, never by the implicit attention
 *   Vp  [b][h][M][d]  block means of V                      (Alg. 1 step 3)
 *   Vt  [b][h][M][d][B] bf16: V of each key block stored channel-major so the P.V product
 *                     reads it like K; tokens past the end of a ragged block are zero.
 *                     Within every run of 16 tokens the two middle groups of four are
 *                     swapped (order 0-3, 8-11, 4-7, 12-15). Opaque to callers: pass it on
 *                     to rsa_sparse_attn_rectified.
 *   Spool [b][h][N][M] raw pooled scores  s^pool = q^pool . k^pool * scale   (Sec. 3.2)
 *   Lmass [b][h][N][M] block log-mass: s^pool + ln(c_m) for a video block (c_m = tokens in
 *                     the block), log-sum-exp over the block's individual token scores
 *                     q^pool . k_t * scale for a text block (Sec. 4.1, isolated pooling)
 *   Apool [b][h][N][M] implicit full attention A^pool = row-softmax(Lmass); equal to the
 *                     paper's reallocation: video block weights times block size, text
 *                     token weights summed per block, renormalised (Sec. 4.1)
 *   Mc_bits [b][h][N][W] compensation mask M_c (Sec. 4.2). gapr_mode 0: all zero;
 *                     2: all ones; 1: bit set iff  |s^pool| > DA + DB  with
 *                     DA = mean_i |(q_i - q^pool_n).k^pool_m| * scale and
 *                     DB = mean_j |q^pool_n.(k_j - k^pool_m)| * scale, i.e. the gain
 *                     |sum_ij s^pool| exceeds the first-order pooling error with the
 *                     absolute value taken per term (the printed signed sum vanishes).
 *   ws / ws_bytes     device scratch, at least pool_ws_bytes, 256-byte aligned.
 */
int rsa_pool(const rsa_shape* shape, const void* Q, const void* K, const void* V,
             float* Qp, float* Kp, float* Vp, void* Vt,
             float* Spool, float* Apool, float* Lmass, uint32_t* Mc_bits, int gapr_mode,
             void* ws, size_t ws_bytes, void* stream);

/*
 * The value part of rsa_pool alone (Alg. 1 step 3 for V): Vp and the channel-major copy Vt of a
 * new V, nothing else. For callers that keep the masks, lists, factors and A^pool of an earlier
 * call (the paper combines the method with caches across diffusion steps, Sec. 5 and appendix
 * "Implementations") and only
 * attend again with new tensors: rsa_pool_values(V') then rsa_sparse_attn_rectified(Q', K', Vt', ...).
 * Same layouts and ownership as in rsa_pool; Vp and Vt are fully overwritten.
 */
int rsa_pool_values(const rsa_shape* shape, const void* V, float* Vp, void* Vt, void* stream);

/*
 * Alg. 1 steps 5-7 alone (Sec. 3.2, Sec. 4.1): the implicit full attention from pooled vectors that
 * an earlier rsa_pool call left in Qp and Kp, together with the text keys of K -- Spool, Lmass and
 * Apool exactly as rsa_pool writes them, nothing else. For callers that re-derive A^pool from stored
 * pooled vectors, and the unit this stage is timed in. Same layouts and ownership as in rsa_pool; the
 * three outputs are fully overwritten.
 */
int rsa_implicit_attention(const rsa_shape* shape, const void* K, const float* Qp, const float* Kp,
                           float* Spool, float* Lmass, float* Apool, void* stream);

/*
 * Alg. 1 steps 13-14 and 19, per video query block n:
 *   keep the k = clamp(M - floor(sparsity*M + 1e-6), 1, M) blocks of largest Lmass (equal
 *   keys: lower block index first); if p > 0 extend, in the same descending order, until
 *   the kept A^pool weight exceeds p; OR with forced_bits (the adjacency mask M_adja,
 *   [b][h][N][W], may be NULL).
 *   mask_bits [b][h][N][W]  the sparse mask
 *   block_idx [b][h][N][M]  kept block indices, ascending, first count[n] entries valid
 *   count     [b][h][N]
 *   R         [b][h][N]     rectification factor: sum of A^pool over kept blocks (Sec. 4.1)
 * sparsity in [0,1], p in [0,1].
 */
int rsa_select_blocks(const rsa_shape* shape, const float* Lmass, const float* Apool,
                      double sparsity, double p, const uint32_t* forced_bits,
                      uint32_t* mask_bits, int32_t* block_idx, int32_t* count, float* R,
                      void* stream);

/*
 * Appendix "Implementations" (the token sequence is reordered before inference so that blocks
 * hold spatially close tokens): moves the rows of one [b][h][T][d] bf16 tensor between raster
 * order (token index (t*H + h)*W + w) and the tile order the other entry points expect (tiles of
 * `tile` in raster order over the (T, H, W) grid, tokens in raster order inside a tile). Text
 * rows [t_video, T) keep their place.
 *   direction 0: dst[tile-order position] = src[raster index]   (before the layer: Q, K, V)
 *   direction 1: dst[raster index] = src[tile-order position]   (after the layer: O)
 *   grid [3], tile [3]: HOST arrays; T*H*W must equal t_video. src and dst: device, both with the
 *   strides of `shape`, must not alias (RSA_E_RANGE). dst is fully overwritten.
 */
int rsa_reorder_tokens(const rsa_shape* shape, const int32_t* grid, const int32_t* tile, int direction,
                       const void* src, void* dst, void* stream);

/*
 * Alg. 1 "Require" and step 14, Sec. 4.3 (spatial-temporal neighbour blocks are always kept):
 * the adjacency mask M_adja for a video latent grid whose tokens are stored tile by tile
 * (tiles in raster order over (T, H, W), tokens in raster order inside a tile, partial tiles
 * at the upper faces of the grid). A video query block n and a video key block m are
 * neighbours when some tile touched by n and some tile touched by m differ by at most
 * `radius` in every tile coordinate (radius 1: the block itself and the surrounding 26 tiles
 * where blocks and tiles coincide). Text key blocks are never set.
 *   grid [3], tile [3]   HOST arrays (T, H, W) and (tile_t, tile_h, tile_w); T*H*W must equal
 *                        t_video (RSA_E_SHAPE otherwise); radius in [0, 64]
 *   forced_bits          device, [b][h][N][W] u32, fully overwritten (same rows for every b, h);
 *                        pass it to rsa_select_blocks
 */
int rsa_adjacency_mask(const rsa_shape* shape, const int32_t* grid, const int32_t* tile, int radius,
                       uint32_t* forced_bits, void* stream);

/*
 * Alg. 1 steps 16-23. For video query block n: online-softmax attention of its tokens over
 * the tokens of the blocks in block_idx[n][0..count[n]) only (masked keys are excluded from
 * the softmax, Sec. 3.1), times R[n] (RSA_RECTIFY_CRITICAL), plus
 * sum_{m: not mask and M_c} Apool[n][m] * Vp[m] (RSA_COMPENSATE). Text query blocks: full
 * attention over all tokens. O has the layout of Q. `lse` (nullable, [b][h][T] fp32)
 * receives the natural-log softmax denominator (including the row maximum) of the
 * un-rectified sparse/dense attention of every row.
 * With RSA_DENSE every list/mask/R/Apool/Mc/Vp pointer may be NULL.
 * ws / ws_bytes: device scratch of at least attn_ws_bytes, 256-byte aligned (RSA_E_WORKSPACE
 * otherwise). It receives the pooled compensation term C_n (fp32 [b][h][N][d], Alg. 1 step 21),
 * an order of the video query blocks (rows with similar lists next to each other, so that they
 * share K/V tiles in the L2 of their XCD) and the schedule that deals the query blocks, in that
 * order and balanced by the length of their lists, to the resident workgroups of the attention
 * kernel; the results do not depend on the order or the schedule. Required with RSA_COMPENSATE
 * (RSA_E_NULL); without that flag it may be NULL, and the query blocks are then dealt in index
 * order. With RSA_DENSE a workspace that is too small or misaligned is ignored (index order).
 * The caller owns it; its contents afterwards are unspecified.
 */
int rsa_sparse_attn_rectified(const rsa_shape* shape, const void* Q, const void* K, const void* Vt,
                              const int32_t* block_idx, const int32_t* count,
                              const uint32_t* mask_bits, const float* R, const float* Apool,
                              const uint32_t* Mc_bits, const float* Vp, int flags,
                              void* O, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * For callers that cannot allocate device memory or hand over a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc. Same computation, arguments,
 * results and error codes as rsa_sparse_attn_rectified, without ws / ws_bytes: the scratch (C_n, the
 * order of the query blocks and their schedule) lives in a device array of RSA_STATIC_SCRATCH_BYTES (16 MiB) that is part of the
 * library image, one copy per GPU, held until the process ends. The call allocates and frees nothing.
 * Its first call on a device looks up that device's copy (hipGetSymbolAddress; RSA_E_LAUNCH if that
 * fails). Shapes whose attn_ws_bytes (rsa_workspace_bytes) exceed RSA_STATIC_SCRATCH_BYTES are
 * refused with RSA_E_WORKSPACE before anything is enqueued: 4 * batch * heads * N * (head_dim + 1)
 * bytes plus the schedule tables and padding, e.g. 11.7 MB for 24 heads of 118 800 + 256 tokens at
 * block 128, head_dim 128.
 * Every call on a GPU uses that GPU's one array and overwrites all of it that it reads (nothing has
 * to start at zero); two calls that overlap in time on one GPU (different streams) race on it.
 * With RSA_DENSE the scratch is not touched (the query blocks are dealt in index order).
 */
int rsa_sparse_attn_rectified_static(const rsa_shape* shape, const void* Q, const void* K, const void* Vt,
                                     const int32_t* block_idx, const int32_t* count,
                                     const uint32_t* mask_bits, const float* R, const float* Apool,
                                     const uint32_t* Mc_bits, const float* Vp, int flags,
                                     void* O, float* lse, void* stream);

/* Static string for a return code. */
const char* rsa_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* RSA_H */
