/* libbct -- the Llama-shaped glue around the bounded-cache attention layer.
 *
 * The paper applies its mechanism to the attention layers of a decoder-only
 * Transformer and obtains the write query and the write key-value vector from
 * the layer input with two learnable matrices (section 3.2 step 1, Algorithm 1:
 * wq_t = W_wq x_t, wv_t = W_wv x_t).  These entry points are the dense pieces
 * of such a stack, so that a token can go through whole layers on the GPU:
 * embedding lookup, RMS normalisation, the projections (W_q, W_wq, W_wv, W_o,
 * the SwiGLU MLP, the output head) and the greedy arg-max.  The attention
 * itself stays bct_decode_step / bct_prefill (include/bct.h).
 *
 * All data pointers are DEVICE memory owned by the caller, bf16, row-major,
 * 16-byte aligned; token ids are int32.  Calls enqueue on the given stream and
 * return.  Status codes are those of include/bct.h.
 */
#ifndef BCT_MODEL_H
#define BCT_MODEL_H

#include <stddef.h>
#include <stdint.h>

#include "bct.h"

#ifdef __cplusplus
extern "C" {
#endif

/* out[r][:] = table[ids[r]][:], r < rows.  table [vocab][dim]; dim a multiple of 8.
 * Ids outside [0, vocab) give a zero row. */
bct_status bctm_embed(const int32_t* ids, const void* table, void* out, uint32_t rows, uint32_t vocab,
                      uint32_t dim, void* hip_stream);

/* Tiled activations.  A [rows][K] activation matrix that feeds a projection can be kept in the order the
 * projection's MFMA reads it, so that every wavefront load is one contiguous kilobyte: rows in groups of
 * 32, columns in groups of 32; group (r / 32, k / 32) is the 2 KB block number (r / 32) * (K / 32) + k / 32,
 * made of two 1 KB halves (rows 0-15, rows 16-31 of the group); in a half, element (r, k) sits at bf16
 * offset 8 * (16 * ((k % 32) / 8) + r % 16) + k % 8.  K must be a multiple of 32 and the buffer holds
 * 32 * ceil(rows / 32) * K bf16; rows past the end are never read for a stored result. */
#define BCTM_X_TILED 1u   /* the input x is tiled */
#define BCTM_OUT_TILED 2u /* the output is written tiled */

/* Row-major x [rows][K] -> tiled (above).  tiled must not be x. */
bct_status bctm_pack_rows(const void* x, void* tiled, uint32_t rows, uint32_t K, void* hip_stream);

/* out[r][:] = x[r][:] * rsqrt(mean(x[r][:]^2) + eps) * gain[:]   (fp32 arithmetic, bf16 in/out).
 * dim a multiple of 8, at most 16384.  flags: BCTM_OUT_TILED (then dim a multiple of 32, out not x). */
bct_status bctm_rmsnorm(const void* x, const void* gain, void* out, uint32_t rows, uint32_t dim, float eps,
                        uint32_t flags, void* hip_stream);

/* Repacks a row-major weight matrix w [N][K] (one output feature per row) into the streaming layout
 * bctm_linear and bctm_swiglu read: 1 KB tiles of 16 features x 32 inputs, tile (n / 16, k / 32) at tile
 * index (n / 16) * (K / 32) + k / 32; inside a tile, element (n, k) sits at bf16 offset
 * 8 * (16 * ((k % 32) / 8) + n % 16) + k % 8.  Done once when weights are loaded.
 * N a multiple of 16, K a multiple of 32; packed holds N * K bf16 and must not be w. */
bct_status bctm_pack_weight(const void* w, void* packed, uint32_t N, uint32_t K, void* hip_stream);

/* out[r][n] = (residual ? residual[r][n] : 0) + sum_k x[r][k] * w[n][k].
 * x [rows][K] row-major, or tiled with flags = BCTM_X_TILED; w_packed = bctm_pack_weight of w [N][K];
 * out/residual [rows][N] row-major;
 * K a multiple of 32, N a multiple of 16; fp32 accumulation (MFMA), one rounding to bf16 at the end.
 * out may alias residual; x must not alias out.  Two kernels: up to 127 rows (a decode batch) the weights
 * are streamed once per 32 rows against activations read from cache; from 128 rows on (a prompt chunk), when
 * N is a multiple of 128 (bctm_swiglu: 64), a tiled matrix-core kernel with 128 x 128 or 256 x 256 workgroups
 * runs instead - fastest with a tiled x.  Both give the sum in fp32 with their own, fixed, summation order. */
bct_status bctm_linear(const void* x, const void* w_packed, const void* residual, void* out, uint32_t rows,
                       uint32_t K, uint32_t N, uint32_t flags, void* hip_stream);

/* One projection with up to three row-major outputs: w_packed holds N0 + N1 + N2 features (packed as one
 * matrix, or matrix by matrix into consecutive parts of one buffer), the first N0 go to out0 [rows][N0], the
 * next N1 to out1 [rows][N1], the last N2 to out2 [rows][N2] (N2 may be 0, out2 then unused).  Every width a
 * multiple of 16.  For W_q, W_wq and W_wv, which read the same input. */
bct_status bctm_linear_split(const void* x, const void* w_packed, void* out0, uint32_t N0, void* out1, uint32_t N1,
                             void* out2, uint32_t N2, uint32_t rows, uint32_t K, uint32_t flags, void* hip_stream);

/* out[r][n] = silu(sum_k x[r][k] w_gate[n][k]) * (sum_k x[r][k] w_up[n][k]),  silu(a) = a / (1 + exp(-a)).
 * Both weights packed; same shape rules as bctm_linear.  flags: BCTM_X_TILED, BCTM_OUT_TILED (the output
 * as tiled activations of N columns, N a multiple of 32, ready to feed the next projection). */
bct_status bctm_swiglu(const void* x, const void* w_gate_packed, const void* w_up_packed, void* out, uint32_t rows,
                       uint32_t K, uint32_t N, uint32_t flags, void* hip_stream);

/* Which kernel bctm_linear / bctm_linear_split (swiglu = 0) or bctm_swiglu (swiglu = 1) launches for a
 * shape: host logic only, no GPU call.  *kernel receives one of the values below. */
#define BCTM_KERNEL_STREAMING 0u /* weights streamed once per 32 rows (one 16-feature tile per workgroup) */
#define BCTM_KERNEL_STREAMING_WIDE 1u /* the same with two feature tiles per workgroup (wide output heads) */
#define BCTM_KERNEL_TILE128 2u   /* matrix-core kernel, 128 rows x 128 features per workgroup */
#define BCTM_KERNEL_TILE256 3u   /* matrix-core kernel, 256 rows x 256 features per workgroup */
#define BCTM_KERNEL_STREAMING_TRIPLE 4u /* streaming with three feature tiles per workgroup */
bct_status bctm_linear_plan(uint32_t rows, uint32_t K, uint32_t N, uint32_t swiglu, uint32_t* kernel);

/* ids[r] = index of the largest logits[r][:] (the lowest index among equal maxima). */
bct_status bctm_argmax(const void* logits, int32_t* ids, uint32_t rows, uint32_t N, void* hip_stream);

/* Thread-local detail of the last failure of a bctm_ call. */
const char* bctm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BCT_MODEL_H */
