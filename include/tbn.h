/*
 * tbn.h -- C ABI of libtbn: inference kernels for tiled-bit layers on AMD MI355X (gfx950).
 *
 * A tiled-bit layer (Tiled Bit Networks, arXiv 2407.12075, Section "Method") stores, for a
 * layer with n weights, one tile of p = n / k entries in {-1,+1} and one or k scalars alpha.
 * The dense weight it stands for is
 *
 *     B_hat[f] = alpha[n_alpha == 1 ? 0 : f / p] * t[f % p],      f = 0 .. n-1
 *
 * where f is the row-major flat index of the weight tensor ((out, in) for a fully-connected
 * layer, (O, C, kh, kw) for a convolution; last index fastest) -- Eq. 4 (tile repeated k times
 * back to back), Eq. 5 (reshape) and the per-tile scaling stated after Eq. 8.  The paper writes
 * N, p, q for what is called n, k, p here.
 *
 * Tile format (the contract for "bit exact"): an array of 32-bit words, little endian; tile
 * entry i lives in word i / 32 at bit i % 32 (least significant bit first); bit 1 means +1,
 * bit 0 means -1; unused high bits of the last word are zero.
 *
 * Conventions for every entry point
 *   - Pointers named below as DEVICE pointers must be device memory of the current HIP device;
 *     the caller owns every buffer.  The library allocates no device memory and keeps no data
 *     from one call for the next.  What it does keep per process: the permission of each kernel
 *     to use more LDS than the default limit (set on the kernel's first launch, thread safe), the
 *     last error text of each thread, and the fixed scratch array of tbn_pack_tile_noalloc.
 *     Calls from several threads are safe; the kernels of two calls that write the same buffer
 *     race like any two kernels.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     on it and the call returns without synchronising.
 *   - On TBN_ERR_NULL / _SHAPE / _UNSUPPORTED / _WORKSPACE nothing has been enqueued and no
 *     output is touched.  TBN_ERR_DEVICE reports a failed HIP launch; work enqueued before the
 *     failing launch may still run and outputs are then undefined.  tbn_last_error() describes
 *     the problem.
 *   - No bias term exists in this layer type (the paper does not use bias parameters).
 */
#ifndef TBN_H
#define TBN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TBN_OK = 0,
    TBN_ERR_NULL = 1,        /* a required pointer is NULL */
    TBN_ERR_SHAPE = 2,       /* non-positive size, n not divisible by k, n_alpha not in {1, k} */
    TBN_ERR_UNSUPPORTED = 3, /* unknown dtype or flag, size beyond the supported range */
    TBN_ERR_DEVICE = 4,      /* a HIP call failed; text in tbn_last_error() */
    TBN_ERR_WORKSPACE = 5    /* workspace missing, misaligned or too small */
} tbn_status;

typedef enum {
    TBN_F32 = 0,  /* IEEE binary32 activations, binary32 accumulation */
    TBN_BF16 = 1  /* bfloat16 activations and outputs, binary32 accumulation, outputs rounded
                     to nearest even */
} tbn_dtype;

/* flags of the forward entry points */
#define TBN_FLAG_RELU 0x1u          /* y = max(0, y): the fused ReLU of Algorithm 1 */
#define TBN_FLAG_FORCE_GENERIC 0x100u /* testing aid: skip the specialised kernels */
#define TBN_FLAG_LARGE_BATCH 0x200u   /* testing aid (linear only): batches above 64 skip the small-batch
                                         kernel, which otherwise also takes small problems at larger batches */
#define TBN_FLAG_BLOCK_KERNEL 0x400u  /* testing aid (linear only): skip the two bfloat16 kernels for tiles of whole
                                         rows, so that their shapes also reach the general matrix-core kernel */
#define TBN_FLAG_STREAM_KERNEL 0x800u /* testing aid (linear only): take the streaming kernel (half tiles, used by
                                         default for grids that leave CUs idle) wherever it supports the shape */
#define TBN_FLAG_SPLIT_K 0x1000u      /* testing aid (tbn_linear_forward_ws only): split the sum over j among
                                         workgroups wherever the shape allows, also where the cost model expects
                                         no gain */
#define TBN_FLAG_TILE_KERNEL 0x2000u  /* testing aid (linear only): take the kernel with one wave per 32 batch rows
                                         wherever it supports the shape */
#define TBN_FLAG_SIGN_OUT 0x4000u     /* tbn_linear_forward_binact only: write the sign bits of the outputs instead
                                         of the outputs (the input format of the next such layer) */

/* Number of 32-bit words of a tile of n / k entries (ceil(n / k / 32)); 0 if n <= 0, k <= 0 or
 * k does not divide n (the paper requires n divisible by the compression factor). */
size_t tbn_tile_words(int64_t n, int32_t k);

/* Message for the last non-OK status returned on the calling thread; never NULL. */
const char *tbn_last_error(void);

/* Library version string, static storage. */
const char *tbn_version(void);

/* Bytes of device workspace tbn_pack_tile needs for these sizes (0 on invalid sizes). */
size_t tbn_pack_workspace_bytes(int64_t n, int32_t k, int32_t n_alpha);

/*
 * Tile construction, Eq. 1-3, and scalars, Eq. 6 (n_alpha == 1) or Eq. 7-8 (n_alpha == k).
 *
 *   s[i]      = sum_{r=0}^{k-1} w_real[r * p + i]      (double precision, r ascending)
 *   tile[i]   = +1 if s[i] > 0, else -1                (zero and NaN give -1)
 *   alpha[0]  = sum_f |a[f]| / n                                        if n_alpha == 1
 *   alpha[r]  = sum_{i<p} |a[r * p + i]| / p,  r = 0..k-1               if n_alpha == k
 *
 * with a = a_real if it is not NULL, else w_real (the paper's separate tensor A for the
 * scalars is optional).  alpha sums are taken in double precision and rounded once to float.
 *
 *   w_real, a_real : DEVICE, n floats each, flattened row-major weight tensor; read only
 *   tile_out       : DEVICE, tbn_tile_words(n, k) words, fully overwritten
 *   alpha_out      : DEVICE, n_alpha floats, overwritten
 *   workspace      : DEVICE, at least tbn_pack_workspace_bytes(n, k, n_alpha) bytes, 8-byte
 *                    aligned; contents on entry are ignored, contents on exit are undefined
 * Errors: TBN_ERR_NULL, TBN_ERR_SHAPE (k <= 0, n <= 0, n % k != 0, n_alpha not 1 or k),
 *         TBN_ERR_WORKSPACE, TBN_ERR_DEVICE.
 */
tbn_status tbn_pack_tile(const float *w_real, const float *a_real, int64_t n, int32_t k,
                         int32_t n_alpha, uint32_t *tile_out, float *alpha_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * tbn_pack_tile for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels, same results as
 * tbn_pack_tile; the partial sums live in an array of TBN_PACK_NOALLOC_SCRATCH_BYTES bytes that is part of the
 * library's code object (each GPU the library runs on holds it until the process ends).  The call allocates and
 * frees nothing.
 *
 *   Sizes are accepted while tbn_pack_workspace_bytes(n, k, n_alpha) <= TBN_PACK_NOALLOC_SCRATCH_BYTES (the
 *   4096 x 4096 weight with k = 8 needs half of it); beyond that TBN_ERR_UNSUPPORTED, nothing is enqueued.
 *   All calls on one GPU share the array: calls that may overlap in time (different streams, different host
 *   threads without ordering between their streams) race and must be serialised by the caller.
 * Other arguments and errors as for tbn_pack_tile.
 */
#define TBN_PACK_NOALLOC_SCRATCH_BYTES (1u << 20)
tbn_status tbn_pack_tile_noalloc(const float *w_real, const float *a_real, int64_t n, int32_t k,
                                 int32_t n_alpha, uint32_t *tile_out, float *alpha_out, void *stream);

/*
 * Fully-connected tiled-bit layer:  Y = X * B_hat^T  (the layer operation applied to B_hat,
 * stated after Eq. 8; Algorithm 1 is the same computation for one input vector).
 *
 *   y[m, o] = sum_{j<in} x[m, j] * alpha[(o*in + j) / p or 0] * t[(o*in + j) % p],  p = in*out/k
 *
 *   x     : DEVICE, M x in, row-major, dense, element type dt; read only
 *   y     : DEVICE, M x out, row-major, dense, element type dt; fully overwritten
 *   tile  : DEVICE, tbn_tile_words(in*out, k) words; read only
 *   alpha : DEVICE, n_alpha floats (n_alpha is 1 or k); read only
 *   flags : 0 or TBN_FLAG_RELU (| TBN_FLAG_FORCE_GENERIC | TBN_FLAG_LARGE_BATCH | TBN_FLAG_BLOCK_KERNEL |
 *           TBN_FLAG_STREAM_KERNEL | TBN_FLAG_TILE_KERNEL | TBN_FLAG_SPLIT_K, which only tbn_linear_forward_ws
 *           looks at)
 * M == 0 is legal and does nothing (x and y may then be NULL).  x and y must not overlap.
 * Errors: TBN_ERR_NULL, TBN_ERR_SHAPE, TBN_ERR_UNSUPPORTED, TBN_ERR_DEVICE.
 */
tbn_status tbn_linear_forward(const void *x, void *y, tbn_dtype dt, int64_t M, int64_t in,
                              int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                              int32_t n_alpha, uint32_t flags, void *stream);

/*
 * Which kernel family tbn_linear_forward would launch for these arguments (the layer operation stated after
 * Eq. 8; the families differ in schedule, never in what is computed).  Host arithmetic only: nothing is launched and
 * no pointer is dereferenced.
 *
 *   x, y : the pointers the forward call would get (any address space; only their alignment is looked at; NULL
 *          counts as aligned).
 * Returns a static string, one of "decode", "small-batch", "tile", "stream", "block", "general", "rows", "direct",
 * "generic"; "" on sizes tbn_linear_forward would reject.  The choice also depends on the current device's number
 * of CUs (256 is assumed where there is no device).  A help for tests and for reading a profile; a caller never
 * needs it.
 */
const char *tbn_linear_forward_kernel(const void *x, const void *y, tbn_dtype dt, int64_t M, int64_t in, int64_t out,
                                      int32_t k, int32_t n_alpha, uint32_t flags);

/*
 * tbn_linear_forward with a caller-supplied workspace.  Same layer (the layer operation stated after Eq. 8), same
 * arguments; the workspace lets shapes whose output blocks would occupy only a fraction of the GPU and whose
 * rows are long (bfloat16, tile of whole weight rows, more than 64 and up to a few thousand batch rows, `in` of
 * about 12288 and more: the split costs a second launch) split the sum over j among several workgroups: each writes float32 partial sums to the workspace, a second kernel adds them in ascending order of
 * j (no floating-point atomics: results are identical from run to run), scales and writes y.  The sums are
 * grouped differently from tbn_linear_forward's, so the two may differ in the last float32 bit before rounding.
 *
 *   tbn_linear_forward_workspace_bytes : bytes with which tbn_linear_forward_ws takes that path for these sizes;
 *                                        0 if no path for them uses a workspace (or on invalid sizes).
 *   workspace : DEVICE, 16-byte aligned, or NULL with workspace_bytes == 0; contents on entry are ignored, on
 *               exit undefined.  With fewer bytes than the query returns the call is exactly tbn_linear_forward.
 *               Calls that share a workspace must be ordered on one stream.
 * Errors: as tbn_linear_forward, and TBN_ERR_WORKSPACE (NULL or misaligned workspace with workspace_bytes > 0).
 */
size_t tbn_linear_forward_workspace_bytes(tbn_dtype dt, int64_t M, int64_t in, int64_t out, int32_t k, uint32_t flags);
tbn_status tbn_linear_forward_ws(const void *x, void *y, tbn_dtype dt, int64_t M, int64_t in,
                                 int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                                 int32_t n_alpha, uint32_t flags, void *workspace, size_t workspace_bytes,
                                 void *stream);

/*
 * Convolutional tiled-bit layer (the paper tiles the flattened (O, C, kh, kw) weight the same
 * way, Section "Method"; Section "CNN Architectures" gives the replicated-channel example):
 * cross-correlation with zero padding, stride (stride_h, stride_w), dilation 1, one group.
 *
 *   y[b, o, yo, xo] = sum_{c, dy, dx} B_hat[o, c, dy, dx] * x[b, c, yo*stride_h + dy - pad_h,
 *                                                                   xo*stride_w + dx - pad_w]
 *   Ho = (H + 2*pad_h - kh) / stride_h + 1,  Wo = (W + 2*pad_w - kw) / stride_w + 1
 *
 *   x : DEVICE, (N, C, H, W) row-major dense, element type dt; read only
 *   y : DEVICE, (N, O, Ho, Wo) row-major dense, element type dt; fully overwritten
 *   tile, alpha, flags : as for tbn_linear_forward with n = O*C*kh*kw
 * N == 0 is legal and does nothing (x and y may then be NULL).
 * Errors: TBN_ERR_NULL, TBN_ERR_SHAPE (also: kernel larger than the padded input),
 *         TBN_ERR_UNSUPPORTED, TBN_ERR_DEVICE.
 */
tbn_status tbn_conv2d_forward(const void *x, void *y, tbn_dtype dt, int64_t N, int64_t C,
                              int64_t H, int64_t W, int64_t O, int32_t kh, int32_t kw,
                              int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                              const uint32_t *tile, int32_t k, const float *alpha,
                              int32_t n_alpha, uint32_t flags, void *stream);

/*
 * Column-tiled variant of the fully-connected layer (Section "GPU Inference Kernel": the out x in weight
 * is kept as one out x q block, q = in / k, which is used again for each of the k column blocks; with the
 * per-copy scalars of Eq. 7-8, or the single scalar of Eq. 6):
 *
 *   W_hat[o, c*q + j] = alpha[c or 0] * t[o, j],  c < k, j < q;     Y = X * W_hat^T
 *
 * The tile holds t row-major: entry (o, j) is bit (o*q + j) % 32 of word (o*q + j) / 32, 1 means +1;
 * it has tbn_tile_words(out*in, k) words.  k must divide in.
 */

/* Bytes of device workspace tbn_pack_coltile needs (0 on invalid sizes). */
size_t tbn_pack_coltile_workspace_bytes(int64_t out, int64_t in, int32_t k, int32_t n_alpha);

/*
 * Tile and scalars of the column-tiled layout from a real out x in weight: Eq. 1-3 with the k column
 * blocks as the k summands, Eq. 6 (n_alpha == 1) or Eq. 7-8 per column block (n_alpha == k).
 *
 *   s[o, j]   = sum_{c<k} w_real[o, c*q + j]           (double precision, c ascending)
 *   t[o, j]   = +1 if s[o, j] > 0, else -1
 *   alpha[c]  = sum_{o, j} |a[o, c*q + j]| / (out*q)   (alpha[0] = sum |a| / (out*in) if n_alpha == 1)
 *
 * Arguments, workspace rules and errors as for tbn_pack_tile, with w_real / a_real of out*in floats,
 * row-major.  TBN_ERR_SHAPE also if k does not divide in.
 */
tbn_status tbn_pack_coltile(const float *w_real, const float *a_real, int64_t out, int64_t in, int32_t k,
                            int32_t n_alpha, uint32_t *tile_out, float *alpha_out, void *workspace,
                            size_t workspace_bytes, void *stream);

/* Bytes of device workspace tbn_linear_coltiled_forward needs (0 on invalid sizes). */
size_t tbn_linear_coltiled_workspace_bytes(tbn_dtype dt, int64_t M, int64_t in, int32_t k);

/*
 * Forward pass of the column-tiled layer, computed as
 *
 *   xf[m, j] = sum_{c<k} alpha[c or 0] * x[m, c*q + j]     (float32 sums, c ascending; rounded to dt)
 *   y[m, o]  = sum_{j<q} xf[m, j] * t[o, j]                (binary32 accumulation)
 *
 * i.e. k times fewer multiply-adds than the dense layer and no repeated output columns.
 *
 *   x, y, tile, alpha, flags : as for tbn_linear_forward
 *   workspace : DEVICE, at least tbn_linear_coltiled_workspace_bytes(dt, M, in, k) bytes, 16-byte
 *               aligned; holds xf during the call; contents on entry are ignored, on exit undefined.
 *               Calls that share a workspace must be ordered on one stream.
 * M == 0 is legal and does nothing.
 * Errors: TBN_ERR_NULL, TBN_ERR_SHAPE, TBN_ERR_WORKSPACE, TBN_ERR_UNSUPPORTED, TBN_ERR_DEVICE.
 */
tbn_status tbn_linear_coltiled_forward(const void *x, void *y, tbn_dtype dt, int64_t M, int64_t in,
                                       int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                                       int32_t n_alpha, uint32_t flags, void *workspace,
                                       size_t workspace_bytes, void *stream);

/*
 * Binary activations (the Conclusion names tiled-bit layers in models with binary weights and binary
 * activations as the first direction of future work and gives no formula).  The reading built here takes the
 * paper's own binarisation: an activation becomes +1 or -1 by the rule that Eq. 3 applies to a weight sum (+1
 * where the value is greater than zero, -1 otherwise: zero and not-a-number give -1), and the layer operation
 * stated after Eq. 8 is applied to those signs unchanged; no scalar is attached to the activations.
 *
 *   s[m, j] = +1 if x[m, j] > 0 else -1
 *   y[m, o] = sum_{j<in} s[m, j] * alpha[(o*in + j) / p or 0] * t[(o*in + j) % p],  p = in*out/k
 *
 * Rows of sign bits: tbn_sign_row_words(in) = ceil(in / 32) words per row; activation j of row m is bit j % 32 of
 * word j / 32 of that row (1 for +1); the unused high bits of a row's last word are written as zero by
 * tbn_sign_pack and ignored by tbn_linear_forward_binact.
 *
 *   tbn_sign_pack             : x DEVICE, M x in, row-major, dense, element type dt, read only;
 *                               xbits DEVICE, M * tbn_sign_row_words(in) words, fully overwritten.
 *   tbn_linear_forward_binact : xbits DEVICE, rows of sign bits as above, read only; y DEVICE, M x out, row-major,
 *                               dense, element type y_dt, fully overwritten; tile, alpha, k, n_alpha as for
 *                               tbn_linear_forward; flags 0 or TBN_FLAG_RELU, TBN_FLAG_SIGN_OUT (| TBN_FLAG_FORCE_GENERIC).
 * With TBN_FLAG_SIGN_OUT the layer hands on what the next binary-activation layer consumes: y is then DEVICE,
 * M * tbn_sign_row_words(out) words, rows of sign bits of the outputs (bit 1 where y[m, o] > 0, unused high bits
 * zero), fully overwritten; y_dt is not looked at beyond its validity and TBN_FLAG_RELU changes nothing (a
 * positive output stays positive).
 * The sums of +-1 products are integers and computed exactly; an output is alpha times such an integer (one
 * float32 product, rounded once more for bfloat16 outputs) unless n_alpha = k and a weight row crosses a tile
 * end, in which case the row's pieces are added in float32 in ascending order of j.
 * M == 0 is legal and does nothing.  xbits and y must not overlap.
 * Errors: TBN_ERR_NULL, TBN_ERR_SHAPE, TBN_ERR_UNSUPPORTED, TBN_ERR_DEVICE.
 */
size_t tbn_sign_row_words(int64_t in);
tbn_status tbn_sign_pack(const void *x, tbn_dtype dt, int64_t M, int64_t in, uint32_t *xbits, void *stream);
tbn_status tbn_linear_forward_binact(const uint32_t *xbits, void *y, tbn_dtype y_dt, int64_t M, int64_t in,
                                     int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                                     int32_t n_alpha, uint32_t flags, void *stream);

/*
 * Measurement aids.  No part of the method (the paper reports no kernel timings; its Section "GPU Inference Kernel"
 * measures memory only): they give the benchmark its denominators, measured the same way as the layer kernels.
 *
 *   tbn_diag_empty_launch : enqueues a kernel of one wave that does nothing (the launch floor).
 *   tbn_diag_stream       : streams `bytes` (rounded down to 16) from src -- to dst if dst is not NULL (copy), else
 *                           into a checksum that is dropped (read only).  DEVICE pointers, 16-byte aligned; sink may
 *                           be NULL or 4 bytes of device memory.
 *   tbn_diag_mfma         : `blocks` workgroups of four waves, every wave issues iters x 8 independent
 *                           32x32x16 bf16 MFMAs (2 * 32 * 32 * 16 flop each); out is NULL or blocks * 256 floats.
 *   tbn_diag_mfma_fp4     : the same with 32x32x64 MFMAs on 4-bit float operands (2 * 32 * 32 * 64 flop each), the
 *                           instruction of tbn_linear_forward_binact.
 * Errors: TBN_ERR_NULL, TBN_ERR_SHAPE, TBN_ERR_DEVICE.
 */
tbn_status tbn_diag_empty_launch(void *stream);
tbn_status tbn_diag_stream(const void *src, void *dst, size_t bytes, void *sink, void *stream);
tbn_status tbn_diag_mfma(int32_t blocks, int32_t iters, float *out, void *stream);
tbn_status tbn_diag_mfma_fp4(int32_t blocks, int32_t iters, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TBN_H */
