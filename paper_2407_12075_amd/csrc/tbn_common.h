// Shared declarations of the libtbn translation units (host dispatch + gfx950 device helpers).
// Notation follows the paper's Method section with the letters of include/tbn.h:
// n weights, k tile repeats, p = n / k tile bits; flat weight index f -> tile bit f % p,
// scalar alpha[f / p] (Eq. 4-5 and the scaling stated after Eq. 8).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/tbn.h"

namespace tbn {

constexpr int kWave = 64;

// ---- host side -----------------------------------------------------------------------------
void set_error(const char *fmt, ...);
tbn_status check_launch(const char *what);

struct LinearArgs {
    const void *x;
    void *y;
    int dt;            // tbn_dtype
    int64_t M, in, out;
    const uint32_t *tile;
    int64_t p;         // tile bits
    int32_t k;
    const float *alpha;
    int32_t n_alpha;
    uint32_t flags;
    hipStream_t stream;
};

struct ConvArgs {
    const void *x;
    void *y;
    int dt;
    int64_t N, C, H, W, O, Ho, Wo;
    int32_t kh, kw, sh, sw, ph, pw;
    const uint32_t *tile;
    int64_t p;
    int32_t k;
    const float *alpha;
    int32_t n_alpha;
    uint32_t flags;
    hipStream_t stream;
};

// kernel families; each returns TBN_OK after enqueueing, or an error with nothing enqueued
// blk > 0: column-tiled layout, summand r of tile position i is element (i / blk) * ld + r * blk + i % blk
tbn_status launch_pack(const float *w, const float *a, int64_t n, int32_t k, int32_t n_alpha,
                       uint32_t *tile_out, float *alpha_out, void *workspace, hipStream_t stream,
                       int64_t blk = 0, int64_t ld = 0);
size_t pack_workspace_bytes(int64_t n, int32_t k, int32_t n_alpha);
tbn_status launch_pack_noalloc(const float *w, const float *a, int64_t n, int32_t k, int32_t n_alpha,
                               uint32_t *tile_out, float *alpha_out, hipStream_t stream);

tbn_status launch_linear_generic(const LinearArgs &a);
bool linear_direct_supported(const LinearArgs &a);   // tile of whole rows, any row length and alignment: vector-ALU kernel
tbn_status launch_linear_direct(const LinearArgs &a);
bool linear_skinny_supported(const LinearArgs &a); // small-batch (decode-shaped) matrix-core kernel
tbn_status launch_linear_skinny(const LinearArgs &a);
bool linear_decode_supported(const LinearArgs &a); // at most 16 batch rows, tile of whole rows: latency-built GEMV kernel
tbn_status launch_linear_decode(const LinearArgs &a);
bool linear_rows_supported(const LinearArgs &a);   // wave-per-row kernel (also repairs tile-end columns)
tbn_status launch_linear_rows(const LinearArgs &a);
tbn_status launch_linear_rows_fixup(const LinearArgs &a);  // recompute the columns whose row holds a tile end
tbn_status launch_linear_tile_ends(const LinearArgs &a);   // the same in one pass over X (falls back to the above)
bool linear_mfma_supported(const LinearArgs &a);   // matrix-core kernel
bool linear_stream_supported(const LinearArgs &a); // streaming matrix-core kernel (bfloat16, tile of whole rows)
tbn_status launch_linear_stream(const LinearArgs &a);
bool linear_block_supported(const LinearArgs &a);  // one block per workgroup with load waves (bfloat16, tile of whole rows)
tbn_status launch_linear_block(const LinearArgs &a);
int linear_split_plan(const LinearArgs &a);         // split K over workgroups for small grids: number of splits, 0 = none
size_t linear_split_workspace_bytes(const LinearArgs &a, int splits);
tbn_status launch_linear_split(const LinearArgs &a, int splits, void *workspace);   // workspace: 16-byte aligned, the bytes above
bool linear_tile_supported(const LinearArgs &a);   // tile of whole rows, at most 512 distinct rows: one wave per 32 batch rows
bool linear_tile_preferred(const LinearArgs &a);   // bfloat16 at a few hundred batch rows: faster than the other kernels
tbn_status launch_linear_tile(const LinearArgs &a);
tbn_status launch_linear_mfma(const LinearArgs &a);

// column-tiled layer: xf[m, j] = sum_c alpha[c] * x[m, c * q + j], and the float 1.0 written to *one_out
tbn_status launch_coltile_fold(const void *x, void *xf, int dt, int64_t M, int64_t in, int32_t k,
                               const float *alpha, int32_t n_alpha, float *one_out, hipStream_t stream);

// binary activations: rows of sign bits (32 per word, ceil(in / 32) words per row) and the layer on them
tbn_status launch_sign_pack(const void *x, int dt, int64_t M, int64_t in, uint32_t *xbits, hipStream_t stream);
tbn_status launch_linear_binact(const uint32_t *xbits, void *y, int dt, int64_t M, int64_t in, int64_t out,
                                const uint32_t *tile, int64_t p, int32_t k, const float *alpha, int32_t n_alpha,
                                uint32_t flags, hipStream_t stream);

tbn_status launch_conv_generic(const ConvArgs &a);
tbn_status launch_conv_generic_tile_ends(const ConvArgs &a);   // only the channels whose filter holds a tile end
bool conv_mfma_supported(const ConvArgs &a);
tbn_status launch_conv_mfma(const ConvArgs &a);
bool conv_direct_supported(const ConvArgs &a);   // tile of whole filters, any window: vector-ALU kernel, 16 filters per workgroup
tbn_status launch_conv_direct(const ConvArgs &a);

// measurement aids (tbn_diag.hip)
tbn_status launch_diag_empty(hipStream_t stream);
tbn_status launch_diag_stream(const void *src, void *dst, size_t bytes, uint32_t *sink, hipStream_t stream);
tbn_status launch_diag_mfma(int32_t blocks, int32_t iters, float *out, hipStream_t stream, bool fp4 = false);

// number of distinct bit rows of the (rows x row_len) weight: row o repeats row o % U
int64_t unique_rows(int64_t rows, int64_t row_len, int64_t p);

// ---- device side ---------------------------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round to nearest even; NaN stays NaN (quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// 32 tile bits starting at bit position `pos` (0 <= pos, pos + 32 may run past the last word:
// the caller guarantees words [pos/32, pos/32 + 1] are readable or passes clamp_words)
__device__ __forceinline__ uint32_t tile_window32(const uint32_t *tile, int64_t pos, int64_t n_words) {
    const int64_t w = pos >> 5;
    const uint32_t sh = static_cast<uint32_t>(pos & 31);
    const uint32_t lo = tile[w];
    const uint32_t hi = (w + 1 < n_words) ? tile[w + 1] : 0u;
    return sh ? __funnelshift_r(lo, hi, sh) : lo;
}

template <typename T> struct ElemIO;
template <> struct ElemIO<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct ElemIO<uint16_t> {   // bfloat16 bit patterns
    static __device__ __forceinline__ float load(const uint16_t *p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t *p, float v) { *p = f32_to_bf16_bits(v); }
};

#endif  // __HIPCC__

}  // namespace tbn
