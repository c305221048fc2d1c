// C ABI of libtbn: argument validation and choice of kernel family.  See include/tbn.h for the
// contract of each entry point and the passages of the paper that define the operations.
#include "tbn_common.h"

#include <cstdarg>
#include <cstdio>
#include <numeric>

namespace tbn {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// An error left behind by an earlier HIP call of the process (outside this library) must not be reported as the
// failure of the launch that follows: the entry points drop it before they enqueue anything.
static void drop_stale_error() { (void)hipGetLastError(); }

tbn_status check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: %s", what, hipGetErrorString(e));
        return TBN_ERR_DEVICE;
    }
    return TBN_OK;
}

int64_t unique_rows(int64_t rows, int64_t row_len, int64_t p) {
    // row o starts at tile bit (o * row_len) % p; that offset has period p / gcd(row_len, p) in o
    const int64_t g = std::gcd(row_len, p);
    const int64_t period = p / g;
    return period < rows ? period : rows;
}

static bool mul_ok(int64_t a, int64_t b, int64_t *r) { return !__builtin_mul_overflow(a, b, r); }

static tbn_status check_tiling(int64_t n, int32_t k, int32_t n_alpha) {
    if (n <= 0 || k <= 0) {
        set_error("n (%lld) and k (%d) must be positive", (long long)n, k);
        return TBN_ERR_SHAPE;
    }
    if (n % k != 0) {
        set_error("the number of weights %lld is not divisible by the compression factor %d", (long long)n, k);
        return TBN_ERR_SHAPE;
    }
    if (n_alpha != 1 && n_alpha != k) {
        set_error("n_alpha must be 1 or k (%d), got %d", k, n_alpha);
        return TBN_ERR_SHAPE;
    }
    return TBN_OK;
}

// The kernel family that serves a fully-connected call (host arithmetic only: shapes, alignment of the pointers, the
// number of CUs of the current device).
enum class LinearKernel { Decode, Tile, Skinny, Stream, Block, Mfma, Rows, Direct, Generic };

static LinearKernel choose_linear(const LinearArgs &a) {
    if (!(a.flags & TBN_FLAG_FORCE_GENERIC)) {
        // at most 16 batch rows: the decode kernel (a workgroup per two distinct columns reads all of X); with many
        // distinct columns and 8 - 16 rows the small-batch kernel, whose workgroups share X sixteen columns at a time,
        // is the faster one (graph replays, 2048 distinct columns, batch 16, in = 1024 / 4096 / 8192: 9.0 / 11.4 / 16.1 us
        // against 7.9 / 8.3 / 13.5; batch 8: 4.6 / 6.5 / 9.0 against 6.6 / 6.9 / 11.0; 4096 columns, batch 8: 7.1 / 9.1 /
        // 13.2 against 6.7 / 7.1 / 11.1)
        if (!(a.flags & TBN_FLAG_LARGE_BATCH) && linear_decode_supported(a) &&
            (a.M * (a.p / a.in) <= 16384 || !linear_skinny_supported(a)))
            return LinearKernel::Decode;
        if (!(a.flags & (TBN_FLAG_BLOCK_KERNEL | TBN_FLAG_STREAM_KERNEL)) && linear_tile_preferred(a)) return LinearKernel::Tile;
        if (linear_skinny_supported(a)) return LinearKernel::Skinny;
        if (!(a.flags & TBN_FLAG_BLOCK_KERNEL)) {
            // bfloat16, tile of whole rows: 128 x 128 blocks with load waves; the streaming kernel (64-row half
            // tiles, twice the workgroups) where the blocks would leave half of the CUs or more idle
            // (4096 x 4096, k = 8, batch 512 / 1024 / 2048: 16 / 17 / 20 us against 23 / 22 / 23)
            const int64_t U = a.p % a.in == 0 ? a.p / a.in : 0;
            const int64_t blocks = ((a.M + 127) / 128) * ((U + 127) / 128);
            if ((a.flags & TBN_FLAG_TILE_KERNEL) && linear_tile_supported(a)) return LinearKernel::Tile;
            const bool stream = (a.flags & TBN_FLAG_STREAM_KERNEL) || blocks <= 128;   // (batch 4096: 25.2 us against 28.3)
            if (stream && linear_stream_supported(a)) return LinearKernel::Stream;
            // (rows of 256: two rounds per block, too few for the persistent form; on grids of more than two blocks per CU
            // the general kernel with two workgroups per CU is 10 - 25 % faster: 8192 x 256 -> 4096 distinct columns 36 us
            // against 43)
            const bool short_rows = a.in < 512 && blocks > 512 && linear_mfma_supported(a);
            if (!short_rows && linear_block_supported(a)) return LinearKernel::Block;
            // float32, tile of whole rows: one wave per 32 batch rows (every shape measured, up to 8192 distinct columns
            // at batch 8192, runs 15 - 70 % faster than in the 128 x 128 blocks of the general kernel: 8192 x 1024 ->
            // 1024 distinct columns 57 us against 84, 8192 x 4096 -> 8192 distinct columns 1379 against 1672)
            if (a.dt == TBN_F32 && linear_tile_supported(a)) return LinearKernel::Tile;
        }
        if (linear_mfma_supported(a)) return LinearKernel::Mfma;
        if (linear_rows_supported(a)) return LinearKernel::Rows;
        // row lengths and alignments that none of the kernels above takes (in no multiple of 8), tile of whole rows
        if (linear_direct_supported(a)) return LinearKernel::Direct;
    }
    return LinearKernel::Generic;
}

static const char *linear_kernel_name(LinearKernel kn) {
    switch (kn) {
        case LinearKernel::Decode: return "decode";
        case LinearKernel::Tile: return "tile";
        case LinearKernel::Skinny: return "small-batch";
        case LinearKernel::Stream: return "stream";
        case LinearKernel::Block: return "block";
        case LinearKernel::Mfma: return "general";
        case LinearKernel::Rows: return "rows";
        case LinearKernel::Direct: return "direct";
        case LinearKernel::Generic: return "generic";
    }
    return "generic";
}

static tbn_status dispatch_linear(const LinearArgs &a) {
    drop_stale_error();
    switch (choose_linear(a)) {
        case LinearKernel::Decode: return launch_linear_decode(a);
        case LinearKernel::Tile: return launch_linear_tile(a);
        case LinearKernel::Skinny: return launch_linear_skinny(a);
        case LinearKernel::Stream: return launch_linear_stream(a);
        case LinearKernel::Block: return launch_linear_block(a);
        case LinearKernel::Mfma: return launch_linear_mfma(a);
        case LinearKernel::Rows: return launch_linear_rows(a);
        case LinearKernel::Direct: return launch_linear_direct(a);
        case LinearKernel::Generic: break;
    }
    return launch_linear_generic(a);
}

static tbn_status check_linear_args(const char *fn, const void *x, const void *y, tbn_dtype dt, int64_t M, int64_t in,
                                    int64_t out, const uint32_t *tile, const float *alpha, uint32_t flags, int64_t *n) {
    if (!tile || !alpha || (M > 0 && (!x || !y))) {  // an empty batch may come with NULL x and y
        set_error("%s: x, y, tile and alpha must not be NULL", fn);
        return TBN_ERR_NULL;
    }
    if (dt != TBN_F32 && dt != TBN_BF16) {
        set_error("%s: unknown dtype %d", fn, (int)dt);
        return TBN_ERR_UNSUPPORTED;
    }
    if (flags & ~(TBN_FLAG_RELU | TBN_FLAG_FORCE_GENERIC | TBN_FLAG_LARGE_BATCH | TBN_FLAG_BLOCK_KERNEL |
                  TBN_FLAG_STREAM_KERNEL | TBN_FLAG_SPLIT_K | TBN_FLAG_TILE_KERNEL)) {
        set_error("%s: unknown flag bits 0x%x", fn, flags);
        return TBN_ERR_UNSUPPORTED;
    }
    if (M < 0 || in <= 0 || out <= 0) {
        set_error("%s: M (%lld) must be >= 0, in (%lld) and out (%lld) positive", fn,
                  (long long)M, (long long)in, (long long)out);
        return TBN_ERR_SHAPE;
    }
    int64_t xs, ys;
    if (!mul_ok(in, out, n) || !mul_ok(M, in, &xs) || !mul_ok(M, out, &ys) || *n > (int64_t(1) << 40) ||
        xs > (int64_t(1) << 40) || ys > (int64_t(1) << 40)) {
        set_error("%s: sizes beyond the supported range", fn);
        return TBN_ERR_UNSUPPORTED;
    }
    return TBN_OK;
}

// Split K with a workspace: not for the batches of the decode and small-batch kernels, not with the flags that name
// another kernel; otherwise where the block kernel's plan says so.
static int workspace_splits(const LinearArgs &a) {
    if (a.flags & (TBN_FLAG_FORCE_GENERIC | TBN_FLAG_BLOCK_KERNEL | TBN_FLAG_STREAM_KERNEL | TBN_FLAG_TILE_KERNEL)) return 0;
    if (a.M <= 64) return 0;
    return linear_split_plan(a);
}

static size_t coltile_xf_bytes(tbn_dtype dt, int64_t M, int64_t q) {
    const size_t raw = static_cast<size_t>(M) * static_cast<size_t>(q) * (dt == TBN_F32 ? 4u : 2u);
    return (raw + 255u) & ~static_cast<size_t>(255u);
}

}  // namespace tbn

using namespace tbn;

extern "C" {

size_t tbn_tile_words(int64_t n, int32_t k) {
    if (n <= 0 || k <= 0 || n % k != 0) return 0;
    return static_cast<size_t>((n / k + 31) / 32);
}

const char *tbn_last_error(void) { return g_err; }

const char *tbn_version(void) { return "libtbn 0.1 (gfx950)"; }

size_t tbn_pack_workspace_bytes(int64_t n, int32_t k, int32_t n_alpha) {
    if (n <= 0 || k <= 0 || n % k != 0 || (n_alpha != 1 && n_alpha != k)) return 0;
    return pack_workspace_bytes(n, k, n_alpha);
}

tbn_status tbn_pack_tile(const float *w_real, const float *a_real, int64_t n, int32_t k,
                         int32_t n_alpha, uint32_t *tile_out, float *alpha_out,
                         void *workspace, size_t workspace_bytes, void *stream) {
    if (!w_real || !tile_out || !alpha_out) {
        set_error("tbn_pack_tile: w_real, tile_out and alpha_out must not be NULL");
        return TBN_ERR_NULL;
    }
    tbn_status st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    const size_t need = pack_workspace_bytes(n, k, n_alpha);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 7u)) {
        set_error("tbn_pack_tile: workspace of %zu bytes, 8-byte aligned, required (got %zu at %p)",
                  need, workspace_bytes, workspace);
        return TBN_ERR_WORKSPACE;
    }
    drop_stale_error();
    return launch_pack(w_real, a_real, n, k, n_alpha, tile_out, alpha_out, workspace,
                       static_cast<hipStream_t>(stream));
}

tbn_status tbn_pack_tile_noalloc(const float *w_real, const float *a_real, int64_t n, int32_t k,
                                 int32_t n_alpha, uint32_t *tile_out, float *alpha_out, void *stream) {
    if (!w_real || !tile_out || !alpha_out) {
        set_error("tbn_pack_tile_noalloc: w_real, tile_out and alpha_out must not be NULL");
        return TBN_ERR_NULL;
    }
    tbn_status st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    drop_stale_error();
    return launch_pack_noalloc(w_real, a_real, n, k, n_alpha, tile_out, alpha_out, static_cast<hipStream_t>(stream));
}

tbn_status tbn_linear_forward(const void *x, void *y, tbn_dtype dt, int64_t M, int64_t in,
                              int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                              int32_t n_alpha, uint32_t flags, void *stream) {
    int64_t n;
    tbn_status st = check_linear_args("tbn_linear_forward", x, y, dt, M, in, out, tile, alpha, flags, &n);
    if (st != TBN_OK) return st;
    st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    if (M == 0) return TBN_OK;

    LinearArgs a{x, y, (int)dt, M, in, out, tile, n / k, k, alpha, n_alpha, flags,
                 static_cast<hipStream_t>(stream)};
    return dispatch_linear(a);
}

const char *tbn_linear_forward_kernel(const void *x, const void *y, tbn_dtype dt, int64_t M, int64_t in, int64_t out,
                                      int32_t k, int32_t n_alpha, uint32_t flags) {
    int64_t n;
    if ((dt != TBN_F32 && dt != TBN_BF16) || M <= 0 || in <= 0 || out <= 0 || k <= 0 || !mul_ok(in, out, &n) || n % k != 0 ||
        (n_alpha != 1 && n_alpha != k))
        return "";
    LinearArgs a{x, const_cast<void *>(y), (int)dt, M, in, out, nullptr, n / k, k, nullptr, n_alpha, flags, nullptr};
    return linear_kernel_name(choose_linear(a));
}

size_t tbn_linear_forward_workspace_bytes(tbn_dtype dt, int64_t M, int64_t in, int64_t out, int32_t k, uint32_t flags) {
    int64_t n;
    if ((dt != TBN_F32 && dt != TBN_BF16) || M <= 0 || in <= 0 || out <= 0 || k <= 0 || !mul_ok(in, out, &n) || n % k != 0) return 0;
    // pointers unknown here: taken as aligned; tbn_linear_forward_ws looks again with the real ones
    LinearArgs a{nullptr, nullptr, (int)dt, M, in, out, nullptr, n / k, k, nullptr, 1, flags, nullptr};
    const int splits = workspace_splits(a);
    return splits ? linear_split_workspace_bytes(a, splits) : 0;
}

tbn_status tbn_linear_forward_ws(const void *x, void *y, tbn_dtype dt, int64_t M, int64_t in,
                                 int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                                 int32_t n_alpha, uint32_t flags, void *workspace, size_t workspace_bytes,
                                 void *stream) {
    int64_t n;
    tbn_status st = check_linear_args("tbn_linear_forward_ws", x, y, dt, M, in, out, tile, alpha, flags, &n);
    if (st != TBN_OK) return st;
    st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    if (M == 0) return TBN_OK;
    if (workspace_bytes > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u))) {
        set_error("tbn_linear_forward_ws: a workspace of %zu bytes must be a 16-byte aligned device pointer (got %p)",
                  workspace_bytes, workspace);
        return TBN_ERR_WORKSPACE;
    }
    LinearArgs a{x, y, (int)dt, M, in, out, tile, n / k, k, alpha, n_alpha, flags,
                 static_cast<hipStream_t>(stream)};
    const int splits = workspace_splits(a);
    if (splits && workspace_bytes >= linear_split_workspace_bytes(a, splits)) return launch_linear_split(a, splits, workspace);
    return dispatch_linear(a);
}

size_t tbn_pack_coltile_workspace_bytes(int64_t out, int64_t in, int32_t k, int32_t n_alpha) {
    int64_t n;
    if (out <= 0 || in <= 0 || k <= 0 || in % k != 0 || (n_alpha != 1 && n_alpha != k) || !mul_ok(out, in, &n)) return 0;
    return pack_workspace_bytes(n, k, n_alpha);
}

tbn_status tbn_pack_coltile(const float *w_real, const float *a_real, int64_t out, int64_t in, int32_t k,
                            int32_t n_alpha, uint32_t *tile_out, float *alpha_out, void *workspace,
                            size_t workspace_bytes, void *stream) {
    if (!w_real || !tile_out || !alpha_out) {
        set_error("tbn_pack_coltile: w_real, tile_out and alpha_out must not be NULL");
        return TBN_ERR_NULL;
    }
    int64_t n;
    if (out <= 0 || in <= 0 || !mul_ok(out, in, &n)) {
        set_error("tbn_pack_coltile: out (%lld) and in (%lld) must be positive", (long long)out, (long long)in);
        return TBN_ERR_SHAPE;
    }
    if (k <= 0 || in % k != 0) {
        set_error("tbn_pack_coltile: in (%lld) is not divisible by the number of column blocks %d", (long long)in, k);
        return TBN_ERR_SHAPE;
    }
    tbn_status st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    const size_t need = pack_workspace_bytes(n, k, n_alpha);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 7u)) {
        set_error("tbn_pack_coltile: workspace of %zu bytes, 8-byte aligned, required (got %zu at %p)",
                  need, workspace_bytes, workspace);
        return TBN_ERR_WORKSPACE;
    }
    return launch_pack(w_real, a_real, n, k, n_alpha, tile_out, alpha_out, workspace,
                       static_cast<hipStream_t>(stream), in / k, in);
}

size_t tbn_linear_coltiled_workspace_bytes(tbn_dtype dt, int64_t M, int64_t in, int32_t k) {
    int64_t xs;
    if ((dt != TBN_F32 && dt != TBN_BF16) || M < 0 || in <= 0 || k <= 0 || in % k != 0 || !mul_ok(M, in, &xs) ||
        xs > (int64_t(1) << 40))
        return 0;
    return coltile_xf_bytes(dt, M, in / k) + 256;
}

tbn_status tbn_linear_coltiled_forward(const void *x, void *y, tbn_dtype dt, int64_t M, int64_t in,
                                       int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                                       int32_t n_alpha, uint32_t flags, void *workspace,
                                       size_t workspace_bytes, void *stream) {
    int64_t n;
    tbn_status st = check_linear_args("tbn_linear_coltiled_forward", x, y, dt, M, in, out, tile, alpha, flags, &n);
    if (st != TBN_OK) return st;
    if (k <= 0 || in % k != 0) {
        set_error("tbn_linear_coltiled_forward: in (%lld) is not divisible by the number of column blocks %d",
                  (long long)in, k);
        return TBN_ERR_SHAPE;
    }
    if (n_alpha != 1 && n_alpha != k) {
        set_error("n_alpha must be 1 or k (%d), got %d", k, n_alpha);
        return TBN_ERR_SHAPE;
    }
    if (M == 0) return TBN_OK;   // an empty batch is legal and needs no workspace
    const int64_t q = in / k;
    const size_t xf_bytes = coltile_xf_bytes(dt, M, q), need = xf_bytes + 256;
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u)) {
        set_error("tbn_linear_coltiled_forward: workspace of %zu bytes, 16-byte aligned, required (got %zu at %p)",
                  need, workspace_bytes, workspace);
        return TBN_ERR_WORKSPACE;
    }
    drop_stale_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (k == 1) {   // one block: the flat layer with one tile copy, nothing to fold
        LinearArgs a{x, y, (int)dt, M, in, out, tile, n, 1, alpha, 1, flags, s};
        return dispatch_linear(a);
    }
    float *one = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + xf_bytes);
    st = launch_coltile_fold(x, workspace, (int)dt, M, in, k, alpha, n_alpha, one, s);
    if (st != TBN_OK) return st;
    // the +-1 product on the folded activations: the flat layer with one tile copy and alpha = 1
    LinearArgs a{workspace, y, (int)dt, M, q, out, tile, out * q, 1, one, 1, flags, s};
    return dispatch_linear(a);
}

size_t tbn_sign_row_words(int64_t in) { return in > 0 ? static_cast<size_t>((in + 31) / 32) : 0; }

tbn_status tbn_sign_pack(const void *x, tbn_dtype dt, int64_t M, int64_t in, uint32_t *xbits, void *stream) {
    if (M > 0 && (!x || !xbits)) {
        set_error("tbn_sign_pack: x and xbits must not be NULL");
        return TBN_ERR_NULL;
    }
    if (dt != TBN_F32 && dt != TBN_BF16) {
        set_error("tbn_sign_pack: unknown dtype %d", (int)dt);
        return TBN_ERR_UNSUPPORTED;
    }
    if (M < 0 || in <= 0) {
        set_error("tbn_sign_pack: M (%lld) must be >= 0 and in (%lld) positive", (long long)M, (long long)in);
        return TBN_ERR_SHAPE;
    }
    int64_t xs;
    if (!mul_ok(M, in, &xs) || xs > (int64_t(1) << 40)) {
        set_error("tbn_sign_pack: sizes beyond the supported range");
        return TBN_ERR_UNSUPPORTED;
    }
    if (M == 0) return TBN_OK;
    drop_stale_error();
    return launch_sign_pack(x, (int)dt, M, in, xbits, static_cast<hipStream_t>(stream));
}

tbn_status tbn_linear_forward_binact(const uint32_t *xbits, void *y, tbn_dtype y_dt, int64_t M, int64_t in,
                                     int64_t out, const uint32_t *tile, int32_t k, const float *alpha,
                                     int32_t n_alpha, uint32_t flags, void *stream) {
    if (flags & ~(TBN_FLAG_RELU | TBN_FLAG_FORCE_GENERIC | TBN_FLAG_SIGN_OUT)) {
        set_error("tbn_linear_forward_binact: unknown flag bits 0x%x", flags);
        return TBN_ERR_UNSUPPORTED;
    }
    int64_t n;
    tbn_status st = check_linear_args("tbn_linear_forward_binact", xbits, y, y_dt, M, in, out, tile, alpha,
                                      flags & ~TBN_FLAG_SIGN_OUT, &n);
    if (st != TBN_OK) return st;
    st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    if (M == 0) return TBN_OK;
    drop_stale_error();
    return launch_linear_binact(xbits, y, (int)y_dt, M, in, out, tile, n / k, k, alpha, n_alpha, flags,
                                static_cast<hipStream_t>(stream));
}

tbn_status tbn_diag_empty_launch(void *stream) { return launch_diag_empty(static_cast<hipStream_t>(stream)); }

tbn_status tbn_diag_stream(const void *src, void *dst, size_t bytes, void *sink, void *stream) {
    if (!src || (reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) {
        set_error("tbn_diag_stream: src must not be NULL; src and dst must be 16-byte aligned");
        return TBN_ERR_NULL;
    }
    if (bytes == 0) return TBN_OK;
    return launch_diag_stream(src, dst, bytes, static_cast<uint32_t *>(sink), static_cast<hipStream_t>(stream));
}

tbn_status tbn_diag_mfma(int32_t blocks, int32_t iters, float *out, void *stream) {
    if (blocks <= 0 || iters < 0 || blocks > (1 << 20)) {
        set_error("tbn_diag_mfma: blocks must be in 1 .. 2^20, iters non-negative");
        return TBN_ERR_SHAPE;
    }
    return launch_diag_mfma(blocks, iters, out, static_cast<hipStream_t>(stream));
}

tbn_status tbn_diag_mfma_fp4(int32_t blocks, int32_t iters, float *out, void *stream) {
    if (blocks <= 0 || iters < 0 || blocks > (1 << 20)) {
        set_error("tbn_diag_mfma_fp4: blocks must be in 1 .. 2^20, iters non-negative");
        return TBN_ERR_SHAPE;
    }
    return launch_diag_mfma(blocks, iters, out, static_cast<hipStream_t>(stream), true);
}

tbn_status tbn_conv2d_forward(const void *x, void *y, tbn_dtype dt, int64_t N, int64_t C,
                              int64_t H, int64_t W, int64_t O, int32_t kh, int32_t kw,
                              int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                              const uint32_t *tile, int32_t k, const float *alpha,
                              int32_t n_alpha, uint32_t flags, void *stream) {
    if (!tile || !alpha || (N > 0 && (!x || !y))) {  // an empty batch may come with NULL x and y
        set_error("tbn_conv2d_forward: x, y, tile and alpha must not be NULL");
        return TBN_ERR_NULL;
    }
    if (dt != TBN_F32 && dt != TBN_BF16) {
        set_error("tbn_conv2d_forward: unknown dtype %d", (int)dt);
        return TBN_ERR_UNSUPPORTED;
    }
    if (flags & ~(TBN_FLAG_RELU | TBN_FLAG_FORCE_GENERIC)) {
        set_error("tbn_conv2d_forward: unknown flag bits 0x%x", flags);
        return TBN_ERR_UNSUPPORTED;
    }
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || O <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 ||
        stride_w <= 0 || pad_h < 0 || pad_w < 0) {
        set_error("tbn_conv2d_forward: sizes and strides must be positive, padding non-negative");
        return TBN_ERR_SHAPE;
    }
    if (H + 2 * (int64_t)pad_h < kh || W + 2 * (int64_t)pad_w < kw) {
        set_error("tbn_conv2d_forward: kernel %dx%d larger than the padded input", kh, kw);
        return TBN_ERR_SHAPE;
    }
    const int64_t lim = int64_t(1) << 40;
    int64_t filt, n, xs, ys;
    const int64_t Ho = (H + 2 * (int64_t)pad_h - kh) / stride_h + 1;
    const int64_t Wo = (W + 2 * (int64_t)pad_w - kw) / stride_w + 1;
    if (!mul_ok(C, (int64_t)kh * kw, &filt) || !mul_ok(filt, O, &n) || n > lim ||
        !mul_ok(N * C, H * W, &xs) || xs > lim || !mul_ok(N * O, Ho * Wo, &ys) || ys > lim ||
        H > (1 << 20) || W > (1 << 20) || C > (1 << 24) || O > (1 << 24) || N > (int64_t(1) << 31) ||
        kh > 4096 || kw > 4096 || pad_h > 4096 || pad_w > 4096) {
        set_error("tbn_conv2d_forward: sizes beyond the supported range");
        return TBN_ERR_UNSUPPORTED;
    }
    tbn_status st = check_tiling(n, k, n_alpha);
    if (st != TBN_OK) return st;
    if (N == 0) return TBN_OK;

    ConvArgs a{x, y, (int)dt, N, C, H, W, O, Ho, Wo, kh, kw, stride_h, stride_w, pad_h, pad_w,
               tile, n / k, k, alpha, n_alpha, flags, static_cast<hipStream_t>(stream)};
    drop_stale_error();
    if (!(flags & TBN_FLAG_FORCE_GENERIC)) {
        // up to 8 input channels (a network's first layer on colour images): the matrix-core kernel would stage chunks of
        // 32 channels that are mostly zeros; the direct kernel is faster (3 -> 64 channels, 3x3, 32 x 32, 128 images:
        // 23 us against 39; 224 x 224, 8 images: 60 against 111; from 12 channels on the matrix cores win: 36 against 48)
        if (a.C <= 8 && conv_direct_supported(a)) return launch_conv_direct(a);
        if (conv_mfma_supported(a)) return launch_conv_mfma(a);
        // other windows (5x5, 7x7, ...) with a tile of whole filters: 16 distinct filters per workgroup on the vector ALUs
        // (ResNet's 7x7, stride 2 first layer on 32 images: 2.0 ms with one thread per output element)
        if (conv_direct_supported(a)) return launch_conv_direct(a);
    }
    return launch_conv_generic(a);
}

}  // extern "C"
