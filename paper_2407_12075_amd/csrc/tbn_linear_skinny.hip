// Small-batch (decode-shaped) kernel for the fully-connected tiled-bit layer: batch <= 64.
//
// Same mathematics as the large-batch kernel (Eq. 4-5, Algorithm 1): only the U = p / gcd(in, p)
// distinct +-1 rows of the weight are multiplied, every output column o = u + t*U is alpha(o) * Z[:, u].
// At these sizes the layer moves a few hundred kilobytes, so the kernel is built for latency:
//   * a workgroup owns 16 batch rows x 16 distinct columns and splits K among its 8 waves;
//   * a wave multiplies with v_mfma_f32_16x16x32_bf16: activations go from global memory straight
//     into the operand layout (a lane reads 64 contiguous bytes of its row per 128 columns of K,
//     so a row is read in 256-byte runs), the sign operand is expanded in registers from one
//     32-bit tile window per lane and 128 columns; nothing is staged in LDS;
//   * float32 activations are split exactly into three bf16 terms in registers;
//   * the 8 partial 16 x 16 blocks are summed through LDS in a fixed order and all replicas are
//     written by the whole workgroup with lanes running along the columns of Y.
// Columns whose weight row contains a tile end (two alphas) are recomputed afterwards by the row
// kernel, as for the large-batch kernel.
#include "tbn_common.h"

namespace tbn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;   // K splits
constexpr int kKBlock = 128;            // columns of K per wave iteration (4 MFMA steps)

struct SkinnyParams {
    int64_t M, in, out, p, n_words, U;
    int32_t n_alpha;
    int aligned;
};

union Frag {
    bf16x8_t v;
    uint32_t u[4];
    u32x4_t q;
};

// +-1 bf16 operand (8 values) from 8 tile bits in natural order (bit 1 -> +1)
__device__ __forceinline__ void expand_byte(Frag &f, uint32_t byte) {
    const uint32_t nb = ~byte;
#pragma unroll
    for (int v = 0; v < 4; ++v)
        f.u[v] = 0x3f803f80u | ((nb << (15 - 2 * v)) & 0x8000u) | ((nb << (30 - 2 * v)) & 0x80000000u);
}

template <typename XT> struct SkTraits;
template <> struct SkTraits<uint16_t> {
    static constexpr int planes = 1;
    static constexpr int blocks_in_flight = 4;
    struct Piece { u32x4_t v; };
    static __device__ __forceinline__ void load(Piece &r, const uint16_t *p) { r.v = *reinterpret_cast<const u32x4_t *>(p); }
    static __device__ __forceinline__ void zero(Piece &r) { r.v = u32x4_t{0u, 0u, 0u, 0u}; }
    static __device__ __forceinline__ void planes_of(const Piece &r, Frag (&a)[1]) { a[0].q = r.v; }
};
template <> struct SkTraits<float> {
    static constexpr int planes = 3;
    static constexpr int blocks_in_flight = 2;
    struct Piece { f32x4_t a, b; };
    static __device__ __forceinline__ void load(Piece &r, const float *p) {
        r.a = *reinterpret_cast<const f32x4_t *>(p);
        r.b = *reinterpret_cast<const f32x4_t *>(p + 4);
    }
    static __device__ __forceinline__ void zero(Piece &r) { r.a = f32x4_t{0.f, 0.f, 0.f, 0.f}; r.b = r.a; }
    // exact split x = t0 + t1 + t2 by truncation (8 + 8 + 8 significand bits)
    static __device__ __forceinline__ void planes_of(const Piece &r, Frag (&a)[3]) {
        const float x[8] = {r.a[0], r.a[1], r.a[2], r.a[3], r.b[0], r.b[1], r.b[2], r.b[3]};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t t[2][3];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float v = x[2 * d + h];
                t[h][0] = __float_as_uint(v) & 0xffff0000u;
                const float r1 = v - __uint_as_float(t[h][0]);
                t[h][1] = __float_as_uint(r1) & 0xffff0000u;
                const float r2 = r1 - __uint_as_float(t[h][1]);
                t[h][2] = __float_as_uint(r2) & 0xffff0000u;
            }
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) a[pl].u[d] = (t[0][pl] >> 16) | t[1][pl];
        }
    }
};

template <typename XT, bool RELU>
__global__ __launch_bounds__(kThreads) void linear_skinny_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                                 const uint32_t *__restrict__ tile,
                                                                 const float *__restrict__ alpha, SkinnyParams P) {
    using T = SkTraits<XT>;
    constexpr int NP = T::planes;
    __shared__ float part[kWaves][16][17];   // partial blocks [wave][batch row][column], padded
    __shared__ float zfin[16][17];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int64_t u0 = int64_t(blockIdx.x) * 16, m0 = int64_t(blockIdx.y) * 16;

    // operand rows of this lane (clamped: results of rows / columns past the end are dropped)
    const int64_t m_l = (m0 + ln) < P.M ? (m0 + ln) : (P.M - 1);
    const int64_t u_l = (u0 + ln) < P.U ? (u0 + ln) : (P.U - 1);
    const XT *xrow = x + m_l * P.in;
    const int64_t off = (u_l * P.in) % P.p;   // start bit of weight row u_l in the tile
    const uint32_t tile_head = tile[0];

    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    const int n_blocks = static_cast<int>((P.in + kKBlock - 1) / kKBlock);

    // K index of (block b, step s, lane group lg, element i) is 128*b + 32*lg + 8*s + i: a lane reads
    // 64 contiguous bytes (bf16) of its batch row per block and one 32-bit tile window.
    constexpr int NB = T::blocks_in_flight;
    typename T::Piece pc[NB][4];
    uint32_t w_lo[NB], w_hi[NB];
    auto issue = [&](int b, typename T::Piece (&dst)[4], uint32_t &lo, uint32_t &hi) {
        const int64_t kb = int64_t(b) * kKBlock + 32 * lg;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            int64_t k = kb + 8 * s;
            k = k < P.in - 8 ? k : P.in - 8;   // in % 8 == 0; pieces past the end are zeroed when used
            T::load(dst[s], xrow + k);
        }
        int64_t pos = off + (kb < P.in ? kb : 0);
        if (pos >= P.p) pos -= P.p;
        const int64_t w = pos >> 5;
        lo = tile[w];
        hi = tile[(w + 1 < P.n_words) ? (w + 1) : w];
    };
    auto consume = [&](int b, typename T::Piece (&src)[4], uint32_t lo, uint32_t hi) {
        const int64_t kb = int64_t(b) * kKBlock + 32 * lg;
        int64_t pos = off + (kb < P.in ? kb : 0);
        if (pos >= P.p) pos -= P.p;
        const uint32_t hi_ok = ((pos >> 5) + 1 < P.n_words) ? hi : 0u;
        uint32_t wbits = __funnelshift_r(lo, hi_ok, static_cast<uint32_t>(pos & 31));
        const int64_t left = P.p - pos;   // bits before the tile end; the window continues at bit 0
        if (left < 32) wbits = (wbits & ((1u << left) - 1u)) | (tile_head << left);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (kb + 8 * s >= P.in) T::zero(src[s]);
            Frag bw, a[NP];
            expand_byte(bw, (wbits >> (8 * s)) & 0xffu);
            T::planes_of(src[s], a);
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[pl].v, bw.v, acc, 0, 0, 0);
        }
    };

    // The wave's blocks are wave, wave + 8, ...; NB of them are loaded at once (for in <= 4096 with
    // bf16 that is all of them: one round trip to memory), then multiplied.
    for (int b0 = wave; b0 < n_blocks; b0 += kWaves * NB) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int b = b0 + j * kWaves;
            issue(b < n_blocks ? b : b0, pc[j], w_lo[j], w_hi[j]);   // a repeated block is loaded but not used
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int b = b0 + j * kWaves;
            if (b < n_blocks) consume(b, pc[j], w_lo[j], w_hi[j]);
        }
    }

    // accumulator layout: lane holds column ln, batch rows 4*lg + i
#pragma unroll
    for (int i = 0; i < 4; ++i) part[wave][4 * lg + i][ln] = acc[i];
    __syncthreads();
    if (tid < 256) {
        const int m = tid >> 4, u = tid & 15;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += part[w][m][u];
        zfin[m][u] = s;
    }
    __syncthreads();

    // epilogue: thread -> (replica t, batch row m, column u); u runs fastest over the lanes
    const int u = tid & 15, m = (tid >> 4) & 15;
    const int64_t reps = (P.out + P.U - 1) / P.U;
    if (u0 + u < P.U && m0 + m < P.M) {
        const float z = zfin[m][u];
        XT *yrow = y + (m0 + m) * P.out;
        for (int64_t t = tid >> 8; t < reps; t += kThreads / 256) {
            const int64_t o = u0 + u + t * P.U;
            if (o >= P.out) break;
            const int64_t ai = (P.n_alpha == 1) ? 0 : (P.aligned ? t : (o * P.in) / P.p);
            float v = alpha[ai] * z;
            if (RELU) v = fmaxf(v, 0.f);
            ElemIO<XT>::store(yrow + o, v);
        }
    }
}

template <typename XT, bool RELU> void launch_sk(const LinearArgs &a, const SkinnyParams &P, dim3 grid) {
    hipLaunchKernelGGL((linear_skinny_kernel<XT, RELU>), grid, dim3(kThreads), 0, a.stream,
                       static_cast<const XT *>(a.x), static_cast<XT *>(a.y), a.tile, a.alpha, P);
}

}  // namespace

bool linear_skinny_supported(const LinearArgs &a) {
    if (a.p < a.in || a.p < 64) return false;   // at most one tile end per row, windows never wrap twice
    if (a.in % 8 != 0) return false;            // 16-byte (bf16) / 32-byte (f32) activation pieces
    if (reinterpret_cast<uintptr_t>(a.x) & 15u) return false;
    return a.M <= 64;
}

tbn_status launch_linear_skinny(const LinearArgs &a) {
    SkinnyParams P;
    P.M = a.M; P.in = a.in; P.out = a.out; P.p = a.p;
    P.n_words = (a.p + 31) / 32;
    P.U = unique_rows(a.out, a.in, a.p);
    P.n_alpha = a.n_alpha;
    P.aligned = (a.p % a.in == 0) ? 1 : 0;
    const int64_t gx = (P.U + 15) / 16, gy = (a.M + 15) / 16;
    if (gx > 0x7fffffffLL) {
        set_error("tbn_linear_forward: too many distinct rows for one launch");
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy));
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    if (a.dt == TBN_F32) {
        if (relu) launch_sk<float, true>(a, P, grid); else launch_sk<float, false>(a, P, grid);
    } else {
        if (relu) launch_sk<uint16_t, true>(a, P, grid); else launch_sk<uint16_t, false>(a, P, grid);
    }
    tbn_status st = check_launch("tbn_linear_forward (small-batch kernel)");
    if (st != TBN_OK) return st;
    // columns whose weight row straddles a tile end need two alphas
    if (a.n_alpha > 1 && !P.aligned) return launch_linear_rows_fixup(a);
    return TBN_OK;
}

}  // namespace tbn
