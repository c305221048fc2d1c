// Small-batch (decode-shaped) kernel for the fully-connected tiled-bit layer: batch <= 64, and larger
// batches as long as the problem is small (see linear_skinny_supported).
//
// Same mathematics as the large-batch kernel (Eq. 4-5, Algorithm 1): only the U = p / gcd(in, p)
// distinct +-1 rows of the weight are multiplied, every output column o = u + t*U is alpha(o) * Z[:, u].
// At these sizes the layer moves a few hundred kilobytes, so the kernel is built for latency:
//   * a workgroup owns 16 batch rows x 16 distinct columns and splits K among its 8 waves;
//   * a wave multiplies with v_mfma_f32_16x16x32_bf16: activations go from global memory straight
//     into the operand layout (the four lane groups of a row read 64 contiguous bytes per load
//     instruction), the sign operand is expanded in registers from the 128-bit cyclic tile window
//     of the lane's column, fetched with one wide load per 128 columns of K; nothing is staged in LDS;
//   * float32 activations are split exactly into three bf16 terms in registers;
//   * the 8 partial 16 x 16 blocks are summed through LDS in a fixed order and all replicas are
//     written by the whole workgroup with lanes running along the columns of Y.
// Columns whose weight row contains a tile start (two alphas) are recomputed afterwards, here and
// after the large-batch kernel, by the same kernel in its FIXUP form at any batch size: the "columns"
// of a workgroup are then the up to k - 1 such rows, the sums before and from the tile start are kept
// in two accumulators (operand elements of the other part are zeroed), and X is read once for all
// of them.
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
    int32_t k;   // tile repeats (FIXUP form: tile starts 1 .. k - 1 are looked at)
};

union Frag {
    bf16x8_t v;
    uint32_t u[4];
    u32x4_t q;
};

// +-1 bf16 operand (8 values) from byte `sel / 0x01010101` of an inverted 32-bit tile window (bit 1 of the
// tile is +1, i.e. sign bit clear): the byte is replicated into both halves, each half is shifted so that
// bits 2v and 2v + 1 land on the two sign positions, and the pattern of 1.0 is merged in.
__device__ __forceinline__ void expand_byte(Frag &f, uint32_t inv_window, uint32_t sel, uint32_t sign_mask, uint32_t one_bits) {
    typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
    const uint32_t rep = __builtin_amdgcn_perm(inv_window, inv_window, sel);
    const u16x2_t r2 = __builtin_bit_cast(u16x2_t, rep);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const u16x2_t sh = {static_cast<uint16_t>(15 - 2 * v), static_cast<uint16_t>(14 - 2 * v)};
        f.u[v] = (__builtin_bit_cast(uint32_t, static_cast<u16x2_t>(r2 << sh)) & sign_mask) | one_bits;
    }
}

// Four tile words fetched with one load (dword alignment is all the hardware asks for) and the word after them.
struct WinWords {
    typedef uint32_t vec4 __attribute__((ext_vector_type(4), aligned(4)));
    vec4 q;
    uint32_t tail;
};

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
            for (int pl = 0; pl < 3; ++pl) a[pl].u[d] = __builtin_amdgcn_perm(t[1][pl], t[0][pl], 0x07060302u);   // high halves
        }
    }
};

// Row of the weight that contains the start of tile number c (FIXUP form), j_e = the start's position in it
// (0: the tile starts with the row, nothing to repair).
__device__ __forceinline__ void tile_start_row(const SkinnyParams &P, int64_t c, int64_t &o_c, uint32_t &j_e) {
    const uint64_t prod = static_cast<uint64_t>(c) * static_cast<uint64_t>(P.p);   // < 2^47
    uint64_t q = static_cast<uint64_t>(static_cast<double>(prod) / static_cast<double>(P.in));
    int64_t r = static_cast<int64_t>(prod - q * static_cast<uint64_t>(P.in));
    if (r < 0) { r += P.in; --q; }
    if (r >= P.in) { r -= P.in; ++q; }
    o_c = static_cast<int64_t>(q);
    j_e = static_cast<uint32_t>(r);
}

template <typename XT, bool RELU, bool FIXUP>
__global__ __launch_bounds__(kThreads) void linear_skinny_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                                 const uint32_t *__restrict__ tile,
                                                                 const float *__restrict__ alpha, SkinnyParams P) {
    using T = SkTraits<XT>;
    constexpr int NP = T::planes;
    constexpr int NA = FIXUP ? 2 : 1;              // accumulators: FIXUP keeps the two alpha segments apart
    __shared__ float part[NA][kWaves][16][17];     // partial blocks [wave][batch row][column], padded
    __shared__ float zfin[NA][16][17];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int64_t u0 = int64_t(blockIdx.x) * 16, m0 = int64_t(blockIdx.y) * 16;

    // operand rows of this lane (clamped: results of rows / columns past the end are dropped)
    const bool row_ok = (m0 + ln) < P.M;
    const int64_t m_l = row_ok ? (m0 + ln) : (P.M - 1);
    const int64_t u_l = (u0 + ln) < P.U ? (u0 + ln) : (P.U - 1);
    const unsigned char *xrow = reinterpret_cast<const unsigned char *>(x + m_l * P.in);
    const uint32_t p32 = static_cast<uint32_t>(P.p), in32 = static_cast<uint32_t>(P.in);
    // start bit of the lane's weight row in the tile
    uint32_t off;
    uint32_t j_e = 0;   // FIXUP: elements before j_e belong to the first alpha segment
    if (FIXUP) {
        // the lane's row is the one that holds the start of tile u0 + ln + 1; its first weight is
        // tile bit p - j_e (lanes past k - 1, or whose tile starts with a row, compute a result nobody reads)
        int64_t c = u0 + ln + 1;
        c = c < P.k ? c : 1;
        int64_t o_c;
        tile_start_row(P, c, o_c, j_e);
        off = j_e == 0 ? 0u : p32 - j_e;
    } else {   // (u_l * in) mod p, the product is below 2^53
        const uint64_t prod = static_cast<uint64_t>(u_l) * in32;
        const uint64_t q = static_cast<uint64_t>(static_cast<double>(prod) / static_cast<double>(p32));
        int64_t r = static_cast<int64_t>(prod - q * p32);
        if (r < 0) r += p32;
        if (r >= static_cast<int64_t>(p32)) r -= p32;
        off = static_cast<uint32_t>(r);
    }
    uint32_t head[5];   // start of the tile: continues a window that runs past the tile end (n_words >= 4)
#pragma unroll
    for (int j = 0; j < 5; ++j) head[j] = tile[j < P.n_words ? j : P.n_words - 1];

    // alphas of this thread's first four replicas: requested now, used in the epilogue
    const int u = tid & 15, m = (tid >> 4) & 15;
    const int64_t reps = (P.out + P.U - 1) / P.U;
    constexpr int kStep = kThreads / 256;   // replicas taken by one thread are kStep apart
    auto alpha_of = [&](int64_t t) {
        t = t < reps ? t : reps - 1;
        int64_t o = u0 + u + t * P.U;
        o = o < P.out ? o : P.out - 1;
        return alpha[(P.n_alpha == 1) ? 0 : (P.aligned ? t : (o * P.in) / P.p)];
    };
    float al_first[4] = {0.f, 0.f, 0.f, 0.f};
    if (!FIXUP) {
#pragma unroll
        for (int j = 0; j < 4; ++j) al_first[j] = alpha_of((tid >> 8) + j * kStep);
    }

    // operand constants kept in registers (two literals do not fit one instruction)
    uint32_t sign_mask = 0x80008000u, one_bits = 0x3f803f80u;
    asm volatile("" : "+v"(sign_mask), "+v"(one_bits));
    const uint32_t byte_sel = 0x01010101u * static_cast<uint32_t>(lg);   // byte lg of a window word

    f32x4_t acc[NA];
#pragma unroll
    for (int h = 0; h < NA; ++h) acc[h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int n_blocks = static_cast<int>((P.in + kKBlock - 1) / kKBlock);

    // K index of (block b, step s, lane group lg, element i) is 128*b + 32*s + 8*lg + i: per load
    // instruction the four lane groups of a batch row read 64 contiguous bytes (bf16); a lane needs
    // byte 4*s + lg of its column's 128-bit tile window of the block.
    constexpr int NB = T::blocks_in_flight;
    typename T::Piece pc[NB][4];
    WinWords wraw[NB];
    uint32_t wpos[NB];
    auto issue = [&](int b, typename T::Piece (&dst)[4], WinWords &wr, uint32_t &wp) {
        const uint32_t kb = static_cast<uint32_t>(b) * kKBlock + 8u * lg;
        if (row_ok) {   // lanes of batch rows past M load nothing (at M = 1 that is 15 of 16 lanes)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint32_t k = kb + 32u * s;
                k = k < in32 - 8 ? k : in32 - 8;   // in % 8 == 0; pieces past the end are zeroed when used
                T::load(dst[s], reinterpret_cast<const XT *>(xrow + k * static_cast<uint32_t>(sizeof(XT))));
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) T::zero(dst[s]);
        }
        uint32_t pos = off + static_cast<uint32_t>(b) * kKBlock;   // < 2p: b * 128 < in <= p
        if (pos >= p32) pos -= p32;
        const uint32_t w = pos >> 5;
        const uint32_t last = static_cast<uint32_t>(P.n_words) - 4u;
        const uint32_t wb = w < last ? w : last;   // the four-word load stays inside the tile
        wr.q = *reinterpret_cast<const WinWords::vec4 *>(reinterpret_cast<const unsigned char *>(tile) + (wb << 2));
        const uint32_t w4 = (wb + 4 < static_cast<uint32_t>(P.n_words)) ? wb + 4 : static_cast<uint32_t>(P.n_words) - 1;
        wr.tail = tile[w4];
        wp = pos;
    };
    auto consume = [&](int b, typename T::Piece (&src)[4], const WinWords &wr, uint32_t pos) {
        const uint32_t kb = static_cast<uint32_t>(b) * kKBlock + 8u * lg;
        const uint32_t sh = pos & 31u;
        const uint32_t last = static_cast<uint32_t>(P.n_words) - 4u;
        uint32_t win[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) win[j] = __funnelshift_r(wr.q[j], j < 3 ? wr.q[j + 1] : wr.tail, sh);
        const uint32_t left = p32 - pos;   // bits before the tile end; the window continues at bit 0
        if (__any((pos >> 5) > last || left < 128u)) {   // rare: near the tile end
            const uint32_t skip = (pos >> 5) > last ? (pos >> 5) - last : 0u;   // words the load was moved back by
            uint32_t t[9];
#pragma unroll
            for (int j = 0; j < 9; ++j) t[j] = j < 4 ? wr.q[j] : (j == 4 ? wr.tail : 0u);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t lo = 0, hi = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (skip == static_cast<uint32_t>(i)) { lo = t[j + i]; hi = t[j + i + 1]; }
                uint32_t raw = __funnelshift_r(lo, hi, sh);
                // bits of this word at or past `left` come from the tile start
                const int32_t lj = static_cast<int32_t>(left) - 32 * j;
                if (lj < 32) {
                    const uint32_t hb = lj <= 0 ? static_cast<uint32_t>(-lj) : 0u;   // first head bit used
                    uint32_t h0 = 0, h1 = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if ((hb >> 5) == static_cast<uint32_t>(i)) { h0 = head[i]; h1 = head[i + 1]; }
                    const uint32_t hw = __funnelshift_r(h0, h1, hb & 31u);
                    raw = lj <= 0 ? hw : ((raw & ((1u << lj) - 1u)) | (hw << lj));
                }
                win[j] = raw;
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (kb + 32u * s >= in32) T::zero(src[s]);
            Frag bw, a[NP];
            expand_byte(bw, ~win[s], byte_sel, sign_mask, one_bits);
            T::planes_of(src[s], a);
            if (FIXUP) {
                // elements kb + 32 s + i with i < na lie before the tile start: keep them in the first
                // operand, the others in the second (0.0 elsewhere)
                const int32_t na = static_cast<int32_t>(j_e) - static_cast<int32_t>(kb + 32u * s);
                Frag bw2;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t keep = (na > 2 * v ? 0x0000ffffu : 0u) | (na > 2 * v + 1 ? 0xffff0000u : 0u);
                    bw2.u[v] = bw.u[v] & ~keep;
                    bw.u[v] &= keep;
                }
#pragma unroll
                for (int pl = 0; pl < NP; ++pl) {
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[pl].v, bw.v, acc[0], 0, 0, 0);
                    acc[NA - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[pl].v, bw2.v, acc[NA - 1], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int pl = 0; pl < NP; ++pl)
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[pl].v, bw.v, acc[0], 0, 0, 0);
            }
        }
    };

    // The wave's blocks are wave, wave + 8, ...; NB of them are loaded at once (for in <= 4096 with
    // bf16 that is all of them: one round trip to memory), then multiplied.
    for (int b0 = wave; b0 < n_blocks; b0 += kWaves * NB) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int b = b0 + j * kWaves;
            issue(b < n_blocks ? b : b0, pc[j], wraw[j], wpos[j]);   // a repeated block is loaded but not used
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int b = b0 + j * kWaves;
            if (b < n_blocks) consume(b, pc[j], wraw[j], wpos[j]);
        }
    }

    // accumulator layout: lane holds column ln, batch rows 4*lg + i
#pragma unroll
    for (int h = 0; h < NA; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) part[h][wave][4 * lg + i][ln] = acc[h][i];
    __syncthreads();
    if (tid < 256) {
        const int mm = tid >> 4, uu = tid & 15;
#pragma unroll
        for (int h = 0; h < NA; ++h) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += part[h][w][mm][uu];
            zfin[h][mm][uu] = s;
        }
    }
    __syncthreads();

    if (FIXUP) {   // one column per (tile start, batch row): y = alpha[c-1] * (sum before) + alpha[c] * (sum from)
        const int64_t c = u0 + u + 1;
        if (tid < 256 && c < P.k && m0 + m < P.M) {
            int64_t o_c;
            uint32_t je;
            tile_start_row(P, c, o_c, je);
            if (je != 0 && o_c < P.out) {
                float v = alpha[c - 1] * zfin[0][m][u] + alpha[c] * zfin[NA - 1][m][u];
                if (RELU) v = fmaxf(v, 0.f);
                ElemIO<XT>::store(y + (m0 + m) * P.out + o_c, v);
            }
        }
        return;
    }

    // epilogue: thread -> (replica t, batch row m, column u); u runs fastest over the lanes
    if (u0 + u < P.U && m0 + m < P.M) {
        const float z = zfin[0][m][u];
        XT *yrow = y + (m0 + m) * P.out;
        for (int64_t t0 = tid >> 8; t0 < reps; t0 += 4 * kStep) {
            float al[4];   // fetched up front: one memory round trip per four replicas
#pragma unroll
            for (int j = 0; j < 4; ++j) al[j] = (t0 == (tid >> 8)) ? al_first[j] : alpha_of(t0 + j * kStep);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t t = t0 + j * kStep;
                const int64_t o = u0 + u + t * P.U;
                if (t < reps && o < P.out) {
                    float v = al[j] * z;
                    if (RELU) v = fmaxf(v, 0.f);
                    ElemIO<XT>::store(yrow + o, v);
                }
            }
        }
    }
}

template <typename XT, bool RELU, bool FIXUP> void launch_sk(const LinearArgs &a, const SkinnyParams &P, dim3 grid) {
    hipLaunchKernelGGL((linear_skinny_kernel<XT, RELU, FIXUP>), grid, dim3(kThreads), 0, a.stream,
                       static_cast<const XT *>(a.x), static_cast<XT *>(a.y), a.tile, a.alpha, P);
}

template <bool FIXUP> void launch_sk_any(const LinearArgs &a, const SkinnyParams &P, dim3 grid) {
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    if (a.dt == TBN_F32) {
        if (relu) launch_sk<float, true, FIXUP>(a, P, grid); else launch_sk<float, false, FIXUP>(a, P, grid);
    } else {
        if (relu) launch_sk<uint16_t, true, FIXUP>(a, P, grid); else launch_sk<uint16_t, false, FIXUP>(a, P, grid);
    }
}

bool shape_ok(const LinearArgs &a) {
    if (a.p < a.in || a.p < 160) return false;  // at most one tile end per row and window; five tile words exist
    if (a.p >= (int64_t(1) << 31) - 256 || a.in > (1 << 21)) return false;   // positions and products in 32 / 53 bits
    if (a.in % 8 != 0) return false;            // 16-byte (bf16) / 32-byte (f32) activation pieces
    if (reinterpret_cast<uintptr_t>(a.x) & 15u) return false;
    return true;
}

SkinnyParams make_params(const LinearArgs &a) {
    SkinnyParams P;
    P.M = a.M; P.in = a.in; P.out = a.out; P.p = a.p;
    P.n_words = (a.p + 31) / 32;
    P.U = unique_rows(a.out, a.in, a.p);
    P.n_alpha = a.n_alpha;
    P.aligned = (a.p % a.in == 0) ? 1 : 0;
    P.k = a.k;
    return P;
}

}  // namespace

// Beyond batch 64 the kernel still takes small problems.  Its workgroups are 16 batch rows x 16 distinct
// columns with K split over 8 waves, so a problem of a few hundred of them fills the chip, where the
// 128 x 128 blocks of the large-batch kernels would leave most CUs idle behind a few long K loops.  Measured
// on 4096 x 4096, k = 8 (this kernel / large-batch kernel, microseconds per call): bf16 9 / 27 at batch 128,
// 16 / 27 at 256, 32 / 27 at 512; float32 13 / 105 at 128, 48 / 105 at 512, 94 / 107 at 1024, 186 / 110 at
// 2048.  With fewer than 256 columns of K most of its waves have nothing to multiply and the large-batch
// kernels win again.
bool linear_skinny_supported(const LinearArgs &a) {
    if (!shape_ok(a)) return false;
    if (a.n_alpha > 1 && a.p % a.in != 0 && a.M > int64_t(65535) * 16) return false;   // the repair pass could not follow
    if (a.M <= 64) return true;
    if ((a.flags & TBN_FLAG_LARGE_BATCH) || a.in < 256) return false;
    const int64_t U = unique_rows(a.out, a.in, a.p);
    return ((U + 15) / 16) * ((a.M + 15) / 16) <= (a.dt == TBN_F32 ? 2048 : 512);
}

// Recomputes the columns whose weight row holds a tile start (two alphas), at any batch size.
tbn_status launch_linear_tile_ends(const LinearArgs &a) {
    const int64_t gy = (a.M + 15) / 16, gx = (int64_t(a.k) - 1 + 15) / 16;
    if (!shape_ok(a) || a.n_alpha != a.k || gy > 65535 || gx > 65535) return launch_linear_rows_fixup(a);
    if (a.k < 2 || a.M == 0) return TBN_OK;
    const SkinnyParams P = make_params(a);
    launch_sk_any<true>(a, P, dim3(static_cast<unsigned>(gx), static_cast<unsigned>(gy)));
    return check_launch("tbn_linear_forward (tile-start repair kernel)");
}

tbn_status launch_linear_skinny(const LinearArgs &a) {
    const SkinnyParams P = make_params(a);
    const int64_t gx = (P.U + 15) / 16, gy = (a.M + 15) / 16;
    if (gx > 0x7fffffffLL) {
        set_error("tbn_linear_forward: too many distinct rows for one launch");
        return TBN_ERR_UNSUPPORTED;
    }
    launch_sk_any<false>(a, P, dim3(static_cast<unsigned>(gx), static_cast<unsigned>(gy)));
    tbn_status st = check_launch("tbn_linear_forward (small-batch kernel)");
    if (st != TBN_OK) return st;
    // columns whose weight row straddles a tile end need two alphas
    if (a.n_alpha > 1 && !P.aligned) return launch_linear_tile_ends(a);
    return TBN_OK;
}

}  // namespace tbn
