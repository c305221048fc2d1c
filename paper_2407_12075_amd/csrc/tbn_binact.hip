// Fully-connected tiled-bit layer with binary activations (the paper's Conclusion names it as the first
// direction of future work and gives no formula; the reading built here: an activation becomes +1 or -1 by the
// rule Eq. 3 applies to a weight sum -- +1 where it is greater than zero -- and the layer operation stated after
// Eq. 8 is applied to those signs unchanged).  Activations travel as rows of sign bits, 32 per word.
//
// Three kernels:
//   * sign_pack: real activations -> rows of sign bits (one pass over X, 16 bytes per lane where rows are whole
//     words, a wave ballot otherwise).
//   * binact_mfma (tile of whole weight rows, in % 256 == 0): Z = S T^T on the matrix cores in the 4-bit float
//     format (E2M1 holds +1 and -1 exactly; v_mfma_f32_32x32x64_f8f6f4, the form without block scales, multiplies 64
//     elements of K per instruction, four times the bfloat16 rate; the float32 sums of +-1 products are exact).
//     A lane's operand for one instruction is 32 sign bits; each byte of them becomes eight 4-bit values through a
//     256-entry table in LDS that is stored once per lane (entry e of lane l at byte 256 e + 4 l: every read is
//     free of bank conflicts and its address is one v_perm_b32 of the bits and the lane offset).  Both operands
//     use the same assignment of K to lanes and registers, so a dot product does not depend on what that
//     assignment is.  The distinct columns are computed once and every replica is written as alpha[t] * Z in whole
//     128-byte lines after a turn through LDS (Section "CNN Architectures": only one of the tile computations needs
//     to be executed).
//   * binact_generic: every other legal shape, one thread per output, XOR and population count on whole words
//     where a word lies inside one tile copy, bit by bit where it crosses a tile end.
#include "tbn_common.h"

#include <type_traits>

namespace tbn {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));   // round to nearest even in hardware
}

// ---- sign bits ------------------------------------------------------------------------------------------

template <typename XT> struct Chunk;   // 16 bytes of activations -> one bit per element
template <> struct Chunk<float> {
    static constexpr int elems = 4;
    static __device__ __forceinline__ uint32_t bits(const u32x4_t &v) {
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) m |= (__uint_as_float(v[i]) > 0.f ? 1u : 0u) << i;
        return m;
    }
};
template <> struct Chunk<uint16_t> {
    static constexpr int elems = 8;
    static __device__ __forceinline__ uint32_t bits(const u32x4_t &v) {
        uint32_t m = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m |= (__uint_as_float(v[i] << 16) > 0.f ? 1u : 0u) << (2 * i);
            m |= (__uint_as_float(v[i] & 0xffff0000u) > 0.f ? 1u : 0u) << (2 * i + 1);
        }
        return m;
    }
};

// Rows of whole words (in % 32 == 0): the rows of sign bits are then one bit stream over the flat activations.
// A lane takes 16 bytes; the 32 / elems lanes of a word OR their pieces together.
template <typename XT>
__global__ __launch_bounds__(256) void sign_pack_flat_kernel(const XT *__restrict__ x, uint32_t *__restrict__ xbits,
                                                             int64_t n_chunks) {
    constexpr int E = Chunk<XT>::elems, LPW = 32 / E;   // lanes per word: 8 (float32) or 4 (bfloat16)
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    // every lane of a wave runs the same number of rounds (the shuffles need all of them)
    const int64_t first = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t wave_first = first - (threadIdx.x & 63);
    for (int64_t base = wave_first; base < n_chunks; base += stride) {
        const int64_t c = base + (threadIdx.x & 63);
        uint32_t m = 0;
        if (c < n_chunks) {
            const u32x4_t v = *reinterpret_cast<const u32x4_t *>(reinterpret_cast<const unsigned char *>(x) + c * 16);
            m = Chunk<XT>::bits(v) << (E * static_cast<int>(c % LPW));
        }
#pragma unroll
        for (int d = 1; d < LPW; d <<= 1) m |= __shfl_xor(m, d);
        if (c < n_chunks && (c % LPW) == 0) xbits[c / LPW] = m;
    }
}

// Any row length: a wave takes 64 consecutive activations of one row; the ballot of "greater than zero" is the
// two words.  Lanes past the row's end vote 0, which is what the unused bits of a row's last word hold.
template <typename XT>
__global__ __launch_bounds__(256) void sign_pack_ballot_kernel(const XT *__restrict__ x, uint32_t *__restrict__ xbits,
                                                               int64_t M, int64_t in, int64_t groups, int64_t row_words) {
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = int64_t(gridDim.x) * (blockDim.x >> 6);
    const int64_t total = M * groups;
    for (int64_t item = int64_t(blockIdx.x) * (blockDim.x >> 6) + (threadIdx.x >> 6); item < total; item += n_waves) {
        const int64_t m = item / groups, g = item - m * groups;
        const int64_t j = g * 64 + lane;
        const bool pos = j < in && ElemIO<XT>::load(x + m * in + j) > 0.f;
        const uint64_t vote = __ballot(pos);
        if (lane < 2 && 2 * g + lane < row_words)
            xbits[m * row_words + 2 * g + lane] = static_cast<uint32_t>(vote >> (32 * lane));
    }
}

// ---- shape-agnostic forward -----------------------------------------------------------------------------

struct BinactArgs {
    const uint32_t *xbits;
    void *y;
    int dt;
    int64_t M, in, out;
    const uint32_t *tile;
    int64_t p;
    int32_t k;
    const float *alpha;
    int32_t n_alpha;
    uint32_t flags;
    hipStream_t stream;
};

// One output of the layer.  The flat weight index of (o, j) is f = o*in + j: tile bit f % p, alpha[f / p].  The
// products of one tile copy are counted as integers (32 minus twice the differing bits per word) and scaled
// once; with one alpha, or a tile of whole rows, an output is a single product of a float and an integer.
__device__ __forceinline__ float binact_output(const uint32_t *__restrict__ xr, int64_t o, int64_t in, int64_t row_words,
                                               const uint32_t *__restrict__ tile, int64_t p, int64_t n_words,
                                               const float *__restrict__ alpha, int32_t n_alpha) {
    const int64_t f0 = o * in;
    int64_t q = f0 % p;          // tile position of the next weight
    int64_t c = f0 / p;          // tile copy it belongs to
    int32_t cnt = 0;             // sum of the +-1 products inside copy c so far
    float acc = 0.f;
    auto flush = [&]() {   // a tile copy ends; with one alpha for all copies the count simply runs on
        if (n_alpha != 1) {
            acc += alpha[c] * static_cast<float>(cnt);
            cnt = 0;
        }
        ++c;
        q = 0;
    };
    for (int64_t w = 0; w < row_words; ++w) {
        const uint32_t xw = xr[w];
        const int32_t nb = (in - 32 * w) < 32 ? static_cast<int32_t>(in - 32 * w) : 32;
        if (q + nb <= p) {
            const uint32_t win = tile_window32(tile, q, n_words);
            const uint32_t mask = nb == 32 ? 0xffffffffu : ((1u << nb) - 1u);
            cnt += nb - 2 * __popc((xw ^ win) & mask);
            q += nb;
            if (q == p) flush();
        } else {   // the word crosses a tile end
            for (int32_t b = 0; b < nb; ++b) {
                const uint32_t tb = (tile[q >> 5] >> (q & 31)) & 1u;
                cnt += (((xw >> b) & 1u) == tb) ? 1 : -1;
                if (++q == p) flush();
            }
        }
    }
    if (n_alpha == 1) acc = alpha[0] * static_cast<float>(cnt);
    else if (q != 0) acc += alpha[c] * static_cast<float>(cnt);   // the copy the row ends in
    return acc;
}

// one thread per output
template <typename YT>
__global__ __launch_bounds__(256) void binact_generic_kernel(const uint32_t *__restrict__ xbits, YT *__restrict__ y,
                                                             int64_t total, int64_t in, int64_t out, int64_t row_words,
                                                             const uint32_t *__restrict__ tile, int64_t p,
                                                             const float *__restrict__ alpha, int32_t n_alpha, int relu) {
    const int64_t n_words = (p + 31) / 32;
    for (int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; idx < total; idx += int64_t(gridDim.x) * blockDim.x) {
        const int64_t m = idx / out, o = idx - m * out;
        float acc = binact_output(xbits + m * row_words, o, in, row_words, tile, p, n_words, alpha, n_alpha);
        if (relu) acc = fmaxf(acc, 0.f);
        ElemIO<YT>::store(y + idx, acc);
    }
}

// sign bits out: one thread per word of 32 outputs
__global__ __launch_bounds__(256) void binact_generic_sign_kernel(const uint32_t *__restrict__ xbits, uint32_t *__restrict__ ybits,
                                                                  int64_t total_words, int64_t in, int64_t out, int64_t row_words,
                                                                  int64_t out_words, const uint32_t *__restrict__ tile, int64_t p,
                                                                  const float *__restrict__ alpha, int32_t n_alpha) {
    const int64_t n_words = (p + 31) / 32;
    for (int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; idx < total_words; idx += int64_t(gridDim.x) * blockDim.x) {
        const int64_t m = idx / out_words, wo = idx - m * out_words;
        uint32_t bits = 0;
        for (int b = 0; b < 32 && 32 * wo + b < out; ++b)
            bits |= (binact_output(xbits + m * row_words, 32 * wo + b, in, row_words, tile, p, n_words, alpha, n_alpha) > 0.f ? 1u : 0u) << b;
        ybits[idx] = bits;
    }
}

// ---- tile of whole rows, any row length: a thread per batch row and 32 distinct columns ---------------------
// For shapes the matrix-core kernel declines (rows that are no multiple of 256, numbers of distinct columns that are
// no multiple of 8).  With p a multiple of `in` only the U = p / in rows of the tile are distinct.  A workgroup owns
// 128 batch rows (one per thread) and 32 distinct columns, whose tile words pass through LDS, 128 words of K at a
// time (cut out of the tile at any bit offset, the last word of a row masked); a thread loads a word of its sign row
// once and counts the differing bits against the 32 columns' words, which every lane reads from the same LDS address:
// a word of 32 products costs an exclusive-or and a bit count.  Integer counts per output, one product with alpha per
// replica, as in binact_output.
constexpr int kDirCols = 32;
constexpr int kDirRows = 128;
constexpr int kDirStage = 128;   // words of K per pass

struct BinactDirectParams {
    int64_t M, in, out, U, row_words, n_words, out_words;
    int32_t reps, n_alpha, relu;
};

template <typename YT, bool SIGN>
__global__ __launch_bounds__(kDirRows) void binact_direct_kernel(const uint32_t *__restrict__ xbits, YT *__restrict__ y,
                                                                const uint32_t *__restrict__ tile,
                                                                const float *__restrict__ alpha, BinactDirectParams P) {
    __shared__ __attribute__((aligned(16))) uint32_t t_lds[kDirStage][kDirCols];
    const int tid = threadIdx.x;
    const int64_t m = int64_t(blockIdx.x) * kDirRows + tid;
    const int64_t u0 = int64_t(blockIdx.y) * kDirCols;
    const bool live = m < P.M;
    const uint32_t *xr = xbits + (live ? m : P.M - 1) * P.row_words;   // rows past M repeat the last one; never written
    const int32_t tail = static_cast<int32_t>(P.in & 31);               // bits in the last word of a row (0: all 32)

    int32_t cnt[kDirCols];   // differing bits
#pragma unroll
    for (int f = 0; f < kDirCols; ++f) cnt[f] = 0;

    for (int64_t w0 = 0; w0 < P.row_words; w0 += kDirStage) {
        const int32_t n = static_cast<int32_t>(P.row_words - w0 < kDirStage ? P.row_words - w0 : kDirStage);
        __syncthreads();   // the previous pass is done with the staged words
        for (int32_t i = tid; i < n * kDirCols; i += kDirRows) {
            const int32_t e = i / kDirCols, f = i % kDirCols;
            const int64_t u = u0 + f < P.U ? u0 + f : P.U - 1;   // columns past U repeat the last one; never written
            uint32_t tw = tile_window32(tile, u * P.in + 32 * (w0 + e), P.n_words);
            if (tail && w0 + e == P.row_words - 1) tw &= (1u << tail) - 1u;
            t_lds[e][f] = tw;
        }
        __syncthreads();
#pragma unroll 2
        for (int32_t e = 0; e < n; ++e) {
            uint32_t xw = xr[w0 + e];
            if (tail && w0 + e == P.row_words - 1) xw &= (1u << tail) - 1u;   // padding bits of a sign row do not count
            const uint4 *tv = reinterpret_cast<const uint4 *>(t_lds[e]);
#pragma unroll
            for (int g = 0; g < kDirCols / 4; ++g) {
                const uint4 t4 = tv[g];
                cnt[4 * g + 0] += __popc(xw ^ t4.x);
                cnt[4 * g + 1] += __popc(xw ^ t4.y);
                cnt[4 * g + 2] += __popc(xw ^ t4.z);
                cnt[4 * g + 3] += __popc(xw ^ t4.w);
            }
        }
    }

    if (!live) return;
    const int32_t in32 = static_cast<int32_t>(P.in);
    if constexpr (SIGN) {   // U is a multiple of 32: the 32 columns are one word of every replica
        uint32_t pos = 0, neg = 0;   // sum > 0, sum < 0
#pragma unroll
        for (int f = 0; f < kDirCols; ++f) {
            const int32_t z = in32 - 2 * cnt[f];
            pos |= (z > 0 ? 1u : 0u) << f;
            neg |= (z < 0 ? 1u : 0u) << f;
        }
        uint32_t *yr = reinterpret_cast<uint32_t *>(y) + m * P.out_words + (u0 >> 5);
        for (int32_t t = 0; t < P.reps; ++t) {
            const float al = alpha[P.n_alpha == 1 ? 0 : t];
            yr[int64_t(t) * (P.U >> 5)] = al > 0.f ? pos : (al < 0.f ? neg : 0u);
        }
    } else {
        YT *yr = y + m * P.out;
        for (int32_t t = 0; t < P.reps; ++t) {
            const float al = alpha[P.n_alpha == 1 ? 0 : t];
#pragma unroll
            for (int f = 0; f < kDirCols; ++f) {
                const int64_t u = u0 + f;
                if (u < P.U) {
                    float v = al * static_cast<float>(in32 - 2 * cnt[f]);
                    if (P.relu) v = fmaxf(v, 0.f);
                    ElemIO<YT>::store(yr + int64_t(t) * P.U + u, v);
                }
            }
        }
    }
}

// ---- matrix-core forward --------------------------------------------------------------------------------

constexpr int kTableBytes = 256 * 256;            // [entry][lane] words
constexpr int kTurnStride = 68;                   // floats per row of a wave's 64 x 64 sums in LDS
constexpr int kTurnBytes = 64 * kTurnStride * 4;  // per wave
constexpr int kMfmaLds = 4 * kTurnBytes > kTableBytes ? 4 * kTurnBytes : kTableBytes;

struct BinactMfmaParams {
    int64_t M;
    int32_t in, out, U;
    int32_t reps;       // out / U
    int32_t n_alpha;
    int32_t tiles_n;    // column blocks of 128
    uint32_t tiles_m;   // row blocks of 128
    int32_t xcd_order;  // deal the column blocks of a row block to one XCD
    int32_t n_super;    // in / 256
    int32_t row_bytes;  // in / 8
};

// 256 threads = 4 waves in 2 x 2; a wave owns 64 batch rows x 64 distinct columns (2 x 2 MFMA tiles) over all of K.
// SIGN: the sign bits of the outputs are written instead of the outputs (U % 32 == 0; YT is then not used).
template <typename YT, bool RELU, bool SIGN>
__global__ __launch_bounds__(256, 2) void binact_mfma_kernel(const uint32_t *__restrict__ xbits, YT *__restrict__ y,
                                                             const uint32_t *__restrict__ tile,
                                                             const float *__restrict__ alpha, BinactMfmaParams P) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, lh = lane >> 5;
    const uint32_t bid = blockIdx.x;
    // Workgroup ids are dealt round-robin to the 8 XCDs: the column blocks of one row block take consecutive slots of
    // one XCD, so that the rows of sign bits they share come from that XCD's L2 (the remaining row blocks: plain order).
    uint32_t tile_m, tile_n;
    {
        const uint32_t tiles_n = static_cast<uint32_t>(P.tiles_n), xcd = bid & 7, slot = bid >> 3;
        // (with real outputs and many column blocks the plain order measured 4 % faster: 8192 x 4096 -> 16384, k = 2 and 8)
        const uint32_t full = P.xcd_order ? (P.tiles_m / 8) * tiles_n : 0u;   // slots per XCD in the regular part
        if (slot < full) {
            const uint32_t q = slot / tiles_n;
            tile_n = slot - q * tiles_n;
            tile_m = q * 8 + xcd;
        } else {
            const uint32_t rest = bid - full * 8;
            const uint32_t q = rest / tiles_n;
            tile_n = rest - q * tiles_n;
            tile_m = (P.xcd_order ? (P.tiles_m / 8) * 8 : 0u) + q;
        }
    }
    const int64_t m0 = int64_t(tile_m) * 128 + (wave >> 1) * 64;   // this wave's first batch row
    const int32_t n0 = static_cast<int32_t>(tile_n) * 128 + (wave & 1) * 64;   // and first distinct column

    // alpha of replica t in lane t (replicas past the 64th are fetched one by one in the epilogue)
    const float alpha_lanes = alpha[P.n_alpha == 1 ? 0 : (lane < P.reps ? lane : P.reps - 1)];

    // table: entry e holds, for bit i of e, the 4-bit float +1.0 (0x2) or -1.0 (0xA) at bits 4i .. 4i+3
    {
        uint32_t v = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) v |= (((tid >> i) & 1) ? 0x2u : 0xAu) << (4 * i);
        const u32x4_t vv = {v, v, v, v};
        u32x4_t *dst = reinterpret_cast<u32x4_t *>(lds + tid * 256);
#pragma unroll
        for (int i = 0; i < 16; ++i) dst[i] = vv;
    }

    // Operand rows.  Activations (second operand): lane (ln, lh) supplies batch row 32*tm + ln.  Tile rows (first
    // operand): lane ln supplies distinct column 32*tn + 16*((ln >> 2) & 1) + 4*(ln >> 3) + (ln & 3); the
    // instruction leaves row 8*(r / 4) + 4*lh + r % 4 of its result in register r, so that register r of a lane
    // is column 32*tn + 16*lh + r: sixteen adjacent columns.  K: bytes 32*S + 16*lh .. + 15 of the row for the
    // four instructions of super-step S, word i for instruction i.
    const unsigned char *a_row[2], *b_row[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int64_t m = m0 + 32 * t + ln;
        m = m < P.M ? m : P.M - 1;
        a_row[t] = reinterpret_cast<const unsigned char *>(xbits) + m * P.row_bytes + 16 * lh;
        int32_t u = n0 + 32 * t + 16 * ((ln >> 2) & 1) + 4 * (ln >> 3) + (ln & 3);
        u = u < P.U ? u : P.U - 1;
        b_row[t] = reinterpret_cast<const unsigned char *>(tile) + int64_t(u) * P.row_bytes + 16 * lh;
    }
    auto load = [&](u32x4_t (&r)[4], int32_t S) {
        r[0] = *reinterpret_cast<const u32x4_t *>(a_row[0] + S * 32);
        r[1] = *reinterpret_cast<const u32x4_t *>(a_row[1] + S * 32);
        r[2] = *reinterpret_cast<const u32x4_t *>(b_row[0] + S * 32);
        r[3] = *reinterpret_cast<const u32x4_t *>(b_row[1] + S * 32);
    };
    // The table starts at LDS address 0 (the kernel has no other LDS object), so the looked-up address needs no base.
    typedef __attribute__((address_space(3))) const int lds_word_t;
    const uint32_t lane_off = static_cast<uint32_t>(lane) * 4u;
    auto expand = [&](i32x8_t &f, uint32_t word) {   // 32 sign bits -> 32 four-bit floats: entry (byte i of word), this lane's copy
        f[0] = *reinterpret_cast<lds_word_t *>(__builtin_amdgcn_perm(word, lane_off, 0x0c0c0400u));
        f[1] = *reinterpret_cast<lds_word_t *>(__builtin_amdgcn_perm(word, lane_off, 0x0c0c0500u));
        f[2] = *reinterpret_cast<lds_word_t *>(__builtin_amdgcn_perm(word, lane_off, 0x0c0c0600u));
        f[3] = *reinterpret_cast<lds_word_t *>(__builtin_amdgcn_perm(word, lane_off, 0x0c0c0700u));
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // Sign bits are fetched two super-steps ahead into three rotating register sets (a super-step is 16
    // instructions, about a quarter of a microsecond: one would not cover a miss in the XCD's L2).
    const int32_t last = P.n_super - 1;
    u32x4_t raw[3][4];
    load(raw[0], 0);
    load(raw[1], 1 < last ? 1 : last);
    __syncthreads();   // the table is written
    i32x8_t F[3][4] = {};   // [operand set][A0, A1, B0, B1]; the upper four words of an operand are not read in this format
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        expand(F[0][f], raw[0][f][0]);
        expand(F[1][f], raw[0][f][1]);
    }
    constexpr int kOne = 0;   // both scale operands zero: the compiler takes the form of the instruction without block scales
    // One super-step: four groups of four instructions.  In front of each instruction one operand of the group after
    // the next is looked up (a lookup takes longer to arrive than two instructions take to run, so one group ahead is
    // not enough), in the order in which that group needs them (A0, B0, B1, A1).  Three operand sets rotate with the
    // groups.  The last super-step loads itself once more and looks up operands nobody multiplies: the body stays one
    // straight line of code, which is what keeps the order written here.
    auto step = [&](auto c_c, int32_t S) __attribute__((always_inline)) {
        constexpr int C = decltype(c_c)::value, N1 = (C + 1) % 3, N2 = (C + 2) % 3;
        load(raw[N2], S + 2 < last ? S + 2 : last);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int s = (C + i) % 3, n = (C + i + 2) % 3;   // group 4 S + i uses set (4 S + i) % 3 = (C + i) % 3
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                constexpr int kOrder[4] = {0, 2, 3, 1};
                const int f = kOrder[q];
                expand(F[n][f], i < 2 ? raw[C][f][i + 2] : raw[N1][f][i - 2]);
                __builtin_amdgcn_sched_group_barrier(0x2, 4, 0);     // the four addresses, then the four reads: a read
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);   // does not follow its own address directly
                __builtin_amdgcn_sched_barrier(0);
                const int tm = q >> 1, tn = q & 1;
                acc[tm][tn] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(F[s][2 + tn], F[s][tm], acc[tm][tn], 4, 4, 0, kOne, 0, kOne);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    int32_t S = 0;
    for (; S + 3 <= P.n_super; S += 3) {
        step(std::integral_constant<int, 0>{}, S);
        step(std::integral_constant<int, 1>{}, S + 1);
        step(std::integral_constant<int, 2>{}, S + 2);
    }
    if (S < P.n_super) {   // one or two super-steps are left; the register sets are back in their first roles
        step(std::integral_constant<int, 0>{}, S);
        if (S + 1 < P.n_super) step(std::integral_constant<int, 1>{}, S + 1);
    }

    // ---- turn the sums round through LDS (the table is no longer needed) and write every replica ----------
    __syncthreads();
    float *zt = reinterpret_cast<float *>(lds + wave * kTurnBytes);
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const f32x4_t v = {acc[tm][tn][4 * a], acc[tm][tn][4 * a + 1], acc[tm][tn][4 * a + 2], acc[tm][tn][4 * a + 3]};
                *reinterpret_cast<f32x4_t *>(zt + (32 * tm + ln) * kTurnStride + 32 * tn + 16 * lh + 4 * a) = v;
            }
    // a lane takes eight adjacent columns of one row; eight lanes cover the 64 columns of a row
    const int c8 = lane & 7, rsub = lane >> 3;
    const int32_t col = n0 + 8 * c8;
    if constexpr (SIGN) {
        // alpha[t] * z is positive where z and alpha[t] have the same sign: the eight bits "z > 0" and the eight bits
        // "z < 0" of a lane are formed once per row and the four lanes of a word OR their bytes together (every lane takes
        // part in the exchanges).  A pass over eight rows has 16 words per replica; they are dealt to the lanes so that
        // one store instruction writes the words of four replicas: lane l stores word l % 16 of the pass (row l / 2 % 8,
        // half l % 2) for replicas l / 16, l / 16 + 4, ..., taking the "positive" or the "negative" word by the sign of
        // that replica's alpha (zero or not a number: no bit).
        uint32_t *yb = reinterpret_cast<uint32_t *>(y);
        const int64_t out_words = P.out >> 5;
        const int slot = lane & 15, t_first = lane >> 4;
        const int owner = (slot >> 1) * 8 + (slot & 1) * 4;   // a lane that holds word `slot` after the exchanges
        const int32_t colw = n0 + 32 * (slot & 1);
        const int32_t words_per_replica = P.U >> 5;
        // the alphas of this lane's first four replicas (up to 16 replicas in all) are fetched once
        float al_own[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int32_t t = t_first + 4 * c;
            al_own[c] = alpha[P.n_alpha == 1 ? 0 : (t < P.reps ? t : P.reps - 1)];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int row = 8 * q + rsub;
            const f32x4_t z0 = *reinterpret_cast<const f32x4_t *>(zt + row * kTurnStride + 8 * c8);
            const f32x4_t z1 = *reinterpret_cast<const f32x4_t *>(zt + row * kTurnStride + 8 * c8 + 4);
            uint32_t wp = 0, wn = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wp |= (z0[i] > 0.f ? 1u : 0u) << i;
                wp |= (z1[i] > 0.f ? 1u : 0u) << (4 + i);
                wn |= (z0[i] < 0.f ? 1u : 0u) << i;
                wn |= (z1[i] < 0.f ? 1u : 0u) << (4 + i);
            }
            uint32_t both = (wp | (wn << 8)) << (16 * (c8 & 1));   // two lanes share a register for the first exchange
            both |= __shfl_xor(both, 1);                           // bytes: pos(c8 even), neg(even), pos(odd), neg(odd)
            const uint32_t pair_p = (both & 0xffu) | ((both >> 8) & 0xff00u), pair_n = ((both >> 8) & 0xffu) | ((both >> 16) & 0xff00u);
            const uint32_t pn = pair_p | (pair_n << 16);           // low half: 16 "positive" bits of the lane pair, high half: "negative"
            const uint32_t other = __shfl_xor(pn, 2);
            const bool upper = (c8 & 2) != 0;                      // this pair holds bits 16 .. 31 of the word
            const uint32_t lo = upper ? other : pn, hi = upper ? pn : other;
            wp = (lo & 0xffffu) | (hi << 16);
            wn = (lo >> 16) | (hi & 0xffff0000u);
            const uint32_t sp = __shfl(wp, owner), sn = __shfl(wn, owner);   // the word this lane stores
            const int64_t m = m0 + 8 * q + (slot >> 1);
            if (m < P.M && colw < P.U) {
                uint32_t *dst = yb + m * out_words + (colw >> 5);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int32_t t = t_first + 4 * c;
                    if (t < P.reps) dst[int64_t(t) * words_per_replica] = al_own[c] > 0.f ? sp : (al_own[c] < 0.f ? sn : 0u);
                }
                for (int32_t t = t_first + 16; t < P.reps; t += 4) {
                    const float al = alpha[P.n_alpha == 1 ? 0 : t];
                    dst[int64_t(t) * words_per_replica] = al > 0.f ? sp : (al < 0.f ? sn : 0u);
                }
            }
        }
        return;
    }
    if (col < P.U) {
#pragma unroll 1
        for (int q = 0; q < 8; ++q) {
            const int row = 8 * q + rsub;
            const int64_t m = m0 + row;
            if (m >= P.M) continue;
            const f32x4_t z0 = *reinterpret_cast<const f32x4_t *>(zt + row * kTurnStride + 8 * c8);
            const f32x4_t z1 = *reinterpret_cast<const f32x4_t *>(zt + row * kTurnStride + 8 * c8 + 4);
            YT *yrow = y + m * P.out + col;
            auto emit = [&](int32_t t, float al) __attribute__((always_inline)) {
                float v[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[i] = al * z0[i];
                    v[4 + i] = al * z1[i];
                }
                if (RELU) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = fmaxf(v[i], 0.f);
                }
                if constexpr (sizeof(YT) == 4) {
                    f32x4_t o0 = {v[0], v[1], v[2], v[3]}, o1 = {v[4], v[5], v[6], v[7]};
                    *reinterpret_cast<f32x4_t *>(yrow + int64_t(t) * P.U) = o0;
                    *reinterpret_cast<f32x4_t *>(yrow + int64_t(t) * P.U + 4) = o1;
                } else {
                    u32x4_t o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
                    *reinterpret_cast<u32x4_t *>(yrow + int64_t(t) * P.U) = o;
                }
            };
            const int32_t reps_in_lanes = P.reps < 64 ? P.reps : 64;
            for (int32_t t = 0; t < reps_in_lanes; ++t)
                emit(t, __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, alpha_lanes), t)));
            for (int32_t t = 64; t < P.reps; ++t) emit(t, alpha[P.n_alpha == 1 ? 0 : t]);
        }
    }
}

bool binact_mfma_supported(const BinactArgs &a) {
    if (a.p % a.in != 0 || a.in % 256 != 0) return false;
    const int64_t U = a.p / a.in;
    if (U % 8 != 0 || a.out % U != 0) return false;
    if ((a.flags & TBN_FLAG_SIGN_OUT) && U % 32 != 0) return false;   // a word of sign bits lies in one replica
    if (a.in > (int64_t(1) << 24) || a.out > (int64_t(1) << 30) || U > (int64_t(1) << 24)) return false;
    if ((reinterpret_cast<uintptr_t>(a.xbits) | reinterpret_cast<uintptr_t>(a.tile) | reinterpret_cast<uintptr_t>(a.y)) & 15u) return false;
    const int64_t blocks = ((a.M + 127) / 128) * ((U + 127) / 128);
    return blocks <= 0x7fffffffLL;
}

// the permission for more than 64 KiB of LDS, once per process
template <typename YT, bool RELU, bool SIGN>
static hipError_t allow_lds() {
    static const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&binact_mfma_kernel<YT, RELU, SIGN>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaLds);
    return e;
}

template <typename YT, bool RELU, bool SIGN = false>
static tbn_status launch_mfma_t(const BinactArgs &a, const BinactMfmaParams &P, unsigned blocks) {
    if (allow_lds<YT, RELU, SIGN>() != hipSuccess) {
        set_error("tbn_linear_forward_binact: the matrix-core kernel was refused %d bytes of LDS", kMfmaLds);
        (void)hipGetLastError();
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL((binact_mfma_kernel<YT, RELU, SIGN>), dim3(blocks), dim3(256), kMfmaLds, a.stream, a.xbits,
                       static_cast<YT *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward_binact (matrix-core kernel)");
}

tbn_status launch_binact_mfma(const BinactArgs &a) {
    const int64_t U = a.p / a.in;
    BinactMfmaParams P;
    P.M = a.M;
    P.in = static_cast<int32_t>(a.in);
    P.out = static_cast<int32_t>(a.out);
    P.U = static_cast<int32_t>(U);
    P.reps = static_cast<int32_t>(a.out / U);
    P.n_alpha = a.n_alpha;
    P.tiles_n = static_cast<int32_t>((U + 127) / 128);
    P.tiles_m = static_cast<uint32_t>((a.M + 127) / 128);
    // (sign bits out with 64 column blocks: the same time in both orders, but the 4 MiB of tile rows of a row block then
    // pass through every XCD's L2 once per row block, 203 MB fetched instead of 40)
    P.xcd_order = P.tiles_n <= ((a.flags & TBN_FLAG_SIGN_OUT) ? 32 : 4) ? 1 : 0;
    P.n_super = static_cast<int32_t>(a.in / 256);
    P.row_bytes = static_cast<int32_t>(a.in / 8);
    const unsigned blocks = static_cast<unsigned>(((a.M + 127) / 128) * P.tiles_n);
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    if (a.flags & TBN_FLAG_SIGN_OUT) return launch_mfma_t<float, false, true>(a, P, blocks);
    if (a.dt == TBN_F32) return relu ? launch_mfma_t<float, true>(a, P, blocks) : launch_mfma_t<float, false>(a, P, blocks);
    return relu ? launch_mfma_t<uint16_t, true>(a, P, blocks) : launch_mfma_t<uint16_t, false>(a, P, blocks);
}

tbn_status launch_binact_generic(const BinactArgs &a) {
    if (a.flags & TBN_FLAG_SIGN_OUT) {
        const int64_t out_words = (a.out + 31) / 32, total_words = a.M * out_words;
        int64_t blocks = (total_words + 255) / 256;
        if (blocks > (1 << 20)) blocks = 1 << 20;
        hipLaunchKernelGGL(binact_generic_sign_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, a.stream, a.xbits,
                           static_cast<uint32_t *>(a.y), total_words, a.in, a.out, (a.in + 31) / 32, out_words, a.tile, a.p,
                           a.alpha, a.n_alpha);
        return check_launch("tbn_linear_forward_binact (generic kernel, sign bits out)");
    }
    const int64_t total = a.M * a.out;
    int64_t blocks = (total + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    const int relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    const int64_t row_words = (a.in + 31) / 32;
    if (a.dt == TBN_F32)
        hipLaunchKernelGGL(binact_generic_kernel<float>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, a.stream, a.xbits,
                           static_cast<float *>(a.y), total, a.in, a.out, row_words, a.tile, a.p, a.alpha, a.n_alpha, relu);
    else
        hipLaunchKernelGGL(binact_generic_kernel<uint16_t>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, a.stream,
                           a.xbits, static_cast<uint16_t *>(a.y), total, a.in, a.out, row_words, a.tile, a.p, a.alpha,
                           a.n_alpha, relu);
    return check_launch("tbn_linear_forward_binact (generic kernel)");
}

bool binact_direct_supported(const BinactArgs &a) {
    if (a.M < 1 || a.p % a.in != 0 || a.in >= (int64_t(1) << 31)) return false;
    const int64_t U = a.p / a.in;
    if (U < 1 || U > a.out || a.out % U != 0 || a.out / U > (1 << 30)) return false;
    if (a.n_alpha != 1 && a.n_alpha != a.out / U) return false;
    if ((a.flags & TBN_FLAG_SIGN_OUT) && U % 32 != 0) return false;   // a word of sign bits lies in one replica
    return (a.M + kDirRows - 1) / kDirRows <= 0x7fffffffLL && (U + kDirCols - 1) / kDirCols <= 65535;
}

tbn_status launch_binact_direct(const BinactArgs &a) {
    BinactDirectParams P;
    P.M = a.M; P.in = a.in; P.out = a.out;
    P.U = a.p / a.in;
    P.row_words = (a.in + 31) / 32;
    P.n_words = (a.p + 31) / 32;
    P.out_words = (a.out + 31) / 32;
    P.reps = static_cast<int32_t>(a.out / P.U);
    P.n_alpha = a.n_alpha;
    P.relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    const dim3 grid(static_cast<unsigned>((a.M + kDirRows - 1) / kDirRows), static_cast<unsigned>((P.U + kDirCols - 1) / kDirCols));
    if (a.flags & TBN_FLAG_SIGN_OUT)
        hipLaunchKernelGGL((binact_direct_kernel<float, true>), grid, dim3(kDirRows), 0, a.stream, a.xbits,
                           static_cast<float *>(a.y), a.tile, a.alpha, P);
    else if (a.dt == TBN_F32)
        hipLaunchKernelGGL((binact_direct_kernel<float, false>), grid, dim3(kDirRows), 0, a.stream, a.xbits,
                           static_cast<float *>(a.y), a.tile, a.alpha, P);
    else
        hipLaunchKernelGGL((binact_direct_kernel<uint16_t, false>), grid, dim3(kDirRows), 0, a.stream, a.xbits,
                           static_cast<uint16_t *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward_binact (direct kernel)");
}

}  // namespace

tbn_status launch_sign_pack(const void *x, int dt, int64_t M, int64_t in, uint32_t *xbits, hipStream_t stream) {
    const int64_t row_words = (in + 31) / 32;
    if (in % 32 == 0 && !(reinterpret_cast<uintptr_t>(x) & 15u)) {
        const int64_t n_chunks = M * in / (dt == TBN_F32 ? 4 : 8);
        int64_t blocks = (n_chunks + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        if (dt == TBN_F32)
            hipLaunchKernelGGL(sign_pack_flat_kernel<float>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                               static_cast<const float *>(x), xbits, n_chunks);
        else
            hipLaunchKernelGGL(sign_pack_flat_kernel<uint16_t>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                               static_cast<const uint16_t *>(x), xbits, n_chunks);
        return check_launch("tbn_sign_pack");
    }
    const int64_t groups = (in + 63) / 64;
    int64_t blocks = (M * groups + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    if (dt == TBN_F32)
        hipLaunchKernelGGL(sign_pack_ballot_kernel<float>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                           static_cast<const float *>(x), xbits, M, in, groups, row_words);
    else
        hipLaunchKernelGGL(sign_pack_ballot_kernel<uint16_t>, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                           static_cast<const uint16_t *>(x), xbits, M, in, groups, row_words);
    return check_launch("tbn_sign_pack");
}

tbn_status launch_linear_binact(const uint32_t *xbits, void *y, int dt, int64_t M, int64_t in, int64_t out,
                                const uint32_t *tile, int64_t p, int32_t k, const float *alpha, int32_t n_alpha,
                                uint32_t flags, hipStream_t stream) {
    const BinactArgs a{xbits, y, dt, M, in, out, tile, p, k, alpha, n_alpha, flags, stream};
    if (!(flags & TBN_FLAG_FORCE_GENERIC)) {
        if (binact_mfma_supported(a)) return launch_binact_mfma(a);
        // (at small batches with short rows one thread per output is level or ahead: 64 rows of 1000 bits 12.7 us
        // against 22.4)
        if ((a.M > 64 || a.in >= 2048) && binact_direct_supported(a)) return launch_binact_direct(a);
    }
    return launch_binact_generic(a);
}

}  // namespace tbn
