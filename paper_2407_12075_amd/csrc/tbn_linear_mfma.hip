// Matrix-core kernels for the fully-connected tiled-bit layer, K split inside the workgroup.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8; Algorithm 1 gives the
// same sums with a running index): the (out x in) weight is the tile repeated along the
// flattened index, so weight row o carries the cyclic tile window that starts at bit
// (o*in) % p.  That start repeats with period U = p / gcd(in, p) rows, hence only U distinct
// +-1 rows exist.  The kernels form Z = X * T_U^T for those U rows once and write every output
// column o = u + t*U as alpha(o) * Z[:, u].
//
// gfx950 mapping, chosen from measurements on the chip: one v_mfma_f32_32x32x16_bf16 keeps a SIMD's
// matrix pipe busy for 32 cycles, a wave issues at most one instruction every four cycles, so about five
// independent VALU / LDS / memory instructions fit in an MFMA's shadow and every further one costs issue
// time.  Turning tile bits into a +-1 bf16 operand costs 9 VALU instructions per operand, so an operand
// has to feed four MFMAs, i.e. a wave needs a 128-row block.  With only U/64 column strips that would
// leave most SIMDs idle for a small U, so K is split instead:
//   * a workgroup (4 waves) owns a 128 x 128 block of Z; wave (g, h) multiplies all 128 rows with
//     column half h over the stages of K congruent to g mod 2 (128 accumulator registers); the two
//     partial blocks are added through LDS at the end and every wave writes 64 rows x 64 columns
//   * bf16 activations go from global memory straight into LDS (global_load_lds_dwordx4, four stage
//     buffers per K group, no staging registers, no LDS stores); rows are unpadded and their
//     16-byte chunks are XOR-swizzled by choosing which chunk each lane fetches, so that the
//     operand reads are free of bank conflicts;
//   * float32 activations are loaded into a register ring and split exactly into three bf16 terms
//     when they are written to LDS (8 + 8 + 8 significand bits; the weights are +-1, so every product
//     is exact and the sums are float32 accumulations in the matrix pipe);
//   * the +-1 operand never exists in memory, nor the tile bits in LDS: lanes fetch the words of
//     their columns' cyclic tile windows (they stay in L1 / L2); the bf16 kernel turns a byte of window
//     bits into the eight +-1 values of an MFMA operand with one read of a 256-entry table in LDS (one
//     bit-field extract and one shift-add per operand), the float32 kernel expands the byte in registers
//     (v_perm, a shift of both 16-bit halves, a merge with the pattern of 1.0);
//   * the +-1 operand is the MFMA's row operand and the activations its column operand, with the
//     operand lanes numbered so that a lane ends up with eight adjacent columns of one row of Y; the
//     epilogue scales by alpha, turns the block round through LDS so that eight lanes hold a whole
//     row of the wave's 64 columns, and writes the replicated column blocks with 16-byte stores.
// Rows whose weights straddle a tile end use two different alphas when one alpha per tile is
// given; those few columns are recomputed afterwards in one pass over X (see tbn_linear_skinny.hip,
// launch_linear_tile_ends).
#include "tbn_common.h"

#include <type_traits>

namespace tbn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));

namespace {

constexpr int kThreads = 256;
constexpr int kKG = 2;                 // K groups per workgroup
constexpr int kGroupThreads = kThreads / kKG;
constexpr int kTM = 4, kTN = 2;        // 32 x 32 MFMA tiles per wave along M and N
constexpr int kBM = kTM * 32;          // 128 rows per workgroup, all of them taken by every wave
constexpr int kWN = kTN * 32;          // 64 columns per wave
constexpr int kBN = 2 * kWN;           // 128 columns per workgroup
constexpr int kTmOut = kTM / 2;        // row blocks a wave writes after the exchange
constexpr int kExchangeBytes = kThreads * kTmOut * kTN * 16 * 4;   // partial sums handed over at the end

union Frag {
    bf16x8_t v;
    u32x4_t q;
};

struct MfmaParams {
    int64_t M, out, U;
    int32_t in, p, n_words;
    int32_t n_alpha;
    int aligned;      // p % in == 0: alpha index of column o is o / U
    int vec_store;    // groups of eight adjacent columns can be written with aligned 16-byte stores
    int tiles_n;      // column blocks of U
    uint32_t tiles_m;
    int32_t reps_all; // out / U when U divides out, else 0
};

// x mod p for x < 2^53 and p < 2^31: the float64 quotient is off by at most one.
__device__ __forceinline__ uint32_t mod_u53(uint64_t x, uint32_t p) {
    const uint64_t q = static_cast<uint64_t>(static_cast<double>(x) / static_cast<double>(p));
    int64_t r = static_cast<int64_t>(x - q * p);
    if (r < 0) r += p;
    if (r >= static_cast<int64_t>(p)) r -= p;
    return static_cast<uint32_t>(r);
}

// floor(x / p) for x < 2^53 and p < 2^31, by the same float64 quotient.
__device__ __forceinline__ uint32_t div_u53(uint64_t x, uint32_t p) {
    uint64_t q = static_cast<uint64_t>(static_cast<double>(x) / static_cast<double>(p));
    const int64_t r = static_cast<int64_t>(x - q * p);
    if (r < 0) --q;
    if (r >= static_cast<int64_t>(p)) ++q;
    return static_cast<uint32_t>(q);
}

// truncation split: t0 = top 8 significand bits, t1 = next 8, t2 = the rest (at most 8 bits)
__device__ __forceinline__ void split3(float x, uint32_t &t0, uint32_t &t1, uint32_t &t2) {
    t0 = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(t0);
    t1 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(t1);
    t2 = __float_as_uint(r2);
}

// high halves of two words in one: (lo >> 16) | (hi & 0xffff0000), a single v_perm_b32
__device__ __forceinline__ uint32_t pack_hi16(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x07060302u); }

// Stores of four adjacent outputs (8-byte aligned bf16, 16-byte aligned float32).
template <typename OT> struct OutPack;
template <> struct OutPack<uint16_t> {
    static __device__ __forceinline__ uint32_t pack2(float a, float b) {
        const f32x2_t f = {a, b};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));   // round to nearest even in hardware
    }
    static __device__ __forceinline__ void store4(uint16_t *p, const float (&v)[4]) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        *reinterpret_cast<u32x2_t *>(p) = u32x2_t{pack2(v[0], v[1]), pack2(v[2], v[3])};
    }
    static __device__ __forceinline__ void store8(uint16_t *p, const float (&v)[8]) {   // 16-byte aligned
        *reinterpret_cast<u32x4_t *>(p) = u32x4_t{pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
    }
};
template <> struct OutPack<float> {
    static __device__ __forceinline__ void store4(float *p, const float (&v)[4]) {
        *reinterpret_cast<f32x4_t *>(p) = f32x4_t{v[0], v[1], v[2], v[3]};
    }
    static __device__ __forceinline__ void store8(float *p, const float (&v)[8]) {   // 16-byte aligned
        *reinterpret_cast<f32x4_t *>(p) = f32x4_t{v[0], v[1], v[2], v[3]};
        *reinterpret_cast<f32x4_t *>(p + 4) = f32x4_t{v[4], v[5], v[6], v[7]};
    }
};

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// Workgroups that share rows of X are given consecutive slots on one XCD (workgroup ids are dealt
// round-robin to the 8 XCDs), so the later column blocks find X in that XCD's L2.
__device__ __forceinline__ void block_coords(const MfmaParams &P, uint32_t &tile_m, uint32_t &tile_n) {
    const uint32_t bid = blockIdx.x;
    const uint32_t xcd = bid & 7, slot = bid >> 3;
    const uint32_t tiles_n = static_cast<uint32_t>(P.tiles_n);
    const uint32_t per_xcd_full = (P.tiles_m / 8) * tiles_n;   // slots per XCD in the regular part
    if (slot < per_xcd_full) {
        const uint32_t q = slot / tiles_n;
        tile_n = slot - q * tiles_n;
        tile_m = q * 8 + xcd;
    } else {  // remaining row blocks: plain order
        const uint32_t rest = bid - per_xcd_full * 8;
        const uint32_t q = rest / tiles_n;
        tile_n = rest - q * tiles_n;
        tile_m = (P.tiles_m / 8) * 8 + q;
    }
}

// The +-1 operand goes into the MFMA as the row operand and the activations as the column operand:
// a lane then holds, for one row of Y, sixteen columns per 32 x 32 tile (accumulator register e is
// operand lane 8*(e/4) + 4*lg + e%4).  Operand lane l of tile tn is given column
// 16*(l/8) + 8*((l/4)%2) + 4*tn + l%4 of the wave's 64, so that registers 4q .. 4q + 3 of the two tiles
// are the eight adjacent columns 16*q + 8*lg .. + 7: one 16-byte store of bf16 (two of float32).
__device__ __forceinline__ int wave_col(int l, int tn) { return 16 * (l >> 3) + 8 * ((l >> 2) & 1) + 4 * tn + (l & 3); }

// Cyclic bit position of the tile window of distinct row `col` at K offset k_off (columns past U
// repeat the last one; they are never written).
__device__ __forceinline__ uint32_t window_start(const MfmaParams &P, int64_t col, int k_off) {
    const int64_t u = col < P.U ? col : P.U - 1;
    return mod_u53(static_cast<uint64_t>(u) * static_cast<uint32_t>(P.in) + static_cast<uint32_t>(k_off),
                   static_cast<uint32_t>(P.p));
}

// WW + 1 tile words with one load instruction (dword alignment is all the hardware asks for).
template <int N> struct WordVec;
template <> struct WordVec<2> { typedef uint32_t type __attribute__((ext_vector_type(2), aligned(4))); };
template <> struct WordVec<3> { typedef uint32_t type __attribute__((ext_vector_type(3), aligned(4))); };

// Issues the load of the WW + 1 tile words that hold the BK window bits from pos on, and moves pos to
// the group's next stage.  Near the tile end the load starts earlier so that it stays inside the tile
// (n_words >= WW + 1); wpos keeps the window's cyclic position.
template <int BK, int STEP = kKG * BK>
__device__ __forceinline__ void load_window_one(const MfmaParams &P, const uint32_t *__restrict__ tile, uint32_t &pos,
                                                uint32_t (&wreg)[BK / 32 + 1], uint32_t &wpos) {
    constexpr int NW = BK / 32 + 1;
    const uint32_t w = pos >> 5;
    const uint32_t last = static_cast<uint32_t>(P.n_words - NW);
    const uint32_t wb = w < last ? w : last;
    const typename WordVec<NW>::type v = *reinterpret_cast<const typename WordVec<NW>::type *>(
        reinterpret_cast<const unsigned char *>(tile) + (wb << 2));
#pragma unroll
    for (int j = 0; j < NW; ++j) wreg[j] = v[j];
    wpos = pos;
    pos += STEP;   // the group's next stage; p >= STEP
    if (pos >= static_cast<uint32_t>(P.p)) pos -= static_cast<uint32_t>(P.p);
}
template <int BK>
__device__ __forceinline__ void load_window(const MfmaParams &P, const uint32_t *__restrict__ tile, uint32_t (&pos)[kTN],
                                            uint32_t (&wreg)[kTN][BK / 32 + 1], uint32_t (&wpos)[kTN]) {
#pragma unroll
    for (int tn = 0; tn < kTN; ++tn) load_window_one<BK>(P, tile, pos[tn], wreg[tn], wpos[tn]);
}

// BK window bits of one column from the cyclic position on (bits past the tile end come from its
// start), inverted: bit 1 is weight +1, i.e. sign bit clear.
template <int BK>
__device__ __forceinline__ void form_window_one(const MfmaParams &P, const uint32_t (&wreg)[BK / 32 + 1], uint32_t wpos,
                                                const uint32_t (&head)[BK / 32], uint32_t (&win)[BK / 32]) {
    constexpr int WW = BK / 32;
    constexpr int NW = WW + 1;
    const uint32_t sh = wpos & 31u;
#pragma unroll
    for (int j = 0; j < WW; ++j) win[j] = __funnelshift_r(wreg[j], wreg[j + 1], sh);
    // One test covers both special cases: the load was moved back (pos >= 32 * n_words - BK >= p - BK) and
    // the window runs past the tile end (pos + BK > p).
    if (__builtin_expect(__any(wpos + static_cast<uint32_t>(BK) >= static_cast<uint32_t>(P.p)), 0)) {   // rare
        const uint32_t last = static_cast<uint32_t>(P.n_words - NW);
        const uint32_t w = wpos >> 5;
        if (w > last) {   // the words were loaded from `last` on: skip w - last of them (zeros follow)
            const uint32_t skip = w - last;   // 1 .. NW - 1
            uint32_t t[NW + 1];
#pragma unroll
            for (int j = 0; j <= NW; ++j) {
                uint32_t x = 0;
#pragma unroll
                for (int i = 1; i < NW; ++i)
                    if (skip == static_cast<uint32_t>(i) && j + i < NW) x = wreg[j + i];
                t[j] = x;
            }
#pragma unroll
            for (int j = 0; j < WW; ++j) win[j] = __funnelshift_r(t[j], t[j + 1], sh);
        }
        const uint32_t left = static_cast<uint32_t>(P.p) - wpos;   // >= 1
        if (left < static_cast<uint32_t>(BK)) {
            if (WW == 2) {
                const uint64_t raw = (uint64_t(win[WW - 1]) << 32) | win[0];
                const uint64_t hd = (uint64_t(head[WW - 1]) << 32) | head[0];
                const uint64_t r = (raw & ((uint64_t(1) << left) - 1)) | (hd << left);
                win[0] = static_cast<uint32_t>(r);
                win[WW - 1] = static_cast<uint32_t>(r >> 32);
            } else {
                win[0] = (win[0] & ((1u << left) - 1u)) | (head[0] << left);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < WW; ++j) win[j] = ~win[j];
}
template <int BK>
__device__ __forceinline__ void form_window(const MfmaParams &P, const uint32_t (&wreg)[kTN][BK / 32 + 1],
                                            const uint32_t (&wpos)[kTN], const uint32_t (&head)[BK / 32],
                                            uint32_t (&win)[kTN][BK / 32]) {
#pragma unroll
    for (int tn = 0; tn < kTN; ++tn) form_window_one<BK>(P, wreg[tn], wpos[tn], head, win[tn]);
}

// The two lane halves (lg = 0 / 1) need the same two windows.  Each half loads and forms the window of
// one column (lg = 0 the first, lg = 1 the second) and the halves trade: v_permlane32_swap of a register
// with itself returns the lower half's value in every lane and the upper half's value in every lane.
template <int BK>
__device__ __forceinline__ void share_window(const uint32_t (&own)[BK / 32], uint32_t (&win)[kTN][BK / 32]) {
    static_assert(kTN == 2, "one column per lane half");
#pragma unroll
    for (int j = 0; j < BK / 32; ++j) {
        const auto r = __builtin_amdgcn_permlane32_swap(own[j], own[j], false, false);
        win[0][j] = r[0];
        win[1][j] = r[1];
    }
}

// The +-1 operand of MFMA step ks: lane group lg supplies K elements 16*ks + 8*lg .. + 7, i.e. byte
// 2*ks + lg of the (inverted) window; register v holds elements 2v and 2v + 1.
__device__ __forceinline__ void expand_operand(uint32_t win_lo, uint32_t win_hi, uint32_t byte_sel, uint32_t sign_mask,
                                               uint32_t one_bits, Frag &b) {
    const uint32_t rep = __builtin_amdgcn_perm(win_hi, win_lo, byte_sel);   // the byte, four times
    const u16x2_t r2 = __builtin_bit_cast(u16x2_t, rep);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const u16x2_t sh = {static_cast<uint16_t>(15 - 2 * v), static_cast<uint16_t>(14 - 2 * v)};
        const uint32_t s = __builtin_bit_cast(uint32_t, static_cast<u16x2_t>(r2 << sh));
        b.q[v] = (s & sign_mask) | one_bits;
    }
}

// Adds up the K groups' partial sums through LDS.  Accumulator index tm of group g stands for row block
// (tm + 2*g) % 4, so every group ends up with the finished sums of its row blocks in its first
// accumulators: each of the two groups hands acc[2..3] to the other.
template <int NT>
__device__ __forceinline__ void hand_over(f32x16_t (&acc)[kTM][kTN], float *red, int from_tm, int to_wave, int wave, int lane) {
    constexpr int kSlotFloats = NT * kTN * 16 * 64;   // per wave
    float *dst = red + to_wave * kSlotFloats + lane * 4;
#pragma unroll
    for (int tm = 0; tm < NT; ++tm)
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x16_t &s = acc[from_tm + tm][tn];
                *reinterpret_cast<f32x4_t *>(dst + ((tm * kTN + tn) * 4 + q) * 256) =
                    f32x4_t{s[4 * q], s[4 * q + 1], s[4 * q + 2], s[4 * q + 3]};
            }
    __syncthreads();
    const float *src = red + wave * kSlotFloats + lane * 4;
#pragma unroll
    for (int tm = 0; tm < NT; ++tm)
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4_t v = *reinterpret_cast<const f32x4_t *>(src + ((tm * kTN + tn) * 4 + q) * 256);
                acc[tm][tn][4 * q] += v[0];
                acc[tm][tn][4 * q + 1] += v[1];
                acc[tm][tn][4 * q + 2] += v[2];
                acc[tm][tn][4 * q + 3] += v[3];
            }
}
__device__ __forceinline__ void exchange_partials(f32x16_t (&acc)[kTM][kTN], unsigned char *lds_raw, int wave, int lane) {
    float *red = reinterpret_cast<float *>(lds_raw);
    __syncthreads();   // all waves are done with the staging buffers
    hand_over<2>(acc, red, 2, wave ^ 2, wave, lane);
}

// The slot of the hand-over that only this wave has read: 16 KiB free for the wave's own use afterwards.
__device__ __forceinline__ float *stage_slot(unsigned char *lds_raw, int wave) {
    constexpr int kSlotFloats = 2 * kTN * 16 * 64;
    return reinterpret_cast<float *>(lds_raw) + wave * kSlotFloats;
}

// Epilogue: y[m, u + t*U] = alpha(u + t*U) * Z[m, u] from acc[0..TMOUT-1].  On entry the lane holds row
// 32*TMOUT*grp + 32*tm + ln of the block and, in registers 4q .. 4q + 3 of tiles 0 and 1, columns
// 16*q + 8*lg .. + 7 of the wave's 64 (n_wave is the wave's first distinct row).  The wave turns its sums
// round through LDS, 32 rows at a time, so that eight lanes hold one row's 64 columns: a store
// instruction then writes whole 128-byte lines of bf16 (eight rows of them), and few enough stores are
// issued that the wave never runs into the limit of stores in flight.
//   LDS row r of the 32 is 256 bytes; the 16-byte chunk ch of it (columns 4*ch .. 4*ch + 3) sits at chunk
//   position ch ^ s(r), s(r) = ((r >> 1) & 7) ^ (2 * (r & 1)): the writes (lanes = rows, served even lanes
//   first) and the reads (eight lanes per row; a lane reads chunks 2g and 2g + 1, the upper four lanes
//   in the other order) are then free of bank conflicts.
template <typename XT, bool RELU, int TMOUT>
__device__ __forceinline__ void write_output(const f32x16_t (&acc)[kTM][kTN], const MfmaParams &P, XT *__restrict__ y,
                                             const float *__restrict__ alpha, int64_t m0, int64_t n_wave, int grp, int lane,
                                             float *stage) {   // stage: 8 KiB of LDS that only this wave touches
    static_assert(kTN == 2, "eight adjacent columns come from two tiles");
    const int ln = lane & 31, lg = lane >> 5;
    const int g = lane & 7, rr = lane >> 3;
    const int ch_a = 2 * g + (g >> 2), ch_b = 2 * g + 1 - (g >> 2);
    const int64_t rows_left = P.M - m0;        // >= 1
    const int64_t u0 = n_wave + 8 * g;         // first of this lane's eight adjacent distinct rows
    const int64_t cols_left = P.U - u0;        // <= 0: nothing to write
    const uint32_t lane_off = (static_cast<uint32_t>(rr) * static_cast<uint32_t>(P.out) + static_cast<uint32_t>(8 * g)) *
                              static_cast<uint32_t>(sizeof(XT));
    // every column has the same number of replicas and alpha depends on the replica only
    const bool uniform_alpha = P.reps_all > 0 && (P.n_alpha == 1 || P.aligned);
#pragma unroll
    for (int tm = 0; tm < TMOUT; ++tm) {
        {
            const int s_w = ((ln >> 1) & 7) ^ (2 * (ln & 1));
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int tn = 0; tn < kTN; ++tn) {
                    const int ch = 4 * q + 2 * lg + tn;
                    const f32x16_t &z = acc[tm][tn];
                    *reinterpret_cast<f32x4_t *>(stage + ln * 64 + ((ch ^ s_w) << 2)) =
                        f32x4_t{z[4 * q], z[4 * q + 1], z[4 * q + 2], z[4 * q + 3]};
                }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float zr[4][8];   // rows rr + 8*i of the 32, columns 8*g .. 8*g + 7
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = rr + 8 * i;
            const int s_r = ((r >> 1) & 7) ^ (2 * (r & 1));
            const f32x4_t za = *reinterpret_cast<const f32x4_t *>(stage + r * 64 + ((ch_a ^ s_r) << 2));
            const f32x4_t zb = *reinterpret_cast<const f32x4_t *>(stage + r * 64 + ((ch_b ^ s_r) << 2));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                zr[i][e] = g < 4 ? za[e] : zb[e];
                zr[i][4 + e] = g < 4 ? zb[e] : za[e];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();   // the next 32 rows overwrite the staging area

        const int row_base = (grp * TMOUT + tm) * 32;
        unsigned char *y_blk = reinterpret_cast<unsigned char *>(y + (m0 + row_base) * P.out + n_wave);
        if (uniform_alpha && P.vec_store) {
            // U is a multiple of 8 and every group of eight is 16-byte aligned; the alphas of four replicas
            // are fetched together
            constexpr int kChunk = 4;
            const int reps_all = P.reps_all;
            for (int t0 = 0; t0 < reps_all; t0 += kChunk) {
                float al[kChunk];
#pragma unroll
                for (int j = 0; j < kChunk; ++j) {
                    const int t = (t0 + j < reps_all) ? (t0 + j) : (reps_all - 1);
                    al[j] = alpha[P.n_alpha == 1 ? 0 : t];
                }
#pragma unroll
                for (int j = 0; j < kChunk; ++j) {
                    if (t0 + j >= reps_all) break;
                    unsigned char *dst_t = y_blk + int64_t(t0 + j) * P.U * static_cast<int64_t>(sizeof(XT));
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (cols_left <= 0 || row_base + rr + 8 * i >= rows_left) continue;
                        float v[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            v[e] = al[j] * zr[i][e];
                            if (RELU) v[e] = fmaxf(v[e], 0.f);
                        }
                        OutPack<XT>::store8(reinterpret_cast<XT *>(dst_t + int64_t(8 * i) * P.out * sizeof(XT) + lane_off), v);
                    }
                }
            }
            continue;
        }
        // General case: odd sizes, or tile ends inside rows so that alpha(o) = alpha[(o*in) / p] differs
        // from column to column (the index is divided out for the lane's first column and stepped on).
        if (cols_left <= 0) continue;
        const int n_cols = cols_left < 8 ? static_cast<int>(cols_left) : 8;
        for (int64_t o0 = u0; o0 < P.out; o0 += P.U) {   // replicas
            float al[8];
            if (P.n_alpha == 1) {
                const float a0 = alpha[0];
#pragma unroll
                for (int e = 0; e < 8; ++e) al[e] = a0;
            } else {
                const uint64_t f = static_cast<uint64_t>(o0) * static_cast<uint32_t>(P.in);
                uint32_t idx = div_u53(f, static_cast<uint32_t>(P.p));
                uint32_t rem = static_cast<uint32_t>(f - static_cast<uint64_t>(idx) * static_cast<uint32_t>(P.p));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    al[e] = alpha[idx < static_cast<uint32_t>(P.n_alpha) ? idx : static_cast<uint32_t>(P.n_alpha) - 1];
                    rem += static_cast<uint32_t>(P.in);   // in <= p < 2^31
                    if (rem >= static_cast<uint32_t>(P.p)) { rem -= static_cast<uint32_t>(P.p); ++idx; }
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = row_base + rr + 8 * i;
                if (row >= rows_left) continue;
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    v[e] = al[e] * zr[i][e];
                    if (RELU) v[e] = fmaxf(v[e], 0.f);
                }
                XT *dst = y + (m0 + row) * P.out + o0;
                if (P.vec_store) {   // then n_cols == 8 and o0 + 7 < out
                    OutPack<XT>::store8(dst, v);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e < n_cols && o0 + e < P.out) ElemIO<XT>::store(dst + e, v[e]);
                }
            }
        }
    }
}

// =====================================================================================================
// bf16 activations: global memory -> LDS directly
// =====================================================================================================
namespace direct {

constexpr int kNB = 4;                         // LDS stage buffers per K group
constexpr int kBias = 3 * 1024;                // keeps the lane offsets non-negative, see below

// The kernel exists in two forms, both with two K groups of two waves.  Stages of 64 elements of K (one wave
// per SIMD, 128 KiB of LDS: one workgroup per CU) is the form for long K loops and one block per CU.  Stages
// of 32 elements take 64 KiB, so that two workgroups share a CU and the index work, pipeline fill and
// epilogue of one hide behind the other's MFMAs: the form for short K loops and for grids of several
// blocks per CU.  (Four K groups, two waves of one workgroup per SIMD, measured about 12 % slower in the
// main loop: the two waves of a SIMD do not alternate on the matrix pipe.)
template <int BKP>
struct Cfg {
    static constexpr int KG = kKG;
    static constexpr int kThreads = KG * 128;
    static constexpr int BK = BKP;                       // K elements per stage
    static constexpr int KS = BK / 16;                   // MFMA steps per stage
    static constexpr int WW = (BK + 31) / 32;            // 32-bit window words per stage
    static constexpr int kRowBytes = BK * 2;             // unpadded
    static constexpr int kSwz = kRowBytes / 16 - 1;      // chunk swizzle mask
    static constexpr int kSwzShift = kRowBytes == 128 ? 1 : 2;    // row bits that drive the swizzle start here
    // With 64-byte rows two row slots share the 32 banks.  The LDS serves the even and the odd lanes of
    // 16 in turn, so rows 2i and 2i + 2 must not sit in the same half: row slots trade their two lowest
    // row bits.
    static __device__ __host__ constexpr int row_slot(int r) { return kRowBytes == 128 ? r : ((r & ~3) | ((r & 1) << 1) | ((r >> 1) & 1)); }
    static constexpr int kStageBytes = kBM * kRowBytes;
    static constexpr int kLoads = kStageBytes / 2 / 1024;   // 1 KiB wave-loads per wave and stage
    static constexpr int kRowsPerLoad = 1024 / kRowBytes;
    static constexpr int kLanesPerRow = kRowBytes / 16;
    static constexpr int kVmPerStage = kLoads + 1;       // vector-memory instructions per stage
    static constexpr int kStagesBytes = KG * kNB * kStageBytes;
    static constexpr int kLdsBytes = kStagesBytes > KG * 32768 ? kStagesBytes : KG * 32768;   // the partial sums handed over at the end need 32 KiB per group
    static constexpr int kTableBytes = 256 * 16;   // the +-1 operand of every byte of tile bits, behind the stage buffers
    static constexpr int kLdsTotal = kLdsBytes + kTableBytes;
    static constexpr int kWavesPerSimd = kLdsBytes <= 65536 ? 2 : 1;   // asked of the compiler: registers for two resident workgroups
    static constexpr int kRot = kTM / KG;                // row blocks a group keeps at the end
    static_assert(KG == 2, "two K groups");
    static_assert(BK == 32 || BK == 64, "stages of 32 or 64 elements");
    static_assert(kLoads == 2 * KS, "two wave-loads per MFMA step");
    static_assert(kLdsBytes == 131072 || kLdsBytes == 65536, "LDS budget");
};

// Operand reads (activation fragments and, from the table, the +-1 operands) are written as inline assembly so that the compiler does not see LDS reads next to the
// asynchronous global -> LDS loads (it would make every read wait for all of those loads).  The
// waits are explicit; tying the destination registers to the wait keeps the MFMAs behind it.
template <int OFF>
__device__ __forceinline__ void lds_read16(u32x4_t &dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// At most N younger LDS operations pending; a whole step's operands are tied to the wait: four activation
// fragments and the two +-1 operands read from the table.
template <int N>
__device__ __forceinline__ void lds_wait_step(Frag (&a)[kTM], Frag (&b)[kTN]) {
    static_assert(kTM == 4 && kTN == 2, "six operand registers sets");
    asm volatile("s_waitcnt lgkmcnt(%6)"
                 : "+v"(a[0].q), "+v"(a[1].q), "+v"(a[2].q), "+v"(a[3].q), "+v"(b[0].q), "+v"(b[1].q)
                 : "n"(N));
}
// The +-1 operand of one MFMA step from the table in LDS: entry e (16 bytes) holds the eight bf16 values
// -1 / +1 for the bits 0 .. 7 of e set / clear (the windows are kept inverted).  Lane group lg takes byte
// 2*ks + lg of the window, i.e. the 8 bits at `shift` of the word that holds it: one bit-field extract, one
// shift-add and the read, where expanding the byte in registers takes nine vector instructions.
__device__ __forceinline__ void table_read(u32x4_t &dst, uint32_t word, uint32_t shift, uint32_t table_addr) {
    const uint32_t byte = __builtin_amdgcn_ubfe(word, shift, 8);
    const uint32_t addr = (byte << 4) + table_addr;
    asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(addr));
}

// One 16-byte-per-lane load from global memory straight into LDS (lane i's bytes land at lds + 16*i).
__device__ __forceinline__ void load_to_lds16(const unsigned char *gptr, unsigned char *lds) {
    __builtin_amdgcn_global_load_lds(gptr, lds, 16, 0, 0);
}
// Wave-load J of a stage (the immediate offset has to be a compile-time constant).
template <int J>
__device__ __forceinline__ void stage_load_one(const unsigned char *src, uint32_t off, unsigned char *dst) {
    __builtin_amdgcn_global_load_lds(src + off, dst + (J >> 2) * 4096, 16, (J & 3) * 1024, 0);
}

template <int BKP, bool RELU>
__global__ __launch_bounds__((Cfg<BKP>::kThreads), (Cfg<BKP>::kWavesPerSimd)) void linear_mfma_bf16_kernel(const uint16_t *__restrict__ x,
                                                                          uint16_t *__restrict__ y,
                                                                          const uint32_t *__restrict__ tile,
                                                                          const float *__restrict__ alpha, MfmaParams P) {
    typedef Cfg<BKP> C;
    constexpr int BK = C::BK, KS = C::KS, WW = C::WW, kRowBytes = C::kRowBytes, kStageBytes = C::kStageBytes;
    constexpr int kLoads = C::kLoads, kVmPerStage = C::kVmPerStage, KG = C::KG;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 1;   // K group
    const int wn = wave & 1;     // column half, also the wave's number inside its group
    const int ln = lane & 31;    // column (B operand) / row (A operand) inside a 32 x 32 tile
    const int lg = lane >> 5;    // K half of the operand registers
    unsigned char *lds_grp = lds_raw + grp * kNB * kStageBytes;

    uint32_t tile_m, tile_n;
    block_coords(P, tile_m, tile_n);
    const int64_t m0 = int64_t(tile_m) * kBM;
    const int64_t n0 = int64_t(tile_n) * kBN;

    // ---- activation loads ---------------------------------------------------------------------------
    // Wave-load j of a wave fills 1 KiB of LDS, piece q = kLoads*wn + j of the stage: lane i writes bytes
    // 16*i .. 16*i + 15 of it, i.e. row slot sr = kRowsPerLoad*q + i/kLanesPerRow, chunk slot
    // i%kLanesPerRow.  Row slot block sr/32 holds row block (sr/32 + kRot*grp) % 4 of X (every K group then
    // keeps its first accumulators at the end), and chunk slot s of row slot sr holds 16-byte chunk
    // s ^ ((sr >> kSwzShift) & kSwz) of the stage's bytes of that row, which keeps the operand reads free of
    // bank conflicts (with 64-byte rows the row slots are permuted as well, see Cfg::row_slot).  Rows past M are clamped to row M-1 (their results are never written).
    // The instruction's immediate offset is added to the LDS address and to the global address alike;
    // loads j = 0..3 and 4..7 share an LDS base and differ in that offset, which the per-lane global
    // offset takes back out; kBias, subtracted from the scalar base instead, keeps it non-negative.
    const unsigned char *x_blk = reinterpret_cast<const unsigned char *>(x + m0 * P.in);
    uint32_t a_off[kLoads];      // bytes from (x_blk - kBias) + 2*k0, without the immediate offset
    uint32_t a_row[kLoads];      // bytes of the row start from x_blk
    int a_chunk[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int sr = C::kRowsPerLoad * (kLoads * wn + j) + lane / C::kLanesPerRow;
        const int r = ((((sr >> 5) + C::kRot * grp) & 3) << 5) + C::row_slot(sr & 31);   // row_slot is its own inverse
        const int64_t last = P.M - 1 - m0;
        const uint32_t rr = static_cast<uint32_t>(r < last ? r : last);
        a_chunk[j] = (lane % C::kLanesPerRow) ^ ((sr >> C::kSwzShift) & C::kSwz);
        a_row[j] = rr * static_cast<uint32_t>(P.in) * 2u;
        a_off[j] = a_row[j] + static_cast<uint32_t>(a_chunk[j]) * 16u + kBias - static_cast<uint32_t>((j & 3) * 1024);
    }

    // ---- tile windows ---------------------------------------------------------------------------
    // Operand lane ln supplies columns wave_col(ln, 0) and wave_col(ln, 1) of the wave's 64; this lane
    // looks after the window of the one with tn = lg (see share_window).
    uint32_t pos = window_start(P, n0 + wn * kWN + wave_col(ln, lg), grp * BK);
    uint32_t head[WW];   // start of the tile: continues a window that runs past the tile end
#pragma unroll
    for (int j = 0; j < WW; ++j) head[j] = tile[j];

    constexpr int D = kNB - 1;   // stages in flight
    uint32_t wreg[kNB][WW + 1];   // slot = stage % kNB, like the LDS buffers
    uint32_t wpos[kNB];
    uint32_t win[kTN][WW];
    auto form_windows = [&](int slot) {
        uint32_t own[WW];
        form_window_one<BK>(P, wreg[slot], wpos[slot], head, own);
        share_window<BK>(own, win);
    };

    // Virtual stage v of group g is stage v*kKG + g.  A group whose stage lies past the end of K
    // still goes through the motions (the barriers are shared); its activations are zeroed.
    auto load_stage_full = [&](int slot, int32_t v) {   // the stage lies entirely inside K
        const int32_t k0 = (v * kKG + grp) * BK;
        const unsigned char *src = x_blk - kBias + static_cast<uint32_t>(k0) * 2u;   // wave-uniform
        asm volatile("" : "+s"(src));   // one scalar base, so that the lane offset stays a 32-bit register
        unsigned char *dst = lds_grp + (v & (kNB - 1)) * kStageBytes + wn * (kStageBytes / 2);
        stage_load_one<0>(src, a_off[0], dst);
        stage_load_one<1>(src, a_off[1], dst);
        stage_load_one<2>(src, a_off[2], dst);
        stage_load_one<3>(src, a_off[3], dst);
        if constexpr (kLoads == 8) {
            stage_load_one<4>(src, a_off[4], dst);
            stage_load_one<5>(src, a_off[5], dst);
            stage_load_one<6>(src, a_off[6], dst);
            stage_load_one<7>(src, a_off[7], dst);
        }
        load_window_one<BK, KG * BK>(P, tile, pos, wreg[slot], wpos[slot]);
    };
    auto load_stage_any = [&](int slot, int32_t v) {
        const int32_t k0 = (v * kKG + grp) * BK;
        if (k0 + BK <= P.in) {
            load_stage_full(slot, v);
            return;
        }
        // chunks past the end of the row are fetched from a clamped address and zeroed before use
        unsigned char *dst = lds_grp + (v & (kNB - 1)) * kStageBytes + wn * (kStageBytes / 2);
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            int32_t c = k0 + a_chunk[j] * 8;
            c = c < P.in - 8 ? c : P.in - 8;
            load_to_lds16(x_blk + (a_row[j] + static_cast<uint32_t>(c) * 2u), dst + j * 1024);
        }
        load_window_one<BK, KG * BK>(P, tile, pos, wreg[slot], wpos[slot]);
    };
    // Zeroes the part of stage v that lies past the end of K (its loads are waited for first).
    auto zero_tail = [&](int32_t v) {
        const int32_t k0 = (v * kKG + grp) * BK;
        if (k0 + BK > P.in) {   // uniform over the group: the last stages only
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            unsigned char *dst = lds_grp + (v & (kNB - 1)) * kStageBytes + wn * (kStageBytes / 2) + lane * 16;
#pragma unroll
            for (int j = 0; j < kLoads; ++j)
                if (k0 + a_chunk[j] * 8 >= P.in) *reinterpret_cast<u32x4_t *>(dst + j * 1024) = u32x4_t{0, 0, 0, 0};
        }
    };
    // The workgroup meets.  A plain barrier, no fence: the waits that matter are explicit, and a fence
    // would make the compiler wait for every asynchronous load in flight.
    auto meet = [&](bool lds_writes_pending) {
        if (lds_writes_pending) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };

    f32x16_t acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand reads: row 32*tm + ln at its row slot, chunk 2*ks + lg at chunk slot (2*ks + lg) ^ ((ln >> kSwzShift) & kSwz)
    uint32_t a_rd[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a_rd[ks] = static_cast<uint32_t>(C::row_slot(ln) * kRowBytes + (((2 * ks + lg) ^ ((ln >> C::kSwzShift) & C::kSwz)) << 4));

    // The +-1 operands come from a table of 256 entries behind the stage buffers (see table_read): entry e,
    // element i is -1 if bit i of e is set (the windows are inverted), +1 otherwise.  Step ks needs byte
    // 2*ks + lg of the window: word ks / 2 (one word with 32-element stages), bits 16*(ks % 2) + 8*lg on.
    typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
    {
        unsigned char *table = lds_raw + C::kLdsBytes;
        for (int e = tid; e < 256; e += C::kThreads) {
            u32x4_t t;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                t[v] = (((e >> (2 * v)) & 1) ? 0xbf80u : 0x3f80u) | ((((e >> (2 * v + 1)) & 1) ? 0xbf80u : 0x3f80u) << 16);
            *reinterpret_cast<u32x4_t *>(table + e * 16) = t;
        }
    }
    const uint32_t table_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte_t *)(lds_raw + C::kLdsBytes)));
    uint32_t bsh[2] = {8u * static_cast<uint32_t>(lg), 16u + 8u * static_cast<uint32_t>(lg)};
    auto read_signs = [&](u32x4_t &dst, const uint32_t (&w)[WW], int ks) {   // ks is a compile-time constant where it is called
        table_read(dst, w[(2 * ks) >> 2], bsh[ks & 1], table_addr);
    };

    // The fragments of step ks + 1 are requested before the MFMAs of step ks are issued.
    const uint32_t lds_grp_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte_t *)lds_grp));
    auto read_frags = [&](Frag (&a)[kTM], uint32_t base, int ks) {
        const uint32_t addr = base + a_rd[ks];
        lds_read16<0 * 32 * kRowBytes>(a[0].q, addr);
        lds_read16<1 * 32 * kRowBytes>(a[1].q, addr);
        lds_read16<2 * 32 * kRowBytes>(a[2].q, addr);
        lds_read16<3 * 32 * kRowBytes>(a[3].q, addr);
    };
    // Multiplies stage v (drain form: every step's operands are requested one step ahead, nothing
    // is carried over from or into the neighbouring stages).
    auto multiply_plain = [&](int32_t v) {
        const uint32_t base = lds_grp_addr + static_cast<uint32_t>((v & (kNB - 1)) * kStageBytes);
        Frag a[2][kTM];
        read_frags(a[0], base, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            Frag b[kTN];
#pragma unroll
            for (int tn = 0; tn < kTN; ++tn) read_signs(b[tn].q, win[tn], ks);
            if (ks + 1 < KS) read_frags(a[(ks + 1) & 1], base, ks + 1);
            // LDS reads complete in order: with the next step's four fragments still pending, this step's
            // fragments and signs have arrived
            if (ks + 1 < KS) lds_wait_step<kTM>(a[ks & 1], b); else lds_wait_step<0>(a[ks & 1], b);
#pragma unroll
            for (int tm = 0; tm < kTM; ++tm)
#pragma unroll
                for (int tn = 0; tn < kTN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[tn].v, a[ks & 1][tm].v, acc[tm][tn], 0, 0, 0);
        }
    };

    // Steady-state round st; D_ = st % kNB names its LDS buffer and ring slot.  On entry the operands of
    // its first step are in pa[0] / pb[0], requested during the round before; stages st + 1 .. st + 3 lie
    // inside K.
    //   * the round opens with the meeting that makes stage st + 1 readable (its loads were issued two
    //     rounds ago) and frees the buffer of stage st - 1 for the loads of stage st + 3;
    //   * those loads are spread between the MFMAs, two per step, so that neither this wave nor the CU's
    //     load path sees them as a burst;
    //   * step ks requests the operands of step ks + 1, the last step those of stage st + 1's first
    //     step; the tile windows of stage st + 1 are formed once the last step's operands exist.
    // Buffer numbers and steps are compile-time constants, so every LDS address is a register that
    // never changes plus an immediate offset.
    Frag pa[2][kTM];
    Frag pb[2][kTN];
    uint32_t a_rdg[KS];   // operand read addresses inside the group's first buffer
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a_rdg[ks] = lds_grp_addr + a_rd[ks];
    unsigned char *lds_wave = lds_grp + wn * (kStageBytes / 2);   // where this wave's loads of buffer 0 go
    auto steady_round = [&](auto d_c, int32_t st) {
        constexpr int D_ = decltype(d_c)::value;
        constexpr int kBufNext = (D_ + 1) & (kNB - 1), kBufLoad = (D_ + D) & (kNB - 1);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(kVmPerStage));   // only the loads of stage st + 2 may be in flight
        meet(false);
        const int32_t k0 = ((st + D) * kKG + grp) * BK;
        const unsigned char *src = x_blk - kBias + static_cast<uint32_t>(k0) * 2u;   // wave-uniform
        asm volatile("" : "+s"(src));   // one scalar base
        unsigned char *dst = lds_wave + kBufLoad * kStageBytes;
        // The lane offsets are widened to 64 bits inside the round (not once, outside the loop), which lets
        // the wave-loads take them as 32-bit offsets to the scalar base.
        asm volatile("" : "+v"(a_off[0]), "+v"(a_off[1]), "+v"(a_off[2]), "+v"(a_off[3]));
        if constexpr (kLoads == 8) asm volatile("" : "+v"(a_off[4]), "+v"(a_off[5]), "+v"(a_off[6]), "+v"(a_off[7]));
        uint32_t own[WW];   // this lane half's window of stage st + 1, before the halves trade
        auto step = [&](auto ks_c) {
            // A wave issues one instruction every four cycles at best, an MFMA runs for 32: between two
            // MFMAs there is room for a handful of other instructions, and LDS reads and wave-loads must
            // not come in runs.  The fences keep the compiler from regrouping the work.
            constexpr int ks = decltype(ks_c)::value;
            constexpr int cur = ks & 1, nx = cur ^ 1, ksn = (ks + 1) % KS;
            constexpr int kRd = (ks + 1 < KS ? D_ : kBufNext) * kStageBytes;   // buffer of the operands requested here
            const uint32_t raddr = a_rdg[ksn];
            auto mfma = [&](int tm, int tn) {
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pb[cur][tn].v, pa[cur][tm].v, acc[tm][tn], 0, 0, 0);
            };
            lds_wait_step<0>(pa[cur], pb[cur]);   // the six reads of the step before (the last was issued five MFMAs ago)
            mfma(0, 0);
            lds_read16<kRd + 0 * 32 * kRowBytes>(pa[nx][0].q, raddr);
            read_signs(pb[nx][0].q, win[0], ksn);
            __builtin_amdgcn_sched_barrier(0);
            mfma(0, 1);
            lds_read16<kRd + 1 * 32 * kRowBytes>(pa[nx][1].q, raddr);
            __builtin_amdgcn_sched_barrier(0);
            mfma(1, 0);
            lds_read16<kRd + 2 * 32 * kRowBytes>(pa[nx][2].q, raddr);
            read_signs(pb[nx][1].q, win[1], ksn);
            __builtin_amdgcn_sched_barrier(0);
            mfma(1, 1);
            lds_read16<kRd + 3 * 32 * kRowBytes>(pa[nx][3].q, raddr);
            __builtin_amdgcn_sched_barrier(0);
            mfma(2, 0);
            stage_load_one<2 * ks>(src, a_off[2 * ks], dst);
            __builtin_amdgcn_sched_barrier(0);
            mfma(2, 1);
            // the window of stage st + 1 (this stage's last operands were expanded in this step): this lane
            // half's column here, the trade with the other half after the step's last MFMA; in the last
            // step the window load of stage st + 3
            if constexpr (ks == KS - 2) form_window_one<BK>(P, wreg[kBufNext], wpos[kBufNext], head, own);
            if constexpr (ks == KS - 1) load_window_one<BK, KG * BK>(P, tile, pos, wreg[kBufLoad], wpos[kBufLoad]);
            __builtin_amdgcn_sched_barrier(0);
            mfma(3, 0);
            stage_load_one<2 * ks + 1>(src, a_off[2 * ks + 1], dst);
            __builtin_amdgcn_sched_barrier(0);
            mfma(3, 1);
            if constexpr (ks == KS - 2) share_window<BK>(own, win);
            __builtin_amdgcn_sched_barrier(0);
        };
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        if constexpr (KS == 4) {
            step(std::integral_constant<int, 2>{});
            step(std::integral_constant<int, 3>{});
        }
    };

    const int32_t n_stages = ((P.in + BK - 1) / BK + kKG - 1) / kKG;   // virtual stages per group
    const int32_t n_full = P.in / (kKG * BK);                           // of which both groups' lie inside K
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < n_stages) load_stage_any(d, d);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    zero_tail(0);
    form_windows(0);
    meet(true);   // stage 0 is readable

    int32_t st0 = 0;
    if (kNB + D <= n_full) {   // the steady loop runs: request the first operands
        read_frags(pa[0], lds_grp_addr, 0);
#pragma unroll
        for (int tn = 0; tn < kTN; ++tn) read_signs(pb[0][tn].q, win[tn], 0);
    }
    for (; st0 + kNB + D <= n_full; st0 += kNB) {
        steady_round(std::integral_constant<int, 0>{}, st0);
        steady_round(std::integral_constant<int, 1>{}, st0 + 1);
        steady_round(std::integral_constant<int, 2>{}, st0 + 2);
        steady_round(std::integral_constant<int, 3>{}, st0 + 3);
    }
    // The last steady round has requested operands nobody will use: let them land before their
    // registers can be given to anything else (unconditionally: a wait with nothing pending costs nothing,
    // and no path exists on which a read is in flight past this point).
    lds_wait_step<0>(pa[0], pb[0]);
    // Drain: st0 is a multiple of kNB, so slot numbers stay static.  Every round opens with the meeting
    // that makes stage st + 1 readable; `win` holds the windows of stage st on entry.
    for (; st0 < n_stages; st0 += kNB) {
#pragma unroll
        for (int d = 0; d < kNB; ++d) {
            const int32_t st = st0 + d;
            if (st < n_stages) {   // uniform
                if (st + 1 < n_stages) {
                    if (st + 2 < n_stages) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kVmPerStage));
                    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                    zero_tail(st + 1);
                    meet(true);
                }
                if (st + D < n_stages) load_stage_any((d + D) & (kNB - 1), st + D);
                multiply_plain(st);
                if (st + 1 < n_stages) form_windows((d + 1) & (kNB - 1));
            }
        }
    }
    static_assert(D == 3 && kNB == 4, "the wait counts are written for three stages in flight");

    exchange_partials(acc, lds_raw, wave, lane);
    write_output<uint16_t, RELU, C::kRot>(acc, P, y, alpha, m0, n0 + wn * kWN, grp, lane, stage_slot(lds_raw, wave));
}

}  // namespace direct

// =====================================================================================================
// float32 activations: register ring, split into three bf16 planes on the way to LDS
// =====================================================================================================
namespace ring {

constexpr int NP = 3;                          // exact split x = t0 + t1 + t2 into bf16 terms
constexpr int BK = 32;                         // K elements per stage
constexpr int KS = BK / 16;
constexpr int WW = BK / 32;
constexpr int D = 3;                           // stages in flight in registers
constexpr int kPieces = BK / 8;                // 8-element pieces per row and stage
constexpr int kRowsPerPass = kGroupThreads / kPieces;
constexpr int kRowItems = kBM / kRowsPerPass;  // rows staged per thread and stage
constexpr int RS = (BK + 8) * 2;               // LDS row stride in bytes (16 B of padding)
constexpr int kPlaneBytes = kBM * RS;
constexpr int kBufferBytes = NP * kPlaneBytes;
constexpr int kLdsBytes = 2 * kKG * kBufferBytes > kExchangeBytes ? 2 * kKG * kBufferBytes : kExchangeBytes;

template <bool RELU>
__global__ __launch_bounds__(kThreads, 1) void linear_mfma_f32_kernel(const float *__restrict__ x,
                                                                         float *__restrict__ y,
                                                                         const uint32_t *__restrict__ tile,
                                                                         const float *__restrict__ alpha, MfmaParams P) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 1;   // K group
    const int wn = wave & 1;     // column half
    const int gt = tid & (kGroupThreads - 1);
    const int ln = lane & 31;    // column (B operand) / row (A operand) inside a 32 x 32 tile
    const int lg = lane >> 5;    // K half of the operand registers
    unsigned char *lds_grp = lds_raw + grp * 2 * kBufferBytes;

    uint32_t tile_m, tile_n;
    block_coords(P, tile_m, tile_n);
    const int64_t m0 = int64_t(tile_m) * kBM;
    const int64_t n0 = int64_t(tile_n) * kBN;

    // ---- staging assignments ---------------------------------------------------------------
    // A thread stages pieces of 8 consecutive K elements of kRowItems rows; the pieces of a row lie
    // on adjacent threads.  Rows past M are clamped to row M-1 (their results are never written).
    // Offsets are relative to the block's first row and fit 32 bits (the launcher checks).
    const unsigned char *x_blk = reinterpret_cast<const unsigned char *>(x + m0 * P.in);
    const int a_piece = gt % kPieces;
    uint32_t a_row_off[kRowItems];   // bytes
    int a_lds[kRowItems];            // bytes inside a plane
#pragma unroll
    for (int i = 0; i < kRowItems; ++i) {
        const int r = gt / kPieces + i * kRowsPerPass;
        const int64_t last = P.M - 1 - m0;
        const uint32_t rr = static_cast<uint32_t>(r < last ? r : last);
        a_row_off[i] = rr * static_cast<uint32_t>(P.in) * 4u;
        a_lds[i] = r * RS + a_piece * 16;
    }

    uint32_t pos[kTN];   // operand lane ln supplies columns wave_col(ln, tn) of the wave's 64
#pragma unroll
    for (int tn = 0; tn < kTN; ++tn) pos[tn] = window_start(P, n0 + wn * kWN + wave_col(ln, tn), grp * BK);
    uint32_t head[WW];
#pragma unroll
    for (int j = 0; j < WW; ++j) head[j] = tile[j];

    u32x4_t areg[D][kRowItems][2];
    uint32_t wreg[D][kTN][WW + 1];
    uint32_t wpos[D][kTN];
    uint32_t win[kTN][WW];

    // Loads are unconditional (addresses are clamped into the tensors) so that they stay in flight
    // across stages; what lies past the end of a row is zeroed when the stage is written to LDS.
    // Virtual stage v of group g is stage v*kKG + g.  A group whose stage lies past the end of K
    // still goes through the motions (the barriers are shared); its activations are zero.
    auto load_stage = [&](int slot, int32_t v) {
        const int32_t k0 = (v * kKG + grp) * BK;
        int32_t c = k0 + a_piece * 8;
        c = c < P.in - 8 ? c : P.in - 8;   // in % 8 == 0: a piece is entirely inside or outside the row
        const uint32_t cb = static_cast<uint32_t>(c) * 4u;
#pragma unroll
        for (int i = 0; i < kRowItems; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                areg[slot][i][h] = *reinterpret_cast<const u32x4_t *>(x_blk + (a_row_off[i] + cb + 16u * h));
        load_window<BK>(P, tile, pos, wreg[slot], wpos[slot]);
    };
    auto store_stage = [&](int slot, int buf, int32_t v) {
        const int32_t k0 = (v * kKG + grp) * BK;
        unsigned char *dst = lds_grp + buf * kBufferBytes;
#pragma unroll
        for (int i = 0; i < kRowItems; ++i) {
            uint32_t o[3][4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const u32x4_t &src = areg[slot][i][d >> 1];
                uint32_t e0, e1, e2, f0, f1, f2;
                split3(__uint_as_float(src[(d & 1) * 2]), e0, e1, e2);
                split3(__uint_as_float(src[(d & 1) * 2 + 1]), f0, f1, f2);
                o[0][d] = pack_hi16(e0, f0);
                o[1][d] = pack_hi16(e1, f1);
                o[2][d] = pack_hi16(e2, f2);
            }
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                *reinterpret_cast<u32x4_t *>(dst + pl * kPlaneBytes + a_lds[i]) =
                    u32x4_t{o[pl][0], o[pl][1], o[pl][2], o[pl][3]};
        }
        if (k0 + BK > P.in) {   // uniform over the group: the last stages only
            if (k0 + a_piece * 8 >= P.in) {   // overwrite what was loaded from the clamped address
#pragma unroll
                for (int i = 0; i < kRowItems; ++i)
#pragma unroll
                    for (int pl = 0; pl < NP; ++pl)
                        *reinterpret_cast<u32x4_t *>(dst + pl * kPlaneBytes + a_lds[i]) = u32x4_t{0, 0, 0, 0};
            }
        }
        form_window<BK>(P, wreg[slot], wpos[slot], head, win);
    };

    f32x16_t acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Accumulator index tm of group g works on row block (tm + 2g) % 4 (see exchange_partials).
    int a_blk[kTM];
#pragma unroll
    for (int tm = 0; tm < kTM; ++tm) a_blk[tm] = (((tm + 2 * grp) & (kTM - 1)) * 32 + ln) * RS + lg * 16;

    uint32_t sign_mask = 0x80008000u, one_bits = 0x3f803f80u;
    asm volatile("" : "+v"(sign_mask), "+v"(one_bits));
    uint32_t byte_sel[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) byte_sel[ks] = 0x01010101u * static_cast<uint32_t>(2 * ks + lg);

    auto multiply_stage = [&](int buf) {
        const unsigned char *src = lds_grp + buf * kBufferBytes;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            Frag b[kTN];
#pragma unroll
            for (int tn = 0; tn < kTN; ++tn)
                expand_operand(win[tn][0], win[tn][WW - 1], byte_sel[ks], sign_mask, one_bits, b[tn]);
#pragma unroll
            for (int pl = 0; pl < NP; ++pl) {
                Frag a[kTM];
#pragma unroll
                for (int tm = 0; tm < kTM; ++tm)
                    a[tm].q = *reinterpret_cast<const u32x4_t *>(src + pl * kPlaneBytes + a_blk[tm] + ks * 32);
#pragma unroll
                for (int tm = 0; tm < kTM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < kTN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[tn].v, a[tm].v, acc[tm][tn], 0, 0, 0);
            }
        }
    };

    const int32_t n_stages = ((P.in + BK - 1) / BK + kKG - 1) / kKG;   // virtual stages per group
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < n_stages) load_stage(d, d);
    store_stage(0, 0, 0);
    __syncthreads();

    // Steady state: every sub-iteration issues the loads of stage st + D, multiplies stage st and
    // moves stage st + 1 from registers to LDS.  No condition depends on the stage number here, so
    // the compiler can count exactly how many younger loads may stay in flight at each wait.
    int32_t st0 = 0;
    for (; st0 + 2 * D <= n_stages; st0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int32_t st = st0 + d;
            const int buf = st & 1;
            load_stage(d, st + D);
            multiply_stage(buf);
            store_stage((d + 1) % D, buf ^ 1, st + 1);
            __syncthreads();
        }
    }
    // Drain: at most 2*D - 1 stages are left; st0 is a multiple of D, so slot numbers stay static.
    for (; st0 < n_stages; st0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int32_t st = st0 + d;
            if (st < n_stages) {   // uniform
                const int buf = st & 1;
                if (st + D < n_stages) load_stage(d, st + D);
                multiply_stage(buf);
                if (st + 1 < n_stages) {
                    store_stage((d + 1) % D, buf ^ 1, st + 1);
                    __syncthreads();
                }
            }
        }
    }

    exchange_partials(acc, lds_raw, wave, lane);
    write_output<float, RELU, kTmOut>(acc, P, y, alpha, m0, n0 + wn * kWN, grp, lane, stage_slot(lds_raw, wave));
}

}  // namespace ring

// Dynamic LDS above the default limit has to be allowed once per kernel.
tbn_status set_lds_limit_once(const void *kernel, int lds) {
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return e == hipSuccess ? TBN_OK : TBN_ERR_DEVICE;
}

// Which form of the bf16 kernel runs (see direct::Cfg).  The form with 32-element stages runs two workgroups
// per CU; it wins where a workgroup's fixed work (index arithmetic, pipeline fill, hand-over of the partial
// sums, epilogue) weighs against a short K loop and some CUs have more than one block to run: 8192 x 512 ->
// 4096 distinct columns 56 us against 77, 8192 x 1024 -> 2048 42 against 55, 8192 x 1024 -> 768 (384 blocks)
// 21 against 26; at in = 4096 the forms are within 4 % of each other, and with one block per CU the
// 64-element stages win (42.6 us against 45.2 on 8192 x 4096, 512 distinct columns).
constexpr int kTwoResidentMaxK = 3072;
constexpr int64_t kTwoResidentMinBlocks = 257;   // more than one per CU

template <int BK, bool RELU>
tbn_status launch_bf16(const LinearArgs &a, const MfmaParams &P, dim3 grid) {
    typedef direct::Cfg<BK> C;
    static const tbn_status attr =   // thread-safe static initialisation: set once per process
        set_lds_limit_once(reinterpret_cast<const void *>(&direct::linear_mfma_bf16_kernel<BK, RELU>), C::kLdsTotal);
    if (attr != TBN_OK) {
        set_error("tbn_linear_forward: cannot reserve %d bytes of LDS", C::kLdsTotal);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL((direct::linear_mfma_bf16_kernel<BK, RELU>), grid, dim3(C::kThreads),
                       C::kLdsTotal, a.stream, static_cast<const uint16_t *>(a.x),
                       static_cast<uint16_t *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward (matrix-core kernel)");
}

template <bool RELU>
tbn_status launch_f32(const LinearArgs &a, const MfmaParams &P, dim3 grid) {
    static const tbn_status attr =
        set_lds_limit_once(reinterpret_cast<const void *>(&ring::linear_mfma_f32_kernel<RELU>), ring::kLdsBytes);
    if (attr != TBN_OK) {
        set_error("tbn_linear_forward: cannot reserve %d bytes of LDS", ring::kLdsBytes);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL((ring::linear_mfma_f32_kernel<RELU>), grid, dim3(kThreads), ring::kLdsBytes, a.stream,
                       static_cast<const float *>(a.x), static_cast<float *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward (matrix-core kernel)");
}

}  // namespace

bool linear_mfma_supported(const LinearArgs &a) {
    if (a.p < a.in || a.p < 128) return false;    // at most one tile end per row and per stage window
    if (a.p >= (int64_t(1) << 31) - 256) return false;   // window positions are kept in 32 bits
    if (a.in % 8 != 0) return false;              // 16-byte (bf16) / 32-byte (f32) activation pieces
    if (a.in > (1 << 21) || a.out > (1 << 22)) return false;   // byte offsets inside a 128-row block fit 32 bits
    if (a.M > (int64_t(1) << 36)) return false;   // row blocks are counted in 32 bits
    if (reinterpret_cast<uintptr_t>(a.x) & 15u) return false;
    if (a.M < 16) return false;
    // two alphas inside rows: the repair pass that follows the main kernel must be able to run (its limit on the
    // batch), so that an unsupported shape is refused before anything is enqueued
    if (a.n_alpha > 1 && a.p % a.in != 0 && a.M > int64_t(65535) * 16) return false;
    return true;
}

tbn_status launch_linear_mfma(const LinearArgs &a) {
    MfmaParams P;
    P.M = a.M; P.out = a.out;
    P.in = static_cast<int32_t>(a.in);
    P.p = static_cast<int32_t>(a.p);
    P.n_words = static_cast<int32_t>((a.p + 31) / 32);
    P.U = unique_rows(a.out, a.in, a.p);
    P.n_alpha = a.n_alpha;
    P.aligned = (a.p % a.in == 0) ? 1 : 0;
    P.vec_store = (P.U % 8 == 0 && a.out % 8 == 0 && (reinterpret_cast<uintptr_t>(a.y) % 16) == 0) ? 1 : 0;
    P.reps_all = (a.out % P.U == 0 && a.out / P.U < (1 << 30)) ? static_cast<int32_t>(a.out / P.U) : 0;
    P.tiles_m = static_cast<uint32_t>((a.M + kBM - 1) / kBM);
    P.tiles_n = static_cast<int>((P.U + kBN - 1) / kBN);
    const int64_t blocks = int64_t(P.tiles_m) * P.tiles_n;
    if (blocks > 0x7fffffffLL) {
        set_error("tbn_linear_forward: problem too large for one launch");
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(blocks));
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    tbn_status st;
    if (a.dt == TBN_F32)
        st = relu ? launch_f32<true>(a, P, grid) : launch_f32<false>(a, P, grid);
    else if (blocks >= kTwoResidentMinBlocks && a.in <= kTwoResidentMaxK)
        st = relu ? launch_bf16<32, true>(a, P, grid) : launch_bf16<32, false>(a, P, grid);
    else
        st = relu ? launch_bf16<64, true>(a, P, grid) : launch_bf16<64, false>(a, P, grid);
    if (st != TBN_OK) return st;
    // columns whose weight row straddles a tile end need two alphas
    if (a.n_alpha > 1 && !P.aligned) return launch_linear_tile_ends(a);
    return TBN_OK;
}

}  // namespace tbn
