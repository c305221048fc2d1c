// Streaming matrix-core kernel for the fully-connected tiled-bit layer with bfloat16 activations and a
// tile that holds whole weight rows (p % in == 0): the large-batch path of the headline shapes.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8): with p a multiple of `in` the
// (out x in) weight is the U = p / in rows of the tile stacked k times, copy t scaled by alpha[t].  So
// Z = X * T^T (M x U, T the +-1 rows of the tile) is formed once and Y[:, t*U + u] = alpha[t] * Z[:, u]
// ("only one of the tile computations needs to be executed", Section "CNN Architectures", applied to
// matrix columns).
//
// How the work is laid out on gfx950 (the reasons are measurements of the earlier one-block-per-tile kernel:
// with one 128 x 128 block per CU the index set-up, the pipeline fill, the hand-over of the K halves and
// above all the replicated-column stores -- 8 of 9 bytes the kernel moves are output -- ran one after the
// other, the matrix pipe idle meanwhile):
//   * a workgroup of four waves stays on its CU and works through a sequence of half tiles, 64 rows of X
//     by 128 tile rows each.  Wave (g, h) multiplies the 64 rows with tile rows 64h .. 64h + 63 over the
//     K slices congruent to g (mod 2): 2 x 2 MFMA tiles of 32 x 32 x 16, the +-1 rows as the row operand;
//   * everything a round of 128 K elements needs streams through LDS rings five rounds ahead of its use,
//     across half-tile borders: the activations (global -> LDS directly, 16 bytes per lane, XOR-swizzled
//     so that operand reads are free of bank conflicts) and the chunk of the packed tile that the
//     workgroup's 128 tile rows need for two rounds (coalesced 16-byte pieces; every wave then reads
//     the 64 window bits of its columns with one LDS instruction per round).  Tile bits are never
//     fetched lane by lane from global memory;
//   * a byte of tile bits becomes the +-1 bf16 MFMA operand through a 256-entry table in LDS;
//   * at the end of a half tile the two K groups add their partial sums through LDS, the wave turns its
//     32 x 64 block round (so that eight lanes hold one row's 64 columns: 16-byte stores that cover whole
//     128-byte lines) and keeps it in registers; the alpha-scaled, replicated stores of that block are
//     issued between the MFMAs of the NEXT half tile, one half replica per round.  Only the last half
//     tile's stores are exposed;
//   * workgroup j of XCD x takes half tiles j, j + W, j + 2W .. of that XCD's share of the rows (row-half
//     major, column block fastest), so at any moment the workgroups of an XCD work on the same few row
//     blocks of X and find them in that XCD's L2.
#include "tbn_common.h"

#include <type_traits>

namespace tbn {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

union Frag {
    bf16x8_t v;
    u32x4_t q;
};

constexpr int kThreads = 256;
constexpr int kHT = 64;                  // rows of X per half tile
constexpr int kBN = 128;                 // tile rows (distinct output columns) per workgroup
constexpr int kRoundK = 128;             // K elements per round: 64 for each of the two K groups
constexpr int kNB = 6;                   // ring slots of activations
constexpr int kLA = kNB - 1;             // rounds the loads run ahead
constexpr int kSlotBytes = 2 * kHT * 128;   // [K group][64 rows][128 bytes]
constexpr int kTileSlots = 4;            // ring of tile chunks, one chunk = two rounds
constexpr int kTileSlotBytes = 4096;     // [16-byte piece (= round parity)][128 columns][16 bytes]
constexpr int kBias = 3 * 1024;          // keeps the lane offsets of the wave-loads non-negative

// LDS map.  The sign table sits at address 0 so that a table read needs no base.
constexpr int kTableOff = 0;                               // 256 entries of 16 bytes
constexpr int kRingOff = 4096;
constexpr int kXchgOff = kRingOff + kNB * kSlotBytes;      // 4 x 8 KiB, one slot per wave
constexpr int kTileOff = kXchgOff + 4 * 8192;
constexpr int kLdsBytes = kTileOff + kTileSlots * kTileSlotBytes;
static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 workgroup");

struct StreamParams {
    int64_t M;
    int32_t in, out, U;
    int32_t reps;         // out / U = k replicas of every distinct column
    int32_t n_alpha;
    int32_t rows_half;    // ceil(M / 64)
    int32_t rows_xcd;     // row halves per XCD
    int32_t tiles_n;      // ceil(U / 128)
    int32_t wg_per_xcd;
    int32_t nr;           // rounds per half tile = in / 128 (even)
};

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// All LDS traffic of this kernel is written as inline assembly: the compiler would otherwise make every
// LDS access wait for all global -> LDS loads in flight, and loads are in flight from the first to the
// last round.  The waits are explicit; a register that a read fills is handed to the compiler only
// through tie() after the wait that covers it.
template <int OFF>
__device__ __forceinline__ void lds_read16(u32x4_t &dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// two 8-byte reads 512 bytes apart: registers 0-1 from addr, 2-3 from addr + 512
__device__ __forceinline__ void lds_read2x8(u32x4_t &dst, uint32_t addr) {
    asm volatile("ds_read2_b64 %0, %1 offset0:0 offset1:64" : "=v"(dst) : "v"(addr));
}
template <int OFF>
__device__ __forceinline__ void lds_write16(uint32_t addr, const u32x4_t &v) {
    asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait() {
    asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ void tie(u32x4_t &r) { asm volatile("" : "+v"(r)); }

// wave-load J of a group of four that share an LDS base: the immediate offset is added to the LDS
// address and to the global address alike (the per-lane offset takes it back out, see a_off)
template <int J>
__device__ __forceinline__ void wave_load(const unsigned char *src, uint32_t off, unsigned char *dst) {
    __builtin_amdgcn_global_load_lds(src + off, dst, 16, J * 1024, 0);
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));   // round to nearest even in hardware
}

// RELU: fused max(0, .) of Algorithm 1.  MASKED: the batch is no multiple of 64 or U no multiple of 128, so
// stores are predicated per lane; otherwise the rounds contain no control flow at all.
template <bool RELU, bool MASKED>
__global__ __launch_bounds__(kThreads, 1) void linear_stream_bf16_kernel(const uint16_t *__restrict__ x,
                                                                           uint16_t *__restrict__ y,
                                                                           const uint32_t *__restrict__ tile,
                                                                           const float *__restrict__ alpha,
                                                                           StreamParams P) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 1;   // K group
    const int wn = wave & 1;     // column half
    const int ln = lane & 31;    // operand lane inside a 32 x 32 tile
    const int lg = lane >> 5;    // K half of the operand registers

    // ---- the half tiles of this workgroup -----------------------------------------------------------
    const int32_t xcd = static_cast<int32_t>(blockIdx.x & 7u), wg = static_cast<int32_t>(blockIdx.x >> 3);
    const int32_t r_lo = xcd * P.rows_xcd;
    const int32_t r_hi = r_lo + P.rows_xcd < P.rows_half ? r_lo + P.rows_xcd : P.rows_half;
    const int32_t n_mine = r_hi > r_lo ? (r_hi - r_lo) * P.tiles_n : 0;
    if (wg >= n_mine) return;   // the whole workgroup leaves: no barrier has been executed yet
    const int32_t W = P.wg_per_xcd;
    const int32_t n_ht = (n_mine - wg + W - 1) / W;
    const int32_t step_r = W / P.tiles_n, step_c = W - step_r * P.tiles_n;
    const int32_t NR = P.nr;
    const int32_t first_row = r_lo + wg / P.tiles_n, first_col = wg % P.tiles_n;
    const int32_t rows_last = static_cast<int32_t>(P.M - int64_t(P.rows_half - 1) * kHT);   // 1 .. 64 rows in the last row half

    // ---- per-lane constants of the activation loads -------------------------------------------------
    // Wave-load j of a wave fills 1 KiB of its K group's 8 KiB: piece q = 4*wn + j, row slot sr = 8*q + lane/8,
    // chunk slot lane%8.  Row-slot block sr/32 holds row block (sr/32 + grp) % 2 of the half tile (so that
    // each K group ends with the sums it keeps in its first accumulators), chunk slot s of row slot sr holds
    // 16-byte chunk s ^ ((sr >> 1) & 7) of the round's 128 bytes of that row.  Rows past M repeat row M - 1.
    uint32_t a_off[4], a_off_last[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int sr = 8 * (4 * wn + j) + (lane >> 3);
        const int xr = ((((sr >> 5) + grp) & 1) << 5) + (sr & 31);
        const int chunk = (lane & 7) ^ ((sr >> 1) & 7);
        const int xr_last = xr < rows_last ? xr : rows_last - 1;
        const uint32_t fix = static_cast<uint32_t>(chunk * 16 + kBias - j * 1024);
        a_off[j] = static_cast<uint32_t>(xr) * static_cast<uint32_t>(P.in) * 2u + fix;
        a_off_last[j] = static_cast<uint32_t>(xr_last) * static_cast<uint32_t>(P.in) * 2u + fix;
    }
    const bool ragged = MASKED && rows_last < kHT;

    // ---- per-lane constants of the tile-chunk loads -----------------------------------------------
    // A chunk holds, for the workgroup's 128 tile rows, the 256 bits of two rounds: two 16-byte pieces per
    // row.  Lane i of wave w fills slot S = 64*w + i of the chunk's 256: piece S / 128, LDS row S % 128.
    // LDS row 64*h + 32*tn + l holds the tile row that operand lane l of wave half h supplies for MFMA tile
    // tn, i.e. column 64*h + 16*(l/8) + 8*((l/4)%2) + 4*tn + l%4 of the block (with this numbering a lane
    // ends up with eight adjacent columns of one row of Y).
    const int t_piece = wave >> 1;
    int t_col;
    {
        const int rho = (64 * wave + lane) & 127;
        const int l = rho & 31;
        t_col = (rho & 64) + 16 * (l >> 3) + 8 * ((l >> 2) & 1) + 4 * ((rho >> 5) & 1) + (l & 3);
    }
    const uint32_t row_bytes = static_cast<uint32_t>(P.in) >> 3;   // bytes of one tile row
    auto tile_lane_off = [&](int32_t col_block) -> uint32_t {
        int32_t u = col_block * kBN + t_col;
        u = u < P.U ? u : P.U - 1;   // columns past U repeat the last one; they are never written
        return static_cast<uint32_t>(u) * row_bytes + static_cast<uint32_t>(t_piece * 16);
    };

    // ---- load cursor: runs kLA rounds ahead of the multiplication --------------------------------------
    // Past the workgroup's last half tile it goes over that half tile again: the rounds stay free of
    // conditions (the wait counts are immediates), the extra loads hit the L2 and land in ring slots that
    // nobody reads.
    int32_t ld_row = first_row, ld_col = first_col, ld_h = 0, ld_r = 0, ld_slot = 0, ld_tslot = 0;
    const unsigned char *x_bytes = reinterpret_cast<const unsigned char *>(x);
    const unsigned char *tile_bytes = reinterpret_cast<const unsigned char *>(tile);
    const unsigned char *ld_x = x_bytes + int64_t(ld_row) * kHT * P.in * 2 + (grp * 128 - kBias);
    uint32_t ld_toff = tile_lane_off(ld_col);
    bool ld_last = ragged && ld_row == P.rows_half - 1;
    unsigned char *const ring_wave = lds_raw + kRingOff + grp * 8192 + wn * 4096;
    unsigned char *const tring_wave = lds_raw + kTileOff + wave * 1024;

    auto issue_x = [&](auto j_c) {
        constexpr int J = decltype(j_c)::value;
        const unsigned char *src = ld_x;
        asm volatile("" : "+s"(src));   // one scalar base, the lane offset stays a 32-bit register
        // widened to 64 bits here, not once outside the loops: the wave-load then takes it as a 32-bit
        // offset to the scalar base
        uint32_t off = ld_last ? a_off_last[J] : a_off[J];
        asm volatile("" : "+v"(off));
        wave_load<J>(src, off, ring_wave + ld_slot * kSlotBytes);
    };
    auto issue_tile = [&]() {   // the chunk of the round under the cursor (an even one) and the next
        const unsigned char *src = tile_bytes + ld_r * 16;   // 128 bits per round
        asm volatile("" : "+s"(src));
        uint32_t off = ld_toff;
        asm volatile("" : "+v"(off));
        __builtin_amdgcn_global_load_lds(src + off, tring_wave + ld_tslot * kTileSlotBytes, 16, 0, 0);
        ld_tslot = (ld_tslot + 1) & (kTileSlots - 1);
    };
    auto advance_load = [&]() {
        ld_slot = ld_slot + 1 == kNB ? 0 : ld_slot + 1;
        ++ld_r;
        ld_x += 2 * kRoundK;
        if (ld_r == NR) {   // uniform
            ld_r = 0;
            if (ld_h + 1 < n_ht) {   // next half tile
                ++ld_h;
                ld_col += step_c;
                ld_row += step_r;
                if (ld_col >= P.tiles_n) { ld_col -= P.tiles_n; ++ld_row; }
                ld_toff = tile_lane_off(ld_col);
                ld_last = ragged && ld_row == P.rows_half - 1;
            }
            ld_x = x_bytes + int64_t(ld_row) * kHT * P.in * 2 + (grp * 128 - kBias);
        }
    };

    // alpha of replica t in lane t (at most 64 replicas), fetched by hand so that the compiler does not
    // place a wait for it inside the rounds; it is the oldest load and covered by the first wait below
    float alpha_lanes;
    {
        const int t = P.n_alpha == 1 ? 0 : (lane < P.reps ? lane : P.reps - 1);
        const uint32_t off = static_cast<uint32_t>(t) * 4u;
        asm volatile("global_load_dword %0, %1, %2" : "=v"(alpha_lanes) : "v"(off), "s"(alpha));
    }

    // ---- prologue: loads of the first kLA rounds ---------------------------------------------------
    // issue order per round, which the wait counts below rely on: four activation wave-loads, then (even
    // rounds) the tile chunk of this round and the next
#pragma unroll
    for (int d = 0; d < kLA; ++d) {
        issue_x(std::integral_constant<int, 0>{});
        issue_x(std::integral_constant<int, 1>{});
        issue_x(std::integral_constant<int, 2>{});
        issue_x(std::integral_constant<int, 3>{});
        if ((d & 1) == 0) issue_tile();
        advance_load();
    }

    // sign table: entry e, element i is +1 if bit i of e is set, else -1
    {
        u32x4_t t;
        const int e = tid;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            t[v] = (((e >> (2 * v)) & 1) ? 0x3f80u : 0xbf80u) | ((((e >> (2 * v + 1)) & 1) ? 0x3f80u : 0xbf80u) << 16);
        lds_write16<kTableOff>(static_cast<uint32_t>(e) * 16u, t);
    }

    // operand read addresses inside a ring slot: row slot 32*tm + ln, K step ks: chunk 2*ks + lg at chunk
    // slot (2*ks + lg) ^ ((ln >> 1) & 7)
    uint32_t a_rd[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        a_rd[ks] = static_cast<uint32_t>(kRingOff + grp * 8192 + ln * 128 + (((2 * ks + lg) ^ ((ln >> 1) & 7)) << 4));
    // window read: LDS row 64*wn + ln (tn = 0) and + 32 (tn = 1) of the chunk, the K group's 8 bytes of the piece
    const uint32_t w_rd = static_cast<uint32_t>(kTileOff + (64 * wn + ln) * 16 + 8 * grp);
    // byte 2*ks + lg of a window: word ks / 2, bits 16*(ks % 2) + 8*lg on
    uint32_t bsh[2] = {8u * static_cast<uint32_t>(lg), 16u + 8u * static_cast<uint32_t>(lg)};
    asm volatile("" : "+v"(bsh[0]), "+v"(bsh[1]));

    // exchange / turn-round addresses
    const uint32_t xchg_mine = static_cast<uint32_t>(kXchgOff + wave * 8192);
    const uint32_t xchg_partner = static_cast<uint32_t>(kXchgOff + (wave ^ 2) * 8192);
    const int g8 = lane & 7, rr = lane >> 3;   // store layout: lane holds columns 8*g8 .. + 7 of rows rr + 8*i

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    Frag A[2][2][2];    // [operand set][K step of the pair][tm]
    Frag B[2][2][2];    // [operand set][K step of the pair][tn]
    u32x4_t win[2];     // [round parity]: words 0-1 the 64 window bits of column tn = 0, words 2-3 of tn = 1
    float zr[4][8];     // finished block of the previous half tile in store layout
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) zr[i][e] = 0.f;
    uint32_t z_mask = 0;               // bit i: row rr + 8*i and the lane's columns are inside Y
    unsigned char *z_base = reinterpret_cast<unsigned char *>(y);   // Y address of the block's row 0, column 0 (replica 0)
    uint32_t z_lane = 0;               // byte offset of the lane's first element
    int32_t z_t = P.reps;              // next replica to store; reps = nothing pending
    const uint32_t out_bytes8 = static_cast<uint32_t>(P.out) * 16u;   // eight rows of Y in bytes
    const uint32_t rep_bytes = static_cast<uint32_t>(P.U) * 2u;

    // multiplication cursor
    int32_t cp_row = first_row, cp_col = first_col, cp_slot = 0, cp_tslot = 0;

#ifndef TBN_X_TABLE
#define TBN_X_TABLE 0
#endif
    uint32_t x_zero = 0;
    asm volatile("" : "+v"(x_zero));
    auto table_read = [&](u32x4_t &dst, uint32_t word, uint32_t shift) {
#if TBN_X_TABLE == 1
        const uint32_t addr = (__builtin_amdgcn_ubfe(word, shift, 8) << 4) & x_zero;   // timing only: one entry
#else
        const uint32_t addr = __builtin_amdgcn_ubfe(word, shift, 8) << 4;
#endif
        lds_read16<kTableOff>(dst, addr);
    };
    auto mfma = [&](int set, int ks, int tm, int tn) {
        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(B[set][ks][tn].v, A[set][ks][tm].v, acc[tm][tn], 0, 0, 0);
    };
    auto alpha_of = [&](int32_t t) -> float {
        return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, alpha_lanes), t));
    };
    // rows rr + 8*I of replica z_t of the held block, in three steps that the rounds spread over MFMA slots
    auto job_scale = [&](auto i_c, float al, float (&v)[8]) {
        constexpr int I = decltype(i_c)::value;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[e] = al * zr[I][e];
            if (RELU) v[e] = fmaxf(v[e], 0.f);
        }
    };
    auto job_pack = [&](const float (&v)[8], u32x4_t &pk) {
        pk = u32x4_t{pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
    };
    auto job_store = [&](auto i_c, const u32x4_t &pk) {
        constexpr int I = decltype(i_c)::value;
        unsigned char *dst = z_base + static_cast<uint32_t>(z_t) * rep_bytes;
        asm volatile("" : "+s"(dst));
#ifdef TBN_X_NOSTORE
        if (z_lane == 0xffffffffu)
#endif
        if (!MASKED || (z_mask & (1u << I)))
            *reinterpret_cast<u32x4_t *>(dst + (z_lane + static_cast<uint32_t>(I) * out_bytes8)) = pk;
    };
    auto store_replica = [&]() {   // all four row groups of replica z_t, outside the rounds
        const float al = alpha_of(z_t);
        float v[8];
        u32x4_t pk;
        job_scale(std::integral_constant<int, 0>{}, al, v); job_pack(v, pk); job_store(std::integral_constant<int, 0>{}, pk);
        job_scale(std::integral_constant<int, 1>{}, al, v); job_pack(v, pk); job_store(std::integral_constant<int, 1>{}, pk);
        job_scale(std::integral_constant<int, 2>{}, al, v); job_pack(v, pk); job_store(std::integral_constant<int, 2>{}, pk);
        job_scale(std::integral_constant<int, 3>{}, al, v); job_pack(v, pk); job_store(std::integral_constant<int, 3>{}, pk);
    };

    // ---- first operands -------------------------------------------------------------------------
    // round 0 is readable once its loads (the oldest) have landed and the workgroup has met
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 + 5 + 4 + 5));   // the loads of rounds 1 .. 4 may be in flight
    asm volatile("" : "+v"(alpha_lanes));
    lds_wait<0>();   // the table
    __builtin_amdgcn_s_barrier();
    lds_read2x8(win[0], w_rd);   // windows of round 0: chunk slot 0, piece 0
    lds_wait<0>();
    tie(win[0]);
    {
        const uint32_t ar0 = a_rd[0], ar1 = a_rd[1];   // ring slot 0
        table_read(B[0][0][0].q, win[0][0], bsh[0]);
        lds_read16<0>(A[0][0][0].q, ar0);
        lds_read16<4096>(A[0][0][1].q, ar0);
        table_read(B[0][0][1].q, win[0][2], bsh[0]);
        table_read(B[0][1][0].q, win[0][0], bsh[1]);
        lds_read16<0>(A[0][1][0].q, ar1);
        lds_read16<4096>(A[0][1][1].q, ar1);
        table_read(B[0][1][1].q, win[0][2], bsh[1]);
    }
    // all of operand set 0 has landed (what a loop is entered with, see below)
    auto settle = [&]() {
        lds_wait<0>();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int t = 0; t < 2; ++t) { tie(A[0][ks][t].q); tie(B[0][ks][t].q); }
    };
    settle();

    // ---- one round: 16 MFMAs per wave ---------------------------------------------------------------
    // PAR: parity of the round (inside its half tile and overall: a half tile has an even number of rounds).
    // JOB: the round also stores two of the eight-row groups of a replica of the previous half tile's block.
    // On entry the operands of the round's first two K steps have been requested (operand set 0).  LDS
    // operations complete in order, so "at most N pending" names exactly which operands have arrived: the
    // eight reads of a pair of K steps are issued one after an MFMA each, in the order in which the next
    // pair's MFMAs need them, and an MFMA waits with six (seven while the window read is among the younger
    // ones) operations pending: every operand has the time of six MFMAs to arrive.
#ifdef TBN_X_NOLOAD
#define X_LOAD(x)
#else
#define X_LOAD(x) x
#endif
#ifdef TBN_X_NOREAD
#define X_READ(x)
#else
#define X_READ(x) x
#endif
    auto round = [&](auto par_c, auto job_c) {
        constexpr int PAR = decltype(par_c)::value;
        constexpr bool JOB = decltype(job_c)::value != 0;
        // Loads that may still be in flight when round + 1 must be readable: those of rounds + 2 .. + 4, four
        // wave-loads each and the tile chunk with the even ones.  (Stores of a job are younger operations
        // too; not counting them errs on the safe side.)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(PAR == 0 ? 14 : 13));
#ifndef TBN_X_NOBAR
        __builtin_amdgcn_s_barrier();   // round + 1 is readable, the slot of round - 1 is free
#endif

        const uint32_t cur_off = static_cast<uint32_t>(cp_slot * kSlotBytes);
        cp_slot = cp_slot + 1 == kNB ? 0 : cp_slot + 1;
        const uint32_t nxt_off = static_cast<uint32_t>(cp_slot * kSlotBytes);
        // windows of the next round: an even round reads the second piece of its own chunk, an odd round
        // the first piece of the next chunk
        if constexpr (PAR == 1) cp_tslot = (cp_tslot + 1) & (kTileSlots - 1);
        const uint32_t w_addr = w_rd + static_cast<uint32_t>(cp_tslot * kTileSlotBytes + (PAR == 0 ? 2048 : 0));
        const uint32_t ar2 = a_rd[2] + cur_off, ar3 = a_rd[3] + cur_off;
        const uint32_t ar0 = a_rd[0] + nxt_off, ar1 = a_rd[1] + nxt_off;
        u32x4_t &wc = win[PAR];        // this round's windows
        u32x4_t &wx = win[PAR ^ 1];    // the next round's
        typedef std::integral_constant<int, 2 * PAR> RowA;
        typedef std::integral_constant<int, 2 * PAR + 1> RowB;
        float al = 0.f, v[8];
        u32x4_t pk;
        if constexpr (JOB) al = alpha_of(z_t);

        // ---- K steps 0 and 1 (operand set 0); requests K steps 2 and 3 into set 1
        lds_wait<6>(); tie(B[0][0][0].q); tie(A[0][0][0].q);
        mfma(0, 0, 0, 0);
        X_READ(table_read(B[1][0][0].q, wc[1], bsh[0]);)
        X_READ(lds_read2x8(wx, w_addr);)
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<7>(); tie(A[0][0][1].q);
        mfma(0, 0, 1, 0);
        X_READ(lds_read16<0>(A[1][0][0].q, ar2);)
        if constexpr (JOB) job_scale(RowA{}, al, v);
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<7>(); tie(B[0][0][1].q);
        mfma(0, 0, 0, 1);
        X_READ(lds_read16<4096>(A[1][0][1].q, ar2);)
        if constexpr (JOB) job_pack(v, pk);
        __builtin_amdgcn_sched_barrier(0);
        mfma(0, 0, 1, 1);
        X_READ(table_read(B[1][0][1].q, wc[3], bsh[0]);)
        X_LOAD(issue_x(std::integral_constant<int, 0>{}));
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<7>(); tie(B[0][1][0].q); tie(A[0][1][0].q);
        mfma(0, 1, 0, 0);
        X_READ(table_read(B[1][1][0].q, wc[1], bsh[1]);)
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<7>(); tie(A[0][1][1].q);
        mfma(0, 1, 1, 0);
        X_READ(lds_read16<0>(A[1][1][0].q, ar3);)
        if constexpr (JOB) job_store(RowA{}, pk);
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<7>(); tie(B[0][1][1].q);
        mfma(0, 1, 0, 1);
        X_READ(lds_read16<4096>(A[1][1][1].q, ar3);)
        __builtin_amdgcn_sched_barrier(0);
        mfma(0, 1, 1, 1);
        X_READ(table_read(B[1][1][1].q, wc[3], bsh[1]);)
        X_LOAD(issue_x(std::integral_constant<int, 1>{}));
        __builtin_amdgcn_sched_barrier(0);

        // ---- K steps 2 and 3 (operand set 1); requests the next round's K steps 0 and 1 into set 0
        lds_wait<6>(); tie(B[1][0][0].q); tie(A[1][0][0].q); tie(wx);
        mfma(1, 0, 0, 0);
        X_READ(table_read(B[0][0][0].q, wx[0], bsh[0]);)
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<6>(); tie(A[1][0][1].q);
        mfma(1, 0, 1, 0);
        X_READ(lds_read16<0>(A[0][0][0].q, ar0);)
        if constexpr (JOB) job_scale(RowB{}, al, v);
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<6>(); tie(B[1][0][1].q);
        mfma(1, 0, 0, 1);
        X_READ(lds_read16<4096>(A[0][0][1].q, ar0);)
        if constexpr (JOB) job_pack(v, pk);
        __builtin_amdgcn_sched_barrier(0);
        mfma(1, 0, 1, 1);
        X_READ(table_read(B[0][0][1].q, wx[2], bsh[0]);)
        X_LOAD(issue_x(std::integral_constant<int, 2>{}));
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<6>(); tie(B[1][1][0].q); tie(A[1][1][0].q);
        mfma(1, 1, 0, 0);
        X_READ(table_read(B[0][1][0].q, wx[0], bsh[1]);)
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<6>(); tie(A[1][1][1].q);
        mfma(1, 1, 1, 0);
        X_READ(lds_read16<0>(A[0][1][0].q, ar1);)
        if constexpr (JOB) job_store(RowB{}, pk);
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<6>(); tie(B[1][1][1].q);
        mfma(1, 1, 0, 1);
        X_READ(lds_read16<4096>(A[0][1][1].q, ar1);)
        __builtin_amdgcn_sched_barrier(0);
        mfma(1, 1, 1, 1);
        X_READ(table_read(B[0][1][1].q, wx[2], bsh[1]);)
        X_LOAD(issue_x(std::integral_constant<int, 3>{}));
        if constexpr (PAR == 1) X_LOAD(issue_tile());
        advance_load();
        if constexpr (JOB && PAR == 1) ++z_t;
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- the half tiles -------------------------------------------------------------------------
    // Two plain loops per half tile: rounds that carry stores of the previous block, then rounds that do
    // not.  Operands requested by a loop's last round are allowed to land before the loop is left
    // (settle), so that a register with a read in flight only ever crosses a loop's own back edge.
    for (int32_t h = 0; h < n_ht; ++h) {
        int32_t pr = 0;
        const int32_t n_pr = NR >> 1;
        if (z_t < P.reps) {
            do {
                round(std::integral_constant<int, 0>{}, std::true_type{});
                round(std::integral_constant<int, 1>{}, std::true_type{});
                ++pr;
            } while (pr < n_pr && z_t < P.reps);
            settle();
        }
        if (pr < n_pr) {
            do {
                round(std::integral_constant<int, 0>{}, std::false_type{});
                round(std::integral_constant<int, 1>{}, std::false_type{});
                ++pr;
            } while (pr < n_pr);
            settle();
        }

        // ---- end of the half tile ---------------------------------------------------------------
        // replicas of the previous block that found no round (short K, many replicas)
        for (; z_t < P.reps; ++z_t) store_replica();

        // The K groups add their partial sums: accumulator index tm of group g stands for row block
        // (tm + g) % 2, so each group keeps acc[0] and hands acc[1] to the other one.  The matrix pipe
        // must have written the accumulators back before the assembly below reads them.
        asm volatile("s_nop 15");
        asm volatile("s_nop 15");
        {
            u32x4_t s[8];
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s[tn * 4 + q][e] = __float_as_uint(acc[1][tn][4 * q + e]);
            const uint32_t dst = xchg_partner + static_cast<uint32_t>(lane) * 16u;
            lds_write16<0 * 1024>(dst, s[0]);
            lds_write16<1 * 1024>(dst, s[1]);
            lds_write16<2 * 1024>(dst, s[2]);
            lds_write16<3 * 1024>(dst, s[3]);
            lds_write16<4 * 1024>(dst, s[4]);
            lds_write16<5 * 1024>(dst, s[5]);
            lds_write16<6 * 1024>(dst, s[6]);
            lds_write16<7 * 1024>(dst, s[7]);
        }
        lds_wait<0>();
        __builtin_amdgcn_s_barrier();
        {
            u32x4_t got[8];
            const uint32_t src = xchg_mine + static_cast<uint32_t>(lane) * 16u;
            lds_read16<0 * 1024>(got[0], src);
            lds_read16<1 * 1024>(got[1], src);
            lds_read16<2 * 1024>(got[2], src);
            lds_read16<3 * 1024>(got[3], src);
            lds_read16<4 * 1024>(got[4], src);
            lds_read16<5 * 1024>(got[5], src);
            lds_read16<6 * 1024>(got[6], src);
            lds_read16<7 * 1024>(got[7], src);
            lds_wait<0>();
#pragma unroll
            for (int i = 0; i < 8; ++i) tie(got[i]);
#pragma unroll
            for (int tn = 0; tn < 2; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[0][tn][4 * q + e] += __uint_as_float(got[tn * 4 + q][e]);
        }
        // Turn the finished 32 x 64 block round inside the wave's own slot (the partner wrote it before the
        // barrier and will not write to it again before the next half tile's hand-over).  On entry the lane
        // holds row ln and, in registers 4q .. 4q + 3 of tiles 0 and 1, columns 16*q + 8*lg .. + 7.  LDS
        // row r is 256 bytes; the 16-byte chunk ch of it (columns 4*ch .. 4*ch + 3) sits at chunk position
        // ch ^ s(r), s(r) = ((r >> 1) & 7) ^ (2 * (r & 1)): the writes (lanes = rows) and the reads (eight
        // lanes per row; a lane reads chunks 2*g8 and 2*g8 + 1, the upper four lanes in the other order)
        // are then free of bank conflicts.
        {
            const int s_w = ((ln >> 1) & 7) ^ (2 * (ln & 1));
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn) {
                    const int ch = 4 * q + 2 * lg + tn;
                    u32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[0][tn][4 * q + e]);
                    lds_write16<0>(xchg_mine + static_cast<uint32_t>(ln * 256 + ((ch ^ s_w) << 4)), v);
                }
            lds_wait<0>();
            __builtin_amdgcn_wave_barrier();
            const int ch_a = 2 * g8 + (g8 >> 2), ch_b = 2 * g8 + 1 - (g8 >> 2);
            u32x4_t za[4], zb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = rr + 8 * i;
                const int s_r = ((r >> 1) & 7) ^ (2 * (r & 1));
                lds_read16<0>(za[i], xchg_mine + static_cast<uint32_t>(r * 256 + ((ch_a ^ s_r) << 4)));
                lds_read16<0>(zb[i], xchg_mine + static_cast<uint32_t>(r * 256 + ((ch_b ^ s_r) << 4)));
            }
            lds_wait<0>();
#pragma unroll
            for (int i = 0; i < 4; ++i) { tie(za[i]); tie(zb[i]); }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    zr[i][e] = __uint_as_float(g8 < 4 ? za[i][e] : zb[i][e]);
                    zr[i][4 + e] = __uint_as_float(g8 < 4 ? zb[i][e] : za[i][e]);
                }
        }
        // where the block goes: rows cp_row*64 + 32*grp + rr + 8*i, columns cp_col*128 + 64*wn + 8*g8 .. + 7
        {
            const int64_t row0 = int64_t(cp_row) * kHT + 32 * grp;
            const int32_t col0 = cp_col * kBN + 64 * wn;
            z_base = reinterpret_cast<unsigned char *>(y) + (row0 * P.out + col0) * 2;
            z_lane = (static_cast<uint32_t>(rr) * static_cast<uint32_t>(P.out) + static_cast<uint32_t>(8 * g8)) * 2u;
            if (MASKED) {
                const int64_t rows_left = P.M - row0;   // may be <= 0 in the last row half
                const bool col_ok = col0 + 8 * g8 < P.U;
                z_mask = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (col_ok && rr + 8 * i < rows_left) z_mask |= 1u << i;
            }
            z_t = 0;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        cp_col += step_c;
        cp_row += step_r;
        if (cp_col >= P.tiles_n) { cp_col -= P.tiles_n; ++cp_row; }
    }

    // ---- the last block's replicas; the loads issued past the end have landed by then -------------------
    for (; z_t < P.reps; ++z_t) store_replica();
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
}

tbn_status set_lds_limit_once(const void *kernel, int lds) {
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) {
        set_error("tbn_linear_forward: cannot reserve %d bytes of LDS: %s", lds, hipGetErrorString(e));
        return TBN_ERR_DEVICE;
    }
    return TBN_OK;
}

}  // namespace

// Shapes the streaming kernel takes: bfloat16, tile of whole rows, K in whole pairs of rounds, 16-byte
// stores possible, every offset inside a half tile in 32 bits.
bool linear_stream_supported(const LinearArgs &a) {
    if (a.dt != TBN_BF16) return false;
    if (a.in % 256 != 0 || a.p % a.in != 0) return false;
    const int64_t U = a.p / a.in;
    if (U > a.out || a.out % U != 0) return false;   // (holds whenever p % in == 0; U = out / k)
    if (U % 8 != 0 || a.out / U > 64) return false;
    if (a.in > (1 << 20) || a.out > (1 << 22) || a.p >= (int64_t(1) << 31)) return false;
    if (a.M < 1 || a.M > (int64_t(1) << 36)) return false;
    if ((reinterpret_cast<uintptr_t>(a.x) & 15u) || (reinterpret_cast<uintptr_t>(a.y) & 15u)) return false;
    if (reinterpret_cast<uintptr_t>(a.tile) & 15u) return false;
    return true;
}

tbn_status launch_linear_stream(const LinearArgs &a) {
    StreamParams P;
    P.M = a.M;
    P.in = static_cast<int32_t>(a.in);
    P.out = static_cast<int32_t>(a.out);
    P.U = static_cast<int32_t>(a.p / a.in);
    P.reps = static_cast<int32_t>(a.out / P.U);
    P.n_alpha = a.n_alpha;
    const int64_t rows_half = (a.M + kHT - 1) / kHT;
    if (rows_half > 0x3fffffff) {
        set_error("tbn_linear_forward: batch too large for one launch");
        return TBN_ERR_UNSUPPORTED;
    }
    P.rows_half = static_cast<int32_t>(rows_half);
    P.rows_xcd = (P.rows_half + 7) / 8;
    P.tiles_n = (P.U + kBN - 1) / kBN;
    P.nr = P.in / kRoundK;
    // one workgroup per CU (the LDS footprint allows no second one): 32 per XCD on the 256 CUs of an
    // MI355X, fewer when an XCD's share of the half tiles is smaller
    int device = 0, cus = 256;
    if (hipGetDevice(&device) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && v >= 8) cus = v;
    }
    const int64_t per_xcd = int64_t(P.rows_xcd) * P.tiles_n;
    P.wg_per_xcd = static_cast<int32_t>(per_xcd < cus / 8 ? per_xcd : cus / 8);
    const dim3 grid(static_cast<unsigned>(8 * P.wg_per_xcd));
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    const bool masked = a.M % kHT != 0 || P.U % kBN != 0;
    typedef void (*kernel_t)(const uint16_t *, uint16_t *, const uint32_t *, const float *, StreamParams);
    static const kernel_t kernels[4] = {&linear_stream_bf16_kernel<false, false>, &linear_stream_bf16_kernel<false, true>,
                                        &linear_stream_bf16_kernel<true, false>, &linear_stream_bf16_kernel<true, true>};
    // dynamic LDS above the default limit has to be allowed once per kernel (thread-safe static initialisation)
    static const tbn_status attr[4] = {set_lds_limit_once(reinterpret_cast<const void *>(kernels[0]), kLdsBytes),
                                       set_lds_limit_once(reinterpret_cast<const void *>(kernels[1]), kLdsBytes),
                                       set_lds_limit_once(reinterpret_cast<const void *>(kernels[2]), kLdsBytes),
                                       set_lds_limit_once(reinterpret_cast<const void *>(kernels[3]), kLdsBytes)};
    const int which = (relu ? 2 : 0) + (masked ? 1 : 0);
    if (attr[which] != TBN_OK) {
        set_error("tbn_linear_forward: cannot reserve %d bytes of LDS for the streaming kernel", kLdsBytes);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL(kernels[which], grid, dim3(kThreads), kLdsBytes, a.stream, static_cast<const uint16_t *>(a.x),
                       static_cast<uint16_t *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward (streaming matrix-core kernel)");
}

}  // namespace tbn
