// Streaming matrix-core kernel for the fully-connected tiled-bit layer with bfloat16 activations and a
// tile that holds whole weight rows (p % in == 0): the large-batch path of the headline shapes.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8): with p a multiple of `in` the
// (out x in) weight is the U = p / in rows of the tile stacked k times, copy t scaled by alpha[t].  So
// Z = X * T^T (M x U, T the +-1 rows of the tile) is formed once and Y[:, t*U + u] = alpha[t] * Z[:, u]
// ("only one of the tile computations needs to be executed", Section "CNN Architectures", applied to
// matrix columns).
//
// How the work is laid out on gfx950.  Measurements of the one-block-per-tile kernel and of a first
// streaming form shaped this: with one 128 x 128 block per CU the index set-up, the pipeline fill, the
// hand-over of the K halves and above all the replicated-column stores (8 of 9 bytes the kernel moves are
// output) ran one after the other with the matrix pipe idle; and a round's cost is set by the instructions
// a wave has to issue beside its MFMAs (LDS reads, wave-loads, the workgroup barrier), not by bank
// conflicts or memory latency.
//   * A workgroup of four waves stays on its CU and works through a sequence of half tiles, 64 rows of X
//     by 128 tile rows each.  The four waves split K in quarters: wave w multiplies all 64 rows with all
//     128 tile rows over K elements w*in/4 .. (w+1)*in/4 - 1 (2 x 4 MFMA tiles of 32 x 32 x 16, the +-1 rows
//     as the row operand: 0.75 LDS operand reads per MFMA).  Nothing a wave reads in the main loop was
//     loaded by another wave, so the loop has no barrier: a wave waits for its own loads only, and the
//     waves drift apart instead of sending their loads to the CU's load path at the same moment.
//   * Everything a round of 32 K elements needs streams through per-wave LDS rings five rounds ahead of
//     its use, across half-tile borders: the activations (global -> LDS directly, 16 bytes per lane,
//     swizzled so that operand reads are free of bank conflicts) and, every fourth round, the 128 bits
//     of each of the 128 tile rows for the next four rounds (coalesced 16-byte pieces; the wave then
//     takes the window words of its columns with four LDS reads per four rounds).  Tile bits are never
//     fetched lane by lane from global memory.
//   * A byte of tile bits becomes the +-1 bf16 MFMA operand through a 256-entry table in LDS.
//   * At the end of a half tile the four waves add their partial sums through LDS (wave w ends with the
//     32 x 64 block of row half w / 2, column half w % 2), turn that block round (eight lanes then hold
//     one row's 64 columns: 16-byte stores that cover whole 128-byte lines) and keep it in registers; its
//     alpha-scaled, replicated stores are issued between the MFMAs of the NEXT half tile, two per round.
//     Only the last half tile's stores are exposed.  The waits for the wave's loads count those stores
//     (the counter is shared and retires in order), so a round never waits for a store to complete.
//   * Workgroup j of XCD x takes half tiles j, j + W, j + 2W .. of that XCD's share of the rows (row-half
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
constexpr int kRoundK = 32;              // K elements per wave and round
constexpr int kNB = 6;                   // ring slots of activations per wave
constexpr int kLA = kNB - 1;             // rounds the loads run ahead
constexpr int kSlotBytes = kHT * kRoundK * 2;   // 64 rows of 64 bytes
constexpr int kTileSlotBytes = 2048;     // 128 tile rows x 16 bytes: the bits of four rounds
constexpr int kBias = 3 * 1024;          // keeps the lane offsets of the wave-loads non-negative

// LDS map.  The sign table sits at address 0 so that a table read needs no base.
constexpr int kTableOff = 0;                               // 256 entries of 16 bytes
constexpr int kRingOff = 4096;                             // per wave kNB slots
constexpr int kXchgOff = kRingOff + 4 * kNB * kSlotBytes;  // 4 x 8 KiB, one slot per wave
constexpr int kTileOff = kXchgOff + 4 * 8192;              // per wave two chunks
constexpr int kLdsBytes = kTileOff + 4 * 2 * kTileSlotBytes;
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
    int32_t n_sr;         // groups of four rounds per wave and half tile = in / 512
};

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// With 64-byte rows two row slots share the 32 banks.  The LDS serves the even and the odd lanes of 16 in
// turn, so rows 2i and 2i + 2 must not sit in the same half: row slots trade their two lowest row bits.
__device__ __host__ constexpr int row_slot(int r) { return (r & ~3) | ((r & 1) << 1) | ((r >> 1) & 1); }

// All LDS traffic of this kernel is written as inline assembly: the compiler would otherwise make every
// LDS access wait for all global -> LDS loads in flight, and loads are in flight from the first to the
// last round.  The waits are explicit; a register that a read fills is handed to the compiler only
// through tie() after the wait that covers it (paper_2407_12075_amd/asm_check.py verifies on the generated
// assembly that nothing touches such a register earlier).
template <int OFF>
__device__ __forceinline__ void lds_read16(u32x4_t &dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
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

template <int V> using Int = std::integral_constant<int, V>;

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
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // K quarter
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
    const int32_t n_sr = P.n_sr;
    const int32_t NR = 4 * n_sr;   // rounds per half tile
    const int32_t first_row = r_lo + wg / P.tiles_n, first_col = wg % P.tiles_n;
    const int32_t rows_last = static_cast<int32_t>(P.M - int64_t(P.rows_half - 1) * kHT);   // 1 .. 64 rows in the last row half
    const bool ragged = MASKED && rows_last < kHT;

    // Which sums a wave keeps at the end: the 32 x 64 block of row half wave / 2, column half wave % 2.  Its
    // accumulator indices are rotated accordingly (index tm stands for row block tm ^ (wave / 2), index tn for
    // column block tn ^ 2 * (wave % 2)), so that every wave keeps acc[0][0..1] and hands the others over with
    // static register indices.
    const int rot_m = wave >> 1, rot_n = wave & 1;

    // ---- per-lane constants of the activation loads -------------------------------------------------
    // Wave-load j fills 1 KiB of the round's 4 KiB slot: row slots 16*j + lane/4, chunk slot lane%4.  Row
    // slot sr holds row 32*((sr / 32) ^ rot_m) + row_slot(sr % 32) of the half tile, chunk slot s of it
    // 16-byte chunk s ^ ((sr >> 2) & 3) of the round's 64 bytes of that row.  Rows past M repeat row M - 1.
    uint32_t a_off[4], a_off_last[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int sr = 16 * j + (lane >> 2);
        const int xr = (((sr >> 5) ^ rot_m) << 5) + row_slot(sr & 31);
        const int chunk = (lane & 3) ^ ((sr >> 2) & 3);
        const int xr_last = xr < rows_last ? xr : rows_last - 1;
        const uint32_t fix = static_cast<uint32_t>(chunk * 16 + kBias - j * 1024);
        a_off[j] = static_cast<uint32_t>(xr) * static_cast<uint32_t>(P.in) * 2u + fix;
        a_off_last[j] = static_cast<uint32_t>(xr_last) * static_cast<uint32_t>(P.in) * 2u + fix;
    }
    const uint32_t quarter_bytes = static_cast<uint32_t>(P.in) >> 1;   // in / 4 elements of 2 bytes

    // ---- per-lane constants of the tile-chunk loads -----------------------------------------------
    // A chunk holds the wave's next 128 bits of each of the workgroup's 128 tile rows, 16 bytes per row: two
    // wave-loads.  LDS row 32*tn + l of the chunk holds the tile row that operand lane l supplies for MFMA
    // tile tn, i.e. column 64*((tn / 2) ^ rot_n) + 16*(l/8) + 8*((l/4)%2) + 4*(tn % 2) + l%4 of the block (with
    // this numbering a lane ends up with eight adjacent columns of one row of Y).
    int t_col[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int rho = 64 * j + lane, tn = rho >> 5, l = rho & 31;
        t_col[j] = 64 * ((tn >> 1) ^ rot_n) + 16 * (l >> 3) + 8 * ((l >> 2) & 1) + 4 * (tn & 1) + (l & 3);
    }
    const uint32_t row_bytes = static_cast<uint32_t>(P.in) >> 3;   // bytes of one tile row
    auto tile_lane_off = [&](int32_t col_block, int j) -> uint32_t {
        int32_t u = col_block * kBN + t_col[j];
        u = u < P.U ? u : P.U - 1;   // columns past U repeat the last one; they are never written
        return static_cast<uint32_t>(u) * row_bytes + static_cast<uint32_t>(wave) * (row_bytes >> 2);
    };

    // ---- load cursors ---------------------------------------------------------------------------
    // The activation cursor runs kLA rounds ahead of the multiplication, the tile cursor two groups of four
    // rounds.  Past the workgroup's last half tile they go over that half tile again: the rounds stay free
    // of conditions (the wait counts are immediates), the extra loads hit the L2 and land where nobody reads.
    const unsigned char *x_bytes = reinterpret_cast<const unsigned char *>(x);
    const unsigned char *tile_bytes = reinterpret_cast<const unsigned char *>(tile);
    unsigned char *const ring_wave = lds_raw + kRingOff + wave * (kNB * kSlotBytes);
    unsigned char *const tring_wave = lds_raw + kTileOff + wave * (2 * kTileSlotBytes);
    auto x_base_of = [&](int32_t row) -> const unsigned char * {
        return x_bytes + int64_t(row) * kHT * P.in * 2 + (static_cast<int64_t>(wave) * quarter_bytes - kBias);
    };
    int32_t ld_row = first_row, ld_col = first_col, ld_h = 0, ld_r = 0, ld_off = 0;   // ld_off: ring slot in bytes
    const unsigned char *ld_x = x_base_of(ld_row);
    bool ld_last = ragged && ld_row == P.rows_half - 1;
    int32_t tl_col = first_col, tl_h = 0, tl_s = 0, tl_slot = 0;
    uint32_t tl_off[2] = {tile_lane_off(tl_col, 0), tile_lane_off(tl_col, 1)};

    // src: the round's scalar base (made opaque once per round, see round()); the lane offset is widened to
    // 64 bits here, not once outside the loops, so that the wave-load takes it as a 32-bit offset to that base
    auto issue_x = [&](auto j_c, const unsigned char *src) {
        constexpr int J = decltype(j_c)::value;
        uint32_t off = ld_last ? a_off_last[J] : a_off[J];
        asm volatile("" : "+v"(off));
        wave_load<J>(src, off, ring_wave + ld_off);
    };
    // after the four loads of a round; CHECK: the cursor may have reached the end of its half tile
    auto advance_x = [&](auto check_c) {
        ld_off = ld_off + kSlotBytes == kNB * kSlotBytes ? 0 : ld_off + kSlotBytes;
        ++ld_r;
        ld_x += 2 * kRoundK;
        if constexpr (decltype(check_c)::value != 0) {
            if (ld_r == NR) {   // uniform
                ld_r = 0;
                if (ld_h + 1 < n_ht) {   // next half tile
                    ++ld_h;
                    ld_col += step_c;
                    ld_row += step_r;
                    if (ld_col >= P.tiles_n) { ld_col -= P.tiles_n; ++ld_row; }
                    ld_last = ragged && ld_row == P.rows_half - 1;
                }
                ld_x = x_base_of(ld_row);
            }
        }
    };
    auto issue_tile = [&](auto j_c) {
        constexpr int J = decltype(j_c)::value;
        const unsigned char *src = tile_bytes + tl_s * 16;   // 128 bits per group of four rounds
        asm volatile("" : "+s"(src));
        uint32_t off = tl_off[J];
        asm volatile("" : "+v"(off));
        __builtin_amdgcn_global_load_lds(src + off, tring_wave + tl_slot * kTileSlotBytes + J * 1024, 16, 0, 0);
    };
    auto advance_tile = [&]() {
        tl_slot ^= 1;
        ++tl_s;
        if (tl_s == n_sr) {   // uniform
            tl_s = 0;
            if (tl_h + 1 < n_ht) {
                ++tl_h;
                tl_col += step_c;
                if (tl_col >= P.tiles_n) tl_col -= P.tiles_n;
                tl_off[0] = tile_lane_off(tl_col, 0);
                tl_off[1] = tile_lane_off(tl_col, 1);
            }
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

    // ---- prologue: tile chunks 0 and 1, activations of rounds 0 .. 4 -----------------------------------
    // in the order the steady state would have issued them (the wait counts rely on it): chunk 0, rounds 0,
    // 1, 2, chunk 1, rounds 3, 4
    issue_tile(Int<0>{}); issue_tile(Int<1>{}); advance_tile();
#pragma unroll
    for (int d = 0; d < kLA; ++d) {
        if (d == 3) { issue_tile(Int<0>{}); issue_tile(Int<1>{}); advance_tile(); }
        issue_x(Int<0>{}, ld_x); issue_x(Int<1>{}, ld_x); issue_x(Int<2>{}, ld_x); issue_x(Int<3>{}, ld_x);
        advance_x(Int<1>{});
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

    // operand read addresses inside a ring slot: row slot 32*tm + row_slot(ln), K step ks: chunk 2*ks + lg at
    // chunk slot (2*ks + lg) ^ ((ln >> 2) & 3)
    uint32_t a_rd[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
        a_rd[ks] = static_cast<uint32_t>(kRingOff + wave * (kNB * kSlotBytes) + row_slot(ln) * 64 + (((2 * ks + lg) ^ ((ln >> 2) & 3)) << 4));
    // window read: LDS row 32*tn + ln of a chunk
    const uint32_t w_rd = static_cast<uint32_t>(kTileOff + wave * (2 * kTileSlotBytes) + ln * 16);
    // byte 2*ks + lg of a window word: bits 16*ks + 8*lg on
    uint32_t bsh[2] = {8u * static_cast<uint32_t>(lg), 16u + 8u * static_cast<uint32_t>(lg)};
    asm volatile("" : "+v"(bsh[0]), "+v"(bsh[1]));

    // exchange / turn-round addresses
    const uint32_t xchg_mine = static_cast<uint32_t>(kXchgOff + wave * 8192);
    const int g8 = lane & 7, rr = lane >> 3;   // store layout: lane holds columns 8*g8 .. + 7 of rows rr + 8*i

    f32x16_t acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    Frag A[2][2];       // [operand set][tm]
    Frag B[2][4];       // [operand set][tn]
    u32x4_t wcur[4];    // [tn]: the 128 window bits of the column for the current four rounds (word = round % 4)
    u32x4_t wnxt[4];    // the same for the next four rounds
    float zr[4][8];     // finished block of the previous half tile in store layout
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) zr[i][e] = 0.f;
    uint32_t z_mask = 0;               // bit i: row rr + 8*i and the lane's columns are inside Y
    unsigned char *z_base = reinterpret_cast<unsigned char *>(y);   // Y address of the block's row 0, column 0 (replica 0)
    uint32_t z_lane = 0;               // byte offset of the lane's first element
    int32_t z_t = P.reps;              // next replica to store; reps = nothing pending
    unsigned char *z_rep = z_base;     // Y address of that replica's row 0, column 0
    const uint32_t out_bytes8 = static_cast<uint32_t>(P.out) * 16u;   // eight rows of Y in bytes
    const uint32_t rep_bytes = static_cast<uint32_t>(P.U) * 2u;

    // multiplication cursor
    int32_t cp_row = first_row, cp_col = first_col, cp_off = 0, cp_tslot = 0;   // cp_off: ring slot in bytes

    auto table_read = [&](u32x4_t &dst, uint32_t word, uint32_t shift) {
        const uint32_t addr = __builtin_amdgcn_ubfe(word, shift, 8) << 4;
        lds_read16<kTableOff>(dst, addr);
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
        typedef __attribute__((address_space(1))) u32x4_t global_u32x4_t;
        unsigned char *dst = z_rep;
        asm volatile("" : "+s"(dst));
        uint32_t off = z_lane + static_cast<uint32_t>(I) * out_bytes8;
        asm volatile("" : "+v"(off));   // scalar base + 32-bit lane offset
        // non-temporal: the output must not push the activations, which the other column blocks of the same
        // rows still need, out of the XCD's L2 (8192 x 4096 -> 16384, k = 8: 174 us against 209 with plain stores)
        if (!MASKED || (z_mask & (1u << I))) __builtin_nontemporal_store(pk, (global_u32x4_t *)(dst + off));
    };
    auto store_replica = [&]() {   // all four row groups of replica z_t, outside the rounds
        const float al = alpha_of(z_t);
        float v[8];
        u32x4_t pk;
        job_scale(Int<0>{}, al, v); job_pack(v, pk); job_store(Int<0>{}, pk);
        job_scale(Int<1>{}, al, v); job_pack(v, pk); job_store(Int<1>{}, pk);
        job_scale(Int<2>{}, al, v); job_pack(v, pk); job_store(Int<2>{}, pk);
        job_scale(Int<3>{}, al, v); job_pack(v, pk); job_store(Int<3>{}, pk);
    };

    // ---- first operands -------------------------------------------------------------------------
    // chunk 0 and round 0 are readable once their loads (the oldest) have landed
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 + 4 + 2 + 4 + 4));   // rounds 1, 2, chunk 1, rounds 3, 4 may be in flight
    asm volatile("" : "+v"(alpha_lanes));
    lds_wait<0>();
    __builtin_amdgcn_s_barrier();   // the table, written by all waves
    lds_read16<0 * 512>(wcur[0], w_rd);
    lds_read16<1 * 512>(wcur[1], w_rd);
    lds_read16<2 * 512>(wcur[2], w_rd);
    lds_read16<3 * 512>(wcur[3], w_rd);
    lds_wait<0>();
    tie(wcur[0]); tie(wcur[1]); tie(wcur[2]); tie(wcur[3]);
    table_read(B[0][0].q, wcur[0][0], bsh[0]);
    lds_read16<0>(A[0][0].q, a_rd[0]);
    lds_read16<2048>(A[0][1].q, a_rd[0]);
    table_read(B[0][1].q, wcur[1][0], bsh[0]);
    table_read(B[0][2].q, wcur[2][0], bsh[0]);
    table_read(B[0][3].q, wcur[3][0], bsh[0]);
    // all of operand set 0 has landed (what a loop is entered with, see below)
    auto settle = [&]() {
        lds_wait<0>();
        tie(A[0][0].q); tie(A[0][1].q);
        tie(B[0][0].q); tie(B[0][1].q); tie(B[0][2].q); tie(B[0][3].q);
    };
    settle();

    // ---- one K step: 8 MFMAs ---------------------------------------------------------------------
    // Multiplies with operand set S and requests the operands of the following K step into the other set: six
    // LDS reads, one in each of the first six MFMA slots, in the order in which the MFMAs of that step need
    // them (+-1 operand of tn = 0, the two activation fragments, +-1 operands of tn = 1, 2, 3).  LDS operations
    // complete in order, so "at most N pending" names exactly which operands have arrived; three waits cover
    // the step, and every operand has the time of at least six MFMAs to arrive.  A slot is: wait, request,
    // MFMA, side work (an instruction between the wait that hands registers over and the MFMA that reads
    // them also saves the compiler a hazard no-op).  W4 = 4: four window reads were issued behind the
    // previous step's requests.  nw: the window words (one per tn) and NKS the K step inside its round of the
    // step requested here.
    auto kstep = [&](auto s_c, auto w4_c, uint32_t n_addr, uint32_t (&nw)[4], auto nks_c, auto &&side) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value, N = S ^ 1, W4 = decltype(w4_c)::value, NKS = decltype(nks_c)::value;
        auto mfma = [&](int tm, int tn) {
            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(B[S][tn].v, A[S][tm].v, acc[tm][tn], 0, 0, 0);
        };
        lds_wait<3 + W4>(); tie(B[S][0].q); tie(A[S][0].q); tie(A[S][1].q);
        side(Int<-1>{});   // what else this wait covers
        table_read(B[N][0].q, nw[0], bsh[NKS]);
        mfma(0, 0);
        side(Int<0>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_read16<0>(A[N][0].q, n_addr);
        mfma(1, 0);
        side(Int<1>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<4 + W4>(); tie(B[S][1].q);
        lds_read16<2048>(A[N][1].q, n_addr);
        mfma(0, 1);
        side(Int<2>{});
        __builtin_amdgcn_sched_barrier(0);
        table_read(B[N][1].q, nw[1], bsh[NKS]);
        mfma(1, 1);
        side(Int<3>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<4 + W4>(); tie(B[S][2].q); tie(B[S][3].q);
        table_read(B[N][2].q, nw[2], bsh[NKS]);
        mfma(0, 2);
        side(Int<4>{});
        __builtin_amdgcn_sched_barrier(0);
        table_read(B[N][3].q, nw[3], bsh[NKS]);
        mfma(1, 2);
        side(Int<5>{});
        __builtin_amdgcn_sched_barrier(0);
        mfma(0, 3);
        side(Int<6>{});
        __builtin_amdgcn_sched_barrier(0);
        mfma(1, 3);
        side(Int<7>{});
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- one round: two K steps, 16 MFMAs --------------------------------------------------------------
    // Q: the round's place in its group of four (window word Q).  JOB: the round stores two eight-row groups
    // of a replica of the previous half tile's block (K step 0).  STORES: how many stores this and the three
    // rounds before have issued.  K step 1 issues the loads of round + 5 (and, for Q = 2, the tile chunk of
    // the group after the next and the reads of the next group's windows).
    auto round = [&](auto q_c, auto job_c, auto stores_c) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value;
        constexpr bool JOB = decltype(job_c)::value != 0;
        constexpr int STORES = decltype(stores_c)::value;
        const uint32_t ar1 = a_rd[1] + static_cast<uint32_t>(cp_off);
        cp_off = cp_off + kSlotBytes == kNB * kSlotBytes ? 0 : cp_off + kSlotBytes;
        const uint32_t ar0 = a_rd[0] + static_cast<uint32_t>(cp_off);
        const unsigned char *src = ld_x;
        asm volatile("" : "+s"(src));   // one scalar base for the round's four wave-loads
        float al = 0.f, v[8];
        u32x4_t pk;
        if constexpr (JOB) al = alpha_of(z_t);
        typedef Int<2 * (Q & 1)> RowA;
        typedef Int<2 * (Q & 1) + 1> RowB;

        // K step 0 (set 0): requests K step 1 of this round
        uint32_t w1[4] = {wcur[0][Q], wcur[1][Q], wcur[2][Q], wcur[3][Q]};
        kstep(Int<0>{}, Int<(Q == 3 ? 4 : 0)>{}, ar1, w1, Int<1>{}, [&](auto slot_c) __attribute__((always_inline)) {
            constexpr int SLOT = decltype(slot_c)::value;
            if constexpr (JOB) {
                if constexpr (SLOT == 1) job_scale(RowA{}, al, v);
                if constexpr (SLOT == 2) job_pack(v, pk);
                if constexpr (SLOT == 3) job_store(RowA{}, pk);
                if constexpr (SLOT == 4) job_scale(RowB{}, al, v);
                if constexpr (SLOT == 5) job_pack(v, pk);
                if constexpr (SLOT == 6) job_store(RowB{}, pk);
            }
        });

        // Round + 1 must be readable from here on.  Vector-memory operations issued after its loads, which
        // may still be in flight: the loads of rounds + 2 .. + 4 (four each, and the two of a tile chunk if a
        // round with Q = 2 is among the three before this one) and the stores counted in STORES.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(12 + (Q == 2 ? 0 : 2) + STORES));

        // K step 1 (set 1): requests K step 0 of the next round
        // (Q = 3: the next group's windows, requested during round Q = 2, are older than this step's operands
        // and handed over behind its first wait; the words are picked there)
        uint32_t w0[4];
        if constexpr (Q < 3) {
#pragma unroll
            for (int tn = 0; tn < 4; ++tn) w0[tn] = wcur[tn][(Q + 1) & 3];
        }
        const uint32_t w_addr = w_rd + static_cast<uint32_t>((cp_tslot ^ 1) * kTileSlotBytes);
        kstep(Int<1>{}, Int<0>{}, ar0, w0, Int<0>{}, [&](auto slot_c) __attribute__((always_inline)) {
            constexpr int SLOT = decltype(slot_c)::value;
            if constexpr (SLOT == -1 && Q == 3) {
#pragma unroll
                for (int tn = 0; tn < 4; ++tn) { tie(wnxt[tn]); w0[tn] = wnxt[tn][0]; }
            }
            if constexpr (SLOT == 1) issue_x(Int<0>{}, src);
            if constexpr (SLOT == 3) issue_x(Int<1>{}, src);
            if constexpr (SLOT == 5) issue_x(Int<2>{}, src);
            if constexpr (Q == 2) {
                if constexpr (SLOT == 2) issue_tile(Int<0>{});
                if constexpr (SLOT == 4) { issue_tile(Int<1>{}); advance_tile(); }
                if constexpr (SLOT == 6) { lds_read16<0 * 512>(wnxt[0], w_addr); lds_read16<1 * 512>(wnxt[1], w_addr); }
                if constexpr (SLOT == 7) { lds_read16<2 * 512>(wnxt[2], w_addr); lds_read16<3 * 512>(wnxt[3], w_addr); }
            }
            if constexpr (SLOT == 7) {
                issue_x(Int<3>{}, src);
                advance_x(Int<(Q == 2)>{});   // the cursor moves on to round + 6: a half tile can only end there if Q = 2
            }
        });
        if constexpr (JOB && (Q & 1) == 1) { ++z_t; z_rep += rep_bytes; }
        if constexpr (Q == 3) {
#pragma unroll
            for (int tn = 0; tn < 4; ++tn) wcur[tn] = wnxt[tn];
            cp_tslot ^= 1;
        }
    };
    // four rounds; JP / J: the previous / this group's rounds carry stores (two each)
    auto group = [&](auto jp_c, auto j_c) __attribute__((always_inline)) {
        constexpr int JP = decltype(jp_c)::value, J = decltype(j_c)::value;
        round(Int<0>{}, j_c, Int<2 * (3 * JP + J)>{});
        round(Int<1>{}, j_c, Int<2 * (2 * JP + 2 * J)>{});
        round(Int<2>{}, j_c, Int<2 * (JP + 3 * J)>{});
        round(Int<3>{}, j_c, Int<2 * (4 * J)>{});
    };

    // ---- the half tiles -------------------------------------------------------------------------
    // Per half tile: groups of rounds that carry stores of the previous block, then groups that do not.
    // Operands requested by a loop's last round are allowed to land before the loop is left (settle), so that
    // a register with a read in flight only ever crosses a loop's own back edge.
    bool jp = false;   // the group before carried stores
    for (int32_t h = 0; h < n_ht; ++h) {
        int32_t sr = 0;
        if (z_t + 2 <= P.reps) {   // a group of four rounds stores two replicas
            if (jp) group(Int<1>{}, Int<1>{}); else group(Int<0>{}, Int<1>{});
            ++sr;
            settle();
            if (sr < n_sr && z_t + 2 <= P.reps) {
                do {
                    group(Int<1>{}, Int<1>{});
                    ++sr;
                } while (sr < n_sr && z_t + 2 <= P.reps);
                settle();
            }
            jp = true;
        }
        if (sr < n_sr) {
            if (jp) group(Int<1>{}, Int<0>{}); else group(Int<0>{}, Int<0>{});
            ++sr;
            settle();
            if (sr < n_sr) {
                do {
                    group(Int<0>{}, Int<0>{});
                    ++sr;
                } while (sr < n_sr);
                settle();
            }
            jp = false;
        }

        // ---- end of the half tile ---------------------------------------------------------------
        // replicas of the previous block that found no round (short K, many replicas, an odd last one)
        if (z_t < P.reps) {
            for (; z_t < P.reps; ++z_t, z_rep += rep_bytes) store_replica();
            jp = false;   // conservative for the wait counts: fewer stores assumed than were issued
        }

        // The waves add their partial sums.  Three steps: in step s = 1, 2, 3 wave w hands the block that wave
        // w ^ s keeps (accumulators [0][2..3], [1][0..1], [1][2..3] by the rotation of the indices) to that
        // wave through its 8 KiB slot.  The matrix pipe must have written the accumulators back before the
        // assembly below reads them.
        asm volatile("s_nop 15");
        asm volatile("s_nop 15");
#pragma unroll
        for (int step = 1; step <= 3; ++step) {
            const int tm = step >> 1, tn0 = 2 * (step & 1);
            u32x4_t s[8];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s[t * 4 + q][e] = __float_as_uint(acc[tm][tn0 + t][4 * q + e]);
            const uint32_t dst = static_cast<uint32_t>(kXchgOff + (wave ^ step) * 8192) + static_cast<uint32_t>(lane) * 16u;
            lds_write16<0 * 1024>(dst, s[0]);
            lds_write16<1 * 1024>(dst, s[1]);
            lds_write16<2 * 1024>(dst, s[2]);
            lds_write16<3 * 1024>(dst, s[3]);
            lds_write16<4 * 1024>(dst, s[4]);
            lds_write16<5 * 1024>(dst, s[5]);
            lds_write16<6 * 1024>(dst, s[6]);
            lds_write16<7 * 1024>(dst, s[7]);
            lds_wait<0>();
            __builtin_amdgcn_s_barrier();
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
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[0][t][4 * q + e] += __uint_as_float(got[t * 4 + q][e]);
            __builtin_amdgcn_s_barrier();   // every slot has been read: the next step (or the turn-round) may write
        }
        // Turn the finished 32 x 64 block round inside the wave's own slot.  On entry the lane holds row ln
        // and, in registers 4q .. 4q + 3 of tiles 0 and 1, columns 16*q + 8*lg .. + 7.  LDS row r is 256
        // bytes; the 16-byte chunk ch of it (columns 4*ch .. 4*ch + 3) sits at chunk position ch ^ s(r),
        // s(r) = ((r >> 1) & 7) ^ (2 * (r & 1)): the writes (lanes = rows) and the reads (eight lanes per row;
        // a lane reads chunks 2*g8 and 2*g8 + 1, the upper four lanes in the other order) are then free of
        // bank conflicts.
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
        __builtin_amdgcn_s_barrier();   // the slots are free for the next half tile's hand-over
        // where the block goes: rows cp_row*64 + 32*rot_m + rr + 8*i, columns cp_col*128 + 64*rot_n + 8*g8 .. + 7
        {
            const int64_t row0 = int64_t(cp_row) * kHT + 32 * rot_m;
            const int32_t col0 = cp_col * kBN + 64 * rot_n;
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
            z_rep = z_base;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        cp_col += step_c;
        cp_row += step_r;
        if (cp_col >= P.tiles_n) { cp_col -= P.tiles_n; ++cp_row; }
    }

    // ---- the last block's replicas; the loads issued past the end have landed by then -------------------
    for (; z_t < P.reps; ++z_t, z_rep += rep_bytes) store_replica();
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

// Shapes the streaming kernel takes: bfloat16, tile of whole rows, K in whole groups of four rounds per wave
// (in % 512 == 0), 16-byte stores possible, every offset inside a half tile in 32 bits.
bool linear_stream_supported(const LinearArgs &a) {
    if (a.dt != TBN_BF16) return false;
    if (a.in % 512 != 0 || a.p % a.in != 0) return false;
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
    P.n_sr = P.in / 512;
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
