// Matrix-core kernel for the fully-connected tiled-bit layer with bfloat16 activations and a tile that
// holds whole weight rows (p % in == 0), one 128 x 128 block of Z per workgroup, with separate load waves.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8): with p a multiple of `in` the
// (out x in) weight is the U = p / in rows of the tile stacked k times, copy t scaled by alpha[t].  So
// Z = X * T^T (M x U, T the +-1 rows of the tile) is formed once and Y[:, t*U + u] = alpha[t] * Z[:, u]
// ("only one of the tile computations needs to be executed", Section "CNN Architectures", applied to
// matrix columns).
//
// Layout on gfx950 and why (every point is a measurement on the chip):
//   * A wave issues one instruction every four cycles at best and a v_mfma_f32_32x32x16_bf16 occupies the
//     matrix pipe for 32, so what bounds the main loop is the number of other instructions the MFMA waves
//     have to issue -- and above all the global -> LDS wave-loads, which block the wave's whole instruction
//     stream whenever the CU's load path is busy.  The workgroup therefore has eight waves: four MFMA waves
//     (one per SIMD) that only read LDS and multiply, and four load waves that issue every wave-load of the
//     main loop and otherwise sleep at the round's barrier (with the MFMA waves loading for themselves, one
//     wave-load in an MFMA slot each, the same kernel measured 46.1 us against 42.6 on 8192 x 4096 -> 4096).
//   * MFMA wave (g, h) owns 128 rows x 64 columns of the block over the K stages congruent to g (mod 2):
//     4 x 2 MFMA tiles, the +-1 rows as the row operand, six LDS operand reads per eight MFMAs.  The two
//     K groups add their partial sums through LDS at the end.
//   * Activations go global -> LDS directly (16 bytes per lane, four ring slots of one stage for both K
//     groups, XOR-swizzled so that operand reads are free of bank conflicts).  The chunk of the packed tile
//     that the block's 128 tile rows need for two rounds travels the same way in coalesced 16-byte pieces;
//     an MFMA wave then takes the 64 window bits of its two columns with one LDS instruction per round.
//     Tile bits are never fetched lane by lane from global memory.
//   * A byte of tile bits becomes the +-1 bf16 MFMA operand through a 256-entry table in LDS.
//   * The replicated, alpha-scaled output is most of the bytes this kernel moves (eight ninths at k = 8).  It
//     is written with 16-byte stores that cover whole 128-byte lines (the sums are turned round through LDS
//     first).  With one block per workgroup the MFMA waves write it themselves with plain stores: all workgroups
//     store at the same time and the last-level cache takes the burst (8192 x 4096 -> 4096, k = 8: 37.7 us
//     against 42.4 with non-temporal stores).
//   * Grids of more blocks than CUs (PERSIST): one workgroup per CU walks blocks, and the stores of a block run
//     under the K loop of the next one.  Of waves 4 .. 7 two load (two quarters of a round each) and two store: the
//     MFMA waves leave the sums of a finished block in LDS, a store wave takes two 64 x 64 quarters into 128
//     registers and writes them, scaled, a few (replica, quarter, 32 rows) units per round, with non-temporal
//     stores (next to a running loop, plain stores push the activations that the other column blocks of the same
//     rows still need out of the XCD's L2: 16384 x 4096 -> 4096, k = 8: 81 us against 65).  Stores and loads have
//     waves of their own because the vector-memory counter counts both, in issue order: a wave that did both
//     waited for its stores whenever it waited for a round of loads (8192 x 4096 -> 16384, k = 8: block loops of
//     28.7 us against 24.7).  The first two rounds of the next block are issued inside the last rounds of the
//     current one, into the two ring slots behind its last round, which are free by then; between two loops lie 2.2 us (the K groups add their
//     sums, the store waves take them over).  8192 x 4096 -> 16384, k = 2 / 4 / 8 / 16: 410 / 211 / 117 / 86 us
//     against 410 / 216 / 127 / 97 with the stores after each loop; 32768 x 4096 -> 4096, k = 8: 137 against 152.
//     What stays exposed is the stores of a workgroup's last block.
//   * Split K (SPLIT = true, for grids that would leave most CUs idle and callers that bring a workspace):
//     the K loop of a block is dealt to S workgroups; each writes its float32 partial sums of the 128 x 128
//     block to the workspace, [split][M][U], and a second kernel adds the S partial sums of every output in
//     ascending split order (no atomics: the result is the same bit for bit from run to run), scales by
//     alpha and writes the replicas.
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

constexpr int kBM = 128, kBN = 128;      // block of Z per workgroup
constexpr int kBK = 64;                  // K elements per K group and round
constexpr int kNB = 4;                   // ring slots
constexpr int kSlotBytes = 2 * kBM * kBK * 2;   // [K group][128 rows][128 bytes]
constexpr int kTileSlots = 3;            // ring of tile chunks, one chunk = two rounds
constexpr int kTileSlotBytes = 4096;     // [16-byte piece (= round parity)][128 columns][16 bytes]
constexpr int kBias = 3 * 1024;          // keeps the lane offsets of the wave-loads non-negative

// LDS map.  The sign table sits at address 0 so that a table read needs no base.
constexpr int kTableOff = 0;             // 256 entries of 16 bytes
constexpr int kRingOff = 4096;
constexpr int kTileOff = kRingOff + kNB * kSlotBytes;
constexpr int kLdsBytes = kTileOff + kTileSlots * kTileSlotBytes;
constexpr int kXchgOff = kRingOff;       // after the main loop the ring holds the partial sums handed over (4 x 16 KiB)
static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 workgroup");

struct BlockParams {
    int64_t M;
    int32_t in, out, U;
    int32_t reps;         // out / U = k replicas of every distinct column
    int32_t n_alpha;
    int32_t tiles_n;      // column blocks of U
    uint32_t tiles_m;
    int32_t n_rounds;     // rounds of 128 elements of K per workgroup (even): in / 128, or in / 128 / splits
    int32_t splits;       // workgroups that share the K loop of a block (1: none)
    uint32_t vrows;       // tiles_m * splits: (row block, split) pairs
    float *partial;       // split K: [split][M][U] float32 partial sums
};

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// All LDS traffic of this kernel is written as inline assembly: the compiler would otherwise make every
// LDS access wait for all global -> LDS loads in flight.  The waits are explicit; a register that a read
// fills is handed to the compiler only through tie() after the wait that covers it
// (paper_2407_12075_amd/asm_check.py verifies on the generated assembly that nothing touches such a
// register earlier).
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

template <int V> using Int = std::integral_constant<int, V>;

// 16-byte store to a scalar base plus a 32-bit lane offset (NT: non-temporal)
template <bool NT>
__device__ __forceinline__ void global_store16(unsigned char *base, uint32_t off, const u32x4_t &v) {
    if constexpr (NT) asm volatile("global_store_dwordx4 %0, %1, %2 nt" : : "v"(off), "v"(v), "s"(base) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, %2" : : "v"(off), "v"(v), "s"(base) : "memory");
}

// Workgroups that share rows of X are given consecutive slots on one XCD (workgroup ids are dealt
// round-robin to the 8 XCDs), so the later column blocks find X in that XCD's L2.
// With split K the unit that shares data is a (row block, split) pair: vrow counts those.
__device__ __forceinline__ void block_coords(const BlockParams &P, uint32_t bid, uint32_t &vrow, uint32_t &tile_n) {
    const uint32_t xcd = bid & 7, slot = bid >> 3;
    const uint32_t tiles_n = static_cast<uint32_t>(P.tiles_n);
    const uint32_t per_xcd_full = (P.vrows / 8) * tiles_n;   // slots per XCD in the regular part
    if (slot < per_xcd_full) {
        const uint32_t q = slot / tiles_n;
        tile_n = slot - q * tiles_n;
        vrow = q * 8 + xcd;
    } else {  // remaining row blocks: plain order
        const uint32_t rest = bid - per_xcd_full * 8;
        const uint32_t q = rest / tiles_n;
        tile_n = rest - q * tiles_n;
        vrow = (P.vrows / 8) * 8 + q;
    }
}

// RELU: fused max(0, .) of Algorithm 1.  SPLIT: the workgroup takes one of P.splits equal parts of K and writes
// float32 partial sums to P.partial instead of Y.  512 threads: waves 0 .. 3 multiply, waves 4 .. 7 load.
// PERSIST (grids of more blocks than CUs; at least four rounds): the workgroup walks blocks blockIdx.x, + gridDim.x, ...;
// waves 4 and 5 load, waves 6 and 7 write the replicas of the block before.  The
// first rounds of the next block start in the ring slot behind the current block's last round, and the hand-over uses
// the slots of the last two rounds.
template <bool RELU, bool SPLIT, bool PERSIST>
__global__ __launch_bounds__(512, 1) void linear_block_bf16_kernel(const uint16_t *__restrict__ x,
                                                                                     uint16_t *__restrict__ y,
                                                                                     const uint32_t *__restrict__ tile,
                                                                                     const float *__restrict__ alpha,
                                                                                     BlockParams P) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = wave & 3;     // MFMA wave: which quarter of the block it owns
    const int grp = li >> 1;     // K group
    const int wn = li & 1;       // column half
    const int ln = lane & 31;    // operand lane inside a 32 x 32 tile
    const int lg = lane >> 5;    // K half of the operand registers

    static_assert(!(SPLIT && PERSIST), "a split grid never has more workgroups than CUs");
    // Ring slot of round g of a block: (g + ph) % 4.  ph is 0 with one block per workgroup; a persistent workgroup
    // starts a block in the slot after the last one of the block before, ph' = (ph + rounds) % 4 (0 or 2: rounds come
    // in pairs).  Hand-over area: with one block per workgroup the start of the ring; PERSIST: the slots of a block's
    // last two rounds, which are the two slots behind those that take the first two rounds of the next block.
    auto xchg_base = [&](int32_t phase) -> uint32_t {
        return PERSIST ? static_cast<uint32_t>(kRingOff + ((P.n_rounds - 2 + phase) & 3) * kSlotBytes) : static_cast<uint32_t>(kXchgOff);
    };
    // Waves 4 .. 7.  One block per workgroup: four load waves, each issues a quarter of a round's loads (quarter q:
    // K group q / 2, row-slot half q % 2).  PERSIST: waves 4 and 5 load (two quarters each: K group = wave - 4),
    // waves 6 and 7 write the replicas of the block before (the quarters of MFMA waves 2*(wave - 6) and + 1).
    constexpr int NQ = PERSIST ? 2 : 1;   // quarters per load wave (and per store wave)
    const int first_q = PERSIST ? 2 * (wave & 1) : (wave & 3);
    const int32_t n_rounds = P.n_rounds;
    const uint32_t n_blocks = P.vrows * static_cast<uint32_t>(P.tiles_n);
    uint32_t bid = blockIdx.x;

    // ---- the loads of a round, a quarter at a time ------------------------------------------------------
    // Activations: wave-load j of quarter q fills 1 KiB of K group q / 2's 16 KiB: piece 8*(q % 2) + j, row slot
    // sr = 8*piece + lane/8, chunk slot lane%8.  Row-slot block sr/32 holds row block (sr/32 + 2*grp) % 4 of the
    // block (so that each K group ends with the sums it keeps in its first accumulators), chunk slot s of row
    // slot sr holds 16-byte chunk s ^ ((sr >> 1) & 7) of the round's 128 bytes of that row.  Rows past M repeat
    // row M - 1.  Tile chunk (two rounds: 256 bits = two 16-byte pieces per tile row): lane i of quarter q fills
    // slot S = 64*q + i of the chunk's 256: piece S / 128, LDS row S % 128; LDS row 64*h + 32*tn + l holds the
    // tile row that operand lane l of column half h supplies for MFMA tile tn, i.e. column
    // 64*h + 16*(l/8) + 8*((l/4)%2) + 4*tn + l%4 of the block (with this numbering a lane ends up with eight
    // adjacent columns of one row of Y).
    uint32_t split = 0;
    int64_t m0 = 0;
    int32_t n0 = 0;
    const unsigned char *x_blk[NQ] = {};
    const unsigned char *tile_bytes = nullptr;
    uint32_t a_off[NQ][8];
    uint32_t t_off[NQ];
    auto set_block = [&](uint32_t b) __attribute__((always_inline)) {
        uint32_t tile_m, tile_n;
        block_coords(P, b, tile_m, tile_n);
        split = 0;
        if (SPLIT) {
            const uint32_t vrow = tile_m;
            tile_m = vrow / static_cast<uint32_t>(P.splits);
            split = vrow - tile_m * static_cast<uint32_t>(P.splits);
        }
        const uint32_t round0 = split * static_cast<uint32_t>(P.n_rounds);   // first round of this workgroup's part of K (even)
        m0 = int64_t(tile_m) * kBM;
        n0 = static_cast<int32_t>(tile_n) * kBN;
        tile_bytes = reinterpret_cast<const unsigned char *>(tile) + round0 * 16u;
        const int64_t last = P.M - 1 - m0;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int lq = first_q + q, gq = lq >> 1, hq = lq & 1;
            x_blk[q] = reinterpret_cast<const unsigned char *>(x) + m0 * P.in * 2 + (gq * 128 - kBias) + round0 * 256u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int sr = 8 * (8 * hq + j) + (lane >> 3);
                const int r = ((((sr >> 5) + 2 * gq) & 3) << 5) + (sr & 31);
                const uint32_t rw = static_cast<uint32_t>(r < last ? r : last);
                const int chunk = (lane & 7) ^ ((sr >> 1) & 7);
                a_off[q][j] = rw * static_cast<uint32_t>(P.in) * 2u + static_cast<uint32_t>(chunk * 16 + kBias - (j & 3) * 1024);
            }
            const int S = 64 * lq + lane, rho = S & 127, l = rho & 31;
            int32_t u = n0 + (rho & 64) + 16 * (l >> 3) + 8 * ((l >> 2) & 1) + 4 * ((rho >> 5) & 1) + (l & 3);
            u = u < P.U ? u : P.U - 1;   // columns past U repeat the last one; they are never written
            t_off[q] = static_cast<uint32_t>(u) * (static_cast<uint32_t>(P.in) >> 3) + static_cast<uint32_t>((S >> 7) * 16);
        }
    };
    set_block(bid);
    // issue order per round, which the wait counts rely on: eight activation wave-loads per quarter, then (even
    // rounds) a quarter's share of the tile chunk of this round and the next
    auto issue_x = [&](auto q_c, auto j_c, int32_t round_, int32_t phase) {
        constexpr int Q = decltype(q_c)::value, J = decltype(j_c)::value;
        const int lq = first_q + Q;
        unsigned char *const ring_q = lds_raw + kRingOff + (lq >> 1) * 16384 + (lq & 1) * 8192;
        const unsigned char *src = x_blk[Q] + static_cast<uint32_t>(round_) * 256u;   // wave-uniform
        asm volatile("" : "+s"(src));   // one scalar base, the lane offset stays a 32-bit register
        uint32_t off = a_off[Q][J];
        asm volatile("" : "+v"(off));
        wave_load<(J & 3)>(src, off, ring_q + ((round_ + phase) & (kNB - 1)) * kSlotBytes + (J >> 2) * 4096);
    };
    auto issue_tile = [&](auto q_c, int32_t round_) {   // round_ is even
        constexpr int Q = decltype(q_c)::value;
        const unsigned char *src = tile_bytes + static_cast<uint32_t>(round_) * 16u;   // 128 bits per round
        asm volatile("" : "+s"(src));
        uint32_t off = t_off[Q];
        asm volatile("" : "+v"(off));
        __builtin_amdgcn_global_load_lds(src + off, lds_raw + kTileOff + (first_q + Q) * 1024 + ((round_ >> 1) % kTileSlots) * kTileSlotBytes, 16, 0, 0);
    };
    auto issue_quarter = [&](auto q_c, int32_t round_, int32_t phase) {
        issue_x(q_c, Int<0>{}, round_, phase); issue_x(q_c, Int<1>{}, round_, phase); issue_x(q_c, Int<2>{}, round_, phase); issue_x(q_c, Int<3>{}, round_, phase);
        issue_x(q_c, Int<4>{}, round_, phase); issue_x(q_c, Int<5>{}, round_, phase); issue_x(q_c, Int<6>{}, round_, phase); issue_x(q_c, Int<7>{}, round_, phase);
    };
    auto issue_round = [&](int32_t round_, int32_t phase = 0) {
        issue_quarter(Int<0>{}, round_, phase);
        if constexpr (NQ == 2) issue_quarter(Int<1>{}, round_, phase);
        if ((round_ & 1) == 0) {
            issue_tile(Int<0>{}, round_);
            if constexpr (NQ == 2) issue_tile(Int<1>{}, round_);
        }
    };
    constexpr int kOdd = 8 * NQ, kEven = 9 * NQ;   // loads of an odd and of an even round per load wave

    // a lane's place in the stores of a replica: eight lanes per row of Y, eight adjacent columns each
    const int g8 = lane & 7, rr = lane >> 3;
    const uint32_t z_lane = (static_cast<uint32_t>(rr) * static_cast<uint32_t>(P.out) + static_cast<uint32_t>(8 * g8)) * 2u;
    const uint32_t out_bytes8 = static_cast<uint32_t>(P.out) * 16u;   // eight rows of Y in bytes
    const uint32_t rep_bytes = static_cast<uint32_t>(P.U) * 2u;

    // =================================================================================================
    // store waves (PERSIST)
    // =================================================================================================
    // MFMA wave q leaves the sums of its 64 x 64 quarter of a finished block in the hand-over area; a store wave
    // takes two quarters into registers (128 per lane) and writes them, scaled, one (replica, quarter, 32 rows)
    // unit after the other, spread evenly over the rounds in which the MFMA waves multiply the next block: the
    // matrix pipe does not wait for the stores, which are most of the bytes this kernel moves.  The stores have
    // waves of their own because the vector-memory counter counts loads and stores alike and in issue order: a
    // wave that did both would wait for its stores whenever it waits for a round of loads.
    if (PERSIST && wave >= 6) {
        float alpha_lanes;
        {
            const int t = P.n_alpha == 1 ? 0 : (lane < P.reps ? lane : P.reps - 1);
            const uint32_t off = static_cast<uint32_t>(t) * 4u;
            asm volatile("global_load_dword %0, %1, %2\n\ts_waitcnt vmcnt(0)" : "=v"(alpha_lanes) : "v"(off), "s"(alpha) : "memory");
        }
        float zr[2][2][4][8];   // [quarter][32-row half][row rr + 8*i][column 8*g8 + e]
        unsigned char *st_base = nullptr;   // &Y[first row of quarter 0][first column of quarter 0], replica 0
        int64_t st_rows = 0;          // rows of the quarters that exist (may be <= 0)
        bool st_col_ok[2] = {false, false};
        int32_t st_rot = 0;           // the replica a block starts with: workgroups that store at the same time write different ones
        int32_t st_next = 0, st_total = 0, st_credit = 0;   // units written / to write; spreads them over the rounds
        auto store_unit = [&](int32_t uidx) __attribute__((always_inline)) {
            const int32_t sub = uidx & 3, half = sub & 1, q = sub >> 1;
            int32_t t = (uidx >> 2) + st_rot;
            t = t >= P.reps ? t - P.reps : t;
            const float al = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, alpha_lanes), t));
            unsigned char *dst = st_base + static_cast<uint32_t>(t) * rep_bytes + static_cast<uint32_t>(half) * 4u * out_bytes8 + static_cast<uint32_t>(q) * 128u;
            const int64_t rows_left = st_rows - 32 * half;
            auto emit = [&](auto q_c, auto half_c) __attribute__((always_inline)) {
                constexpr int Q = decltype(q_c)::value, H = decltype(half_c)::value;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        v[e] = al * zr[Q][H][i][e];
                        if (RELU) v[e] = fmaxf(v[e], 0.f);
                    }
                    const u32x4_t pk = {pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
                    if (st_col_ok[Q] && rr + 8 * i < rows_left) global_store16<true>(dst, z_lane + static_cast<uint32_t>(i) * out_bytes8, pk);
                }
            };
            if (sub == 0) emit(Int<0>{}, Int<0>{});
            else if (sub == 1) emit(Int<0>{}, Int<1>{});
            else if (sub == 2) emit(Int<1>{}, Int<0>{});
            else emit(Int<1>{}, Int<1>{});
        };
        int32_t ph = 0;
        for (;;) {
            const int64_t cur_m0 = m0;
            const int32_t cur_n0 = n0;
            __builtin_amdgcn_s_barrier();   // the block's first barrier
            for (int32_t g = 0; g < n_rounds; ++g) {
                __builtin_amdgcn_s_barrier();
                st_credit += st_total;
                for (; st_credit >= n_rounds && st_next < st_total; st_credit -= n_rounds) store_unit(st_next++);
            }
            while (st_next < st_total) store_unit(st_next++);
            const uint32_t next = bid + gridDim.x;
            const bool more = next < n_blocks;
            if (more) {
                bid = next;
                set_block(bid);
            }
            __builtin_amdgcn_s_barrier();   // the two barriers of the hand-over
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_s_barrier();   // the sums of the finished block are in the hand-over area
            // the same turn-round as in the epilogue of the MFMA waves below: eight lanes take one row's 64 columns
            {
                const int ch_a = 2 * g8 + (g8 >> 2), ch_b = 2 * g8 + 1 - (g8 >> 2);
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const uint32_t area = xchg_base(ph) + static_cast<uint32_t>((first_q + q) * 16384);
                    u32x4_t za[2][4], zb[2][4];
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int r = rr + 8 * i;
                            const int s_r = ((r >> 1) & 7) ^ (2 * (r & 1));
                            lds_read16<0>(za[h][i], area + static_cast<uint32_t>(h * 8192 + r * 256 + ((ch_a ^ s_r) << 4)));
                            lds_read16<0>(zb[h][i], area + static_cast<uint32_t>(h * 8192 + r * 256 + ((ch_b ^ s_r) << 4)));
                        }
                    lds_wait<0>();
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            tie(za[h][i]);
                            tie(zb[h][i]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                zr[q][h][i][e] = __uint_as_float(g8 < 4 ? za[h][i][e] : zb[h][i][e]);
                                zr[q][h][i][4 + e] = __uint_as_float(g8 < 4 ? zb[h][i][e] : za[h][i][e]);
                            }
                        }
                }
            }
            {
                const int64_t row0 = cur_m0 + 64 * (first_q >> 1);
                st_base = reinterpret_cast<unsigned char *>(y) + (row0 * P.out + cur_n0) * 2;
                st_rows = P.M - row0;
                st_col_ok[0] = cur_n0 + 8 * g8 < P.U;
                st_col_ok[1] = cur_n0 + 64 + 8 * g8 < P.U;
                st_rot = static_cast<int32_t>(static_cast<uint32_t>(cur_m0 >> 7) % static_cast<uint32_t>(P.reps));
                st_next = 0;
                st_total = 4 * P.reps;
                st_credit = 0;
                ph = (ph + n_rounds) & 3;
            }
            if (!more) {
                while (st_next < st_total) store_unit(st_next++);
                return;
            }
        }
    }

    // =================================================================================================
    // load waves
    // =================================================================================================
    if (wave >= 4) {
        if constexpr (PERSIST) {
            // One workgroup walks blocks.  The last three rounds of a block load nothing for it, and the two ring slots behind its last round
            // are free by then: the activations of the next block's rounds 0 and 1 are issued there, one round each,
            // and its first tile chunk behind the last round's barrier (that slot of the tile ring is read until then),
            // so the hand-over between two blocks waits for no load to be issued.
            issue_round(0);
            issue_round(1);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOdd));   // round 0 and its tile chunk; round 1's loads are younger
            int32_t ph = 0;
            for (;;) {
                __builtin_amdgcn_s_barrier();   // meets the MFMA waves' "round 0 readable; the hand-over area is free"
                issue_round(2, ph);
                const int32_t ph_next = (ph + n_rounds) & 3;
                const uint32_t next = bid + gridDim.x;
                const bool more = next < n_blocks;
                for (int32_t g = 0; g < n_rounds; ++g) {
                    // round g + 1 has to be readable when the MFMA waves pass this barrier; what was issued after its
                    // loads may stay in flight: round g + 2 (with the tile chunk if that round is even), or, at the end of
                    // a block, the next block's round 0
                    if (g + 2 < n_rounds) {
                        if (g & 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOdd));
                        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(kEven));
                    } else if (!more) {
                        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                    } else if (g + 2 == n_rounds) {
                        __builtin_amdgcn_s_waitcnt(vmcnt_imm(8 * NQ));
                    }
                    __builtin_amdgcn_s_barrier();
                    if (g + 3 < n_rounds) {
                        issue_round(g + 3, ph);
                    } else if (more) {
                        if (g + 3 == n_rounds) {
                            bid = next;
                            set_block(bid);
                            issue_quarter(Int<0>{}, 0, ph_next);
                            issue_quarter(Int<1>{}, 0, ph_next);
                        } else if (g + 2 == n_rounds) {
                            issue_quarter(Int<0>{}, 1, ph_next);
                            issue_quarter(Int<1>{}, 1, ph_next);
                        } else {
                            issue_tile(Int<0>{}, 0);
                            issue_tile(Int<1>{}, 0);
                        }
                    }
                }
                __builtin_amdgcn_s_barrier();   // the two barriers of the hand-over
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_s_barrier();   // the store waves take the sums of the finished block
                if (!more) return;
                ph = ph_next;
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // rounds 0 and 1 and the tile chunk of the next block
            }
        } else {
            // rounds 0 .. 2 at once; then, at the top of every round, the loads of round + 3 into the slot that the
            // barrier has just freed
            for (int32_t d = 0; d < 3 && d < n_rounds; ++d) issue_round(d);
            // round 0 is readable once it has landed (two younger rounds may be in flight)
            if (n_rounds >= 3) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOdd + kEven));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __builtin_amdgcn_s_barrier();   // meets the MFMA waves' "table written, round 0 readable"
            for (int32_t g = 0; g < n_rounds; ++g) {
                // round g + 1 has to be readable when the MFMA waves pass this barrier; the loads of round g + 2 (with
                // the tile chunk if that round is even) are younger and may stay in flight
                if (g + 2 < n_rounds) {
                    if (g & 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOdd));
                    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(kEven));
                } else {
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                }
                __builtin_amdgcn_s_barrier();
                if (g + 3 < n_rounds) issue_round(g + 3);
            }
            __builtin_amdgcn_s_barrier();   // the two barriers of the hand-over
            __builtin_amdgcn_s_barrier();
            return;
        }
    }

    // =================================================================================================
    // MFMA waves
    // =================================================================================================
    // alpha of replica t in lane t (at most 64 replicas), fetched by hand so that the compiler places no wait
    // for it inside the rounds
    float alpha_lanes;
    {
        const int t = P.n_alpha == 1 ? 0 : (lane < P.reps ? lane : P.reps - 1);
        const uint32_t off = static_cast<uint32_t>(t) * 4u;
        asm volatile("global_load_dword %0, %1, %2" : "=v"(alpha_lanes) : "v"(off), "s"(alpha));
    }

    int32_t ph = 0;   // ring phase of the current block

    // sign table: entry e, element i is +1 if bit i of e is set, else -1
    if (tid < 256) {
        u32x4_t t;
        const int e = tid;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            t[v] = (((e >> (2 * v)) & 1) ? 0x3f80u : 0xbf80u) | ((((e >> (2 * v + 1)) & 1) ? 0x3f80u : 0xbf80u) << 16);
        lds_write16<kTableOff>(static_cast<uint32_t>(e) * 16u, t);
    }

    // operand read addresses inside a ring slot: row slot 32*tm + ln, K step ks: chunk 2*ks + lg at chunk slot
    // (2*ks + lg) ^ ((ln >> 1) & 7)
    uint32_t a_rd[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        a_rd[ks] = static_cast<uint32_t>(kRingOff + grp * 16384 + ln * 128 + (((2 * ks + lg) ^ ((ln >> 1) & 7)) << 4));
    // window read: LDS row 64*wn + ln (tn = 0) and + 32 (tn = 1) of the chunk, the K group's 8 bytes of the piece
    const uint32_t w_rd = static_cast<uint32_t>(kTileOff + (64 * wn + ln) * 16 + 8 * grp);
    // byte 2*ks + lg of a window: word ks / 2, bits 16*(ks % 2) + 8*lg on
    uint32_t bsh[2] = {8u * static_cast<uint32_t>(lg), 16u + 8u * static_cast<uint32_t>(lg)};
    asm volatile("" : "+v"(bsh[0]), "+v"(bsh[1]));

    f32x16_t acc[4][2];
    Frag A[2][4];       // [operand set][tm]
    Frag B[2][2];       // [operand set][tn]
    u32x4_t win[2];     // [round parity]: words 0-1 the 64 window bits of column tn = 0, words 2-3 of tn = 1

    auto table_read = [&](u32x4_t &dst, uint32_t word, uint32_t shift) {
        const uint32_t addr = __builtin_amdgcn_ubfe(word, shift, 8) << 4;
        lds_read16<kTableOff>(dst, addr);
    };

    auto settle = [&]() {   // all of operand set 0 has landed
        lds_wait<0>();
        tie(B[0][0].q); tie(B[0][1].q);
        tie(A[0][0].q); tie(A[0][1].q); tie(A[0][2].q); tie(A[0][3].q);
    };

    // ---- one K step: 8 MFMAs ---------------------------------------------------------------------
    // Multiplies with operand set S and requests the operands of the following K step into the other set: six
    // LDS reads, one in each of the first six MFMA slots, in the order in which that step's MFMAs need them
    // (+-1 operand of tn = 0, activation fragment of tm = 0, +-1 operand of tn = 1, fragments of tm = 1, 2, 3).
    // LDS operations complete in order, so "at most N pending" names exactly which operands have arrived;
    // three waits cover the step, and every operand has the time of at least six MFMAs to arrive.  A slot is:
    // wait, request, MFMA, side work.  W1 = 1: the window read of the next round was issued behind the previous
    // step's requests.
    auto kstep = [&](auto s_c, auto w1_c, uint32_t n_addr, uint32_t nw0, uint32_t nw1, auto nks_c, auto &&side) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value, N = S ^ 1, W1 = decltype(w1_c)::value, NKS = decltype(nks_c)::value;
        auto mfma = [&](int tm, int tn) {
            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(B[S][tn].v, A[S][tm].v, acc[tm][tn], 0, 0, 0);
        };
        lds_wait<3 + W1>(); tie(B[S][0].q); tie(A[S][0].q); tie(B[S][1].q);
        side(Int<-1>{});   // what else this wait covers
        table_read(B[N][0].q, nw0, bsh[NKS]);
        mfma(0, 0);
        side(Int<0>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_read16<0>(A[N][0].q, n_addr);
        mfma(0, 1);
        side(Int<1>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<4 + W1>(); tie(A[S][1].q);
        table_read(B[N][1].q, nw1, bsh[NKS]);
        mfma(1, 0);
        side(Int<2>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_read16<4096>(A[N][1].q, n_addr);
        mfma(1, 1);
        side(Int<3>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_wait<4 + W1>(); tie(A[S][2].q); tie(A[S][3].q);
        lds_read16<8192>(A[N][2].q, n_addr);
        mfma(2, 0);
        side(Int<4>{});
        __builtin_amdgcn_sched_barrier(0);
        lds_read16<12288>(A[N][3].q, n_addr);
        mfma(2, 1);
        side(Int<5>{});
        __builtin_amdgcn_sched_barrier(0);
        mfma(3, 0);
        side(Int<6>{});
        __builtin_amdgcn_sched_barrier(0);
        mfma(3, 1);
        side(Int<7>{});
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- one round: four K steps, 32 MFMAs -------------------------------------------------------------
    // PAR: parity of the round.  The round opens with the barrier that makes round + 1 readable (its loads were
    // issued two rounds ago) and frees the slot of round - 1 for the loads of round + 3.  On entry the operands
    // of the first K step have been requested into set 0.
    auto round = [&](auto par_c, int32_t g) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_c)::value;
        __builtin_amdgcn_s_barrier();
        const uint32_t cur = static_cast<uint32_t>(((g + ph) & (kNB - 1)) * kSlotBytes);
        const uint32_t nxt = static_cast<uint32_t>(((g + 1 + ph) & (kNB - 1)) * kSlotBytes);
        // windows of the next round: an even round reads the second piece of its own chunk, an odd round the
        // first piece of the next chunk
        const uint32_t w_addr = w_rd + static_cast<uint32_t>((((g + 1) >> 1) % kTileSlots) * kTileSlotBytes + (PAR == 0 ? 2048 : 0));
        u32x4_t &wc = win[PAR];       // this round's windows
        u32x4_t &wx = win[PAR ^ 1];   // the next round's
        kstep(Int<0>{}, Int<0>{}, a_rd[1] + cur, wc[0], wc[2], Int<1>{}, [&](auto slot_c) __attribute__((always_inline)) {
            constexpr int SLOT = decltype(slot_c)::value;
            if constexpr (SLOT == 6) lds_read2x8(wx, w_addr);
        });
        kstep(Int<1>{}, Int<1>{}, a_rd[2] + cur, wc[1], wc[3], Int<0>{}, [&](auto) __attribute__((always_inline)) {});
        kstep(Int<0>{}, Int<0>{}, a_rd[3] + cur, wc[1], wc[3], Int<1>{}, [&](auto slot_c) __attribute__((always_inline)) {
            constexpr int SLOT = decltype(slot_c)::value;
            if constexpr (SLOT == -1) tie(wx);   // the window read is older than this step's operands
        });
        kstep(Int<1>{}, Int<0>{}, a_rd[0] + nxt, wx[0], wx[2], Int<0>{}, [&](auto) __attribute__((always_inline)) {});
    };

    lds_wait<0>();   // the table
    for (;;) {   // one block per pass (a single pass unless PERSIST)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- first operands -------------------------------------------------------------------------
    __builtin_amdgcn_s_barrier();   // table written, round 0 readable (PERSIST: and every wave is done with the hand-over area)
    lds_read2x8(win[0], w_rd);      // windows of round 0: chunk slot 0, piece 0
    lds_wait<0>();
    tie(win[0]);
    {
        const uint32_t first = a_rd[0] + static_cast<uint32_t>(ph * kSlotBytes);
        table_read(B[0][0].q, win[0][0], bsh[0]);
        lds_read16<0>(A[0][0].q, first);
        table_read(B[0][1].q, win[0][2], bsh[0]);
        lds_read16<4096>(A[0][1].q, first);
        lds_read16<8192>(A[0][2].q, first);
        lds_read16<12288>(A[0][3].q, first);
    }
    settle();

    // One plain loop over pairs of rounds; the operands that its last round requests (of a round that does not
    // exist) land before anything else touches their registers.
    for (int32_t g = 0; g < n_rounds; g += 2) {
        round(Int<0>{}, g);
        round(Int<1>{}, g + 1);
    }
    settle();

    // ---- the K groups add their partial sums ---------------------------------------------------------
    // Accumulator index tm of group g stands for row block (tm + 2g) % 4: each group keeps acc[0..1] and hands
    // acc[2..3] to the other one through its 16 KiB slot (the ring is free: every load has landed, every read
    // of it is done once all waves are here).  The matrix pipe must have written the accumulators back before
    // the assembly below reads them.
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    asm volatile("" : "+v"(alpha_lanes));
    __builtin_amdgcn_s_barrier();
    asm volatile("s_nop 15");
    asm volatile("s_nop 15");
    const uint32_t xchg_mine = xchg_base(ph) + static_cast<uint32_t>(li * 16384);
    {
        const uint32_t dst = xchg_base(ph) + static_cast<uint32_t>((li ^ 2) * 16384) + static_cast<uint32_t>(lane) * 16u;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4_t s[8];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s[t * 4 + q][e] = __float_as_uint(acc[2 + half][t][4 * q + e]);
            const uint32_t d = dst + static_cast<uint32_t>(half * 8192);
            lds_write16<0 * 1024>(d, s[0]);
            lds_write16<1 * 1024>(d, s[1]);
            lds_write16<2 * 1024>(d, s[2]);
            lds_write16<3 * 1024>(d, s[3]);
            lds_write16<4 * 1024>(d, s[4]);
            lds_write16<5 * 1024>(d, s[5]);
            lds_write16<6 * 1024>(d, s[6]);
            lds_write16<7 * 1024>(d, s[7]);
        }
    }
    lds_wait<0>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        u32x4_t got[8];
        const uint32_t src = xchg_mine + static_cast<uint32_t>(half * 8192) + static_cast<uint32_t>(lane) * 16u;
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
                for (int e = 0; e < 4; ++e) acc[half][t][4 * q + e] += __uint_as_float(got[t * 4 + q][e]);
    }

    // ---- epilogue: y[m, u + t*U] = alpha[t] * Z[m, u] ---------------------------------------------------
    // The lane holds, for row block tm, row 32*tm + ln and, in registers 4q .. 4q + 3 of tiles 0 and 1, columns
    // 16*q + 8*lg .. + 7 of the wave's 64.  The wave turns 32 rows at a time round through the part of its slot
    // that it has read already, so that eight lanes hold one row's 64 columns: a store instruction then writes
    // eight whole 128-byte lines.  LDS row r is 256 bytes; the 16-byte chunk ch of it (columns 4*ch .. 4*ch + 3)
    // sits at chunk position ch ^ s(r), s(r) = ((r >> 1) & 7) ^ (2 * (r & 1)): the writes (lanes = rows) and the
    // reads (eight lanes per row; a lane reads chunks 2*g8 and 2*g8 + 1, the upper four lanes in the other
    // order) are then free of bank conflicts.
    if constexpr (PERSIST) {
        // the store waves write the replicas: leave both 32-row halves in this wave's part of the hand-over area (all of
        // which the wave has read by now), in the layout described above
        const int s_w = ((ln >> 1) & 7) ^ (2 * (ln & 1));
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn) {
                    const int ch = 4 * q + 2 * lg + tn;
                    u32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[tm][tn][4 * q + e]);
                    lds_write16<0>(xchg_mine + static_cast<uint32_t>(tm * 8192 + ln * 256 + ((ch ^ s_w) << 4)), v);
                }
        lds_wait<0>();
        __builtin_amdgcn_s_barrier();   // the store waves take the sums from here
            const uint32_t next = bid + gridDim.x;
        if (next >= n_blocks) break;
        bid = next;
        ph = (ph + n_rounds) & 3;
        continue;
    }
    const bool col_ok = n0 + 64 * wn + 8 * g8 < P.U;
#pragma unroll
    for (int tm = 0; tm < 2; ++tm) {
        float zr[4][8];
        {
            const int s_w = ((ln >> 1) & 7) ^ (2 * (ln & 1));
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn) {
                    const int ch = 4 * q + 2 * lg + tn;
                    u32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[tm][tn][4 * q + e]);
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
            __builtin_amdgcn_wave_barrier();   // the next 32 rows overwrite the staging area
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    zr[i][e] = __uint_as_float(g8 < 4 ? za[i][e] : zb[i][e]);
                    zr[i][4 + e] = __uint_as_float(g8 < 4 ? zb[i][e] : za[i][e]);
                }
        }
        // rows m0 + 64*grp + 32*tm + rr + 8*i, columns n0 + 64*wn + 8*g8 .. + 7
        const int64_t row0 = m0 + 64 * grp + 32 * tm;
        const int64_t rows_left = P.M - row0;   // may be <= 0
        if constexpr (SPLIT) {
            typedef __attribute__((address_space(1))) u32x4_t global_u32x4_t;
            unsigned char *dst = reinterpret_cast<unsigned char *>(P.partial + (int64_t(split) * P.M + row0) * P.U + n0 + 64 * wn);
            const uint32_t lane_off = (static_cast<uint32_t>(rr) * static_cast<uint32_t>(P.U) + static_cast<uint32_t>(8 * g8)) * 4u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (col_ok && rr + 8 * i < rows_left) {
                    const uint32_t off = lane_off + static_cast<uint32_t>(i) * static_cast<uint32_t>(P.U) * 32u;   // eight rows on
                    u32x4_t lo, hi;
#pragma unroll
                    for (int e = 0; e < 4; ++e) { lo[e] = __float_as_uint(zr[i][e]); hi[e] = __float_as_uint(zr[i][4 + e]); }
                    *(global_u32x4_t *)(dst + off) = lo;
                    *(global_u32x4_t *)(dst + off + 16) = hi;
                }
            }
            continue;
        }
        unsigned char *z_rep = reinterpret_cast<unsigned char *>(y) + (row0 * P.out + n0 + 64 * wn) * 2;
        for (int32_t t = 0; t < P.reps; ++t, z_rep += rep_bytes) {
            const float al = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, alpha_lanes), t));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    v[e] = al * zr[i][e];
                    if (RELU) v[e] = fmaxf(v[e], 0.f);
                }
                const u32x4_t pk = {pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
                typedef __attribute__((address_space(1))) u32x4_t global_u32x4_t;
                unsigned char *dst = z_rep;
                asm volatile("" : "+s"(dst));
                uint32_t off = z_lane + static_cast<uint32_t>(i) * out_bytes8;
                asm volatile("" : "+v"(off));   // scalar base + 32-bit lane offset
                if (col_ok && rr + 8 * i < rows_left) *(global_u32x4_t *)(dst + off) = pk;
            }
        }
    }
    break;   // one block per workgroup
    }
}

// Second pass of split K: z = partial[0] + partial[1] + ... (ascending, float32), y[m, u + t*U] = alpha[t] * z.
// One thread per eight adjacent distinct columns of a row.
template <bool RELU>
__global__ __launch_bounds__(128) void linear_split_reduce_kernel(const float *__restrict__ partial, uint16_t *__restrict__ y,
                                                                  const float *__restrict__ alpha, BlockParams P) {
    const int64_t groups = P.U / 8;
    const int64_t idx = int64_t(blockIdx.x) * 128 + threadIdx.x;
    if (idx >= P.M * groups) return;
    const int64_t m = idx / groups, g = idx - m * groups;
    const int64_t plane = P.M * int64_t(P.U);
    const float *src = partial + m * P.U + 8 * g;
    float z[8];
    {
        const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
        z[0] = a.x; z[1] = a.y; z[2] = a.z; z[3] = a.w; z[4] = b.x; z[5] = b.y; z[6] = b.z; z[7] = b.w;
    }
    for (int32_t s = 1; s < P.splits; ++s) {
        const float4 a = *reinterpret_cast<const float4 *>(src + s * plane), b = *reinterpret_cast<const float4 *>(src + s * plane + 4);
        z[0] += a.x; z[1] += a.y; z[2] += a.z; z[3] += a.w; z[4] += b.x; z[5] += b.y; z[6] += b.z; z[7] += b.w;
    }
    uint16_t *dst = y + m * P.out + 8 * g;
    for (int32_t t = 0; t < P.reps; ++t, dst += P.U) {
        const float al = alpha[P.n_alpha == 1 ? 0 : t];
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[e] = al * z[e];
            if (RELU) v[e] = fmaxf(v[e], 0.f);
        }
        *reinterpret_cast<u32x4_t *>(dst) = u32x4_t{pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
    }
}

int device_cus() {
    int device = 0, cus = 256;
    if (hipGetDevice(&device) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && v > 0) cus = v;
    }
    return cus;
}

void fill_params(const LinearArgs &a, BlockParams &P) {
    P.M = a.M;
    P.in = static_cast<int32_t>(a.in);
    P.out = static_cast<int32_t>(a.out);
    P.U = static_cast<int32_t>(a.p / a.in);
    P.reps = static_cast<int32_t>(a.out / P.U);
    P.n_alpha = a.n_alpha;
    P.tiles_m = static_cast<uint32_t>((a.M + kBM - 1) / kBM);
    P.tiles_n = (P.U + kBN - 1) / kBN;
    P.n_rounds = P.in / 128;
    P.splits = 1;
    P.vrows = P.tiles_m;
    P.partial = nullptr;
}

tbn_status set_lds_limit_once(const void *kernel, int lds) {
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return e == hipSuccess ? TBN_OK : TBN_ERR_DEVICE;
}

}  // namespace

// Shapes this kernel takes: bfloat16, tile of whole rows, K in whole pairs of rounds (in % 256 == 0), 16-byte
// stores possible, every offset inside a block in 32 bits.
bool linear_block_supported(const LinearArgs &a) {
    if (a.dt != TBN_BF16) return false;
    if (a.in % 256 != 0 || a.p % a.in != 0) return false;
    const int64_t U = a.p / a.in;
    if (U > a.out || a.out % U != 0) return false;   // (holds whenever p % in == 0; U = out / k)
    if (U % 8 != 0 || a.out / U > 64) return false;
    if (a.in > (1 << 20) || a.out > (1 << 22) || a.p >= (int64_t(1) << 31)) return false;
    if (a.M < 1 || a.M > (int64_t(1) << 36)) return false;
    if ((reinterpret_cast<uintptr_t>(a.x) & 15u) || (reinterpret_cast<uintptr_t>(a.y) & 15u)) return false;
    if (reinterpret_cast<uintptr_t>(a.tile) & 15u) return false;
    const int64_t blocks = ((a.M + kBM - 1) / kBM) * ((U + kBN - 1) / kBN);
    return blocks <= 0x7fffffffLL;
}

// Split K: how many workgroups share a block's K loop so that the grid about fills the chip (0: no split).  A part
// is a whole number of round pairs (256 elements of K) and at least one.  The split costs a second launch and a
// round trip of the float32 partial sums, about 12 us more fixed time than one kernel on MI355X, so it is taken
// only where a cost model fitted to measurements at 512 distinct columns predicts a gain of more than 10 %
// (R = in / 128 rounds; one kernel: 8 + 0.26 R (1 + blocks / 256) us on the streaming kernel's grids, 12 + 0.55 R us
// at 128 blocks and more; split: 20 + 0.55 R / S + 8 blocks / 128 us.  Measured, out = 4096, k = 8:
// in = 16384, batch 512 / 1024 / 2048 / 4096: 26 / 26 / 38 / 64 us against 40 / 44 / 47 / 72; in = 8192: equal;
// in = 4096: 22 / 22 / 25 / 31 against 15 / 16 / 17 / 27, not taken).  TBN_FLAG_SPLIT_K skips the model.
int linear_split_plan(const LinearArgs &a) {
    if (!linear_block_supported(a)) return 0;
    const int64_t U = a.p / a.in;
    const int64_t blocks = ((a.M + kBM - 1) / kBM) * ((U + kBN - 1) / kBN);
    const int64_t pairs = a.in / 256;
    const int cus = device_cus();
    int best = 0;
    for (int s = 2; s <= 16; s *= 2)
        if (blocks * s <= cus && pairs % s == 0) best = s;
    if (!best || (a.flags & TBN_FLAG_SPLIT_K)) return best;
    const double R = double(a.in) / 128.0;
    const double one = blocks <= 128 ? 8.0 + 0.26 * R * (1.0 + double(blocks) / 256.0) : 12.0 + 0.55 * R;
    const double split = 20.0 + 0.55 * R / best + 8.0 * double(blocks) / 128.0;
    return split < 0.9 * one ? best : 0;
}

size_t linear_split_workspace_bytes(const LinearArgs &a, int splits) {
    return static_cast<size_t>(splits) * static_cast<size_t>(a.M) * static_cast<size_t>(a.p / a.in) * sizeof(float);
}

tbn_status launch_linear_split(const LinearArgs &a, int splits, void *workspace) {
    BlockParams P;
    fill_params(a, P);
    P.splits = splits;
    P.n_rounds = P.in / 128 / splits;
    P.vrows = P.tiles_m * static_cast<uint32_t>(splits);
    P.partial = static_cast<float *>(workspace);
    const int64_t wgs = int64_t(P.vrows) * P.tiles_n;
    typedef void (*kernel_t)(const uint16_t *, uint16_t *, const uint32_t *, const float *, BlockParams);
    static const kernel_t kernel = &linear_block_bf16_kernel<false, true, false>;
    static const tbn_status attr = set_lds_limit_once(reinterpret_cast<const void *>(kernel), kLdsBytes);
    if (attr != TBN_OK) {
        set_error("tbn_linear_forward_ws: cannot reserve %d bytes of LDS for the block kernel", kLdsBytes);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(wgs)), dim3(512), kLdsBytes, a.stream,
                       static_cast<const uint16_t *>(a.x), static_cast<uint16_t *>(a.y), a.tile, a.alpha, P);
    tbn_status st = check_launch("tbn_linear_forward_ws (split-K matrix-core kernel)");
    if (st != TBN_OK) return st;
    const int64_t threads = a.M * (P.U / 8);
    const dim3 grid(static_cast<unsigned>((threads + 127) / 128));
    if (a.flags & TBN_FLAG_RELU)
        hipLaunchKernelGGL(linear_split_reduce_kernel<true>, grid, dim3(128), 0, a.stream, P.partial, static_cast<uint16_t *>(a.y), a.alpha, P);
    else
        hipLaunchKernelGGL(linear_split_reduce_kernel<false>, grid, dim3(128), 0, a.stream, P.partial, static_cast<uint16_t *>(a.y), a.alpha, P);
    return check_launch("tbn_linear_forward_ws (sum of the split-K partial sums)");
}

tbn_status launch_linear_block(const LinearArgs &a) {
    BlockParams P;
    fill_params(a, P);
    const dim3 grid(static_cast<unsigned>(int64_t(P.tiles_m) * P.tiles_n));
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    typedef void (*kernel_t)(const uint16_t *, uint16_t *, const uint32_t *, const float *, BlockParams);
    // more blocks than CUs and at least four rounds: one persistent workgroup per CU
    int cus = device_cus() & ~7;
    if (cus < 8) cus = 8;
    const bool persist = int64_t(P.tiles_m) * P.tiles_n > cus && P.n_rounds >= 4;
    // (its store waves write with non-temporal stores whatever the shape: next to a running K loop, plain stores push
    // the activations that the other column blocks of the same rows still need out of the XCD's L2)
    static const kernel_t kernels[4] = {&linear_block_bf16_kernel<false, false, false>, &linear_block_bf16_kernel<true, false, false>,
                                        &linear_block_bf16_kernel<false, false, true>, &linear_block_bf16_kernel<true, false, true>};
    // dynamic LDS above the default limit has to be allowed once per kernel (thread-safe static initialisation)
    static const tbn_status attr[4] = {set_lds_limit_once(reinterpret_cast<const void *>(kernels[0]), kLdsBytes),
                                       set_lds_limit_once(reinterpret_cast<const void *>(kernels[1]), kLdsBytes),
                                       set_lds_limit_once(reinterpret_cast<const void *>(kernels[2]), kLdsBytes),
                                       set_lds_limit_once(reinterpret_cast<const void *>(kernels[3]), kLdsBytes)};
    const int which = (relu ? 1 : 0) + (persist ? 2 : 0);
    if (attr[which] != TBN_OK) {
        set_error("tbn_linear_forward: cannot reserve %d bytes of LDS for the block kernel", kLdsBytes);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL(kernels[which], persist ? dim3(static_cast<unsigned>(cus)) : grid, dim3(512), kLdsBytes, a.stream,
                       static_cast<const uint16_t *>(a.x), static_cast<uint16_t *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward (matrix-core kernel with load waves)");
}

}  // namespace tbn
