// Kernel for the fully-connected tiled-bit layer with a tile of whole weight rows (p % in == 0) and few distinct
// rows or few batch rows: one wave per 32 batch rows, many small workgroups, no workgroup-wide pipeline.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8): with p a multiple of `in` only the
// U = p / in rows of the tile are distinct; Z = X * T^T (M x U) is formed once and Y[:, t*U + u] = alpha[t] * Z[:, u].
//
// Why another kernel.  (1) The layers that come with float32 activations (the MLP of a small vision transformer,
// 384 -> 1536 -> 384 on 12608 tokens, k = 4) have short rows and few distinct columns.  They move about 100 MB
// for 5 us of matrix work, so what counts is how many bytes are in flight, not how the matrix pipe is fed; a
// workgroup that owns a 128 x 128 block with a deep LDS pipeline spends its time filling and draining that
// pipeline (297 or 99 blocks of 20 us each on 256 CUs).  (2) bfloat16 layers at a few hundred batch rows give the
// block kernels 16 - 64 blocks for 256 CUs, each running the whole K loop alone.  Here
//   * a wave owns 32 batch rows and up to 128 distinct columns over one K slice; the workgroup's waves (1, 4 or 8)
//     take different K slices and add their sums through LDS at the end (in wave order: the result does not depend
//     on timing), so that a layer with 99 row blocks of 128, or a batch of 512 on a 4096 x 4096 layer, still puts
//     more than 1000 waves on the chip's 1024 SIMDs;
//   * a load instruction reads whole 128-byte lines (eight lanes per row); a chunk of 256 bytes per row (64 floats,
//     128 bfloat16) of the wave's 32 rows passes through 8 KiB of LDS that only this wave touches, to reach the
//     operand layout (a lane of the matrix instruction holds eight consecutive elements of one row), while the next
//     chunk's loads are in flight; no barrier in the K loop;
//   * every float is split exactly into three bfloat16 terms (8 + 8 + 8 significand bits); the weights are +-1,
//     so every product is exact and the sums are float32 accumulations in the matrix pipe
//     (v_mfma_f32_32x32x16_bf16, three per column tile and step; one for bfloat16 activations);
//   * the +-1 operand comes from the tile bits through a 256-entry table in LDS (one read per operand); K is
//     consumed in an order that suits the loads: lane half lg takes the elements of its half of the chunk, eight
//     per step, for both operands alike;
//   * the sums are turned round through LDS, 32 x 32 at a time, so that a store instruction writes whole
//     lines of Y (a lane of the accumulator layout holds four adjacent columns of one row only).
#include "tbn_common.h"

#include <type_traits>

namespace tbn {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));   // round to nearest even in hardware
}

union Frag {
    bf16x8_t v;
    u32x4_t q;
};

constexpr int kChunkBytes = 256;   // bytes of a row per chunk: 64 floats (four MFMA steps) or 128 bfloat16 (eight)
template <typename XT> constexpr int chunk_elems() { return kChunkBytes / static_cast<int>(sizeof(XT)); }
constexpr int kMaxNT = 4;       // column tiles of 32 per wave (two or three measure 3 - 50 % slower: more waves read X again)

struct TileParams {
    int64_t M;
    int32_t in, out, U;
    int32_t reps, n_alpha;
    int32_t col_groups;   // groups of NT * 32 distinct columns
    uint32_t row_tiles;   // tiles of 32 batch rows
    int32_t k_per_wave;   // K slice of a wave (whole chunks)
};

// truncation split of eight floats into three bf16x8 operands: term 0 = top 8 significand bits, term 1 = the next 8,
// term 2 = the rest (at most 8 bits, so its truncation to bfloat16 is exact)
__device__ __forceinline__ void split8(const float (&x)[8], Frag (&t)[3]) {
    uint32_t h[3][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t t0 = __float_as_uint(x[i]) & 0xffff0000u;
        const float r1 = x[i] - __uint_as_float(t0);
        const uint32_t t1 = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(t1);
        h[0][i] = t0; h[1][i] = t1; h[2][i] = __float_as_uint(r2);
    }
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v)   // high halves of two words in one: (lo >> 16) | (hi & 0xffff0000)
            t[j].q[v] = __builtin_amdgcn_perm(h[j][2 * v + 1], h[j][2 * v], 0x07060302u);
}

// LDS of a workgroup: the sign table, then one region per wave.  During the K loop a wave's region holds its
// current chunk of X, 32 rows of 256 bytes with the 16-byte pieces of a row XOR-swizzled by the row number (so that
// both the row-wise writes and the column-wise operand reads spread over the banks); afterwards the regions hold
// the partial sums that the waves hand over, and at last the 32 x 32 block a wave turns round for its stores.
template <int NT, int KW>
struct Lds {
    static constexpr int SL = (NT == KW) ? NT - 1 : NT;   // hand-over slots per wave: a wave keeps the tile it finishes
    static constexpr int kStage = 8192;                    // bytes per wave during the loop
    static constexpr int kPart = KW > 1 ? SL * 4096 : 0;
    static constexpr int kRegion = kStage > kPart ? kStage : kPart;
    static constexpr int kBytes = 4096 + KW * kRegion;
};

template <typename XT, bool RELU, int NT, int KW>
__global__ __launch_bounds__(64 * KW) void linear_tile_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                              const uint32_t *__restrict__ tile,
                                                              const float *__restrict__ alpha, TileParams P) {
    typedef Lds<NT, KW> L;
    constexpr bool kF32 = std::is_same<XT, float>::value;
    constexpr int kCE = chunk_elems<XT>();          // elements of K per chunk
    constexpr int kSteps = kCE / 16;                // MFMA steps per chunk
    constexpr int kWords = kCE / 64;                // tile words per lane half, column and chunk
    extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
    u32x4_t *s_table = reinterpret_cast<u32x4_t *>(s_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, lg = lane >> 5;
    unsigned char *region_b = s_raw + 4096 + wave * L::kRegion;   // this wave's
    float *region = reinterpret_cast<float *>(region_b);

    // sign table: entry e, element i is +1 if bit i of e is set, else -1
    for (int e = tid; e < 256; e += 64 * KW) {
        u32x4_t t;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            t[v] = (((e >> (2 * v)) & 1) ? 0x3f80u : 0xbf80u) | ((((e >> (2 * v + 1)) & 1) ? 0x3f80u : 0xbf80u) << 16);
        s_table[e] = t;
    }
    __syncthreads();

    // Workgroup ids are dealt round-robin to the 8 XCDs: the column groups of one row tile take consecutive slots of
    // one XCD, so that the rows of X they share are fetched from HBM once and then found in that XCD's L2 (plain order
    // fetched X once per column group: 58 MB instead of 19 on 12608 x 384 -> 1536, float32).
    uint32_t rt;
    int32_t cg;
    {
        const uint32_t bid = blockIdx.x, groups = static_cast<uint32_t>(P.col_groups), xcd = bid & 7, slot = bid >> 3;
        const uint32_t full = (P.row_tiles / 8) * groups;   // slots per XCD in the regular part
        if (slot < full) {
            const uint32_t q = slot / groups;
            cg = static_cast<int32_t>(slot - q * groups);
            rt = q * 8 + xcd;
        } else {   // the remaining row tiles: plain order
            const uint32_t rest = bid - full * 8, q = rest / groups;
            cg = static_cast<int32_t>(rest - q * groups);
            rt = (P.row_tiles / 8) * 8 + q;
        }
    }
    const int64_t m0 = int64_t(rt) * 32;
    const int32_t u0 = cg * (NT * 32);
    const int32_t k_begin = wave * P.k_per_wave;

    // loads: instruction (i, h) of a chunk reads rows 8i + lane/8, bytes 128h + 16*(lane%8) .. + 15 of the chunk's 256:
    // eight lanes cover a whole 128-byte line.  Rows past M repeat the last one; they are never written.
    const unsigned char *x_blk = reinterpret_cast<const unsigned char *>(x + m0 * P.in + k_begin);
    const int64_t last = P.M - 1 - m0;   // >= 0
    uint32_t ld_off[4];                  // byte offsets from x_blk
    uint32_t st_pos[4][2];               // byte positions in the wave's region
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 8 * i + (lane >> 3);
        ld_off[i] = static_cast<uint32_t>(r < last ? r : last) * static_cast<uint32_t>(P.in) * static_cast<uint32_t>(sizeof(XT)) +
                    static_cast<uint32_t>(16 * (lane & 7));
#pragma unroll
        for (int h = 0; h < 2; ++h) st_pos[i][h] = static_cast<uint32_t>(r * 256 + (((8 * h + (lane & 7)) ^ (r & 15)) << 4));
    }
    // operand reads of row ln.  float32: step s of lane half lg takes floats 32*lg + 8*s .. + 7, pieces 8*lg + 2*s and + 1;
    // bfloat16: elements 64*lg + 8*s .. + 7, piece 8*lg + s.
    constexpr int kReads = kF32 ? 2 : 1;
    uint32_t rd_pos[kSteps][kReads];
#pragma unroll
    for (int s4 = 0; s4 < kSteps; ++s4)
#pragma unroll
        for (int j = 0; j < kReads; ++j)
            rd_pos[s4][j] = static_cast<uint32_t>(ln * 256 + (((8 * lg + kReads * s4 + j) ^ (ln & 15)) << 4));

    // tile words of this lane's column in every column tile: bit u * in + k; a lane half covers kWords words per chunk
    const uint32_t *tp[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int32_t u = u0 + 32 * t + ln;
        u = u < P.U ? u : P.U - 1;   // columns past U repeat the last one; never written
        tp[t] = tile + ((int64_t(u) * P.in + k_begin) >> 5) + kWords * lg;
    }

    f32x16_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

    // one chunk ahead: requesting two or four chunks before the first use measured 5 - 10 % slower at small batches
    u32x4_t xr[8];        // the chunk in flight: [i][h]
    uint32_t wr[NT][kWords];
    auto load_chunk = [&](int32_t c) {
        const unsigned char *src = x_blk + c * kChunkBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) xr[2 * i + h] = *reinterpret_cast<const u32x4_t *>(src + ld_off[i] + 128 * h);
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int w = 0; w < kWords; ++w) wr[t][w] = tp[t][c * 2 * kWords + w];
    };

    const int32_t chunks = P.k_per_wave / kCE;   // >= 1
    load_chunk(0);
    for (int32_t c = 0; c < chunks; ++c) {
        // the chunk goes to LDS, the next one is requested, then this one is multiplied from LDS
        uint32_t wc[NT][kWords];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int w = 0; w < kWords; ++w) wc[t][w] = wr[t][w];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) *reinterpret_cast<u32x4_t *>(region_b + st_pos[i][h]) = xr[2 * i + h];
        __builtin_amdgcn_wave_barrier();   // lanes read what other lanes of the wave wrote (LDS operations of a wave stay in order)
        if (c + 1 < chunks) load_chunk(c + 1);
#pragma unroll
        for (int s4 = 0; s4 < kSteps; ++s4) {
            constexpr int kTerms = kF32 ? 3 : 1;
            Frag xt[kTerms];
            if constexpr (kF32) {
                const f32x4_t a = *reinterpret_cast<const f32x4_t *>(region_b + rd_pos[s4][0]);
                const f32x4_t b = *reinterpret_cast<const f32x4_t *>(region_b + rd_pos[s4][kReads - 1]);
                const float xs[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
                split8(xs, xt);
            } else {
                xt[0].q = *reinterpret_cast<const u32x4_t *>(region_b + rd_pos[s4][0]);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                Frag sg;
                sg.q = s_table[(wc[t][s4 / 4] >> (8 * (s4 % 4))) & 0xffu];
#pragma unroll
                for (int j = 0; j < kTerms; ++j)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sg.v, xt[j].v, acc[t], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();   // the next chunk overwrites the region
    }

    // ---- the waves of the workgroup add their K slices: wave w ends up with column tile w ------------------------
    // (sums in ascending wave order whatever the timing: results are the same from run to run)
    int t_mine = 0;            // column tiles this wave writes: [t_mine, t_end)
    int t_end = NT;
    if constexpr (KW > 1) {
        static_assert(KW >= NT, "every column tile needs a wave");
        constexpr int SL = L::SL;
        __syncthreads();   // every wave is done with its chunk: the regions change their use
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (t == wave) continue;                       // kept in registers
            const int slot = (NT == KW && t > wave) ? t - 1 : t;
#pragma unroll
            for (int r = 0; r < 16; ++r) region[(slot * 16 + r) * 64 + lane] = acc[t][r];
        }
        __syncthreads();
        t_mine = wave;
        t_end = wave < NT ? wave + 1 : wave;   // waves past NT write nothing
        if (wave < NT) {
            f32x16_t sum;
            bool first = true;
#pragma unroll
            for (int w = 0; w < KW; ++w) {
                f32x16_t v;
                if (w == wave) {
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        if (t == wave) v = acc[t];
                } else {
                    const int slot = (NT == KW && wave > w) ? wave - 1 : wave;
                    const float *other = reinterpret_cast<const float *>(s_raw + 4096 + w * L::kRegion);
#pragma unroll
                    for (int r = 0; r < 16; ++r) v[r] = other[(slot * 16 + r) * 64 + lane];
                }
                if (first) { sum = v; first = false; }
                else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum[r] += v[r];
                }
            }
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (t == wave) acc[t] = sum;
        }
        __syncthreads();   // all hand-over reads are done: a wave's region is its own again
        (void)SL;
    }

    // ---- y[m, u + t*U] = alpha[t] * Z[m, u] ----------------------------------------------------------------------
    // Register 4q + e of a column tile is column 8q + 4lg + e of row ln.  The wave turns every 32 x 32 tile round
    // through its region (row r at r * 128 bytes, 16-byte piece c at position c ^ (r & 7)) so that a few lanes hold a
    // row's 32 columns: eight lanes with four float32 each, or four lanes with eight bfloat16 each, and a store
    // instruction writes whole lines.
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (t < t_mine || t >= t_end) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<f32x4_t *>(region + ln * 32 + (((2 * q + lg) ^ (ln & 7)) << 2)) =
                f32x4_t{acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if constexpr (kF32) {
            const int r8 = lane >> 3, c8 = lane & 7;
            f32x4_t z[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = r8 + 8 * i;
                z[i] = *reinterpret_cast<const f32x4_t *>(region + r * 32 + ((c8 ^ (r & 7)) << 2));
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the next tile overwrites the region
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int32_t u = u0 + 32 * t + 4 * c8;
            if (u >= P.U) continue;   // U % 4 == 0: a group of four is inside or outside
            for (int32_t rep = 0; rep < P.reps; ++rep) {
                const float al = alpha[P.n_alpha == 1 ? 0 : rep];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t m = m0 + r8 + 8 * i;
                    if (m >= P.M) continue;
                    f32x4_t v = al * z[i];
                    if (RELU) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
                    f32x4_t *dst = reinterpret_cast<f32x4_t *>(y + m * P.out + int64_t(rep) * P.U + u);
                    // Non-temporal where K is split among the waves of a workgroup (long rows: the layer then reads more
                    // than it writes and the output should not push X out of the L2: 12608 x 1536 -> 384 20.1 us against
                    // 21.3); plain otherwise (384 -> 1536: 27.0 against 28.7 non-temporal).  A compile-time choice: the
                    // compiler merges the two stores of a run-time one into a plain store.
                    if constexpr (KW > 1) __builtin_nontemporal_store(v, dst);
                    else *dst = v;
                }
            }
        } else {
            const int r4 = lane >> 2, c4 = lane & 3;   // row of 16, eight columns 8*c4 .. + 7: pieces 2*c4 and 2*c4 + 1
            f32x4_t za[2], zb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = r4 + 16 * i;
                za[i] = *reinterpret_cast<const f32x4_t *>(region + r * 32 + (((2 * c4) ^ (r & 7)) << 2));
                zb[i] = *reinterpret_cast<const f32x4_t *>(region + r * 32 + (((2 * c4 + 1) ^ (r & 7)) << 2));
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the next tile overwrites the region
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int32_t u = u0 + 32 * t + 8 * c4;
            if (u >= P.U) continue;   // U % 8 == 0: a group of eight is inside or outside
            for (int32_t rep = 0; rep < P.reps; ++rep) {
                const float al = alpha[P.n_alpha == 1 ? 0 : rep];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int64_t m = m0 + r4 + 16 * i;
                    if (m >= P.M) continue;
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[e] = al * za[i][e]; v[4 + e] = al * zb[i][e]; }
                    if (RELU) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
                    }
                    const u32x4_t pk = {pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
                    *reinterpret_cast<u32x4_t *>(y + m * P.out + int64_t(rep) * P.U + u) = pk;
                }
            }
        }
    }
}

template <typename XT, bool RELU, int NT, int KW>
tbn_status launch_one(const LinearArgs &a, const TileParams &P, unsigned grid) {
    typedef Lds<NT, KW> L;
    // dynamic LDS above the default limit has to be allowed once per kernel (thread-safe static initialisation)
    static const hipError_t attr = L::kBytes > 65536
        ? hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_tile_kernel<XT, RELU, NT, KW>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes)
        : hipSuccess;
    if (attr != hipSuccess) {
        set_error("tbn_linear_forward: cannot reserve %d bytes of LDS", L::kBytes);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL((linear_tile_kernel<XT, RELU, NT, KW>), dim3(grid), dim3(64 * KW), L::kBytes, a.stream,
                       static_cast<const XT *>(a.x), static_cast<XT *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward (one wave per 32 batch rows)");
}

template <typename XT, bool RELU, int NT>
tbn_status launch_kw(const LinearArgs &a, const TileParams &P, unsigned grid, int kw) {
    if (kw == 8) return launch_one<XT, RELU, NT, 8>(a, P, grid);
    if (kw == 4) return launch_one<XT, RELU, NT, 4>(a, P, grid);
    return launch_one<XT, RELU, NT, 1>(a, P, grid);
}

template <typename XT, bool RELU>
tbn_status launch_nt(const LinearArgs &a, const TileParams &P, unsigned grid, int nt, int kw) {
    if (nt == 1) return launch_kw<XT, RELU, 1>(a, P, grid, kw);
    if (nt == 2) return launch_kw<XT, RELU, 2>(a, P, grid, kw);
    if constexpr (std::is_same<XT, float>::value) {   // the plan gives bfloat16 at most two tiles per wave
        if (nt == 3) return launch_kw<XT, RELU, 3>(a, P, grid, kw);
        return launch_kw<XT, RELU, 4>(a, P, grid, kw);
    }
    set_error("tbn_linear_forward: no kernel for %d column tiles per wave", nt);
    return TBN_ERR_UNSUPPORTED;
}

// column tiles per wave: as few groups as possible, then as even as possible (float32, U = 384: three groups of four, see below
// tiles; U = 96: one group of three; bfloat16 takes at most two tiles per wave: its use is small batches, where more
// waves count for more than fewer passes over X: 4096 x 4096, k = 8 at batch 256 / 512 9.3 / 10.3 us against 13.6 /
// 14.0 with four); K slices per workgroup: as many (8, 4) as leave a wave at least two chunks and the chip at most
// about two waves per SIMD
void plan(const LinearArgs &a, int &nt, int &groups, int &kw) {
    const int64_t U = a.p / a.in;
    const int64_t tiles = (U + 31) / 32;
    const int max_nt = a.dt == TBN_F32 ? kMaxNT : 2;
    groups = static_cast<int>((tiles + max_nt - 1) / max_nt);
    nt = static_cast<int>((tiles + groups - 1) / groups);
    const int64_t ce = a.dt == TBN_F32 ? chunk_elems<float>() : chunk_elems<uint16_t>();
    const int64_t waves1 = ((a.M + 31) / 32) * groups;
    kw = 1;
    for (int cand : {8, 4}) {
        if (a.in % (cand * ce) == 0 && a.in / cand >= 2 * ce && waves1 * cand <= 2048 && cand >= nt) {
            kw = cand;
            break;
        }
    }
    // float32 with K in one slice (one wave per workgroup) and fewer than one and a half waves per SIMD: one more
    // column group where the tiles divide evenly, for more waves in flight (12608 x 384 -> 384 distinct columns: four
    // groups of three tiles 25.8 us against three groups of four 27.8; with more waves the extra pass over X costs more
    // than it gains: 1536 distinct columns 51.4 against 49.5)
    if (a.dt == TBN_F32 && kw == 1 && waves1 < 1536 && nt > 2 && tiles % (groups + 1) == 0) {
        groups += 1;
        nt = static_cast<int>(tiles / groups);
    }
}

}  // namespace

// Shapes this kernel takes: tile of whole rows, K in chunks of 256 bytes, 16-byte loads and stores possible.  Every
// group of 64 (bfloat16) or up to 128 (float32) distinct columns reads its rows of X again, from L2: with many distinct
// columns the kernel is for small batches only, which linear_tile_preferred and the dispatch see to.
bool linear_tile_supported(const LinearArgs &a) {
    if (a.dt != TBN_F32 && a.dt != TBN_BF16) return false;
    const int64_t ce = a.dt == TBN_F32 ? chunk_elems<float>() : chunk_elems<uint16_t>();
    if (a.in % ce != 0 || a.p % a.in != 0) return false;
    const int64_t U = a.p / a.in;
    if (U > a.out || a.out % U != 0 || U % (a.dt == TBN_F32 ? 4 : 8) != 0 || U > (1 << 20)) return false;
    if (a.in > (1 << 20) || a.out > (1 << 22) || a.p >= (int64_t(1) << 36)) return false;
    if (a.M < 1 || a.M > (int64_t(1) << 34)) return false;
    if ((reinterpret_cast<uintptr_t>(a.x) & 15u) || (reinterpret_cast<uintptr_t>(a.y) & 15u)) return false;
    int nt, groups, kw;
    plan(a, nt, groups, kw);
    return ((a.M + 31) / 32) * groups <= 0x7fffffffLL;
}

// bfloat16: where this kernel beats the small-batch, the streaming and the block kernels.  Graph replays, microseconds
// per call, this kernel / what the dispatch would take otherwise:
//   * at least four K slices and at most about two waves per SIMD.  512 distinct columns, in = 4096, batch 256 / 512 /
//     1024 / 2048: 8.8 / 8.9 / 10.3 / 15.8 against 16.6 / 15.6 / 15.0 / 15.4; in = 2048, batch 1024 / 2048: 7.2 / 10.5
//     against 10.7 / 10.9; 128 distinct columns, batch 4096, in = 2048 / 4096: 7.2 / 10.4 against 10.7 / 17.8.  Batch
//     17 - 64, 512 distinct columns, in = 1024 / 1536 / 2048 / 3072 / 8192: 5.1 / 5.6 / 6.3 / 7.4 / 12.8 against 7.9 / 7.5 /
//     8.0 / 8.1 / 13.6 for the small-batch kernel; at in = 4096 that kernel keeps those batches (8.3 against 8.5).
//     The number of distinct columns is not limited: 4096 of them at batch 100 / 256, in = 1024: 5.4 / 7.3 against
//     10.6 / 10.0 with the streaming kernel, in = 4096: 9.0 / 15.1 against 20.4 / 20.6;
//   * short rows (fewer K slices), up to 512 waves, where the small-batch kernel would need more than one workgroup
//     per CU: in = 512, 512 distinct columns, batch 512 / 1024 / 2048: 6.0 / 6.4 / 7.2 against 7.4 / 7.6 / 7.7 (batch
//     4096: 9.4 against 9.0, left to the block kernel); batch 160 / 256, in = 256 / 768: 4.7 / 7.0 against 6.7 - 6.9 /
//     11.0 - 11.4 (with 256 workgroups or fewer the small-batch kernel is the faster one: 4.2 / 6.4 against 4.7 / 7.1).
// float32: the small-batch kernel's time grows with every further 256 workgroups (one per CU), this kernel's hardly
// with the batch.  512 distinct columns, batch 197 / 400 / 800, this kernel / the small-batch kernel: in = 1024:
// 10.1 / 10.3 / 10.6 against 14.0 / 26.5 / 46.0; in = 4096: 23.0 / 23.2 / 23.6 against 24.2 / 47.0 / 80.8; in = 384:
// 12.6 / 12.8 / 13.2 against 8.3 / 15.2 / 25.6.  So: more than 512 of its workgroups, or more than 256 with rows of at
// least 1024.
bool linear_tile_preferred(const LinearArgs &a) {
    if (a.M <= 16 || !linear_tile_supported(a)) return false;
    if (a.dt == TBN_F32) {
        const int64_t grid = ((a.p / a.in + 15) / 16) * ((a.M + 15) / 16);   // workgroups of the small-batch kernel
        return a.M > 64 && grid <= 2048 && (grid > 512 || (grid > 256 && a.in >= 1024));   // beyond 2048 that kernel declines
    }
    int nt, groups, kw;
    plan(a, nt, groups, kw);
    const int64_t waves1 = ((a.M + 31) / 32) * groups;
    if (kw >= 4) return waves1 * kw <= 2048 && (a.M > 64 || a.in < 4096 || a.in >= 8192);
    const int64_t U = a.p / a.in;
    const int64_t small_grid = ((U + 15) / 16) * ((a.M + 15) / 16);   // workgroups of the small-batch kernel
    return a.M > 64 && small_grid > 256 && waves1 <= 512;
}

tbn_status launch_linear_tile(const LinearArgs &a) {
    TileParams P;
    P.M = a.M;
    P.in = static_cast<int32_t>(a.in);
    P.out = static_cast<int32_t>(a.out);
    P.U = static_cast<int32_t>(a.p / a.in);
    P.reps = static_cast<int32_t>(a.out / P.U);
    P.n_alpha = a.n_alpha;
    int nt, groups, kw;
    plan(a, nt, groups, kw);
    P.col_groups = groups;
    P.row_tiles = static_cast<uint32_t>((a.M + 31) / 32);
    P.k_per_wave = P.in / kw;
    const unsigned grid = static_cast<unsigned>(((a.M + 31) / 32) * groups);
    const bool relu = (a.flags & TBN_FLAG_RELU) != 0;
    if (a.dt == TBN_F32) return relu ? launch_nt<float, true>(a, P, grid, nt, kw) : launch_nt<float, false>(a, P, grid, nt, kw);
    return relu ? launch_nt<uint16_t, true>(a, P, grid, nt, kw) : launch_nt<uint16_t, false>(a, P, grid, nt, kw);
}

}  // namespace tbn
