// Matrix-core kernel for the fully-connected tiled-bit layer at medium and large batch.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8; Algorithm 1 gives the
// same sums with a running index): the (out x in) weight is the tile repeated along the
// flattened index, so weight row o carries the cyclic tile window that starts at bit
// (o*in) % p.  That start repeats with period U = p / gcd(in, p) rows, hence only U distinct
// +-1 rows exist.  The kernel forms Z = X * T_U^T for those U rows once and writes every output
// column o = u + t*U as alpha(o) * Z[:, u] -- the "compute one tile, replicate the others"
// observation the paper makes for convolution channels, applied to matrix columns.
//
// gfx950 mapping
//   * one workgroup (4 waves, 2 x 2) owns a 128 x 128 block of Z; X is staged in LDS as bf16 and
//     read back as operands of v_mfma_f32_32x32x16_bf16; a ring of stages is kept in flight in
//     registers between global memory and LDS so that HBM latency is covered even when only one
//     workgroup fits the problem per CU;
//   * float32 activations are split exactly into three bf16 terms (8 + 8 + 8 significand bits;
//     the weights are +-1, so each product is exact and the sums are float32 accumulations);
//   * the +-1 operand never exists in memory: 32-bit tile windows (shifted to the row's start
//     bit, continued at the tile start after the tile end) are staged in LDS with even and odd
//     bits separated, so that the two bits of a packed bf16 pair sit 16 apart and one shift plus
//     one and-or turns a window into an operand register;
//   * the epilogue scales by alpha and writes the replicated column blocks straight from the
//     accumulators; a lane owns adjacent columns so that a half-wave writes a contiguous run.
// Rows whose weights straddle a tile end use two different alphas when one alpha per tile is
// given; those few columns are recomputed afterwards by the row kernel (see tbn_linear_rows.hip).
#include "tbn_common.h"

namespace tbn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;
constexpr int kWavesM = 2, kWavesN = 2;
constexpr int kTM = 2, kTN = 2;                  // 32x32 MFMA tiles per wave along M and N
constexpr int kBM = kWavesM * kTM * 32;          // 128
constexpr int kBN = kWavesN * kTN * 32;          // 128
constexpr int kBK = 64;                          // K elements per pipeline stage
constexpr int kKB = kBK / 32;                    // 32-bit tile windows per stage and row
constexpr int kPieces = kBK / 8;                 // 8-element (16-byte bf16) pieces per row and stage
constexpr int kRowStride = kBK + 8;              // LDS row stride in bf16 elements (16 B of padding)
constexpr int kPlaneElems = kBM * kRowStride;
constexpr int kItems = kBM * kPieces / kThreads; // pieces staged per thread and stage

union Frag {
    bf16x8_t v;
    uint32_t u[4];
    uint4 q;
};

template <typename XT> struct Traits;
template <> struct Traits<uint16_t> {
    static constexpr int planes = 1;   // bf16 activations go to LDS as they are
    static constexpr int depth = 3;    // stages in flight in registers
    struct Piece { uint4 v; };
    static __device__ __forceinline__ void load(Piece &r, const uint16_t *src) {
        r.v = *reinterpret_cast<const uint4 *>(src);
    }
    static __device__ __forceinline__ void zero(Piece &r) { r.v = make_uint4(0, 0, 0, 0); }
    static __device__ __forceinline__ void store(const Piece &r, uint16_t *dst) {
        *reinterpret_cast<uint4 *>(dst) = r.v;
    }
};
template <> struct Traits<float> {
    static constexpr int planes = 3;   // exact split x = t0 + t1 + t2 into bf16 terms
    static constexpr int depth = 2;
    struct Piece { float4 a, b; };
    static __device__ __forceinline__ void load(Piece &r, const float *src) {
        r.a = *reinterpret_cast<const float4 *>(src);
        r.b = *reinterpret_cast<const float4 *>(src + 4);
    }
    static __device__ __forceinline__ void zero(Piece &r) {
        r.a = make_float4(0.f, 0.f, 0.f, 0.f);
        r.b = r.a;
    }
    // truncation split: t0 = top 8 significand bits, t1 = next 8, t2 = the rest (at most 8 bits)
    static __device__ __forceinline__ void split3(float x, uint32_t &t0, uint32_t &t1, uint32_t &t2) {
        t0 = __float_as_uint(x) & 0xffff0000u;
        const float r1 = x - __uint_as_float(t0);
        t1 = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(t1);
        t2 = __float_as_uint(r2);
    }
    static __device__ __forceinline__ void store(const Piece &r, uint16_t *dst) {
        const float x[8] = {r.a.x, r.a.y, r.a.z, r.a.w, r.b.x, r.b.y, r.b.z, r.b.w};
        uint32_t o[3][4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t e0, e1, e2, f0, f1, f2;
            split3(x[2 * d], e0, e1, e2);
            split3(x[2 * d + 1], f0, f1, f2);
            o[0][d] = (e0 >> 16) | f0;
            o[1][d] = (e1 >> 16) | f1;
            o[2][d] = (e2 >> 16) | (f2 & 0xffff0000u);
        }
#pragma unroll
        for (int pl = 0; pl < 3; ++pl)
            *reinterpret_cast<uint4 *>(dst + pl * kPlaneElems) = make_uint4(o[pl][0], o[pl][1], o[pl][2], o[pl][3]);
    }
};

// even bits of x to the low half, odd bits to the high half (both in order)
__device__ __forceinline__ uint32_t unshuffle_bits(uint32_t x) {
    uint32_t t;
    t = (x ^ (x >> 1)) & 0x22222222u; x ^= t ^ (t << 1);
    t = (x ^ (x >> 2)) & 0x0c0c0c0cu; x ^= t ^ (t << 2);
    t = (x ^ (x >> 4)) & 0x00f000f0u; x ^= t ^ (t << 4);
    t = (x ^ (x >> 8)) & 0x0000ff00u; x ^= t ^ (t << 8);
    return x;
}

template <typename OT> struct OutPack;
template <> struct OutPack<uint16_t> {
    static __device__ __forceinline__ void store2(uint16_t *p, float a, float b) {
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        typedef float f32x2_t __attribute__((ext_vector_type(2)));
        const f32x2_t f = {a, b};
        const bf16x2_t h = __builtin_convertvector(f, bf16x2_t);   // round to nearest even in hardware
        *reinterpret_cast<bf16x2_t *>(p) = h;
    }
};
template <> struct OutPack<float> {
    static __device__ __forceinline__ void store2(float *p, float a, float b) {
        *reinterpret_cast<float2 *>(p) = make_float2(a, b);
    }
};

struct MfmaParams {
    int64_t M, in, out, p, n_words, U;
    int32_t n_alpha;
    int relu;
    int aligned;      // p % in == 0: alpha index of column o is o / U
    int vec_store;    // adjacent column pairs can be written with one aligned vector store
    int tiles_n;      // column blocks of U
    int64_t tiles_m;
};

template <typename XT, bool RELU>
__global__ __launch_bounds__(kThreads, 2) void linear_mfma_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                               const uint32_t *__restrict__ tile,
                                                               const float *__restrict__ alpha, MfmaParams P) {
    using T = Traits<XT>;
    constexpr int NP = T::planes;
    constexpr int D = T::depth;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    typedef uint16_t (*LdsA)[NP][kPlaneElems];
    typedef uint32_t (*LdsBits)[kKB][kBN];
    LdsA lds_a = reinterpret_cast<LdsA>(lds_raw);
    LdsBits lds_bits = reinterpret_cast<LdsBits>(lds_raw + sizeof(uint16_t) * 2 * NP * kPlaneElems);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / kWavesN, wn = wave % kWavesN;
    const int ln = lane & 31;   // column (B operand) / row (A operand) inside a 32 x 32 tile
    const int lg = lane >> 5;   // K half of the operand registers

    // Workgroups that share rows of X are given consecutive slots on one XCD (workgroup ids are
    // dealt round-robin to the 8 XCDs), so the later column blocks find X in that XCD's L2.
    int64_t tile_m, tile_n;
    {
        const int64_t bid = blockIdx.x;
        const int64_t xcd = bid & 7, slot = bid >> 3;
        const int64_t per_xcd_full = (P.tiles_m / 8) * P.tiles_n;   // slots per XCD in the regular part
        if (slot < per_xcd_full) {
            tile_n = slot % P.tiles_n;
            tile_m = (slot / P.tiles_n) * 8 + xcd;
        } else {  // remaining row blocks: plain order
            const int64_t rest = bid - per_xcd_full * 8;
            tile_n = rest % P.tiles_n;
            tile_m = (P.tiles_m / 8) * 8 + rest / P.tiles_n;
        }
    }
    const int64_t m0 = tile_m * kBM;
    const int64_t n0 = tile_n * kBN;

    // ---- staging assignments ---------------------------------------------------------------
    // activations: item i of a thread = 8 consecutive columns (one 16-byte bf16 piece) of one row;
    // 8 consecutive threads cover the 64 columns of a row.  Rows past M are clamped to row M-1
    // (their results are never written).
    const int a_piece = tid % kPieces;
    const XT *a_src[kItems];
    int a_lds[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int r = tid / kPieces + i * (kThreads / kPieces);
        const int64_t m = (m0 + r) < P.M ? (m0 + r) : (P.M - 1);
        a_src[i] = x + m * P.in;
        a_lds[i] = r * kRowStride + a_piece * 8;
    }
    // tile windows: one (column, window) per thread and stage (kBN * kKB == kThreads)
    static_assert(kBN * kKB == kThreads, "one tile window per thread and stage");
    const int b_col = tid % kBN, b_kb = tid / kBN;
    const bool b_ok = (n0 + b_col) < P.U;
    int64_t b_pos = 0;  // cyclic bit position of this thread's window at k0 = 0
    if (b_ok) {
        b_pos = ((n0 + b_col) * P.in) % P.p + b_kb * 32;
        if (b_pos >= P.p) b_pos -= P.p;
    }
    const uint32_t tile_head = tile[0];   // continues a window that runs past the tile end

    typename T::Piece areg[D][kItems];
    uint32_t breg_lo[D], breg_hi[D];

    // Loads are unconditional (addresses are clamped into the tensors) so that they stay in flight
    // across stages; what lies past the end of a row is zeroed when the stage is written to LDS.
    auto load_stage = [&](int slot, int64_t k0) {
        int64_t c = k0 + a_piece * 8;
        c = c < P.in - 8 ? c : P.in - 8;   // in % 8 == 0: a piece is entirely inside or outside the row
#pragma unroll
        for (int i = 0; i < kItems; ++i) T::load(areg[slot][i], a_src[i] + c);
        int64_t pos = b_pos + k0;
        if (pos >= P.p) pos -= P.p;
        const int64_t w = pos >> 5;
        breg_lo[slot] = tile[w];
        breg_hi[slot] = tile[(w + 1 < P.n_words) ? (w + 1) : w];
    };
    auto store_stage = [&](int slot, int buf, int64_t k0) {
        if (k0 + a_piece * 8 >= P.in) {
#pragma unroll
            for (int i = 0; i < kItems; ++i) T::zero(areg[slot][i]);
        }
#pragma unroll
        for (int i = 0; i < kItems; ++i) T::store(areg[slot][i], &lds_a[buf][0][a_lds[i]]);
        // 32 tile bits from the window's cyclic position on; bits past the tile end come from its start
        int64_t pos = b_pos + k0;
        if (pos >= P.p) pos -= P.p;
        const uint32_t sh = static_cast<uint32_t>(pos & 31);
        const uint32_t hi = ((pos >> 5) + 1 < P.n_words) ? breg_hi[slot] : 0u;
        uint32_t wbits = __funnelshift_r(breg_lo[slot], hi, sh);   // shift 0 returns the low word
        const int64_t left = P.p - pos;
        if (left < 32) wbits = (wbits & ((1u << left) - 1u)) | (tile_head << left);
        lds_bits[buf][b_kb][b_col] = b_ok ? unshuffle_bits(wbits) : 0u;
    };

    f32x16_t acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int a_row_base = (wm * kTM * 32 + ln) * kRowStride;   // + tm*32*kRowStride
    const int b_col_base = wn * kTN * 32 + ln * kTN;            // + tn  (a lane owns kTN adjacent columns)

    // One MFMA step covers 16 columns; lane group lg supplies columns 16*s + 8*lg .. + 7 of the
    // 32-column window, i.e. element pairs 8*s + 4*lg + v (v = register).  After unshuffle_bits the
    // two bits of pair i are bits i and i + 16 of the window.
    auto multiply_stage = [&](int buf) {
#pragma unroll
        for (int kb = 0; kb < kKB; ++kb) {
            uint32_t nw[kTN];
#pragma unroll
            for (int tn = 0; tn < kTN; ++tn) nw[tn] = (~lds_bits[buf][kb][b_col_base + tn]) >> (4 * lg);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                Frag b[kTN];
#pragma unroll
                for (int tn = 0; tn < kTN; ++tn)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        b[tn].u[v] = ((nw[tn] << (15 - 8 * s - v)) & 0x80008000u) | 0x3f803f80u;
#pragma unroll
                for (int pl = 0; pl < NP; ++pl) {
                    Frag a[kTM];
#pragma unroll
                    for (int tm = 0; tm < kTM; ++tm)
                        a[tm].q = *reinterpret_cast<const uint4 *>(
                            &lds_a[buf][pl][a_row_base + tm * 32 * kRowStride + kb * 32 + s * 16 + lg * 8]);
#pragma unroll
                    for (int tm = 0; tm < kTM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < kTN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm].v, b[tn].v, acc[tm][tn], 0, 0, 0);
                }
            }
        }
    };

    const int64_t n_stages = (P.in + kBK - 1) / kBK;
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < n_stages) load_stage(d, int64_t(d) * kBK);
    store_stage(0, 0, 0);
    __syncthreads();

    // Steady state: every sub-iteration issues the loads of stage st + D, multiplies stage st and
    // moves stage st + 1 from registers to LDS.  No condition depends on the stage number here, so
    // the compiler can count exactly how many younger loads may stay in flight at each wait.
    int64_t st0 = 0;
    for (; st0 + 2 * D <= n_stages; st0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int64_t st = st0 + d;
            const int buf = static_cast<int>(st & 1);
            load_stage(d, (st + D) * kBK);
            multiply_stage(buf);
            store_stage((d + 1) % D, buf ^ 1, (st + 1) * kBK);
            __syncthreads();
        }
    }
    // Drain: at most 2*D - 1 stages are left; st0 is a multiple of D, so slot numbers stay static.
    for (; st0 < n_stages; st0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int64_t st = st0 + d;
            if (st < n_stages) {   // uniform
                const int buf = static_cast<int>(st & 1);
                if (st + D < n_stages) load_stage(d, (st + D) * kBK);
                multiply_stage(buf);
                if (st + 1 < n_stages) {
                    store_stage((d + 1) % D, buf ^ 1, (st + 1) * kBK);
                    __syncthreads();
                }
            }
        }
    }

    // ---- epilogue: y[m, u + t*U] = alpha(u + t*U) * Z[m, u] --------------------------------------
    const int64_t u_base = n0 + b_col_base;   // first of this lane's kTN adjacent unique columns
    static_assert(kTN == 2, "the epilogue writes column pairs");
    if (u_base >= P.U) return;
    const bool pair_ok = (u_base + 1 < P.U);
    const int64_t m_wave = m0 + wm * kTM * 32 + 4 * lg;

    const int64_t reps = (P.out - u_base + P.U - 1) / P.U;   // replicas of column u_base
    const bool all_pairs = pair_ok && (u_base + (reps - 1) * P.U + 1 < P.out);
    if ((P.n_alpha == 1 || P.aligned) && P.vec_store && all_pairs) {
        // alpha depends on the replica only and every replica is a whole, aligned column pair.
        // Replicas are taken in chunks whose alphas are fetched up front; inside a chunk the rows
        // are outermost, so the stores of one row of Y are issued back to back.
        constexpr int kChunk = 8;
        for (int64_t t0 = 0; t0 < reps; t0 += kChunk) {
            float al[kChunk];
#pragma unroll
            for (int j = 0; j < kChunk; ++j) {
                const int64_t t = (t0 + j < reps) ? (t0 + j) : (reps - 1);
                al[j] = alpha[P.n_alpha == 1 ? 0 : t];
            }
            const int n_here = static_cast<int>((reps - t0) < kChunk ? (reps - t0) : kChunk);
#pragma unroll
            for (int tm = 0; tm < kTM; ++tm) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int64_t m = m_wave + tm * 32 + 8 * (e >> 2) + (e & 3);
                    if (m >= P.M) continue;
                    XT *dst = y + m * P.out + u_base + t0 * P.U;
                    const float z0 = acc[tm][0][e], z1 = acc[tm][1][e];
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) {
                        if (j < n_here) {
                            float v0 = al[j] * z0, v1 = al[j] * z1;
                            if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
                            OutPack<XT>::store2(dst + j * P.U, v0, v1);
                        }
                    }
                }
            }
        }
        return;
    }

    // general case (odd sizes, or tile ends inside rows so that alpha(o) = alpha[(o*in) / p] differs
    // per lane): replicas outermost
    for (int64_t t = 0; t < reps; ++t) {
        const int64_t o0 = u_base + t * P.U, o1 = o0 + 1;
        const bool ok1 = pair_ok && (o1 < P.out);
        float al0, al1;
        if (P.n_alpha == 1) {
            al0 = al1 = alpha[0];
        } else {
            al0 = alpha[(o0 * P.in) / P.p];
            al1 = ok1 ? alpha[(o1 * P.in) / P.p] : 0.f;
        }
#pragma unroll
        for (int tm = 0; tm < kTM; ++tm) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m_wave + tm * 32 + 8 * (e >> 2) + (e & 3);
                if (m >= P.M) continue;
                float v0 = al0 * acc[tm][0][e];
                float v1 = al1 * acc[tm][1][e];
                if (RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
                XT *dst = y + m * P.out + o0;
                if (P.vec_store && ok1) {
                    OutPack<XT>::store2(dst, v0, v1);
                } else {
                    ElemIO<XT>::store(dst, v0);
                    if (ok1) ElemIO<XT>::store(dst + 1, v1);
                }
            }
        }
    }
}

template <typename XT> size_t lds_bytes() {
    return sizeof(uint16_t) * 2 * Traits<XT>::planes * kPlaneElems + sizeof(uint32_t) * 2 * kKB * kBN;
}

template <typename XT, bool RELU> tbn_status launch_typed(const LinearArgs &a, const MfmaParams &P, dim3 grid) {
    static bool attr_set = false;   // dynamic LDS above the default limit has to be allowed once
    const size_t lds = lds_bytes<XT>();
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_mfma_kernel<XT, RELU>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) {
            set_error("tbn_linear_forward: cannot reserve %zu bytes of LDS: %s", lds, hipGetErrorString(e));
            return TBN_ERR_DEVICE;
        }
        attr_set = true;
    }
    hipLaunchKernelGGL((linear_mfma_kernel<XT, RELU>), grid, dim3(kThreads), lds, a.stream, static_cast<const XT *>(a.x),
                       static_cast<XT *>(a.y), a.tile, a.alpha, P);
    return check_launch("tbn_linear_forward (matrix-core kernel)");
}

}  // namespace

bool linear_mfma_supported(const LinearArgs &a) {
    if (a.p < a.in || a.p < 64) return false;   // at most one tile end per row, windows never wrap twice
    if (a.in % 8 != 0) return false;            // 16-byte (bf16) / 32-byte (f32) activation pieces
    if (reinterpret_cast<uintptr_t>(a.x) & 15u) return false;
    if (a.M < 16) return false;
    return true;
}

tbn_status launch_linear_mfma(const LinearArgs &a) {
    MfmaParams P;
    P.M = a.M; P.in = a.in; P.out = a.out; P.p = a.p;
    P.n_words = (a.p + 31) / 32;
    P.U = unique_rows(a.out, a.in, a.p);
    P.n_alpha = a.n_alpha;
    P.relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    P.aligned = (a.p % a.in == 0) ? 1 : 0;
    const size_t esz = (a.dt == TBN_F32) ? 4 : 2;
    P.vec_store = (P.U % 2 == 0 && a.out % 2 == 0 && (reinterpret_cast<uintptr_t>(a.y) % (2 * esz)) == 0) ? 1 : 0;
    P.tiles_m = (a.M + kBM - 1) / kBM;
    P.tiles_n = static_cast<int>((P.U + kBN - 1) / kBN);
    const int64_t blocks = P.tiles_m * P.tiles_n;
    if (blocks > 0x7fffffffLL) {
        set_error("tbn_linear_forward: problem too large for one launch");
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(blocks));
    tbn_status st;
    if (a.dt == TBN_F32)
        st = P.relu ? launch_typed<float, true>(a, P, grid) : launch_typed<float, false>(a, P, grid);
    else
        st = P.relu ? launch_typed<uint16_t, true>(a, P, grid) : launch_typed<uint16_t, false>(a, P, grid);
    if (st != TBN_OK) return st;
    // columns whose weight row straddles a tile end need two alphas
    if (a.n_alpha > 1 && !P.aligned) return launch_linear_rows_fixup(a);
    return TBN_OK;
}

}  // namespace tbn
