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
//   * one workgroup (4 waves, 2 x 2) owns a 128 x 128 block of Z; X is staged in LDS as bf16 in
//     the operand order of v_mfma_f32_32x32x16_bf16 and double buffered against global loads;
//   * float32 activations are split exactly into three bf16 terms (8 + 8 + 8 significand bits;
//     the weights are +-1, so each product is exact and the sums are float32 accumulations);
//   * the +-1 operand never exists in memory: 32-bit tile windows (aligned for the row's start
//     bit, wrapped at the tile end) are staged in LDS and expanded in registers, two VALU
//     operations per packed bf16 pair, using an operand order in which bits j and j+16 of a
//     window share one register;
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
constexpr int kRowPad = 8;                       // bf16 elements of padding per LDS row (16 B)
constexpr int kRowStride = kBK + kRowPad;        // in bf16 elements

union Frag {
    bf16x8_t v;
    uint32_t u[4];
    uint4 q;
};

template <typename XT> struct Planes;
template <> struct Planes<uint16_t> { static constexpr int n = 1; };
template <> struct Planes<float> { static constexpr int n = 3; };

// one staging item: 8 + 8 activations (columns c..c+7 and c+16..c+23 of a 32-column block)
template <typename XT> struct StageRegs;
template <> struct StageRegs<uint16_t> { uint4 lo, hi; };
template <> struct StageRegs<float> { float4 lo0, lo1, hi0, hi1; };

__device__ __forceinline__ void stage_load(StageRegs<uint16_t> &r, const uint16_t *src, bool ok_lo, bool ok_hi) {
    r.lo = ok_lo ? *reinterpret_cast<const uint4 *>(src) : make_uint4(0, 0, 0, 0);
    r.hi = ok_hi ? *reinterpret_cast<const uint4 *>(src + 16) : make_uint4(0, 0, 0, 0);
}
__device__ __forceinline__ void stage_load(StageRegs<float> &r, const float *src, bool ok_lo, bool ok_hi) {
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    r.lo0 = ok_lo ? *reinterpret_cast<const float4 *>(src) : z;
    r.lo1 = ok_lo ? *reinterpret_cast<const float4 *>(src + 4) : z;
    r.hi0 = ok_hi ? *reinterpret_cast<const float4 *>(src + 16) : z;
    r.hi1 = ok_hi ? *reinterpret_cast<const float4 *>(src + 20) : z;
}

// interleave: out element 2c+h = (h ? hi : lo)[c]  -> register d holds (lo[d], hi[d]) as (low, high) half
__device__ __forceinline__ void stage_store(const StageRegs<uint16_t> &r, uint16_t *dst, int /*plane_stride*/) {
    const uint32_t lo[4] = {r.lo.x, r.lo.y, r.lo.z, r.lo.w};
    const uint32_t hi[4] = {r.hi.x, r.hi.y, r.hi.z, r.hi.w};
    uint32_t o[8];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        o[2 * d] = __byte_perm(lo[d], hi[d], 0x5410);      // (lo[d].low16, hi[d].low16)
        o[2 * d + 1] = __byte_perm(lo[d], hi[d], 0x7632);  // (lo[d].high16, hi[d].high16)
    }
    uint4 *d4 = reinterpret_cast<uint4 *>(dst);
    d4[0] = make_uint4(o[0], o[1], o[2], o[3]);
    d4[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

// exact three-way split of a float into bf16 terms by truncation: x = t0 + t1 + t2
__device__ __forceinline__ void split3(float x, uint32_t &t0, uint32_t &t1, uint32_t &t2) {
    const uint32_t b0 = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(b0);
    const uint32_t b1 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(b1);
    t0 = b0;
    t1 = b1;
    t2 = __float_as_uint(r2);  // at most 8 significant bits are left, the low half is zero
}

__device__ __forceinline__ void stage_store(const StageRegs<float> &r, uint16_t *dst, int plane_stride) {
    const float lo[8] = {r.lo0.x, r.lo0.y, r.lo0.z, r.lo0.w, r.lo1.x, r.lo1.y, r.lo1.z, r.lo1.w};
    const float hi[8] = {r.hi0.x, r.hi0.y, r.hi0.z, r.hi0.w, r.hi1.x, r.hi1.y, r.hi1.z, r.hi1.w};
    uint32_t o[3][8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        uint32_t l0, l1, l2, h0, h1, h2;
        split3(lo[c], l0, l1, l2);
        split3(hi[c], h0, h1, h2);
        o[0][c] = (l0 >> 16) | h0;   // the masked high terms already have a zero low half
        o[1][c] = (l1 >> 16) | h1;
        o[2][c] = (l2 >> 16) | (h2 & 0xffff0000u);
    }
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
        uint4 *d4 = reinterpret_cast<uint4 *>(dst + pl * plane_stride);
        d4[0] = make_uint4(o[pl][0], o[pl][1], o[pl][2], o[pl][3]);
        d4[1] = make_uint4(o[pl][4], o[pl][5], o[pl][6], o[pl][7]);
    }
}

// 32 tile bits at cyclic position pos (0 <= pos < p), continuing at bit 0 after bit p-1.  p >= 32.
__device__ __forceinline__ uint32_t cyclic_window(const uint32_t *__restrict__ tile, int64_t pos, int64_t p,
                                                  int64_t n_words) {
    uint32_t w = tile_window32(tile, pos, n_words);
    const int64_t left = p - pos;  // bits before the tile end
    if (left < 32) {
        const uint32_t head = tile[0];
        w = (w & ((1u << left) - 1u)) | (head << left);
    }
    return w;
}

template <typename OT> struct OutPack;
template <> struct OutPack<uint16_t> {
    static __device__ __forceinline__ void store2(uint16_t *p, float a, float b) {
        *reinterpret_cast<uint32_t *>(p) = uint32_t(f32_to_bf16_bits(a)) | (uint32_t(f32_to_bf16_bits(b)) << 16);
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

template <typename XT>
__global__ __launch_bounds__(kThreads) void linear_mfma_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                               const uint32_t *__restrict__ tile,
                                                               const float *__restrict__ alpha, MfmaParams P) {
    constexpr int NP = Planes<XT>::n;
    constexpr int kPlaneElems = kBM * kRowStride;
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
    int64_t bid = blockIdx.x;
    int64_t tile_m, tile_n;
    {
        const int64_t xcd = bid & 7, slot = bid >> 3;
        const int64_t total = P.tiles_m * P.tiles_n;
        const int64_t per_xcd_full = (total / (8 * P.tiles_n)) * P.tiles_n;  // slots per XCD in the regular part
        if (slot < per_xcd_full) {
            tile_n = slot % P.tiles_n;
            tile_m = (slot / P.tiles_n) * 8 + xcd;
        } else {  // remainder: plain order
            const int64_t rest = bid - per_xcd_full * 8;
            const int64_t base_m = (per_xcd_full / P.tiles_n) * 8;
            tile_n = rest % P.tiles_n;
            tile_m = base_m + rest / P.tiles_n;
        }
    }
    const int64_t m0 = tile_m * kBM;
    const int64_t n0 = tile_n * kBN;

    // ---- staging assignments -------------------------------------------------------------
    // activations: item = (row r, window kb, pair pr) -> columns kb*32 + pr*8 + {0..7, 16..23}
    constexpr int kItems = kBM * kKB * 2 / kThreads;  // per thread
    int a_row[kItems], a_col[kItems];
    const XT *a_src[kItems];
    bool a_row_ok[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int id = tid + i * kThreads;
        const int pr = id & 1, kb = (id >> 1) % kKB, r = id / (2 * kKB);
        a_row[i] = r;
        a_col[i] = kb * 32 + pr * 8;
        a_row_ok[i] = (m0 + r) < P.M;
        a_src[i] = x + (a_row_ok[i] ? (m0 + r) : 0) * P.in + a_col[i];
    }
    // tile windows: item = (column c, window kb); one per thread (kBN * kKB == kThreads)
    static_assert(kBN * kKB == kThreads, "one tile window per thread and stage");
    const int b_col = tid % kBN, b_kb = tid / kBN;
    const int64_t b_u = n0 + b_col;
    const bool b_ok = b_u < P.U;
    int64_t b_pos = 0;  // cyclic bit position of this window at k0 = 0
    if (b_ok) {
        b_pos = (b_u * P.in) % P.p + b_kb * 32;
        if (b_pos >= P.p) b_pos -= P.p;
    }

    StageRegs<XT> areg[kItems];
    uint32_t breg = 0;

    auto load_stage = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t c = k0 + a_col[i];
            stage_load(areg[i], a_src[i] + k0, a_row_ok[i] && c < P.in, a_row_ok[i] && (c + 16) < P.in);
        }
        if (b_ok && k0 + b_kb * 32 < P.in) {
            int64_t pos = b_pos + k0;
            if (pos >= P.p) pos -= P.p;
            breg = cyclic_window(tile, pos, P.p, P.n_words);
        } else {
            breg = 0;
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kItems; ++i)
            stage_store(areg[i], &lds_a[buf][0][a_row[i] * kRowStride + 2 * a_col[i] - (a_col[i] & ~31)], kPlaneElems);
        lds_bits[buf][b_kb][b_col] = breg;
    };
    // LDS element offset of an item inside its row: window kb occupies [kb*32, kb*32+32); pair pr
    // fills the 16 elements at pr*16.  a_col = kb*32 + pr*8, so kb*32 + pr*16 = 2*a_col - kb*32
    // and kb*32 = a_col & ~31 (pr*8 < 32).

    f32x16_t acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int a_row_base = (wm * kTM * 32 + ln) * kRowStride;   // + tm*32*kRowStride
    const int b_col_base = wn * kTN * 32 + ln * kTN;            // + tn  (a lane owns kTN adjacent columns)

    const int64_t n_stages = (P.in + kBK - 1) / kBK;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int64_t st = 0; st < n_stages; ++st) {
        const int buf = st & 1;
        if (st + 1 < n_stages) load_stage((st + 1) * kBK);
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
                            &lds_a[buf][pl][a_row_base + tm * 32 * kRowStride + kb * 32 + (s * 2 + lg) * 8]);
#pragma unroll
                    for (int tm = 0; tm < kTM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < kTN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm].v, b[tn].v, acc[tm][tn], 0, 0, 0);
                }
            }
        }
        if (st + 1 < n_stages) {
            store_stage(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: y[m, u + t*U] = alpha(u + t*U) * Z[m, u] --------------------------------------
    const int64_t u_base = n0 + b_col_base;   // first of this lane's kTN adjacent unique columns
    static_assert(kTN == 2, "the epilogue writes column pairs");
    for (int64_t t = 0; u_base + t * P.U < P.out && u_base < P.U; ++t) {
        const int64_t o0 = u_base + t * P.U, o1 = o0 + 1;
        const bool ok1 = (u_base + 1 < P.U) && (o1 < P.out);
        float al0, al1;
        if (P.n_alpha == 1) {
            al0 = al1 = alpha[0];
        } else if (P.aligned) {
            al0 = al1 = alpha[t];
        } else {
            al0 = alpha[(o0 * P.in) / P.p];
            al1 = ok1 ? alpha[(o1 * P.in) / P.p] : 0.f;
        }
#pragma unroll
        for (int tm = 0; tm < kTM; ++tm) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + wm * kTM * 32 + tm * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
                if (m >= P.M) continue;
                float v0 = al0 * acc[tm][0][e];
                float v1 = al1 * acc[tm][1][e];
                if (P.relu) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
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

}  // namespace

bool linear_mfma_supported(const LinearArgs &a) {
    if (a.p < a.in || a.p < 64) return false;   // at most one tile end per row, windows never wrap twice
    if (a.in % 8 != 0) return false;            // 16-byte activation loads
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
    const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    const int planes = (a.dt == TBN_F32) ? 3 : 1;
    const size_t lds = sizeof(uint16_t) * 2 * planes * kBM * kRowStride + sizeof(uint32_t) * 2 * kKB * kBN;
    static bool attr_set[2] = {false, false};   // large dynamic LDS has to be allowed once per kernel
    if (!attr_set[a.dt == TBN_F32]) {
        hipError_t e = (a.dt == TBN_F32)
                           ? hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_mfma_kernel<float>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                           : hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_mfma_kernel<uint16_t>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            set_error("tbn_linear_forward: cannot reserve %zu bytes of LDS: %s", lds, hipGetErrorString(e));
            return TBN_ERR_DEVICE;
        }
        attr_set[a.dt == TBN_F32] = true;
    }
    if (a.dt == TBN_F32)
        hipLaunchKernelGGL(linear_mfma_kernel<float>, grid, block, lds, a.stream, static_cast<const float *>(a.x),
                           static_cast<float *>(a.y), a.tile, a.alpha, P);
    else
        hipLaunchKernelGGL(linear_mfma_kernel<uint16_t>, grid, block, lds, a.stream,
                           static_cast<const uint16_t *>(a.x), static_cast<uint16_t *>(a.y), a.tile, a.alpha, P);
    tbn_status st = check_launch("tbn_linear_forward (matrix-core kernel)");
    if (st != TBN_OK) return st;
    // columns whose weight row straddles a tile end need two alphas
    if (a.n_alpha > 1 && !P.aligned) return launch_linear_rows_fixup(a);
    return TBN_OK;
}

}  // namespace tbn
