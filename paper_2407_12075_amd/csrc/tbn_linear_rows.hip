// Small-batch kernel for the fully-connected tiled-bit layer (GEMV-shaped work): one wave per
// pair of distinct weight rows, +-1 applied to coalesced activation loads, wave-level reduction.
//
// Semantics follow Algorithm 1: the weight of flat position f = o*in + j is t[f % p] scaled by
// alpha[f / p].  Row o starts at tile bit (o*in) % p; if the tile ends inside the row (column
// j0 = p - start < in) the sum is split there, because the two parts are scaled by consecutive
// alphas.  Rows repeat with period U = p / gcd(in, p); each distinct row is summed once and
// written to all its replicas o = u + t*U with that replica's alpha(s).
//
// The same kernel, launched over the list of rows that contain a tile end, repairs those
// columns after the matrix-core kernel (which scales a whole row by its first alpha).
#include "tbn_common.h"

namespace tbn {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerWave = 2;
constexpr int kRowsPerBlock = kRowsPerWave * (kThreads / kWave);  // 8
constexpr int kMaxMB = 16;                                        // most batch rows per workgroup

struct RowsParams {
    int64_t M, in, out, p, n_words, U;
    int32_t k, n_alpha;
    int relu;
    int fixup;   // 0: rows are the distinct rows u (all replicas written); 1: rows are those holding a tile end
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// 8 tile bits at cyclic position pos (any pos in [0, 2p)); p >= 64
__device__ __forceinline__ uint32_t cyclic_byte(const uint32_t *__restrict__ tile, int64_t pos, int64_t p,
                                                int64_t n_words) {
    if (pos >= p) pos -= p;
    uint32_t w = tile_window32(tile, pos, n_words);
    const int64_t left = p - pos;
    if (left < 8) w = (w & ((1u << left) - 1u)) | (tile[0] << left);
    return w & 0xffu;
}

template <typename XT> struct XChunk;
template <> struct XChunk<uint16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const uint16_t *p, bool ok) {
        v = ok ? *reinterpret_cast<const uint4 *>(p) : make_uint4(0, 0, 0, 0);
    }
};
template <> struct XChunk<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float *p, bool ok) {
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        a = ok ? *reinterpret_cast<const float4 *>(p) : z;
        b = ok ? *reinterpret_cast<const float4 *>(p + 4) : z;
    }
};

// weights of 8 consecutive columns: sign bits from `bits` (1 -> +1), zero where `valid` is 0
struct SignPairs {   // bf16 operands for v_dot2_f32_bf16
    uint32_t w[4];
    __device__ __forceinline__ void build(uint32_t bits, uint32_t valid) {
        const uint32_t nb = ~bits;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t lo = 0x3f80u | (((nb >> (2 * i)) & 1u) << 15);
            uint32_t hi = 0x3f80u | (((nb >> (2 * i + 1)) & 1u) << 15);
            lo = ((valid >> (2 * i)) & 1u) ? lo : 0u;
            hi = ((valid >> (2 * i + 1)) & 1u) ? hi : 0u;
            w[i] = lo | (hi << 16);
        }
    }
    __device__ __forceinline__ float dot(const XChunk<uint16_t> &x, float acc) const {
        const uint32_t xs[4] = {x.v.x, x.v.y, x.v.z, x.v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            bf16x2_t a, b;
            __builtin_memcpy(&a, &xs[i], 4);
            __builtin_memcpy(&b, &w[i], 4);
            acc = __builtin_amdgcn_fdot2_f32_bf16(a, b, acc, false);
        }
        return acc;
    }
};

struct SignMasks {   // float32: sign flip by xor, zero by and
    uint32_t flip[8], keep[8];
    __device__ __forceinline__ void build(uint32_t bits, uint32_t valid) {
        const uint32_t nb = ~bits;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            flip[i] = ((nb >> i) & 1u) << 31;
            keep[i] = ((valid >> i) & 1u) ? 0xffffffffu : 0u;
        }
    }
    __device__ __forceinline__ float dot(const XChunk<float> &x, float acc) const {
        const float xs[8] = {x.a.x, x.a.y, x.a.z, x.a.w, x.b.x, x.b.y, x.b.z, x.b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += __uint_as_float((__float_as_uint(xs[i]) ^ flip[i]) & keep[i]);
        return acc;
    }
};

template <typename XT> struct Weights;
template <> struct Weights<uint16_t> { using type = SignPairs; };
template <> struct Weights<float> { using type = SignMasks; };

template <typename XT, int kMB>
__global__ __launch_bounds__(kThreads) void linear_rows_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                               const uint32_t *__restrict__ tile,
                                                               const float *__restrict__ alpha, RowsParams P) {
    __shared__ float s_sum[2][kMB][kRowsPerBlock];
    __shared__ int64_t s_row[kRowsPerBlock];     // output column of replica 0, or -1 if the slot is empty
    __shared__ int s_wrap[kRowsPerBlock];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t m_base = int64_t(blockIdx.y) * kMB;
    const int mcount = static_cast<int>((P.M - m_base) < kMB ? (P.M - m_base) : kMB);

    // rows of this wave
    int64_t row[kRowsPerWave], off[kRowsPerWave], j0[kRowsPerWave];
    bool any_wrap = false;
#pragma unroll
    for (int r = 0; r < kRowsPerWave; ++r) {
        const int64_t slot = int64_t(blockIdx.x) * kRowsPerBlock + wave * kRowsPerWave + r;
        int64_t o = -1;
        if (!P.fixup) {
            if (slot < P.U) o = slot;
        } else if (slot + 1 < P.k) {
            const int64_t f = (slot + 1) * P.p;           // flat index where tile number slot+1 starts
            if (f % P.in != 0) o = f / P.in;              // it starts inside row o
        }
        row[r] = o;
        off[r] = (o >= 0) ? (o * P.in) % P.p : 0;
        j0[r] = (o >= 0 && P.p - off[r] < P.in) ? (P.p - off[r]) : P.in;
        any_wrap |= (j0[r] < P.in);
        if (lane == 0) {
            s_row[wave * kRowsPerWave + r] = o;
            s_wrap[wave * kRowsPerWave + r] = (j0[r] < P.in) ? 1 : 0;
        }
    }

    const int n_seg = any_wrap ? 2 : 1;   // uniform per wave
    for (int seg = 0; seg < n_seg; ++seg) {
        float acc[kRowsPerWave][kMB];
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
            for (int m = 0; m < kMB; ++m) acc[r][m] = 0.f;

        for (int64_t c0 = 0; c0 < P.in; c0 += 64 * 8) {
            const int64_t j8 = c0 + lane * 8;
            const bool in_range = j8 < P.in;     // in % 8 == 0: a group of 8 is all inside or all outside
            XChunk<XT> xc[kMB];
#pragma unroll
            for (int m = 0; m < kMB; ++m) xc[m].load(x + (m_base + (m < mcount ? m : 0)) * P.in + j8, in_range && m < mcount);
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                if (row[r] < 0) continue;
                const int64_t jlo = seg ? j0[r] : 0, jhi = seg ? P.in : j0[r];
                int64_t lo = jlo - j8, hi = jhi - j8;
                lo = lo < 0 ? 0 : (lo > 8 ? 8 : lo);
                hi = hi < 0 ? 0 : (hi > 8 ? 8 : hi);
                const uint32_t valid = (in_range && hi > lo) ? (((1u << hi) - 1u) & ~((1u << lo) - 1u)) : 0u;
                uint32_t bits = 0;
                if (valid) bits = cyclic_byte(tile, off[r] + j8, P.p, P.n_words);
                // a group that crosses the tile end reads its tail bits from the tile start
                typename Weights<XT>::type wts;
                wts.build(bits, valid);
#pragma unroll
                for (int m = 0; m < kMB; ++m) acc[r][m] = wts.dot(xc[m], acc[r][m]);
            }
        }
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
#pragma unroll
            for (int m = 0; m < kMB; ++m) {
                const float s = wave_sum(acc[r][m]);
                if (lane == 0) s_sum[seg][m][wave * kRowsPerWave + r] = s;
            }
    }
    __syncthreads();

    // epilogue: thread -> (local row lr, batch row m, replica t); consecutive threads write consecutive columns
    const int64_t reps = P.fixup ? 1 : (P.out + P.U - 1) / P.U;
    const int64_t work = reps * mcount * kRowsPerBlock;
    for (int64_t id = tid; id < work; id += kThreads) {
        const int lr = static_cast<int>(id % kRowsPerBlock);
        const int m = static_cast<int>((id / kRowsPerBlock) % mcount);
        const int64_t t = id / (int64_t(kRowsPerBlock) * mcount);
        const int64_t o_first = s_row[lr];
        if (o_first < 0) continue;
        const int64_t o = o_first + t * P.U;
        if (o >= P.out) continue;
        const int64_t ai = (P.n_alpha == 1) ? 0 : (o * P.in) / P.p;
        float v = alpha[ai] * s_sum[0][m][lr];
        if (s_wrap[lr]) v += alpha[P.n_alpha == 1 ? 0 : ai + 1] * s_sum[1][m][lr];
        if (P.relu) v = fmaxf(v, 0.f);
        ElemIO<XT>::store(y + (m_base + m) * P.out + o, v);
    }
}

tbn_status launch_rows(const LinearArgs &a, int fixup) {
    RowsParams P;
    P.M = a.M; P.in = a.in; P.out = a.out; P.p = a.p;
    P.n_words = (a.p + 31) / 32;
    P.U = unique_rows(a.out, a.in, a.p);
    P.k = a.k; P.n_alpha = a.n_alpha;
    P.relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    P.fixup = fixup;
    const int64_t rows = fixup ? (a.k - 1) : P.U;
    if (rows <= 0) return TBN_OK;
    const int64_t gx = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
    const int mb = a.M >= 16 ? 16 : (a.M > 4 ? 8 : (a.M > 2 ? 4 : (a.M > 1 ? 2 : 1)));
    const int64_t gy = (a.M + mb - 1) / mb;
    if (gx > 0x7fffffffLL || gy > 65535) {
        set_error("tbn_linear_forward: problem too large for the row kernel");
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy)), block(kThreads);
#define TBN_ROWS_LAUNCH(MB)                                                                                        \
    do {                                                                                                           \
        if (a.dt == TBN_F32)                                                                                       \
            hipLaunchKernelGGL((linear_rows_kernel<float, MB>), grid, block, 0, a.stream,                          \
                               static_cast<const float *>(a.x), static_cast<float *>(a.y), a.tile, a.alpha, P);    \
        else                                                                                                       \
            hipLaunchKernelGGL((linear_rows_kernel<uint16_t, MB>), grid, block, 0, a.stream,                       \
                               static_cast<const uint16_t *>(a.x), static_cast<uint16_t *>(a.y), a.tile, a.alpha, \
                               P);                                                                                 \
    } while (0)
    switch (mb) {
        case 1: TBN_ROWS_LAUNCH(1); break;
        case 2: TBN_ROWS_LAUNCH(2); break;
        case 4: TBN_ROWS_LAUNCH(4); break;
        case 8: TBN_ROWS_LAUNCH(8); break;
        default: TBN_ROWS_LAUNCH(16); break;
    }
#undef TBN_ROWS_LAUNCH
    return check_launch(fixup ? "tbn_linear_forward (tile-end columns)" : "tbn_linear_forward (row kernel)");
}

}  // namespace

bool linear_rows_supported(const LinearArgs &a) {
    if (a.p < a.in || a.p < 64) return false;  // at most one tile end per row
    if (a.in % 8 != 0) return false;           // 16-byte (bf16) / 32-byte (f32) activation groups
    if (reinterpret_cast<uintptr_t>(a.x) & 15u) return false;
    return a.M <= 32;
}

tbn_status launch_linear_rows(const LinearArgs &a) { return launch_rows(a, 0); }

tbn_status launch_linear_rows_fixup(const LinearArgs &a) {
    if (a.M > int64_t(65535) * kMaxMB) {
        set_error("tbn_linear_forward: batch too large for the tile-end pass");
        return TBN_ERR_UNSUPPORTED;
    }
    return launch_rows(a, 1);
}

}  // namespace tbn
