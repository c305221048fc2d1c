// Decode-shaped kernel for the fully-connected tiled-bit layer: at most 16 batch rows, tile of whole weight
// rows (p % in == 0).  GEMV-shaped work, built for latency.
//
// Same sums as Algorithm 1 (Section "GPU Inference Kernel" / microcontroller listing), Eq. 4-5: weight (o, j) is
// tile bit (o*in + j) % p scaled by alpha[(o*in + j) / p]; with whole rows per tile only the U = p / in rows of
// the tile are distinct, each is summed once and written to its k replicas o = u + t*U scaled by alpha[t].
//
// At these sizes the layer moves a few hundred kilobytes: tens of nanoseconds of HBM time under a launch of
// about 1.7 us, so what counts is how few dependent steps stand between the launch and the last store, and that
// the whole chip takes part (the matrix-core small-batch kernel gives a 4096 x 4096, k = 8 layer to 32
// workgroups; its loads queue at 32 CUs' load paths for 2 us).  Here a workgroup owns R = 2 or 4 distinct rows
// (512 rows -> 256 or 128 workgroups), its four waves split K in interleaved chunks of 512 elements, a lane
// takes 8 consecutive elements of a chunk: one 16-byte (bf16) or two 16-byte (float32) loads per batch row, all
// issued before the first use, and one byte of tile bits per row.  +-1 is applied as a sign flip on the loaded
// activations (v_dot2_f32_bf16 against +-1 pairs for bf16, xor of the sign bit for float32), sums are float32.
// The R * MB sums of a lane are reduced over the wave with a butterfly that halves the number of values at
// every step (32 shuffles for 32 values instead of 192), the four waves' sums are added in wave order through
// LDS, and every thread takes part in the replicated, alpha-scaled stores.
#include "tbn_common.h"

namespace tbn {

namespace {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kChunk = kWave * 8;     // K elements a wave covers per step

struct DecodeParams {
    int64_t M, in, out, U;
    int32_t reps, n_alpha, relu;
};

template <typename XT> struct XGroup;   // 8 consecutive activations
template <> struct XGroup<uint16_t> {
    uint32_t w[4];
    __device__ __forceinline__ void load(const uint16_t *p) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    }
    __device__ __forceinline__ void zero() { w[0] = w[1] = w[2] = w[3] = 0u; }
};
template <> struct XGroup<float> {
    float f[8];
    __device__ __forceinline__ void load(const float *p) {
        const float4 a = *reinterpret_cast<const float4 *>(p);
        const float4 b = *reinterpret_cast<const float4 *>(p + 4);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = 0.f;
    }
};

// +-1 weights of 8 consecutive columns from 8 tile bits (1 -> +1)
template <typename XT> struct Signs;
template <> struct Signs<uint16_t> {   // bf16 pairs for v_dot2_f32_bf16
    uint32_t w[4];
    __device__ __forceinline__ void build(uint32_t bits) {
        const uint32_t nb = ~bits;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = 0x3f803f80u | (((nb >> (2 * i)) & 1u) << 15) | (((nb >> (2 * i + 1)) & 1u) << 31);
    }
    __device__ __forceinline__ float dot(const XGroup<uint16_t> &x, float acc) const {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, x.w[i]), __builtin_bit_cast(bf16x2_t, w[i]), acc, false);
        return acc;
    }
};
template <> struct Signs<float> {   // sign flip by xor
    uint32_t flip[8];
    __device__ __forceinline__ void build(uint32_t bits) {
        const uint32_t nb = ~bits;
#pragma unroll
        for (int i = 0; i < 8; ++i) flip[i] = ((nb >> i) & 1u) << 31;
    }
    __device__ __forceinline__ float dot(const XGroup<float> &x, float acc) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += __uint_as_float(__float_as_uint(x.f[i]) ^ flip[i]);
        return acc;
    }
};

// Sums V = 2^LOGV values per lane over the 64 lanes.  A step with lane distance d: while more than one value is
// left, a lane keeps one half of its values (which half is its bit d) and receives the partner's sums of that half;
// afterwards plain sums.  On exit v[0] of lane l is the total of value l >> (6 - LOGV).
template <int LOGV, int D, int N>
__device__ __forceinline__ void wave_reduce_step(float (&v)[1 << LOGV], int lane) {
    if constexpr (D >= 1) {
        if constexpr (N > 1) {
            constexpr int H = N / 2;
            const bool upper = (lane & D) != 0;
#pragma unroll
            for (int i = 0; i < H; ++i) {
                const float keep = upper ? v[i + H] : v[i];
                const float send = upper ? v[i] : v[i + H];
                v[i] = keep + __shfl_xor(send, D, kWave);
            }
            wave_reduce_step<LOGV, D / 2, H>(v, lane);
        } else {
            v[0] += __shfl_xor(v[0], D, kWave);
            wave_reduce_step<LOGV, D / 2, 1>(v, lane);
        }
    }
}
template <int LOGV>
__device__ __forceinline__ void wave_reduce_values(float (&v)[1 << LOGV], int lane) {
    wave_reduce_step<LOGV, 32, (1 << LOGV)>(v, lane);
}

template <typename XT, int LOGMB, int LOGR>
__global__ __launch_bounds__(kThreads) void linear_decode_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                                 const unsigned char *__restrict__ tile_bytes,
                                                                 const float *__restrict__ alpha, DecodeParams P) {
    constexpr int MB = 1 << LOGMB, R = 1 << LOGR, V = MB * R, LOGV = LOGMB + LOGR;
    __shared__ float s_part[kWaves][V];
    __shared__ float s_z[V];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t u0 = int64_t(blockIdx.x) * R;
    const int mcount = static_cast<int>(P.M < MB ? P.M : MB);

    // the scalar of this thread's first store, requested before everything else: its latency would otherwise
    // follow the reduction
    const int work = P.reps * mcount * R;
    const int t_first = (tid >> LOGR) / mcount;
    const float alpha_first = alpha[(P.n_alpha == 1 || tid >= work) ? 0 : t_first];

    float acc[V];   // [r][m]
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;

    int64_t row_bits[R];   // bit position of the row start in the tile (rows past U repeat the last one; never written)
#pragma unroll
    for (int r = 0; r < R; ++r) row_bits[r] = (u0 + r < P.U ? u0 + r : P.U - 1) * P.in;

    const int64_t n_chunks = (P.in + kChunk - 1) / kChunk;
    // S chunks of this wave per step, all their loads issued before the first use (one chunk where two would not
    // fit the registers: float32 at 8 or 16 batch rows)
    constexpr int S = (sizeof(XT) == 4 && MB >= 8) ? 1 : 2;
    for (int64_t c = wave; c < n_chunks; c += S * kWaves) {
        XGroup<XT> xg[S][MB];
        uint32_t bits[S][R];
        bool ok[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int64_t j8 = (c + s * kWaves) * kChunk + lane * 8;
            ok[s] = j8 < P.in;   // in % 8 == 0: a group of 8 is all inside or all outside
            if (ok[s]) {
#pragma unroll
                for (int r = 0; r < R; ++r) bits[s][r] = tile_bytes[(row_bits[r] + j8) >> 3];
#pragma unroll
                for (int m = 0; m < MB; ++m) xg[s][m].load(x + int64_t(m < mcount ? m : 0) * P.in + j8);
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) bits[s][r] = 0;
#pragma unroll
                for (int m = 0; m < MB; ++m) xg[s][m].zero();
            }
        }
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                Signs<XT> w;
                w.build(bits[s][r]);
#pragma unroll
                for (int m = 0; m < MB; ++m) acc[r * MB + m] = w.dot(xg[s][m], acc[r * MB + m]);
            }
    }

    wave_reduce_values<LOGV>(acc, lane);
    if ((lane & ((kWave >> LOGV) - 1)) == 0) s_part[wave][lane >> (6 - LOGV)] = acc[0];
    __syncthreads();
    if (tid < V) {
        float z = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) z += s_part[wv][tid];   // fixed order
        s_z[tid] = z;
    }
    __syncthreads();

    // y[m, u0 + r + t*U] = alpha[t] * z[r][m]; consecutive threads write the R adjacent columns of a replica
    for (int id = tid; id < work; id += kThreads) {
        const int r = id & (R - 1);
        const int m = (id >> LOGR) % mcount;
        const int t = (id >> LOGR) / mcount;
        if (u0 + r >= P.U) continue;
        const float al = id == tid ? alpha_first : alpha[P.n_alpha == 1 ? 0 : t];
        float v = al * s_z[r * MB + m];
        if (P.relu) v = fmaxf(v, 0.f);
        ElemIO<XT>::store(y + int64_t(m) * P.out + u0 + r + int64_t(t) * P.U, v);
    }
}

template <typename XT, int LOGMB>
void launch_decode_r(const LinearArgs &a, const DecodeParams &P, int log_r) {
    const unsigned char *tb = reinterpret_cast<const unsigned char *>(a.tile);
    const XT *x = static_cast<const XT *>(a.x);
    XT *y = static_cast<XT *>(a.y);
    if (log_r == 1) {
        const dim3 grid(static_cast<unsigned>((P.U + 1) / 2));
        hipLaunchKernelGGL((linear_decode_kernel<XT, LOGMB, 1>), grid, dim3(kThreads), 0, a.stream, x, y, tb, a.alpha, P);
    } else {
        const dim3 grid(static_cast<unsigned>((P.U + 3) / 4));
        hipLaunchKernelGGL((linear_decode_kernel<XT, LOGMB, 2>), grid, dim3(kThreads), 0, a.stream, x, y, tb, a.alpha, P);
    }
}

template <typename XT>
void launch_decode_t(const LinearArgs &a, const DecodeParams &P) {
    // two rows per workgroup (4096 x 4096, k = 8, batch 16: 5.3 us against 6.4 with four: the 256 workgroups fill
    // the chip, the 128 do not); four only where the grid is large anyway and every workgroup re-reads all of X
    const int log_r = (a.M >= 8 && P.U >= 4096) ? 2 : 1;
    if (a.M <= 1) launch_decode_r<XT, 0>(a, P, log_r);
    else if (a.M <= 2) launch_decode_r<XT, 1>(a, P, log_r);
    else if (a.M <= 4) launch_decode_r<XT, 2>(a, P, log_r);
    else if (a.M <= 8) launch_decode_r<XT, 3>(a, P, log_r);
    else launch_decode_r<XT, 4>(a, P, log_r);
}

}  // namespace

bool linear_decode_supported(const LinearArgs &a) {
    if (a.M < 1 || a.M > 16) return false;
    if (a.p % a.in != 0 || a.in % 8 != 0) return false;   // whole rows per tile; 8 bits and 16 / 32 bytes per lane and step
    const int64_t U = a.p / a.in;
    if (U > a.out || a.out % U != 0 || a.out / U > (1 << 20)) return false;
    if (U > (int64_t(1) << 31) - 8) return false;
    if (reinterpret_cast<uintptr_t>(a.x) & 15u) return false;
    return true;
}

tbn_status launch_linear_decode(const LinearArgs &a) {
    DecodeParams P;
    P.M = a.M; P.in = a.in; P.out = a.out;
    P.U = a.p / a.in;
    P.reps = static_cast<int32_t>(a.out / P.U);
    P.n_alpha = a.n_alpha;
    P.relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    if (a.dt == TBN_F32) launch_decode_t<float>(a, P);
    else launch_decode_t<uint16_t>(a, P);
    return check_launch("tbn_linear_forward (decode kernel)");
}

}  // namespace tbn
