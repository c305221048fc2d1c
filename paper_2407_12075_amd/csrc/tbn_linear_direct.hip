// Fully-connected tiled-bit layer for row lengths the matrix-core kernels do not take (in no multiple of 8, or
// activations that are not 16-byte aligned: the 196-token mixing layers of an MLP-Mixer, 300- or 2050-wide rows),
// with a tile of whole weight rows.
//
// What is computed (Section "Method", Eq. 4-5 and the scaling after Eq. 8): with p a multiple of `in` the weight is
// the U = p / in rows of the tile stacked k times, copy t scaled by alpha[t]; Z = X * T^T is formed once and
// Y[:, t*U + u] = alpha[t] * Z[:, u].
//
// A thread owns one batch row and 16 distinct columns: it walks its row of X one or two elements at a time (a lane's
// loads hit the same cache line many times in a row, whatever the row's alignment) and feeds every element to 16 sums with
// +-1 values that all lanes read from the same LDS address.  The +-1 weights of the workgroup's 16 tile rows pass
// through LDS as float32, 512 positions of K at a time.  Vector-ALU work, an order of magnitude above one thread per
// output element (8192 x 196 -> 384, k = 4: 34 us against 382; 8192 x 2050 -> 1026, k = 2: 0.50 ms against 8.9).
#include "tbn_common.h"

namespace tbn {

namespace {

constexpr int kFG = 16;       // distinct columns per workgroup
constexpr int kRows = 128;    // batch rows per workgroup, one per thread
constexpr int kStage = 512;   // positions of K staged per pass

struct DirectLinearParams {
    int64_t M, in, out, U;
    int32_t reps, n_alpha, relu;
};

// VEC consecutive activations with one load (the caller has checked the alignment)
template <typename T, int VEC> struct XVec;
template <> struct XVec<float, 1> { static __device__ __forceinline__ void load(const float *p, float (&v)[1]) { v[0] = *p; } };
template <> struct XVec<float, 2> {
    static __device__ __forceinline__ void load(const float *p, float (&v)[2]) {
        const float2 t = *reinterpret_cast<const float2 *>(p);
        v[0] = t.x; v[1] = t.y;
    }
};
template <> struct XVec<uint16_t, 1> { static __device__ __forceinline__ void load(const uint16_t *p, float (&v)[1]) { v[0] = bf16_bits_to_f32(*p); } };
template <> struct XVec<uint16_t, 2> {
    static __device__ __forceinline__ void load(const uint16_t *p, float (&v)[2]) {
        const uint32_t t = *reinterpret_cast<const uint32_t *>(p);
        v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xffff0000u);
    }
};

template <typename T, int VEC>
__global__ __launch_bounds__(kRows) void linear_direct_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                             const uint32_t *__restrict__ tile,
                                                             const float *__restrict__ alpha, DirectLinearParams P) {
    __shared__ __attribute__((aligned(16))) float w_lds[kStage][kFG];   // +1 / -1
    const int tid = threadIdx.x;
    const int64_t m = int64_t(blockIdx.x) * kRows + tid;
    const int64_t u0 = int64_t(blockIdx.y) * kFG;
    const bool live = m < P.M;
    const T *xr = x + (live ? m : P.M - 1) * P.in;   // rows past M repeat the last one; never written

    float acc[kFG];
#pragma unroll
    for (int f = 0; f < kFG; ++f) acc[f] = 0.f;

    for (int64_t j0 = 0; j0 < P.in; j0 += kStage) {
        const int32_t n = static_cast<int32_t>(P.in - j0 < kStage ? P.in - j0 : kStage);
        __syncthreads();   // the previous pass is done with the staged weights
        for (int32_t e = tid; e < n; e += kRows) {
#pragma unroll
            for (int f = 0; f < kFG; ++f) {
                const int64_t u = u0 + f < P.U ? u0 + f : P.U - 1;   // columns past U repeat the last one; never written
                const int64_t bit = u * P.in + j0 + e;               // < p
                w_lds[e][f] = ((tile[bit >> 5] >> (bit & 31)) & 1u) ? 1.f : -1.f;
            }
        }
        __syncthreads();
        const T *xs = xr + j0;
#pragma unroll 4
        for (int32_t e = 0; e < n; e += VEC) {   // n is a multiple of VEC: `in` is, and so is the stage
            float xv[VEC];
            XVec<T, VEC>::load(xs + e, xv);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float4 *wv = reinterpret_cast<const float4 *>(w_lds[e + i]);
#pragma unroll
                for (int g = 0; g < kFG / 4; ++g) {
                    const float4 s = wv[g];
                    acc[4 * g + 0] = fmaf(xv[i], s.x, acc[4 * g + 0]);
                    acc[4 * g + 1] = fmaf(xv[i], s.y, acc[4 * g + 1]);
                    acc[4 * g + 2] = fmaf(xv[i], s.z, acc[4 * g + 2]);
                    acc[4 * g + 3] = fmaf(xv[i], s.w, acc[4 * g + 3]);
                }
            }
        }
    }

    if (!live) return;
    T *yr = y + m * P.out;
    for (int32_t t = 0; t < P.reps; ++t) {
        const float al = alpha[P.n_alpha == 1 ? 0 : t];
#pragma unroll
        for (int f = 0; f < kFG; ++f) {
            const int64_t u = u0 + f;
            if (u < P.U) {
                float v = al * acc[f];
                if (P.relu) v = fmaxf(v, 0.f);
                ElemIO<T>::store(yr + int64_t(t) * P.U + u, v);
            }
        }
    }
}

}  // namespace

// Shapes this kernel takes: tile of whole rows; it is meant for what the matrix-core kernels decline.
bool linear_direct_supported(const LinearArgs &a) {
    if (a.dt != TBN_F32 && a.dt != TBN_BF16) return false;
    if (a.M < 1 || a.in < 1 || a.p % a.in != 0) return false;
    const int64_t U = a.p / a.in;
    if (U < 1 || U > a.out || a.out % U != 0 || a.out / U > (1 << 30)) return false;
    if (a.n_alpha != 1 && a.n_alpha != a.out / U) return false;
    if ((a.M + kRows - 1) / kRows > 0x7fffffffLL || (U + kFG - 1) / kFG > 65535) return false;
    return true;
}

tbn_status launch_linear_direct(const LinearArgs &a) {
    DirectLinearParams P;
    P.M = a.M; P.in = a.in; P.out = a.out;
    P.U = a.p / a.in;
    P.reps = static_cast<int32_t>(a.out / P.U);
    P.n_alpha = a.n_alpha;
    P.relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    const dim3 grid(static_cast<unsigned>((a.M + kRows - 1) / kRows), static_cast<unsigned>((P.U + kFG - 1) / kFG));
    // activations per load: two where the row length and the alignment of x allow
    const size_t esz = a.dt == TBN_F32 ? 4 : 2;
    const uintptr_t xa = reinterpret_cast<uintptr_t>(a.x);
    const int vec = (a.in % 2 == 0 && xa % (2 * esz) == 0) ? 2 : 1;   // (four per load measured slower: 48 us against 37 at in = 196)
#define TBN_DIRECT_LAUNCH(T, V)                                                                                          \
    hipLaunchKernelGGL((linear_direct_kernel<T, V>), grid, dim3(kRows), 0, a.stream, static_cast<const T *>(a.x),           \
                       static_cast<T *>(a.y), a.tile, a.alpha, P)
    if (a.dt == TBN_F32) {
        if (vec == 2) TBN_DIRECT_LAUNCH(float, 2); else TBN_DIRECT_LAUNCH(float, 1);
    } else {
        if (vec == 2) TBN_DIRECT_LAUNCH(uint16_t, 2); else TBN_DIRECT_LAUNCH(uint16_t, 1);
    }
#undef TBN_DIRECT_LAUNCH
    return check_launch("tbn_linear_forward (direct kernel)");
}

}  // namespace tbn
