// Column-tiled fully-connected layer (GPU Inference Kernel section: an out x in weight kept as one
// out x q block, q = in / k, that serves all k column blocks).
//
//   y[m, o] = sum_c alpha[c] * sum_j x[m, c*q + j] * t[o, j] = sum_j xf[m, j] * t[o, j],
//   xf[m, j] = sum_c alpha[c] * x[m, c*q + j]
//
// so the layer is one pass over X that folds its k column blocks (this file) followed by a +-1 product of
// M x q by q x out, which is the flat-tiled layer with k = 1 on q inputs: the tile words are the same and the
// matrix-core kernels run it as they are, with a k times shorter K loop and no replicated columns.
//
// The fold is bound by memory: it reads M * in elements once and writes M * q.  A thread owns 16 bytes of one
// row of xf and walks the k blocks in ascending order with eight loads in flight; sums are float32 (bfloat16
// activations are rounded once, to nearest even, when xf is written).
#include "tbn_common.h"

namespace tbn {

namespace {

constexpr int kFoldThreads = 256;
constexpr int kFoldDepth = 8;   // column blocks requested before the first is used

template <typename XT> struct FoldIO;
template <> struct FoldIO<float> {
    static constexpr int kVec = 4;
    struct Raw { float4 v; };
    static __device__ __forceinline__ void load(Raw &r, const float *p) { r.v = *reinterpret_cast<const float4 *>(p); }
    static __device__ __forceinline__ void add(float (&s)[kVec], const Raw &r, float a) {
        s[0] += a * r.v.x; s[1] += a * r.v.y; s[2] += a * r.v.z; s[3] += a * r.v.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&s)[kVec]) {
        *reinterpret_cast<float4 *>(p) = make_float4(s[0], s[1], s[2], s[3]);
    }
};
template <> struct FoldIO<uint16_t> {
    static constexpr int kVec = 8;
    struct Raw { uint4 v; };
    static __device__ __forceinline__ void load(Raw &r, const uint16_t *p) { r.v = *reinterpret_cast<const uint4 *>(p); }
    static __device__ __forceinline__ void add(float (&s)[kVec], const Raw &r, float a) {
        const uint32_t w[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[2 * i] += a * __uint_as_float(w[i] << 16);
            s[2 * i + 1] += a * __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(uint16_t *p, const float (&s)[kVec]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = static_cast<uint32_t>(f32_to_bf16_bits(s[2 * i])) | (static_cast<uint32_t>(f32_to_bf16_bits(s[2 * i + 1])) << 16);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// WIDE: a thread owns 16 bytes of xf (q a multiple of the vector length, aligned pointers), else one element
template <typename XT, bool WIDE>
__global__ __launch_bounds__(kFoldThreads) void coltile_fold_kernel(const XT *__restrict__ x, XT *__restrict__ xf,
                                                                    const float *__restrict__ alpha, int32_t n_alpha,
                                                                    int64_t M, int64_t in, int64_t q, int32_t k,
                                                                    float *__restrict__ one_out) {
    using IO = FoldIO<XT>;
    constexpr int VEC = WIDE ? IO::kVec : 1;
    if (blockIdx.x == 0 && threadIdx.x == 0) *one_out = 1.0f;
    const int64_t per_row = q / VEC;   // WIDE is only used when q % kVec == 0
    const int64_t idx = int64_t(blockIdx.x) * kFoldThreads + threadIdx.x;
    if (idx >= M * per_row) return;
    const int64_t m = idx / per_row, j = (idx - m * per_row) * VEC;
    const XT *src = x + m * in + j;
    float s[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) s[v] = 0.f;
    for (int32_t c0 = 0; c0 < k; c0 += kFoldDepth) {
        if constexpr (WIDE) {
            typename IO::Raw r[kFoldDepth];
            float a[kFoldDepth];
#pragma unroll
            for (int d = 0; d < kFoldDepth; ++d) {
                const int32_t c = c0 + d < k ? c0 + d : k - 1;   // a repeated block is loaded but not added
                IO::load(r[d], src + int64_t(c) * q);
                a[d] = alpha[n_alpha == 1 ? 0 : c];
            }
#pragma unroll
            for (int d = 0; d < kFoldDepth; ++d)
                if (c0 + d < k) IO::add(s, r[d], a[d]);
        } else {
            float r[kFoldDepth], a[kFoldDepth];
#pragma unroll
            for (int d = 0; d < kFoldDepth; ++d) {
                const int32_t c = c0 + d < k ? c0 + d : k - 1;
                r[d] = ElemIO<XT>::load(src + int64_t(c) * q);
                a[d] = alpha[n_alpha == 1 ? 0 : c];
            }
#pragma unroll
            for (int d = 0; d < kFoldDepth; ++d)
                if (c0 + d < k) s[0] += a[d] * r[d];
        }
    }
    XT *dst = xf + m * q + j;
    if constexpr (WIDE) IO::store(dst, s); else ElemIO<XT>::store(dst, s[0]);
}

template <typename XT>
tbn_status launch_fold_typed(const void *x, void *xf, int64_t M, int64_t in, int32_t k, const float *alpha,
                             int32_t n_alpha, float *one_out, hipStream_t stream) {
    const int64_t q = in / k;
    constexpr int kVec = FoldIO<XT>::kVec;
    // 16-byte accesses need every block of every row to start on a 16-byte boundary
    const bool wide = q % kVec == 0 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(xf)) & 15u) == 0;
    const int64_t items = M * (wide ? q / kVec : q);
    const int64_t blocks = (items + kFoldThreads - 1) / kFoldThreads;
    if (blocks > 0x7fffffffLL) {
        set_error("tbn_linear_coltiled_forward: %lld x %lld folded activations are beyond one launch", (long long)M, (long long)q);
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(blocks)), block(kFoldThreads);
    if (wide)
        hipLaunchKernelGGL((coltile_fold_kernel<XT, true>), grid, block, 0, stream, static_cast<const XT *>(x),
                           static_cast<XT *>(xf), alpha, n_alpha, M, in, q, k, one_out);
    else
        hipLaunchKernelGGL((coltile_fold_kernel<XT, false>), grid, block, 0, stream, static_cast<const XT *>(x),
                           static_cast<XT *>(xf), alpha, n_alpha, M, in, q, k, one_out);
    return check_launch("tbn_linear_coltiled_forward (fold kernel)");
}

}  // namespace

tbn_status launch_coltile_fold(const void *x, void *xf, int dt, int64_t M, int64_t in, int32_t k,
                               const float *alpha, int32_t n_alpha, float *one_out, hipStream_t stream) {
    if (dt == TBN_F32) return launch_fold_typed<float>(x, xf, M, in, k, alpha, n_alpha, one_out, stream);
    return launch_fold_typed<uint16_t>(x, xf, M, in, k, alpha, n_alpha, one_out, stream);
}

}  // namespace tbn
