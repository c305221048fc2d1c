// Measurement aids of libtbn: kernels with no part in the method, launched the same way as the layer kernels,
// that give the denominators the benchmark quotes next to the datasheet peaks -- the duration of a launch that
// does nothing (the floor under the small-batch rows), the rate of a plain streaming read and copy (what HBM
// gives a kernel that does nothing else), and the rate of a loop of nothing but bf16 MFMAs (what the matrix
// pipes sustain at the clock they settle at).
#include "tbn_common.h"

namespace tbn {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ void diag_empty_kernel() {}

// grid-stride over 16-byte pieces, four loads in flight per thread
template <bool COPY>
__global__ __launch_bounds__(256) void diag_stream_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst,
                                                          int64_t n16, uint32_t *__restrict__ sink) {
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    u32x4_t acc = {0, 0, 0, 0};
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u32x4_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (COPY) __builtin_nontemporal_store(v[j], dst + i + j * stride);
            else acc ^= v[j];
        }
    }
    for (; i < n16; i += stride) {
        const u32x4_t v = src[i];
        if (COPY) dst[i] = v;
        else acc ^= v;
    }
    if (!COPY) {   // keeps the loads alive; never true for data that is not all ones
        if ((acc[0] & acc[1] & acc[2] & acc[3]) == 0xffffffffu && sink) sink[0] = acc[0];
    }
}

// every wave: iters x 8 independent 32x32x16 bf16 MFMAs on register operands
__global__ __launch_bounds__(256) void diag_mfma_kernel(int32_t iters, float *__restrict__ out) {
    bf16x8_t a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = static_cast<__bf16>(1.0f + 0.125f * static_cast<float>((threadIdx.x + e) & 3));
        b[e] = static_cast<__bf16>((e & 1) ? 1.0f : -1.0f);
    }
    f32x16_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) s += acc[t][0];
    if (out) out[int64_t(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

// the same with the 4-bit float form of the MFMA (32x32x64, both operands E2M1, no block scales): the instruction
// of the binary-activation kernel
__global__ __launch_bounds__(256) void diag_mfma_fp4_kernel(int32_t iters, float *__restrict__ out) {
    typedef int i32x8_t __attribute__((ext_vector_type(8)));
    i32x8_t a = {}, b = {};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        a[e] = static_cast<int>(0x2a2a2a2au ^ (0x88888888u * ((threadIdx.x + e) & 1)));   // nibbles 0x2 / 0xA: +1 and -1
        b[e] = static_cast<int>(0xa2a2a2a2u);
    }
    f32x16_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    for (int32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[t], 4, 4, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) s += acc[t][0];
    if (out) out[int64_t(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

}  // namespace

tbn_status launch_diag_empty(hipStream_t stream) {
    hipLaunchKernelGGL(diag_empty_kernel, dim3(1), dim3(64), 0, stream);
    return check_launch("tbn_diag_empty_launch");
}

tbn_status launch_diag_stream(const void *src, void *dst, size_t bytes, uint32_t *sink, hipStream_t stream) {
    const int64_t n16 = static_cast<int64_t>(bytes / 16);
    const dim3 grid(256 * 16), block(256);
    if (dst)
        hipLaunchKernelGGL((diag_stream_kernel<true>), grid, block, 0, stream, static_cast<const u32x4_t *>(src),
                           static_cast<u32x4_t *>(dst), n16, sink);
    else
        hipLaunchKernelGGL((diag_stream_kernel<false>), grid, block, 0, stream, static_cast<const u32x4_t *>(src),
                           static_cast<u32x4_t *>(nullptr), n16, sink);
    return check_launch("tbn_diag_stream");
}

tbn_status launch_diag_mfma(int32_t blocks, int32_t iters, float *out, hipStream_t stream, bool fp4) {
    if (fp4) {
        hipLaunchKernelGGL(diag_mfma_fp4_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, iters, out);
        return check_launch("tbn_diag_mfma_fp4");
    }
    hipLaunchKernelGGL(diag_mfma_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, iters, out);
    return check_launch("tbn_diag_mfma");
}

}  // namespace tbn
