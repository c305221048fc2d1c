// Direct convolution for tiles of whole filters and window shapes the matrix-core kernel does not take
// (5x5, 7x7, ...: a network's first layer, if it is tiled at all).
//
// What is computed (Section "Method", Eq. 4-5, and Section "CNN Architectures"): weight (o, c, dy, dx) is tile bit
// (o*F + w) % p, F = C*kh*kw, w = (c*kh + dy)*kw + dx, scaled by alpha[(o*F + w) / p].  With p a multiple of F only
// the U = p / F filters of the tile are distinct and filter o = u + t*U is filter u scaled by alpha[t]: each distinct
// filter is applied once and its output channel is written k times.
//
// A workgroup owns 256 output pixels of one image (one per thread, so loads and stores run along the image rows)
// and 16 distinct filters.  The +-1 weights of those filters go through LDS as float32, 512 (channel, tap) positions
// at a time; a thread loads an input value once and feeds it to its 16 sums with values that every lane reads from
// the same LDS address (a broadcast), so an input element costs one load, four LDS reads and 16 multiply-adds.
// This is vector-ALU work (the 7x7, stride 2 first layer of a ResNet on 32 images: 3.8 G multiply-adds), far from
// the matrix cores' rate but an order of magnitude above one thread per output element.
#include "tbn_common.h"

namespace tbn {

namespace {

constexpr int kMaxFG = 16;     // distinct filters per workgroup: 16, or 4 where 16 would leave most of the chip idle
constexpr int kPixels = 256;   // output pixels per workgroup
constexpr int kStage = 512;    // (channel, tap) positions of a filter staged per pass

struct DirectParams {
    int64_t C, H, W, O, Ho, Wo;
    int32_t kh, kw, sh, sw, ph, pw;
    int64_t F;      // weights per filter
    int64_t U;      // distinct filters
    int32_t reps;   // O / U
    int32_t n_alpha, relu;
};

template <typename T, int kFG>
__global__ __launch_bounds__(kPixels) void conv_direct_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                              const uint32_t *__restrict__ tile,
                                                              const float *__restrict__ alpha, DirectParams P) {
    __shared__ __attribute__((aligned(16))) float w_lds[kStage][kFG];   // +1 / -1
    const int tid = threadIdx.x;
    const int64_t b = blockIdx.z;
    const int64_t u0 = int64_t(blockIdx.y) * kFG;
    const int64_t q = int64_t(blockIdx.x) * kPixels + tid;   // output pixel of the image, row-major
    const int64_t pixels = P.Ho * P.Wo;
    const bool live = q < pixels;
    const int32_t yo = live ? static_cast<int32_t>(q / P.Wo) : 0, xo = live ? static_cast<int32_t>(q % P.Wo) : 0;
    const int32_t yi0 = yo * P.sh - P.ph, xi0 = xo * P.sw - P.pw;
    const int32_t H = static_cast<int32_t>(P.H), W = static_cast<int32_t>(P.W);
    const int32_t plane = H * W;
    const T *xb = x + b * P.C * plane;

    float acc[kFG];
#pragma unroll
    for (int f = 0; f < kFG; ++f) acc[f] = 0.f;

    // (channel, row, column) of the window position, stepped along with the position (wave-uniform)
    int32_t c = 0, dy = 0, dx = 0;
    for (int64_t w0 = 0; w0 < P.F; w0 += kStage) {
        const int32_t n = static_cast<int32_t>(P.F - w0 < kStage ? P.F - w0 : kStage);
        __syncthreads();   // the previous pass is done with the staged weights
        for (int32_t e = tid; e < n; e += kPixels) {
#pragma unroll
            for (int f = 0; f < kFG; ++f) {
                const int64_t u = u0 + f < P.U ? u0 + f : P.U - 1;   // filters past U repeat the last one; never written
                const int64_t bit = u * P.F + w0 + e;               // < p
                w_lds[e][f] = ((tile[bit >> 5] >> (bit & 31)) & 1u) ? 1.f : -1.f;
            }
        }
        __syncthreads();
#pragma unroll 4
        for (int32_t e = 0; e < n; ++e) {
            const int32_t yi = yi0 + dy, xi = xi0 + dx;
            float xv = 0.f;
            if (live && yi >= 0 && yi < H && xi >= 0 && xi < W) xv = ElemIO<T>::load(xb + (c * plane + yi * W + xi));
            const float4 *wv = reinterpret_cast<const float4 *>(w_lds[e]);
#pragma unroll
            for (int g = 0; g < kFG / 4; ++g) {
                const float4 s = wv[g];
                acc[4 * g + 0] = fmaf(xv, s.x, acc[4 * g + 0]);
                acc[4 * g + 1] = fmaf(xv, s.y, acc[4 * g + 1]);
                acc[4 * g + 2] = fmaf(xv, s.z, acc[4 * g + 2]);
                acc[4 * g + 3] = fmaf(xv, s.w, acc[4 * g + 3]);
            }
            if (++dx == P.kw) {
                dx = 0;
                if (++dy == P.kh) { dy = 0; ++c; }
            }
        }
    }

    if (!live) return;
    T *yb = y + b * P.O * pixels + q;
#pragma unroll
    for (int f = 0; f < kFG; ++f) {
        const int64_t u = u0 + f;
        if (u >= P.U) break;
        for (int32_t t = 0; t < P.reps; ++t) {
            float v = alpha[P.n_alpha == 1 ? 0 : t] * acc[f];
            if (P.relu) v = fmaxf(v, 0.f);
            ElemIO<T>::store(yb + (u + int64_t(t) * P.U) * pixels, v);
        }
    }
}

}  // namespace

// Shapes this kernel takes: tile of whole filters, one image plane addressable in 32 bits, grid within the limits.
bool conv_direct_supported(const ConvArgs &a) {
    if (a.dt != TBN_F32 && a.dt != TBN_BF16) return false;
    const int64_t F = a.C * a.kh * a.kw;
    if (F <= 0 || a.p % F != 0) return false;
    const int64_t U = a.p / F;
    if (U < 1 || U > a.O || a.O % U != 0) return false;
    if (a.n_alpha != 1 && a.n_alpha != a.O / U) return false;
    if (a.C * a.H * a.W >= (int64_t(1) << 31) || a.Ho * a.Wo >= (int64_t(1) << 31)) return false;
    if (a.N > 65535 || (U + 3) / 4 > 65535 || (a.Ho * a.Wo + kPixels - 1) / kPixels > 0x7fffffffLL) return false;
    return true;
}

tbn_status launch_conv_direct(const ConvArgs &a) {
    if (a.N == 0 || a.Ho <= 0 || a.Wo <= 0 || a.O == 0) return TBN_OK;
    DirectParams P;
    P.C = a.C; P.H = a.H; P.W = a.W; P.O = a.O; P.Ho = a.Ho; P.Wo = a.Wo;
    P.kh = a.kh; P.kw = a.kw; P.sh = a.sh; P.sw = a.sw; P.ph = a.ph; P.pw = a.pw;
    P.F = a.C * a.kh * a.kw;
    P.U = a.p / P.F;
    P.reps = static_cast<int32_t>(a.O / P.U);
    P.n_alpha = a.n_alpha;
    P.relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    // 16 distinct filters per workgroup; 4 where that would give the chip fewer than two workgroups per CU (an input
    // element then feeds four sums instead of 16, but four times the threads work: 5x5, 64 -> 64 channels on 28 x 28
    // maps, 32 images, 16 distinct filters: 128 workgroups at 16)
    const int64_t pix_blocks = (a.Ho * a.Wo + kPixels - 1) / kPixels;
    const bool narrow = pix_blocks * a.N * ((P.U + kMaxFG - 1) / kMaxFG) < 512;
    const int fg = narrow ? 4 : kMaxFG;
    const dim3 grid(static_cast<unsigned>(pix_blocks), static_cast<unsigned>((P.U + fg - 1) / fg), static_cast<unsigned>(a.N));
#define TBN_CONV_DIRECT_LAUNCH(T, FG)                                                                                     \
    hipLaunchKernelGGL((conv_direct_kernel<T, FG>), grid, dim3(kPixels), 0, a.stream, static_cast<const T *>(a.x),          \
                       static_cast<T *>(a.y), a.tile, a.alpha, P)
    if (a.dt == TBN_F32) {
        if (narrow) TBN_CONV_DIRECT_LAUNCH(float, 4); else TBN_CONV_DIRECT_LAUNCH(float, kMaxFG);
    } else {
        if (narrow) TBN_CONV_DIRECT_LAUNCH(uint16_t, 4); else TBN_CONV_DIRECT_LAUNCH(uint16_t, kMaxFG);
    }
#undef TBN_CONV_DIRECT_LAUNCH
    return check_launch("tbn_conv2d_forward (direct kernel)");
}

}  // namespace tbn
