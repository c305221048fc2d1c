// Shape-agnostic kernels: one thread per output element, walking the flattened weight with a
// running tile index exactly as Algorithm 1 does (the index is never reset at a row start, it
// returns to zero after tile entry p-1 and the scalar index then moves on).  They accept every
// legal combination of sizes (tile shorter than a row, tile ends mid-row, k = 1, p = 1, ...) and
// serve as the fallback behind the specialised kernels.
#include "tbn_common.h"

namespace tbn {

template <typename T>
__global__ __launch_bounds__(256) void linear_generic_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t M,
                                                             int64_t in, int64_t out,
                                                             const uint32_t *__restrict__ tile, int64_t p,
                                                             const float *__restrict__ alpha, int32_t n_alpha,
                                                             int relu) {
    const int64_t o = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (o >= out) return;
    for (int64_t m = blockIdx.y; m < M; m += gridDim.y) {
        const T *xr = x + m * in;
        const int64_t f0 = o * in;
        int64_t ti = f0 % p;
        int64_t ai = (n_alpha == 1) ? 0 : f0 / p;
        float total = 0.f, seg = 0.f;
        int64_t j = 0;
        while (j < in) {
            const uint32_t word = tile[ti >> 5] >> (ti & 31);
            int64_t run = 32 - (ti & 31);
            if (run > in - j) run = in - j;
            if (run > p - ti) run = p - ti;
            for (int t = 0; t < (int)run; ++t) {
                const float xv = ElemIO<T>::load(xr + j + t);
                seg += ((word >> t) & 1u) ? xv : -xv;
            }
            j += run;
            ti += run;
            if (ti == p) {  // end of the tile: close the segment that used alpha[ai]
                total += alpha[ai] * seg;
                seg = 0.f;
                ti = 0;
                if (n_alpha != 1) ++ai;
            }
        }
        if (ai < n_alpha) total += alpha[ai] * seg;  // seg is empty when the row ended on a tile end
        if (relu) total = fmaxf(total, 0.f);
        ElemIO<T>::store(y + m * out + o, total);
    }
}

tbn_status launch_linear_generic(const LinearArgs &a) {
    const int relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    const int64_t gx = (a.out + 255) / 256;
    if (gx > 0x7fffffffLL) {
        set_error("tbn_linear_forward: out beyond the supported range");
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(a.M < 65535 ? a.M : 65535));
    if (a.dt == TBN_F32)
        hipLaunchKernelGGL(linear_generic_kernel<float>, grid, dim3(256), 0, a.stream, static_cast<const float *>(a.x),
                           static_cast<float *>(a.y), a.M, a.in, a.out, a.tile, a.p, a.alpha, a.n_alpha, relu);
    else
        hipLaunchKernelGGL(linear_generic_kernel<uint16_t>, grid, dim3(256), 0, a.stream,
                           static_cast<const uint16_t *>(a.x), static_cast<uint16_t *>(a.y), a.M, a.in, a.out, a.tile,
                           a.p, a.alpha, a.n_alpha, relu);
    return check_launch("tbn_linear_forward (generic kernel)");
}

// ends == 0: every output element.  ends > 0: only the output channels whose filter contains the
// start of tile number c = 1 .. ends (used after the matrix-core kernel, which scales such a
// channel by its first alpha only); `total` then counts N * ends * Ho * Wo candidates.
template <typename T>
__global__ __launch_bounds__(256) void conv_generic_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t total,
                                                           int64_t C, int64_t H, int64_t W, int64_t O, int64_t Ho,
                                                           int64_t Wo, int kh, int kw, int sh, int sw, int ph, int pw,
                                                           const uint32_t *__restrict__ tile, int64_t p,
                                                           const float *__restrict__ alpha, int32_t n_alpha,
                                                           int relu, int32_t ends) {
    const int64_t chans = ends > 0 ? ends : O;
    for (int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; idx < total;
         idx += int64_t(gridDim.x) * blockDim.x) {
        int64_t r = idx;
        const int64_t xo = r % Wo; r /= Wo;
        const int64_t yo = r % Ho; r /= Ho;
        int64_t o = r % chans;
        const int64_t b = r / chans;
        if (ends > 0) {
            const int64_t f = (o + 1) * p;             // flat index where tile number o + 1 starts
            if (f % (C * kh * kw) == 0) continue;      // it starts on a filter boundary: nothing to repair
            o = f / (C * kh * kw);
        }
        const int64_t f0 = o * C * kh * kw;  // flat index of this filter's first weight
        int64_t ti = f0 % p;
        int64_t ai = (n_alpha == 1) ? 0 : f0 / p;
        float acc = 0.f, seg = 0.f;
        for (int64_t c = 0; c < C; ++c) {
            const T *xc = x + (b * C + c) * H * W;
            for (int dy = 0; dy < kh; ++dy) {
                const int64_t yi = yo * sh + dy - ph;
                const bool row_ok = (yi >= 0 && yi < H);
                for (int dx = 0; dx < kw; ++dx) {
                    const int64_t xi = xo * sw + dx - pw;
                    if (row_ok && xi >= 0 && xi < W) {
                        const float xv = ElemIO<T>::load(xc + yi * W + xi);
                        seg += ((tile[ti >> 5] >> (ti & 31)) & 1u) ? xv : -xv;
                    }
                    if (++ti == p) {
                        acc += alpha[ai] * seg;
                        seg = 0.f;
                        ti = 0;
                        if (n_alpha != 1) ++ai;
                    }
                }
            }
        }
        if (ai < n_alpha) acc += alpha[ai] * seg;
        if (relu) acc = fmaxf(acc, 0.f);
        ElemIO<T>::store(y + ((b * O + o) * Ho + yo) * Wo + xo, acc);
    }
}

static tbn_status launch_conv_generic_impl(const ConvArgs &a, int32_t ends) {
    const int relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    const int64_t total = a.N * (ends > 0 ? ends : a.O) * a.Ho * a.Wo;
    if (total == 0) return TBN_OK;
    int64_t blocks = (total + 255) / 256;
    if (blocks > (1 << 20)) blocks = 1 << 20;
    const dim3 grid(static_cast<unsigned>(blocks));
    if (a.dt == TBN_F32)
        hipLaunchKernelGGL(conv_generic_kernel<float>, grid, dim3(256), 0, a.stream, static_cast<const float *>(a.x),
                           static_cast<float *>(a.y), total, a.C, a.H, a.W, a.O, a.Ho, a.Wo, a.kh, a.kw, a.sh, a.sw,
                           a.ph, a.pw, a.tile, a.p, a.alpha, a.n_alpha, relu, ends);
    else
        hipLaunchKernelGGL(conv_generic_kernel<uint16_t>, grid, dim3(256), 0, a.stream,
                           static_cast<const uint16_t *>(a.x), static_cast<uint16_t *>(a.y), total, a.C, a.H, a.W, a.O,
                           a.Ho, a.Wo, a.kh, a.kw, a.sh, a.sw, a.ph, a.pw, a.tile, a.p, a.alpha, a.n_alpha, relu, ends);
    return check_launch("tbn_conv2d_forward (generic kernel)");
}

tbn_status launch_conv_generic(const ConvArgs &a) { return launch_conv_generic_impl(a, 0); }

tbn_status launch_conv_generic_tile_ends(const ConvArgs &a) { return launch_conv_generic_impl(a, a.k - 1); }

}  // namespace tbn
