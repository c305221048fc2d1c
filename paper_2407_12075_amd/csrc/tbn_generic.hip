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

// Repair pass behind the matrix-core conv kernel, which scales a channel by one alpha: the (at most k - 1)
// output channels whose filter contains the start of a tile need two (Eq. 4-5: alpha changes where the
// tile index returns to zero).  Requires p >= C*kh*kw, so a filter holds at most one tile start.
// Workgroup = 64 output pixels of one (image, such channel); its four waves split the input channels,
// each thread keeps the sums before and after the tile start apart, LDS adds the four slices.
template <typename T, int TAPS>
__global__ __launch_bounds__(256) void conv_tile_end_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t C,
                                                            int64_t H, int64_t W, int64_t O, int64_t Ho, int64_t Wo,
                                                            int kh, int kw, int sh, int sw, int ph, int pw,
                                                            const uint32_t *__restrict__ tile, int64_t p,
                                                            const float *__restrict__ alpha, int relu) {
    __shared__ float part[4][64][2];
    const int64_t F = C * TAPS;
    const int64_t c_idx = int64_t(blockIdx.y) + 1;   // tile number whose start is looked at
    const int64_t f = c_idx * p;                     // flat index where it starts
    if (f % F == 0) return;                          // it starts on a filter boundary: nothing to repair (whole block)
    const int64_t o = f / F;
    if (o >= O) return;
    const int64_t b = blockIdx.z;
    const int px = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int64_t q = int64_t(blockIdx.x) * 64 + px;
    const bool live = q < Ho * Wo;
    const int64_t yo = live ? q / Wo : 0, xo = live ? q % Wo : 0;
    // element offsets of the taps inside a channel plane, -1 where the tap falls into the padding
    int32_t off[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
        const int64_t yi = yo * sh - ph + t / kw, xi = xo * sw - pw + t % kw;
        off[t] = (live && yi >= 0 && yi < H && xi >= 0 && xi < W) ? static_cast<int32_t>(yi * W + xi) : -1;
    }
    const int32_t cs = static_cast<int32_t>((C + 3) / 4);
    const int32_t c_lo = slice * cs, c_hi = (c_lo + cs) < C ? (c_lo + cs) : static_cast<int32_t>(C);
    const int64_t g0 = o * F + int64_t(c_lo) * TAPS;   // flat index of this slice's first weight
    int64_t ti = g0 % p;                               // its tile position
    int64_t before = f - g0;                           // weights of this slice before the tile start (may be <= 0)
    const int64_t n_words = (p + 31) / 32;
    float seg_a = 0.f, seg_b = 0.f;                    // sums over weights before / from the tile start
    const T *xc = x + (b * C + c_lo) * H * W;
    for (int32_t c = c_lo; c < c_hi; ++c, xc += H * W, before -= TAPS) {
        float xv[TAPS];
#pragma unroll
        for (int t = 0; t < TAPS; ++t) xv[t] = off[t] >= 0 ? ElemIO<T>::load(xc + off[t]) : 0.f;
        // the channel's TAPS tile bits: a window from ti on; the tile start may lie inside it
        uint32_t bits;
        if (ti + TAPS <= p) {
            const int64_t w = ti >> 5;
            const uint32_t lo = tile[w], hi = tile[(w + 1 < n_words) ? (w + 1) : w];
            bits = __funnelshift_r(lo, hi, static_cast<uint32_t>(ti & 31));
            ti += TAPS;
            if (ti == p) ti = 0;
        } else {   // once per tile
            bits = 0;
            for (int t = 0; t < TAPS; ++t) {
                bits |= ((tile[ti >> 5] >> (ti & 31)) & 1u) << t;
                if (++ti == p) ti = 0;
            }
        }
        float sa = 0.f, sb = 0.f;
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const float sv = ((bits >> t) & 1u) ? xv[t] : -xv[t];
            if (t < before) sa += sv; else sb += sv;
        }
        seg_a += sa;
        seg_b += sb;
    }
    part[slice][px][0] = seg_a;
    part[slice][px][1] = seg_b;
    __syncthreads();
    if (slice == 0 && live) {
        const float sa = (part[0][px][0] + part[1][px][0]) + (part[2][px][0] + part[3][px][0]);
        const float sb = (part[0][px][1] + part[1][px][1]) + (part[2][px][1] + part[3][px][1]);
        float v = alpha[c_idx - 1] * sa + alpha[c_idx] * sb;
        if (relu) v = fmaxf(v, 0.f);
        ElemIO<T>::store(y + ((b * O + o) * Ho + yo) * Wo + xo, v);
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

template <typename T, int TAPS>
static void launch_tile_end(const ConvArgs &a, dim3 grid, int relu) {
    hipLaunchKernelGGL((conv_tile_end_kernel<T, TAPS>), grid, dim3(256), 0, a.stream, static_cast<const T *>(a.x),
                       static_cast<T *>(a.y), a.C, a.H, a.W, a.O, a.Ho, a.Wo, a.kh, a.kw, a.sh, a.sw, a.ph, a.pw, a.tile,
                       a.p, a.alpha, relu);
}

tbn_status launch_conv_generic_tile_ends(const ConvArgs &a) {
    const int64_t F = a.C * a.kh * a.kw;
    const int taps = a.kh * a.kw;
    const int64_t pix_blocks = (a.Ho * a.Wo + 63) / 64;
    if (a.n_alpha != a.k || a.p < F || (taps != 1 && taps != 9) || a.H * a.W >= (int64_t(1) << 31) || a.k - 1 > 65535 ||
        a.N > 65535 || pix_blocks > 0x7fffffffLL)
        return launch_conv_generic_impl(a, a.k - 1);   // shapes the repair kernel does not take
    if (a.k < 2 || a.N == 0 || pix_blocks == 0) return TBN_OK;
    const int relu = (a.flags & TBN_FLAG_RELU) ? 1 : 0;
    const dim3 grid(static_cast<unsigned>(pix_blocks), static_cast<unsigned>(a.k - 1), static_cast<unsigned>(a.N));
    if (a.dt == TBN_F32) {
        if (taps == 1) launch_tile_end<float, 1>(a, grid, relu); else launch_tile_end<float, 9>(a, grid, relu);
    } else {
        if (taps == 1) launch_tile_end<uint16_t, 1>(a, grid, relu); else launch_tile_end<uint16_t, 9>(a, grid, relu);
    }
    return check_launch("tbn_conv2d_forward (tile-end repair kernel)");
}

}  // namespace tbn
