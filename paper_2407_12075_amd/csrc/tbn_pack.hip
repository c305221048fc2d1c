// tbn_pack_tile: tile construction (Eq. 1-3) and scalars (Eq. 6, Eq. 7-8) in one pass over
// the real weights.
//
// The flattened weight is viewed as k rows of p entries (Eq. 1).  A thread owns a few tile
// positions i and walks the k rows in ascending order, so its loads of row r are coalesced
// with its neighbours' and each weight is read exactly once.  Column sums s_i (Eq. 2) are kept
// in double precision in row order, which makes the sign (Eq. 3) independent of the launch
// shape and identical to a sequential double-precision sum.  |a| is summed per row in double
// precision: a wave reduces its share of row r and writes one partial per (wave, r) to the
// workspace; a second small kernel adds the partials in a fixed order and divides (Eq. 6 / 8).
// No floating-point atomics are used, so results are reproducible bit for bit.
//
// The same kernels build the tile of the column-tiled layout (GPU Inference Kernel section): there the k
// summands of tile position i = o * blk + j are the entries (o, r * blk + j) of an out x in matrix with
// blk = in / k, i.e. summand r of position i sits at (i / blk) * ld + r * blk + i % blk with ld = in.  The flat
// layout of Eq. 1 is the case blk = p (one "row" holds the whole tile).
#include "tbn_common.h"

#include <mutex>

namespace tbn {

constexpr int kPackThreads = 256;
constexpr int kPackWaves = kPackThreads / kWave;
constexpr int kPackQ = 4;  // loads per row per thread

template <int VEC> struct PackVec;
template <> struct PackVec<4> { using type = float4; };
template <> struct PackVec<1> { using type = float; };

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// positions handled by one block: kPackThreads * VEC * kPackQ, a multiple of 64
template <int VEC, bool SEPARATE_A>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(const float *__restrict__ w,
                                                            const float *__restrict__ a, int64_t p, int32_t k,
                                                            int64_t blk, int64_t ld,
                                                            uint32_t *__restrict__ tile_out, int64_t n_words,
                                                            double *__restrict__ partial) {
    constexpr int64_t kChunk = int64_t(kPackThreads) * VEC;   // positions covered by one load round
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int64_t block_base = int64_t(blockIdx.x) * kChunk * kPackQ;

    double s[kPackQ][VEC];
#pragma unroll
    for (int q = 0; q < kPackQ; ++q)
#pragma unroll
        for (int v = 0; v < VEC; ++v) s[q][v] = 0.0;

    int64_t pos[kPackQ];   // offset of summand 0 of the thread's positions
    bool live[kPackQ];
#pragma unroll
    for (int q = 0; q < kPackQ; ++q) {
        const int64_t i = block_base + q * kChunk + int64_t(tid) * VEC;
        live[q] = i < p;  // VEC == 4 is only used when p % 4 == 0: a vector is all in or all out
        pos[q] = (blk == p || !live[q]) ? i : (i / blk) * ld + i % blk;   // blk % 4 == 0 with VEC == 4: no vector spans two rows
    }

    double *my_partial = partial + (int64_t(blockIdx.x) * kPackWaves + wave) * k;

    for (int32_t r = 0; r < k; ++r) {
        const float *wr = w + int64_t(r) * blk;
        const float *ar = SEPARATE_A ? a + int64_t(r) * blk : wr;
        float wv[kPackQ][VEC];
        float av[kPackQ][VEC];
#pragma unroll
        for (int q = 0; q < kPackQ; ++q) {
            if (live[q]) {
                if constexpr (VEC == 4) {
                    const float4 t = *reinterpret_cast<const float4 *>(wr + pos[q]);
                    wv[q][0] = t.x; wv[q][1] = t.y; wv[q][2] = t.z; wv[q][3] = t.w;
                    if constexpr (SEPARATE_A) {
                        const float4 u = *reinterpret_cast<const float4 *>(ar + pos[q]);
                        av[q][0] = u.x; av[q][1] = u.y; av[q][2] = u.z; av[q][3] = u.w;
                    }
                } else {
                    wv[q][0] = wr[pos[q]];
                    if constexpr (SEPARATE_A) av[q][0] = ar[pos[q]];
                }
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) { wv[q][v] = 0.f; av[q][v] = 0.f; }
            }
        }
        double l1 = 0.0;
#pragma unroll
        for (int q = 0; q < kPackQ; ++q)
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                s[q][v] += static_cast<double>(wv[q][v]);
                l1 += static_cast<double>(fabsf(SEPARATE_A ? av[q][v] : wv[q][v]));
            }
        l1 = wave_sum_f64(l1);
        if (lane == 0) my_partial[r] = l1;
    }

    // Eq. 3 and bit packing, LSB first
#pragma unroll
    for (int q = 0; q < kPackQ; ++q) {
        if constexpr (VEC == 4) {
            uint32_t nib = 0;
#pragma unroll
            for (int v = 0; v < 4; ++v) nib |= (s[q][v] > 0.0 ? 1u : 0u) << v;
            uint32_t word = nib << (4 * (lane & 7));
            word |= __shfl_xor(word, 1, kWave);
            word |= __shfl_xor(word, 2, kWave);
            word |= __shfl_xor(word, 4, kWave);
            const int64_t wi = (block_base + q * kChunk + int64_t(tid & ~7) * 4) >> 5;
            if ((lane & 7) == 0 && wi < n_words) tile_out[wi] = word;
        } else {
            const unsigned long long mask = __ballot(s[q][0] > 0.0);
            const int64_t wi = (block_base + q * kChunk + int64_t(wave) * kWave) >> 5;
            if (lane == 0 && wi < n_words) tile_out[wi] = static_cast<uint32_t>(mask);
            if (lane == 1 && wi + 1 < n_words) tile_out[wi + 1] = static_cast<uint32_t>(mask >> 32);
        }
    }
}

// alpha[r] = (sum over all (block, wave) partials of row r) / p, or one alpha = total / n.
// One block per output scalar; fixed strided order + fixed tree -> reproducible.
__global__ __launch_bounds__(256) void pack_alpha_kernel(const double *__restrict__ partial, int64_t n_part,
                                                         int32_t k, int32_t n_alpha, int64_t p,
                                                         float *__restrict__ alpha_out) {
    __shared__ double red[256 / kWave];
    const int tid = threadIdx.x;
    const int32_t r_begin = (n_alpha == 1) ? 0 : blockIdx.x;
    const int32_t r_end = (n_alpha == 1) ? k : blockIdx.x + 1;
    double acc = 0.0;
    for (int32_t r = r_begin; r < r_end; ++r) {
        int64_t i = tid;
        for (; i + 7 * 256 < n_part; i += 8 * 256) {   // eight independent loads in flight
            double t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = partial[(i + j * 256) * k + r];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += t[j];
        }
        for (; i < n_part; i += 256) acc += partial[i * k + r];
    }
    acc = wave_sum_f64(acc);
    if ((tid & (kWave - 1)) == 0) red[tid / kWave] = acc;
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
#pragma unroll
        for (int wv = 0; wv < 256 / kWave; ++wv) total += red[wv];
        const double denom = (n_alpha == 1) ? static_cast<double>(p) * static_cast<double>(k) : static_cast<double>(p);
        alpha_out[blockIdx.x] = static_cast<float>(total / denom);
    }
}

static int64_t pack_blocks(int64_t p, int vec) {
    const int64_t per_block = int64_t(kPackThreads) * vec * kPackQ;
    return (p + per_block - 1) / per_block;
}

size_t pack_workspace_bytes(int64_t n, int32_t k, int32_t /*n_alpha*/) {
    // sized for the scalar-load variant (the larger grid) so the choice of variant, which
    // depends on pointer alignment, never changes the requirement
    const int64_t p = n / k;
    return static_cast<size_t>(pack_blocks(p, 1) * kPackWaves * k) * sizeof(double);
}

tbn_status launch_pack(const float *w, const float *a, int64_t n, int32_t k, int32_t n_alpha,
                       uint32_t *tile_out, float *alpha_out, void *workspace, hipStream_t stream,
                       int64_t blk, int64_t ld) {
    const int64_t p = n / k;
    const int64_t n_words = (p + 31) / 32;
    if (blk <= 0) { blk = p; ld = 0; }   // flat layout
    const bool vec4 = (p % 4 == 0) && (blk % 4 == 0) && (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(w) & 15u) == 0) &&
                      (!a || (reinterpret_cast<uintptr_t>(a) & 15u) == 0);
    const int64_t blocks = pack_blocks(p, vec4 ? 4 : 1);
    if (blocks > 0x7fffffffLL) {
        set_error("tbn_pack_tile: tile of %lld bits is beyond the supported range", (long long)p);
        return TBN_ERR_UNSUPPORTED;
    }
    double *partial = static_cast<double *>(workspace);
    const dim3 grid(static_cast<unsigned>(blocks)), block(kPackThreads);
    if (vec4) {
        if (a) hipLaunchKernelGGL((pack_kernel<4, true>), grid, block, 0, stream, w, a, p, k, blk, ld, tile_out, n_words, partial);
        else   hipLaunchKernelGGL((pack_kernel<4, false>), grid, block, 0, stream, w, a, p, k, blk, ld, tile_out, n_words, partial);
    } else {
        if (a) hipLaunchKernelGGL((pack_kernel<1, true>), grid, block, 0, stream, w, a, p, k, blk, ld, tile_out, n_words, partial);
        else   hipLaunchKernelGGL((pack_kernel<1, false>), grid, block, 0, stream, w, a, p, k, blk, ld, tile_out, n_words, partial);
    }
    tbn_status st = check_launch("tbn_pack_tile (tile kernel)");
    if (st != TBN_OK) return st;
    hipLaunchKernelGGL(pack_alpha_kernel, dim3(static_cast<unsigned>(n_alpha)), dim3(256), 0, stream, partial,
                       blocks * kPackWaves, k, n_alpha, p, alpha_out);
    return check_launch("tbn_pack_tile (alpha kernel)");
}

// ---- tbn_pack_tile_noalloc: the same two kernels with the partial sums in a file-scope device array ----------
// Every GPU the library runs on holds its own copy of the array at its own address until the process ends.  In
// host code the array's name is only a stand-in for the symbol: the device address is looked up once per device,
// with that device current, and that pointer is what the kernels and every other use get.
static __device__ __align__(256) unsigned char scratch[TBN_PACK_NOALLOC_SCRATCH_BYTES];

static tbn_status pack_scratch_address(void **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *address[kMaxDevices] = {};
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess || device < 0 || device >= kMaxDevices) {
        set_error("tbn_pack_tile_noalloc: cannot identify the current device: %s",
                  e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
        return TBN_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!address[device]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_error("tbn_pack_tile_noalloc: cannot resolve the scratch array on device %d: %s", device,
                      hipGetErrorString(e));
            return TBN_ERR_DEVICE;
        }
        address[device] = ptr;
    }
    *out = address[device];
    return TBN_OK;
}

tbn_status launch_pack_noalloc(const float *w, const float *a, int64_t n, int32_t k, int32_t n_alpha,
                               uint32_t *tile_out, float *alpha_out, hipStream_t stream) {
    const size_t need = pack_workspace_bytes(n, k, n_alpha);
    if (need > sizeof(scratch)) {
        set_error("tbn_pack_tile_noalloc: these sizes need %zu bytes of scratch memory, the built-in array holds %zu; "
                  "use tbn_pack_tile with a workspace", need, sizeof(scratch));
        return TBN_ERR_UNSUPPORTED;
    }
    void *ptr = nullptr;
    tbn_status st = pack_scratch_address(&ptr);
    if (st != TBN_OK) return st;
    // nothing in the array has to start at zero: every partial sum that the second kernel reads is written by
    // the first one of the same call
    return launch_pack(w, a, n, k, n_alpha, tile_out, alpha_out, ptr, stream);
}

}  // namespace tbn
