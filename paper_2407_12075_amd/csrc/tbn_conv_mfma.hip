// Matrix-core kernel for the convolutional tiled-bit layer.
//
// The flattened (O, C, kh, kw) weight is the tile repeated k times (Eq. 4-5), so the filter of
// output channel o is the cyclic tile window that starts at bit (o*F) % p, F = C*kh*kw.  That start
// has period R = p / gcd(F, p) in o: only R distinct +-1 filters exist and, as the paper notes for
// its two-channel example (Section "CNN Architectures"), the other output channels are copies up
// to alpha.  The kernel computes the R distinct channels once per image block and writes every
// replica o = u + t*R as alpha(o) * Z[u].  When the tile holds whole filters (p % F == 0), R = p / F
// and alpha(o) = alpha[t]; otherwise alpha(o) = alpha[(o*F) / p] and the few channels whose filter
// contains a tile end (two alphas) are recomputed afterwards by the shape-agnostic kernel.
//
// gfx950 mapping (implicit GEMM on v_mfma_f32_16x16x32_bf16, filters as rows, pixels as columns):
//   * workgroup = one image, a block of output rows (<= 128 pixels = 8 tiles of 16; a row whose input patch is too
//     wide to stage is cut into equal column blocks) and 32 distinct filters:
//     8 waves, each owning one pixel tile x the 2 tiles of 16 filters (64 filters for bf16 inputs where that
//     many exist: then 4 waves of two pixel tiles x 4 filter tiles);
//   * K runs over chunks of 32 input channels (a short last chunk is filled with zeros); inside a chunk over the kh*kw taps, so that one MFMA
//     step (K = 32) is "32 channels of one tap".  The input patch of a chunk (with its zero halo)
//     is staged in LDS channel-last as bf16, which makes the 8 channels a lane needs one 16-byte
//     LDS read at (pixel + tap offset); float32 inputs are split exactly into three bf16 planes
//     (the weights are +-1, so products are exact; sums are float32 in the matrix pipe);
//   * the filter bits are reordered once per workgroup from (channel, tap) to (tap, channel) order
//     into LDS, 32 channels per word; a lane expands its byte of a word into a +-1 bf16 operand by
//     replicating it (v_perm), shifting both halves so that two neighbouring bits land on the two sign
//     positions (v_pk_lshlrev_b16) and merging with the pattern of 1.0;
//   * the operand reads run several MFMAs ahead of their use (explicit waits); the next chunk's input
//     is on its way from global memory while the current one is multiplied and is converted in the
//     shadow of the last taps' MFMAs.
#include "tbn_common.h"

#include <algorithm>
#include <type_traits>

namespace tbn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

namespace {

// Waves per workgroup.  With 32 distinct filters per workgroup 8 waves share the 8 pixel tiles, one each: two
// waves per SIMD cover each other's waits (a 14 x 14 layer's waves spent 41 % of their life waiting with one
// wave per SIMD) and the prologue and the staging are spread over twice the threads: 4 - 18 % faster.  With 64
// filters (bf16) 4 waves of two pixel tiles each measured faster: the expanded filter operands serve twice the
// MFMAs.
constexpr int waves_of(int nft) { return nft == 4 ? 4 : 8; }
constexpr int kFtSmall = 2;        // MFMA row tiles of 16 distinct filters per workgroup: 32 filters,
constexpr int kFtLarge = 4;        // or 64 where there are that many (the staged input then feeds twice the MFMAs)
constexpr int kCK = 32;            // input channels per chunk (one MFMA step per tap)
constexpr int kMaxPix = 128;       // output pixels per workgroup (8 MFMA column tiles)
constexpr int kItemsSmall = 2560;   // staged (channel pair, pixel) items per workgroup and chunk: patches up to 160 pixels
constexpr int kItemsLarge = 3072;   // ... up to 192 pixels (one output row of a 56- to 62-wide image with its 3x3 halo)
constexpr int kPixStride = kCK * 2 + 16;   // bytes per patch pixel in LDS: 32 bf16 channels + 16 B padding

constexpr __host__ __device__ int n_chunks_of(int64_t C) { return static_cast<int>((C + kCK - 1) / kCK); }

struct ConvMfmaParams {
    int64_t N, C, H, W, O, Ho, Wo;
    int32_t kh, kw, sh, sw, ph, pw;
    int64_t F;            // filter length C*kh*kw
    int64_t R;            // distinct filters
    int64_t p, n_words;   // tile bits / words
    int32_t aligned;      // p % F == 0
    int32_t n_alpha;
    int32_t rows_per_blk; // output rows per workgroup
    int32_t cols_per_blk; // output columns per workgroup (Wo unless a row's patch is too wide to stage)
    int32_t n_colblk;     // column blocks per row block
    int32_t PR, PC;       // input patch rows / columns (with halo)
    int32_t plane_bytes;  // PR*PC*kPixStride
};

template <typename XT> struct CTraits;
template <> struct CTraits<float> { static constexpr int planes = 3; };
template <> struct CTraits<uint16_t> { static constexpr int planes = 1; };

// truncation split of a float into three bf16 terms (top 8 significand bits, next 8, the rest)
__device__ __forceinline__ void split3(float x, uint32_t &t0, uint32_t &t1, uint32_t &t2) {
    t0 = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(t0);
    t1 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(t1);
    t2 = __float_as_uint(r2);
}

// high halves of two words in one: (lo >> 16) | (hi & 0xffff0000), a single v_perm_b32
__device__ __forceinline__ uint32_t pack_hi16(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x07060302u); }

// Staged inputs stay as loaded (float32 values / zero-extended bf16 patterns): nothing is computed from them
// before the conversion step, so no wait for the loads is placed ahead of it.
__device__ __forceinline__ uint32_t load_raw(const float *p) { return __float_as_uint(*p); }
__device__ __forceinline__ uint32_t load_raw(const uint16_t *p) { return *p; }

// FIX: the repair pass behind the main pass when tiles end inside filters (one alpha per tile).  The main pass
// scales a whole output channel by the alpha of its first weight; a channel whose filter contains the start of tile
// number c (flat index c * p, at most one per filter since p >= F) needs alpha[c - 1] for the weights before it and
// alpha[c] from it on.  Here the "distinct filters" of a workgroup are pairs of masked copies of such filters:
// pseudo-filter 2i keeps the weights before the start of tile u0 / 2 + i + 1 and has zeros after it, pseudo-filter
// 2i + 1 the rest (a zero weight is the +-1 pattern ANDed away: +0.0 in bfloat16).  A lane's accumulators hold both
// halves of a pair, so the epilogue writes alpha[c - 1] * before + alpha[c] * after over what the main pass wrote.
// SHORT: C is no multiple of 32; the channels that the last chunk lacks are staged as zeros (a form of its own: the
// extra selects in the loads cost the other form registers it does not have).
template <typename XT, int T, bool RELU, int kBudget, int NFT, bool FIX, bool SHORT>
__global__ __launch_bounds__((64 * waves_of(NFT)), (waves_of(NFT) == 8 ? 4 : 2)) void conv_mfma_kernel(const XT *__restrict__ x, XT *__restrict__ y,
                                                                  const uint32_t *__restrict__ tile,
                                                                  const float *__restrict__ alpha, ConvMfmaParams P) {
    constexpr int NP = CTraits<XT>::planes;
    constexpr int kFB = 16 * NFT;   // distinct filters per workgroup
    constexpr int kWaves = waves_of(NFT), kThreads = 64 * kWaves;
    constexpr int kTilesPerWave = 8 / kWaves;      // pixel tiles of 16 per wave
    constexpr int kMaxItems = kBudget / kThreads;  // staged items per thread and chunk
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    // layout: patch buffers [2][NP][PR*PC][kPixStride bytes], then filter bits [chunk][tap][kFB filters]
    unsigned char *lds_patch = lds_raw;
    const int buf_bytes = NP * P.plane_bytes;
    uint32_t *lds_bits = reinterpret_cast<uint32_t *>(lds_raw + 2 * buf_bytes);
    uint32_t *lds_mask = lds_bits + T * n_chunks_of(P.C) * kFB;   // FIX only: which weights a pseudo-filter keeps, same layout

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    const int n_chunks = static_cast<int>((P.C + kCK - 1) / kCK);   // the last chunk may be short: its missing channels are staged as zeros
    // Workgroups are dispatched in the order of their linear id and dealt round-robin to the 8 XCDs.  All workgroups of
    // one image -- its row and column blocks, whose patches overlap, and its filter blocks, which stage the same input --
    // take consecutive slots of one XCD, so that the image is fetched from HBM once and then found in that XCD's L2
    // (plain order fetched 219 MB for 26 MB of input on 128 x 256 x 14 x 14 with eight filter blocks).
    uint32_t blk_x, blk_z;
    int64_t img;
    {
        const uint32_t lid = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
        const uint32_t per_img = gridDim.x * gridDim.z, n_img = gridDim.y;
        const uint32_t xcd = lid & 7, slot = lid >> 3, full = (n_img / 8) * per_img;   // slots per XCD in the regular part
        uint32_t inner;
        if (slot < full) {
            const uint32_t q = slot / per_img;
            inner = slot - q * per_img;
            img = q * 8 + xcd;
        } else {   // the remaining images: plain order
            const uint32_t rest = lid - full * 8, q = rest / per_img;
            inner = rest - q * per_img;
            img = (n_img / 8) * 8 + q;
        }
        blk_z = inner / gridDim.x;
        blk_x = inner - blk_z * gridDim.x;
    }
    const int rb = static_cast<int>(blk_x) / P.n_colblk, cb = static_cast<int>(blk_x) - rb * P.n_colblk;
    const int row0 = rb * P.rows_per_blk;                                 // first output row of the block
    const int col0 = cb * P.cols_per_blk;                                 // first output column
    const int rows = (P.Ho - row0) < P.rows_per_blk ? static_cast<int>(P.Ho - row0) : P.rows_per_blk;
    const int cols = (P.Wo - col0) < P.cols_per_blk ? static_cast<int>(P.Wo - col0) : P.cols_per_blk;
    const int PX = rows * cols;                                           // output pixels of the block, row-major
    const int64_t u0 = int64_t(blk_z) * kFB;                              // first distinct filter of the block

    // ---- staging items: (channel pair cp, valid patch pixel) -> registers -> LDS --------------------
    // valid patch pixels = patch positions inside the image, enumerated row-major
    const int iy_first = row0 * P.sh - P.ph;                               // image row of patch row 0 (may be < 0)
    const int ix_first = col0 * P.sw - P.pw;                               // image column of patch column 0 (may be < 0)
    const int py_lo = iy_first < 0 ? -iy_first : 0;
    const int py_hi = (iy_first + P.PR) > P.H ? static_cast<int>(P.H - iy_first) : P.PR;   // exclusive
    const int px_lo = ix_first < 0 ? -ix_first : 0;
    const int px_hi = (ix_first + P.PC) > P.W ? static_cast<int>(P.W - ix_first) : P.PC;   // exclusive
    const int vrows = py_hi > py_lo ? py_hi - py_lo : 0, vcols = px_hi > px_lo ? px_hi - px_lo : 0;
    const int npix = vrows * vcols;
    const int n_items = npix * (kCK / 2);
    int32_t it_goff[kMaxItems];   // element offset inside the chunk's first channel plane, or -1
    int32_t it_loff[kMaxItems];   // byte offset inside a patch plane: pixel * kPixStride + 4 * channel pair
    {
        // item q = tid + i * kThreads is (channel pair, valid row, valid column) = (q / npix, (q % npix) / vcols,
        // q % vcols); the thread divides once and then steps by kThreads items with carries
        const int np1 = npix > 0 ? npix : 1, vc1 = vcols > 0 ? vcols : 1;
        int cp = tid / np1, pix = tid % np1;
        int ry = pix / vc1, rx = pix % vc1;
        const int d_cp = kThreads / np1, d_pix = kThreads % np1;   // uniform
        const int d_ry = d_pix / vc1, d_rx = d_pix % vc1;
        const int vr1 = vrows > 0 ? vrows : 1;
#pragma unroll
        for (int i = 0; i < kMaxItems; ++i) {
            const int q = tid + i * kThreads;
            if (q < n_items) {
                const int py = py_lo + ry, px = px_lo + rx;
                it_goff[i] = static_cast<int32_t>((2 * cp) * P.H * P.W + int64_t(iy_first + py) * P.W + (ix_first + px));
                it_loff[i] = (py * P.PC + px) * kPixStride + cp * 4;
            } else {
                it_goff[i] = -1;
                it_loff[i] = 0;
            }
            rx += d_rx; ry += d_ry; cp += d_cp;
            if (rx >= vc1) { rx -= vc1; ++ry; }
            if (ry >= vr1) { ry -= vr1; ++cp; }
        }
    }
    const int64_t plane_hw = P.H * P.W;
    const XT *x_img = x + img * P.C * plane_hw;

    uint32_t st_a[1][kMaxItems], st_b[1][kMaxItems];   // the two channels of a pair, as loaded
    uint32_t st_pk[kMaxItems][NP];                  // ... split and packed, ready for LDS
    auto load_chunk = [&](int chunk, int slot) {
        const XT *base = x_img + int64_t(chunk) * kCK * plane_hw;
        const int c_left = static_cast<int>(P.C) - chunk * kCK;   // channels of this chunk that exist (uniform)
        if (!SHORT || c_left >= kCK) {
#pragma unroll
            for (int i = 0; i < kMaxItems; ++i) {
                const int32_t g = it_goff[i] < 0 ? 0 : it_goff[i];
                st_a[slot][i] = load_raw(base + g);
                st_b[slot][i] = load_raw(base + g + plane_hw);
            }
        } else {   // short last chunk: channels past C read as zero (and nothing past the end of x is touched)
#pragma unroll
            for (int i = 0; i < kMaxItems; ++i) {
                const int ch = (it_loff[i] % kPixStride) / 2;   // first channel of the pair inside the chunk
                const bool ok_a = it_goff[i] >= 0 && ch < c_left, ok_b = it_goff[i] >= 0 && ch + 1 < c_left;
                const uint32_t va = load_raw(base + (ok_a ? it_goff[i] : 0));
                const uint32_t vb = load_raw(base + (ok_b ? it_goff[i] + plane_hw : 0));
                st_a[slot][i] = ok_a ? va : 0u;
                st_b[slot][i] = ok_b ? vb : 0u;
            }
        }
    };
    auto pack_item = [&](int i, int slot) {   // VALU only
        if (NP == 3) {
            uint32_t a0, a1, a2, b0, b1, b2;
            split3(__uint_as_float(st_a[slot][i]), a0, a1, a2);
            split3(__uint_as_float(st_b[slot][i]), b0, b1, b2);
            st_pk[i][0] = pack_hi16(a0, b0);
            st_pk[i][NP > 1 ? 1 : 0] = pack_hi16(a1, b1);
            st_pk[i][NP > 2 ? 2 : 0] = pack_hi16(a2, b2);
        } else {   // bf16 input: the two patterns side by side, a single v_perm_b32
            st_pk[i][0] = __builtin_amdgcn_perm(st_b[slot][i], st_a[slot][i], 0x05040100u);
        }
    };
    auto store_chunk = [&](int buf) {
        unsigned char *dst = lds_patch + buf * buf_bytes;
#pragma unroll
        for (int i = 0; i < kMaxItems; ++i) {
            if (it_goff[i] < 0) continue;
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
                *reinterpret_cast<uint32_t *>(dst + pl * P.plane_bytes + it_loff[i]) = st_pk[i][pl];
        }
    };

    // The first chunk's loads are issued before the zero fill and the filter-bit transposition, which hide their
    // trip to memory.
    load_chunk(0, 0);

    // ---- zero both patch buffers (halo positions and padding stay zero for the whole kernel) ----
    for (int i = tid * 16; i < 2 * buf_bytes; i += kThreads * 16)
        *reinterpret_cast<u32x4_t *>(lds_patch + i) = u32x4_t{0u, 0u, 0u, 0u};

    const uint32_t tile_head = tile[0];
    // ---- filter bits: (channel, tap) order in the tile -> one word per (chunk, tap, filter) -------
    // A thread transposes the 32 x T bit block of one (filter, chunk): T consecutive words in, T out.
    for (int id = tid; id < kFB * n_chunks; id += kThreads) {
        const int u = id % kFB, chunk = id / kFB;
        uint32_t w[T], o[T];
        int64_t filt = u0 + u;          // filter whose bits are read
        bool live = filt < P.R;
        int64_t keep_before = 0;        // FIX: weights of the filter before the tile start
        if constexpr (FIX) {
            const int64_t c = (u0 + u) / 2 + 1;              // tile number whose start is looked at
            const int64_t f = c * P.p;                       // flat index where it starts
            filt = f / P.F;
            keep_before = f - filt * P.F;
            live = c < P.n_alpha && keep_before != 0 && filt < P.O;   // n_alpha == k; a start on a filter boundary needs no repair
            if (!live) filt = 0;
        }
        if (!FIX && !SHORT && P.aligned) {
            // whole filters per tile and whole chunks (so F % 32 == 0): the block is T consecutive words of the tile
            const int64_t word0 = (filt * P.F) / 32 + int64_t(chunk) * T;
#pragma unroll
            for (int i = 0; i < T; ++i) w[i] = live ? tile[word0 + i] : 0u;
        } else {
            // the 32*T bits of this (filter, chunk) start at cyclic tile position pos; all loads are
            // issued first (unconditionally, with clamped indices) so that they overlap
            int64_t pos = live ? (filt * P.F + int64_t(chunk) * 32 * T) % P.p : 0;
            uint32_t lo[T], hi[T];
            int64_t wpos[T];
    #pragma unroll
            for (int i = 0; i < T; ++i) {
                wpos[i] = pos;
                const int64_t wi = pos >> 5;
                lo[i] = tile[wi];
                hi[i] = tile[(wi + 1 < P.n_words) ? (wi + 1) : wi];
                pos += 32;
                if (pos >= P.p) pos -= P.p;
            }
    #pragma unroll
            for (int i = 0; i < T; ++i) {
                const uint32_t hi_ok = ((wpos[i] >> 5) + 1 < P.n_words) ? hi[i] : 0u;
                uint32_t v = __funnelshift_r(lo[i], hi_ok, static_cast<uint32_t>(wpos[i] & 31));
                const int64_t left = P.p - wpos[i];   // bits before the tile end; the window continues at bit 0
                if (left < 32) v = (v & ((1u << left) - 1u)) | (tile_head << left);
                w[i] = live ? v : 0u;
            }
        }
#pragma unroll
        for (int tap = 0; tap < T; ++tap) {
            uint32_t acc = 0;
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int pos = j * T + tap;   // bit of channel j, this tap, inside the block
                acc |= __builtin_amdgcn_ubfe(w[pos >> 5], pos & 31, 1) << j;   // bit extract, shift-or
            }
            o[tap] = acc;   // bit j = channel j of the chunk
        }
#pragma unroll
        for (int tap = 0; tap < T; ++tap) lds_bits[(chunk * T + tap) * kFB + u] = o[tap];
        if constexpr (FIX) {
            // weight (channel j of the chunk, tap) has index chunk * 32 * T + j * T + tap inside the filter: the channels
            // with an index below keep_before are j < ceil((keep_before - chunk * 32 * T - tap) / T)
            const int64_t rem = keep_before - int64_t(chunk) * 32 * T;
#pragma unroll
            for (int tap = 0; tap < T; ++tap) {
                int64_t cnt = (rem - tap + T - 1) / T;
                if (rem - tap <= 0) cnt = 0;
                if (cnt > 32) cnt = 32;
                const uint32_t before = cnt >= 32 ? 0xffffffffu : ((1u << cnt) - 1u);
                const uint32_t m = ((u0 + u) & 1) ? ~before : before;
                lds_mask[(chunk * T + tap) * kFB + u] = live ? m : 0u;
            }
        }
    }

    // ---- MFMA operands of this lane -----------------------------------------------------------------
    // pixel tiles of the wave: wave and wave + 4; lane column = pixel ln of the tile
    int pix_off[kTilesPerWave];
    bool tile_live[kTilesPerWave];
#pragma unroll
    for (int j = 0; j < kTilesPerWave; ++j) {
        const int pt = wave + kWaves * j;
        tile_live[j] = pt * 16 < PX;
        int q = pt * 16 + ln;
        q = q < PX ? q : (PX > 0 ? PX - 1 : 0);   // lanes past the block read a valid pixel; results are dropped
        const int yo = q / cols, xo = q % cols;
        pix_off[j] = ((yo * P.sh) * P.PC + xo * P.sw) * kPixStride + lg * 16;
    }
    f32x4_t acc[NFT][kTilesPerWave];   // [filter tile][pixel tile]
#pragma unroll
    for (int a = 0; a < NFT; ++a)
#pragma unroll
        for (int b = 0; b < kTilesPerWave; ++b) acc[a][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    union Frag { bf16x8_t v; uint32_t u[4]; u32x4_t q; };
    int tap_off[T];   // byte offset of a tap inside the patch (uniform)
#pragma unroll
    for (int tap = 0; tap < T; ++tap) tap_off[tap] = ((tap / P.kw) * P.PC + (tap % P.kw)) * kPixStride;

    // operand constants kept in registers (two literals do not fit one instruction)
    uint32_t sign_mask = 0x80008000u, one_bits = 0x3f803f80u;
    asm volatile("" : "+v"(sign_mask), "+v"(one_bits));
    const uint32_t byte_sel = 0x01010101u * static_cast<uint32_t>(lg);
    typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
    const uint32_t patch_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte_t *)lds_patch));

    // One chunk of the product for a wave with J live pixel tiles.  The work is a chain of units
    // (tap, pixel tile, plane): one 16-byte LDS read of the input operand, then one MFMA per filter
    // tile.  The reads are written as inline assembly and run kDepth units ahead of their MFMAs, with
    // explicit waits tied to the destination registers (LDS operations complete in order, so extra
    // operations the compiler puts in between only make a wait more conservative).  The +-1 operands
    // of the next tap and the conversion of the next chunk's staged input are computed in the shadow
    // of the MFMAs.
    auto multiply_chunk = [&](int buf, int chunk, bool stage_next, int next_slot, auto j_c) {
        constexpr int J = decltype(j_c)::value;
        constexpr int U = T * J * NP;
        constexpr int kDepth = U < 6 ? U : 6;
        const uint32_t src = patch_addr + static_cast<uint32_t>(buf * buf_bytes);
        const uint32_t *bits = lds_bits + chunk * T * kFB + ln;
        uint32_t nw[T][NFT];   // inverted filter bits of the chunk (bit 1 of the tile is +1: sign bit clear)
        uint32_t mw[FIX ? T : 1][NFT];   // FIX: the weights kept
#pragma unroll
        for (int tap = 0; tap < T; ++tap)
#pragma unroll
            for (int ft = 0; ft < NFT; ++ft) {
                nw[tap][ft] = ~bits[tap * kFB + ft * 16];
                if constexpr (FIX) mw[tap][ft] = (lds_mask + chunk * T * kFB + ln)[tap * kFB + ft * 16];
            }
        auto unit_addr = [&](int u) {
            const int tap = u / (J * NP), j = (u / NP) % J, pl = u % NP;
            return src + static_cast<uint32_t>(pix_off[j] + tap_off[tap] + pl * P.plane_bytes);
        };
        auto expand = [&](int tap, Frag (&wf)[NFT]) {
            // lane group lg holds channels 8*lg .. 8*lg + 7 of the step: byte lg of the word; register v
            // holds channels 2v and 2v + 1
            typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int ft = 0; ft < NFT; ++ft) {
                const u16x2_t r2 = __builtin_bit_cast(u16x2_t, __builtin_amdgcn_perm(nw[tap][ft], nw[tap][ft], byte_sel));
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const u16x2_t sh = {static_cast<uint16_t>(15 - 2 * v), static_cast<uint16_t>(14 - 2 * v)};
                    wf[ft].u[v] = (__builtin_bit_cast(uint32_t, static_cast<u16x2_t>(r2 << sh)) & sign_mask) | one_bits;
                }
                if constexpr (FIX) {   // zero where the pseudo-filter has no weight: the kept bit spread over its half word
                    typedef int16_t i16x2_t __attribute__((ext_vector_type(2)));
                    const u16x2_t m2 = __builtin_bit_cast(u16x2_t, __builtin_amdgcn_perm(mw[tap][ft], mw[tap][ft], byte_sel));
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const u16x2_t sh = {static_cast<uint16_t>(15 - 2 * v), static_cast<uint16_t>(14 - 2 * v)};
                        const i16x2_t top = __builtin_bit_cast(i16x2_t, static_cast<u16x2_t>(m2 << sh));
                        const i16x2_t fifteen = {15, 15};
                        wf[ft].u[v] &= __builtin_bit_cast(uint32_t, static_cast<i16x2_t>(top >> fifteen));
                    }
                }
            }
        };
        Frag xf[kDepth + 1];
        Frag wf[2][NFT];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) asm volatile("ds_read_b128 %0, %1" : "=v"(xf[u].q) : "v"(unit_addr(u)));
        expand(0, wf[0]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tap = u / (J * NP), j = (u / NP) % J;
            if (u + kDepth < U)
                asm volatile("ds_read_b128 %0, %1" : "=v"(xf[(u + kDepth) % (kDepth + 1)].q) : "v"(unit_addr(u + kDepth)));
            if (u % (J * NP) == 0 && tap + 1 < T) expand(tap + 1, wf[(tap + 1) & 1]);
            Frag &x = xf[u % (kDepth + 1)];
            // younger reads in flight: min(kDepth, U - 1 - u)
            if (U - 1 - u >= kDepth) asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x.q) : "n"(kDepth));
            else if (U - 1 - u == 5) asm volatile("s_waitcnt lgkmcnt(5)" : "+v"(x.q));
            else if (U - 1 - u == 4) asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(x.q));
            else if (U - 1 - u == 3) asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(x.q));
            else if (U - 1 - u == 2) asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(x.q));
            else if (U - 1 - u == 1) asm volatile("s_waitcnt lgkmcnt(1)" : "+v"(x.q));
            else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x.q));
#pragma unroll
            for (int ft = 0; ft < NFT; ++ft)
                acc[ft][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[tap & 1][ft].v, x.v, acc[ft][j], 0, 0, 0);
            // one staged item of the next chunk per tap
            // conversion of the next chunk's staged input: as late as possible (its loads were issued at the
            // start of the chunk), two items per tap over the last two taps and the rest after the last MFMA
            if (u % (J * NP) == J * NP - 1 && stage_next) {
                constexpr int kFirst = T > 2 ? T - 2 : 0;
                if (tap >= kFirst) {
                    const int i0 = 2 * (tap - kFirst);
                    if (i0 < kMaxItems) pack_item(i0, next_slot);
                    if (i0 + 1 < kMaxItems) pack_item(i0 + 1, next_slot);
                }
            }
        }
        if (stage_next) {
            constexpr int kFirst = T > 2 ? T - 2 : 0;
            constexpr int kDone = 2 * (T - kFirst) < kMaxItems ? 2 * (T - kFirst) : kMaxItems;
#pragma unroll
            for (int i = kDone; i < kMaxItems; ++i) pack_item(i, next_slot);
        }
    };

    // ---- main loop over channel chunks -----------------------------------------------------------------
    // Chunk c is multiplied from LDS buffer c % 2 while chunk c + 1 arrives in registers, is converted
    // in the shadow of the MFMAs and written to the other buffer at the end.
#pragma unroll
    for (int i = 0; i < kMaxItems; ++i) pack_item(i, 0);
    __syncthreads();            // zero fill and filter bits are in place
    store_chunk(0);
    __syncthreads();
    auto main_loop = [&](auto j_c) {
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            const int buf = chunk & 1;
            const bool more = chunk + 1 < n_chunks;
            if (more) load_chunk(chunk + 1, 0);
            if constexpr (decltype(j_c)::value > 0) {
                multiply_chunk(buf, chunk, more, 0, j_c);
            } else if (more) {   // a wave without pixels of its own still stages its share of the input
#pragma unroll
                for (int i = 0; i < kMaxItems; ++i) pack_item(i, 0);
            }
            if (more) store_chunk(buf ^ 1);
            __syncthreads();
        }
    };
    if constexpr (kTilesPerWave == 2) {
        if (tile_live[1]) main_loop(std::integral_constant<int, 2>{});
        else if (tile_live[0]) main_loop(std::integral_constant<int, 1>{});
        else main_loop(std::integral_constant<int, 0>{});
    } else {
        if (tile_live[0]) main_loop(std::integral_constant<int, 1>{});
        else main_loop(std::integral_constant<int, 0>{});
    }

    // ---- epilogue: y[img, u + t*R, row0.., :] = alpha[t] * Z[u] ---------------------------------------------
    // lane holds pixel ln of its tiles and filters 4*lg + i of each filter tile
    const int64_t plane_out = P.Ho * P.Wo;
    // pixel q of the block (row-major over rows x cols) sits at (q / cols) * Wo + q % cols from the block's first pixel
    int out_pix[kTilesPerWave];
    bool out_live[kTilesPerWave];
#pragma unroll
    for (int j = 0; j < kTilesPerWave; ++j) {
        const int q = (wave + kWaves * j) * 16 + ln;
        out_live[j] = q < PX;
        const int yo = q / cols, xo = q - yo * cols;
        out_pix[j] = yo * static_cast<int>(P.Wo) + xo;
    }
    if constexpr (FIX) {
        // registers i = 0, 1 and i = 2, 3 of a filter tile are the two halves of a pair
#pragma unroll
        for (int ft = 0; ft < NFT; ++ft)
#pragma unroll
            for (int i = 0; i < 4; i += 2) {
                const int64_t c = (u0 + ft * 16 + 4 * lg + i) / 2 + 1;
                if (c >= P.n_alpha) continue;
                const int64_t f = c * P.p, o = f / P.F;
                if (f == o * P.F || o >= P.O) continue;
                const float a_before = alpha[c - 1], a_after = alpha[c];
                XT *dst = y + ((img * P.O + o) * plane_out) + int64_t(row0) * P.Wo + col0;
#pragma unroll
                for (int j = 0; j < kTilesPerWave; ++j) {
                    if (!out_live[j]) continue;
                    float v = a_before * acc[ft][j][i] + a_after * acc[ft][j][i + 1];
                    if (RELU) v = fmaxf(v, 0.f);
                    ElemIO<XT>::store(dst + out_pix[j], v);
                }
            }
        return;
    }
    const int64_t reps = (P.O + P.R - 1) / P.R;
    const bool per_replica = (P.n_alpha == 1) || P.aligned;   // alpha depends on the replica only (uniform)
    auto write_all = [&](auto per_replica_c) __attribute__((always_inline)) {
        constexpr bool kPerReplica = decltype(per_replica_c)::value;
        for (int64_t t = 0; t < reps; ++t) {
            const float al_t = kPerReplica ? alpha[P.n_alpha == 1 ? 0 : t] : 0.f;
#pragma unroll
            for (int ft = 0; ft < NFT; ++ft) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t u = u0 + ft * 16 + 4 * lg + i;
                    const int64_t o = u + t * P.R;
                    if (u >= P.R || o >= P.O) continue;
                    const float al = kPerReplica ? al_t : alpha[(o * P.F) / P.p];
                    XT *dst = y + ((img * P.O + o) * plane_out) + int64_t(row0) * P.Wo + col0;
#pragma unroll
                    for (int j = 0; j < kTilesPerWave; ++j) {
                        if (!out_live[j]) continue;
                        float v = al * acc[ft][j][i];
                        if (RELU) v = fmaxf(v, 0.f);
                        ElemIO<XT>::store(dst + out_pix[j], v);
                    }
                }
            }
        }
    };
    if (per_replica) write_all(std::true_type{}); else write_all(std::false_type{});
}

constexpr int kPlanLdsMax = 150 * 1024;   // most LDS a plan may ask for

struct ConvPlan {
    bool ok;
    int rows_per_blk, cols_per_blk, n_colblk, PR, PC, nblk;   // nblk: row blocks
    size_t lds;
    int items;   // kItemsSmall or kItemsLarge
    int nft;     // kFtSmall or kFtLarge
    bool fix;    // launch the repair pass (pairs of masked filters) instead of the main pass
};

ConvPlan plan_conv(const ConvArgs &a) {
    ConvPlan pl{false, 0, 0, 0, 0, 0, 0, 0, kItemsSmall, kFtSmall, false};
    const int64_t F = a.C * a.kh * a.kw;
    const int T = a.kh * a.kw;
    if (T != 1 && T != 9) return pl;                     // instantiated tap counts: 1x1 and 3x3
    if (a.p < F || a.p < 64) return pl;                  // at most one tile end per filter
    if (a.Wo <= 0 || a.Ho <= 0 || a.Wo > (1 << 20) || a.Ho > (1 << 20)) return pl;
    if (a.C * a.H * a.W >= (int64_t(1) << 31)) return pl;   // 32-bit element offsets inside an image
    if (a.N > 65535) return pl;
    const int planes = (a.dt == TBN_F32) ? 3 : 1;
    const int64_t R = unique_rows(a.O, F, a.p);
    // 64 filters per workgroup for bf16 inputs where that many exist and enough workgroups remain to fill
    // the chip (measured 12 % faster; with float32 inputs, three planes per operand, it measured 8 % slower)
    pl.nft = (a.dt != TBN_F32 && a.C % kCK == 0 && R >= 16 * kFtLarge && ((R + 16 * kFtLarge - 1) / (16 * kFtLarge)) * a.N >= 256)
                 ? kFtLarge : kFtSmall;
    const int kFB = 16 * pl.nft;
    const size_t bits_bytes = size_t(T) * n_chunks_of(a.C) * kCK * 4 * (kFB / 32);   // kFB filters * T * ceil(C/32) words
    // A workgroup's block of output pixels is rows x cols (at most kMaxPix) whose input patch fits a staging budget.
    // What a pixel costs is mostly the staging of its share of the patch, so among the ways to cut a row into equal
    // column blocks (one block where the patch of a whole row fits) the plan takes the one with the fewest staged
    // patch pixels per output pixel: a 56-wide map is cut into blocks of 4 rows x 28 columns (patch 6 x 30, 1.6 staged
    // pixels per output) rather than 1 row x 56 (3 x 58, 3.1), a 14-wide map stays whole.
    const int64_t fblocks = (R + kFB - 1) / kFB;
    double best_cost = 0;
    for (int64_t n_colblk = 1; n_colblk <= 16; ++n_colblk) {
        const int64_t cols = (a.Wo + n_colblk - 1) / n_colblk;
        if (n_colblk > 1 && (cols < 7 || (a.Wo + cols - 1) / cols != n_colblk)) continue;
        if (cols > kMaxPix) continue;
        // balanced row blocks of at most kMaxPix pixels
        int64_t rows = kMaxPix / cols;
        if (rows > a.Ho) rows = a.Ho;
        int64_t nblk0 = (a.Ho + rows - 1) / rows;
        // With fewer workgroups than CUs (256), halve the row blocks as long as a block keeps at least 3 rows.
        while (nblk0 * n_colblk * a.N * fblocks < 256 && (a.Ho + 2 * nblk0 - 1) / (2 * nblk0) >= 3) nblk0 *= 2;
        rows = (a.Ho + nblk0 - 1) / nblk0;
        bool found = false;
        // the smaller staging budget first (less work per thread for the patches it covers)
        for (int items : {kItemsSmall, kItemsLarge}) {
            for (int64_t r = rows; r >= 1 && !found; --r) {
                const int64_t PR = (r - 1) * a.sh + a.kh, PC = (cols - 1) * a.sw + a.kw;
                const int64_t vrows = PR < a.H ? PR : a.H, vcols = PC < a.W ? PC : a.W;
                const size_t lds = 2 * size_t(planes) * PR * PC * kPixStride + bits_bytes;
                if (vrows * vcols * (kCK / 2) > int64_t(items) || lds > size_t(kPlanLdsMax)) continue;
                const int64_t nblk = (a.Ho + r - 1) / r;
                // the kernel numbers its workgroups in 32 bits (main pass: fblocks filter blocks; repair pass: at most k - 1)
                if (nblk * n_colblk * a.N * std::max<int64_t>(fblocks, a.k) > 0x7fffffffLL) continue;
                found = true;
                // one block more per row has to pay for itself: 10 % per extra column block
                const double cost = double(vrows * vcols) / double(r * cols) * (1.0 + 0.1 * double(n_colblk - 1));
                if (!pl.ok || cost < best_cost) {
                    best_cost = cost;
                    pl.ok = true;
                    pl.rows_per_blk = static_cast<int>(r);
                    pl.cols_per_blk = static_cast<int>(cols);
                    pl.n_colblk = static_cast<int>(n_colblk);
                    pl.PR = static_cast<int>(PR);
                    pl.PC = static_cast<int>(PC);
                    pl.nblk = static_cast<int>(nblk);
                    pl.lds = lds;
                    pl.items = items;
                }
            }
            if (found) break;
        }
    }
    return pl;
}

template <typename XT, int T, bool RELU, int ITEMS, int NFT, bool FIX, bool SHORT>
tbn_status launch_conv_fix(const ConvArgs &a, const ConvMfmaParams &P, size_t lds, dim3 grid) {
    // Dynamic LDS above the default limit has to be allowed once per kernel: the plan's upper bound, set by the
    // thread-safe initialisation of a static.
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_kernel<XT, T, RELU, ITEMS, NFT, FIX, SHORT>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kPlanLdsMax);
    if (attr != hipSuccess || lds > size_t(kPlanLdsMax)) {
        set_error("tbn_conv2d_forward: cannot reserve %zu bytes of LDS", lds);
        return TBN_ERR_DEVICE;
    }
    hipLaunchKernelGGL((conv_mfma_kernel<XT, T, RELU, ITEMS, NFT, FIX, SHORT>), grid, dim3(64 * waves_of(NFT)), lds, a.stream,
                       static_cast<const XT *>(a.x), static_cast<XT *>(a.y), a.tile, a.alpha, P);
    return check_launch(FIX ? "tbn_conv2d_forward (matrix-core repair pass)" : "tbn_conv2d_forward (matrix-core kernel)");
}

template <typename XT, int T, bool RELU, int ITEMS, int NFT>
tbn_status launch_conv_typed(const ConvArgs &a, const ConvMfmaParams &P, const ConvPlan &pl, dim3 grid) {
    if constexpr (NFT == kFtSmall) {
        if (pl.fix) return launch_conv_fix<XT, T, RELU, ITEMS, NFT, true, false>(a, P, pl.lds, grid);   // whole chunks only
        if (a.C % kCK != 0) return launch_conv_fix<XT, T, RELU, ITEMS, NFT, false, true>(a, P, pl.lds, grid);
    }
    return launch_conv_fix<XT, T, RELU, ITEMS, NFT, false, false>(a, P, pl.lds, grid);
}

template <typename XT, int T, bool RELU>
tbn_status launch_conv_items(const ConvArgs &a, const ConvMfmaParams &P, const ConvPlan &pl, dim3 grid) {
    if constexpr (!std::is_same<XT, float>::value) {
        if (pl.nft == kFtLarge)
            return pl.items == kItemsSmall ? launch_conv_typed<XT, T, RELU, kItemsSmall, kFtLarge>(a, P, pl, grid)
                                           : launch_conv_typed<XT, T, RELU, kItemsLarge, kFtLarge>(a, P, pl, grid);
    }
    return pl.items == kItemsSmall ? launch_conv_typed<XT, T, RELU, kItemsSmall, kFtSmall>(a, P, pl, grid)
                                   : launch_conv_typed<XT, T, RELU, kItemsLarge, kFtSmall>(a, P, pl, grid);
}

template <typename XT, int T>
tbn_status launch_conv_relu(const ConvArgs &a, const ConvMfmaParams &P, const ConvPlan &pl, dim3 grid) {
    return (a.flags & TBN_FLAG_RELU) ? launch_conv_items<XT, T, true>(a, P, pl, grid)
                                     : launch_conv_items<XT, T, false>(a, P, pl, grid);
}

template <typename XT>
tbn_status launch_conv_taps(const ConvArgs &a, const ConvMfmaParams &P, const ConvPlan &pl, dim3 grid) {
    return (a.kh * a.kw == 1) ? launch_conv_relu<XT, 1>(a, P, pl, grid) : launch_conv_relu<XT, 9>(a, P, pl, grid);
}

}  // namespace

bool conv_mfma_supported(const ConvArgs &a) { return plan_conv(a).ok; }

tbn_status launch_conv_mfma(const ConvArgs &a) {
    const ConvPlan pl = plan_conv(a);
    if (!pl.ok) {
        set_error("tbn_conv2d_forward: shape not supported by the matrix-core kernel");
        return TBN_ERR_UNSUPPORTED;
    }
    ConvMfmaParams P;
    P.N = a.N; P.C = a.C; P.H = a.H; P.W = a.W; P.O = a.O; P.Ho = a.Ho; P.Wo = a.Wo;
    P.kh = a.kh; P.kw = a.kw; P.sh = a.sh; P.sw = a.sw; P.ph = a.ph; P.pw = a.pw;
    P.F = a.C * a.kh * a.kw;
    P.R = unique_rows(a.O, P.F, a.p);
    P.p = a.p;
    P.n_words = (a.p + 31) / 32;
    P.aligned = (a.p % P.F == 0) ? 1 : 0;
    P.n_alpha = a.n_alpha;
    P.rows_per_blk = pl.rows_per_blk;
    P.cols_per_blk = pl.cols_per_blk;
    P.n_colblk = pl.n_colblk;
    P.PR = pl.PR; P.PC = pl.PC;
    P.plane_bytes = pl.PR * pl.PC * kPixStride;
    const int64_t fblocks = (P.R + 16 * pl.nft - 1) / (16 * pl.nft);
    if (fblocks > 65535) {
        set_error("tbn_conv2d_forward: too many distinct filters for one launch");
        return TBN_ERR_UNSUPPORTED;
    }
    const dim3 grid(static_cast<unsigned>(pl.nblk * pl.n_colblk), static_cast<unsigned>(a.N), static_cast<unsigned>(fblocks));
    tbn_status st = (a.dt == TBN_F32) ? launch_conv_taps<float>(a, P, pl, grid) : launch_conv_taps<uint16_t>(a, P, pl, grid);
    if (st != TBN_OK) return st;
    if (a.n_alpha == 1 || P.aligned) return TBN_OK;
    // Channels whose filter contains a tile start are scaled by two alphas: a second pass of the same kernel over
    // pairs of masked filters, 16 such channels per workgroup, where the doubled filter-bit area still fits the LDS
    // (else the plain kernel for those channels).
    ConvPlan fp = pl;
    fp.fix = true;
    fp.nft = kFtSmall;
    const size_t bits_small = size_t(a.kh * a.kw) * n_chunks_of(a.C) * kCK * 4 * (16 * kFtSmall / 32);
    const size_t bits_main = size_t(a.kh * a.kw) * n_chunks_of(a.C) * kCK * 4 * (16 * pl.nft / 32);
    fp.lds = pl.lds - bits_main + 2 * bits_small;
    const int64_t pairs_per_blk = 16 * kFtSmall / 2;
    const int64_t fix_blocks = (int64_t(a.k) - 1 + pairs_per_blk - 1) / pairs_per_blk;
    if (fp.lds > size_t(kPlanLdsMax) || fix_blocks > 65535 || a.C % kCK != 0) return launch_conv_generic_tile_ends(a);
    const dim3 fgrid(static_cast<unsigned>(pl.nblk * pl.n_colblk), static_cast<unsigned>(a.N), static_cast<unsigned>(fix_blocks));
    return (a.dt == TBN_F32) ? launch_conv_taps<float>(a, P, fp, fgrid) : launch_conv_taps<uint16_t>(a, P, fp, fgrid);
}

}  // namespace tbn
