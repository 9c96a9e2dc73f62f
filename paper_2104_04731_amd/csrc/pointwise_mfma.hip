// GEMM stage for 1x1 convolutions (stride 1, no padding) that reads NCHW itself.
//
// A 1x1 convolution is out[n] = W [K x C] * X[n] [C x HW]: the weights are depth-contiguous as
// they are, but an image is depth-major, the pixels contiguous.  Channel blocking (Pad + Split +
// Reorder of Table 2) exists to turn that around; here a workgroup turns its own 32 pixels
// around in LDS instead, so nothing rewritten is stored and the layer is one launch.
//
// One workgroup (4 waves) = 32 consecutive pixels of one image x 128 output channels:
//   1. each wave fetches the MFMA weight operands of its 32 output channels straight into
//      registers (16 bytes of row lane%32 per 32-deep step; rows are 16-byte multiples);
//   2. a thread fetches four channel rows x four pixels (one dword each), transposes the 4x4
//      bytes with eight v_perm_b32 and writes each pixel's four channels into the LDS tile
//      XT[pixel][channel] (pitch C + 16 bytes: 32 rows start in different bank groups);
//   3. v_mfma_i32_32x32x32_i8, channels x pixels, activation operand = 16 bytes of XT row lane%32;
//   4. the D block (column = pixel = lane%32) goes straight to NKPQ in 128-byte runs.
// All global loads of a thread are issued before its first LDS store; a workgroup that has more
// than one tile keeps its weight operands and fetches the next tile's pixels during the current one.
// Two more forms of the same layer follow it: one for grids too small to fill the chip (a workgroup of 32 pixels x 32
// output channels whose waves share the depth) and one for large batches (a workgroup owns 224 pixels of an image).
#include "kernels.h"
#include "rewrite_bodies.h"

namespace c2i8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

struct PointArgs {
    const int8_t *in;
    const int8_t *wt;
    int32_t *out;
    int C, HW, K, tiles;  // tiles of 32 pixels per image
    int ntiles;           // N * tiles
    unsigned m_tiles;
    int W;                // image width (the activation epilogue needs a pixel's row and column)
    unsigned m_W;
    ActOut act;           // activation epilogue (act.out != null): `out` is not written
};

__device__ __forceinline__ unsigned ld_u32(const void *p)  // any alignment
{
    unsigned x;
    __builtin_memcpy(&x, p, 4);
    return x;
}
__device__ __forceinline__ v4i ld_v4(const void *p)  // any alignment
{
    v4i x;
    __builtin_memcpy(&x, p, 16);
    return x;
}

template <int NKK, bool ACT>  // C = 32 * NKK; ACT: the activation epilogue (a kernel of its own: the plain one stays as lean as it was)
__global__ void __launch_bounds__(256) conv_pointwise_kernel(const PointArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int C = 32 * NKK, PITCH = C + 16;
    constexpr int QUADS = C / 4;                  // groups of four channels
    constexpr int PASSES = (QUADS + 31) / 32;     // 256 threads = 8 pixel groups x 32 quads per pass

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, half = lane >> 5;
    const int k0 = blockIdx.y * 128 + wave * 32;

    // A workgroup keeps its weight operands in registers and walks over pixel tiles gridDim.x apart.
    const int g = tid & 7, cq = tid >> 3;
    // The next tile's pixels are fetched while this tile is multiplied and stored.
    unsigned xv[PASSES][4];
    // 2. activations: pixels px0 + 4g .. +3 (HW is a multiple of 4: a group is inside the image or past it)
    auto fetch = [&](int tile) {
        const int n = fast_div_any(tile, a.tiles, a.m_tiles), px0 = (tile - n * a.tiles) * 32;
        const int px = min(px0 + 4 * g, a.HW - 4);
        const int8_t *img = a.in + (size_t)n * C * a.HW + px;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int q = min(cq + 32 * ps, QUADS - 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[ps][j] = ld_u32(img + (size_t)(4 * q + j) * a.HW);
        }
    };
    const int lid0 = xcd_contiguous(blockIdx.x, gridDim.x);
    if (lid0 < a.ntiles) fetch(lid0);
    // 1. weights (waves past the last output channel compute on row K-1 and store nothing).  Asked for after the
    //    first tile's pixels: loads return in order, and the pixels are needed first (turned around and written to
    //    LDS while the four times larger weight operand is still arriving).
    v4i wf[NKK];
    {
        const int8_t *row = a.wt + (size_t)min(k0 + l31, a.K - 1) * C + half * 16;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) wf[kk] = ld_v4(row + kk * 32);
    }
    for (int lid = lid0; lid < a.ntiles; lid += gridDim.x) {
    const int n = fast_div_any(lid, a.tiles, a.m_tiles), px0 = (lid - n * a.tiles) * 32;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int q = cq + 32 * ps;
        if (q < QUADS) {
            // rows = channels 4q .. 4q+3, bytes = pixels: out_i = byte i of each row
            const unsigned lo01 = __builtin_amdgcn_perm(xv[ps][1], xv[ps][0], 0x05010400u);
            const unsigned hi01 = __builtin_amdgcn_perm(xv[ps][1], xv[ps][0], 0x07030602u);
            const unsigned lo23 = __builtin_amdgcn_perm(xv[ps][3], xv[ps][2], 0x05010400u);
            const unsigned hi23 = __builtin_amdgcn_perm(xv[ps][3], xv[ps][2], 0x07030602u);
            unsigned *dst = reinterpret_cast<unsigned *>(smem + (4 * g) * PITCH + 4 * q);
            dst[0 * PITCH / 4] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
            dst[1 * PITCH / 4] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
            dst[2 * PITCH / 4] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
            dst[3 * PITCH / 4] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
        }
    }
    __syncthreads();
    if (lid + (int)gridDim.x < a.ntiles) fetch(lid + (int)gridDim.x);

    // 3. MFMA
    v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
    const unsigned char *xrow = smem + l31 * PITCH + half * 16;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
        const v4i xf = *reinterpret_cast<const v4i *>(xrow + kk * 32);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[kk], xf, acc, 0, 0, 0);
    }

    // 4. D block: column = lane%32 = pixel, row = 8*(v/4) + 4*(lane/32) + v%4 = channel
    const int p = px0 + l31;
    if (ACT) {
        if (p < a.HW) {
            const int py = fast_div_any(p, a.W, a.m_W), qx = p - py * a.W;
#pragma unroll
            for (int vg = 0; vg < 4; ++vg)
                act_store4(a.act, n, py, qx, k0 + 8 * vg + 4 * half, a.K, acc[4 * vg], acc[4 * vg + 1], acc[4 * vg + 2],
                           acc[4 * vg + 3]);
        }
    } else if (p < a.HW) {
        int32_t *base = a.out + ((size_t)n * a.K + k0 + 4 * half) * a.HW + p;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int kr = 8 * (v >> 2) + (v & 3);
            if (k0 + 4 * half + kr < a.K) base[(size_t)kr * a.HW] = acc[v];
        }
    }
    if (lid + (int)gridDim.x >= a.ntiles) break;
    __syncthreads();  // the next tile's pixels replace these in LDS
    }
}

// ---- the same layer when the grid above would leave most of the chip idle: the depth split over the waves ----
// Eight images of 14x14 pixels and 128 output channels are 56 pixel tiles x 1 channel group = 56 workgroups
// for 256 compute units, each waiting for sixteen 16-byte weight loads per lane and then running sixteen
// dependent MFMAs.  Here a workgroup is 32 pixels x 32 output channels and each of its four waves takes a
// quarter of the channels: four weight loads and four MFMAs per lane, four times as many workgroups.  A wave
// turns around only the channels it multiplies, in an LDS tile of its own, so nothing waits for another wave
// until the four partial D blocks are added: each wave leaves its block in LDS, one barrier, and wave w adds
// up and stores rows 8w .. 8w+7 of the 32.
template <int NKK>  // C = 32 * NKK, NKK a multiple of 4
__global__ void __launch_bounds__(256) conv_pointwise_split_kernel(const PointArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    static_assert(NKK % 4 == 0, "four waves share the depth");
    constexpr int C = 32 * NKK, CW = C / 4, PITCH = CW + 16;   // CW: channels of one wave
    constexpr int NK = NKK / 4;                                // 32-deep steps of one wave
    constexpr int PASSES = CW / 32;                            // 64 lanes = 8 pixel groups x 8 quads of channels per pass

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, half = lane >> 5;
    const int k0 = blockIdx.y * 32, c0 = wave * CW;
    const int tile = blockIdx.x;
    const int n = fast_div_any(tile, a.tiles, a.m_tiles), px0 = (tile - n * a.tiles) * 32;
    const int g = lane & 7, cq = lane >> 3;

    // pixels before weights: loads return in order and the pixels are needed first
    unsigned xv[PASSES][4];
    {
        const int px = min(px0 + 4 * g, a.HW - 4);   // HW is a multiple of 4: a group is inside the image or past it
        const int8_t *img = a.in + ((size_t)n * C + c0) * a.HW + px;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[ps][j] = ld_u32(img + (size_t)(4 * (cq + 8 * ps) + j) * a.HW);
    }
    v4i wf[NK];
    {
        const int8_t *row = a.wt + (size_t)min(k0 + l31, a.K - 1) * C + c0 + half * 16;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) wf[kk] = ld_v4(row + kk * 32);
    }
    unsigned char *xt = smem + wave * (32 * PITCH);   // this wave's XT[pixel][its channels]
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int q = cq + 8 * ps;
        const unsigned lo01 = __builtin_amdgcn_perm(xv[ps][1], xv[ps][0], 0x05010400u);
        const unsigned hi01 = __builtin_amdgcn_perm(xv[ps][1], xv[ps][0], 0x07030602u);
        const unsigned lo23 = __builtin_amdgcn_perm(xv[ps][3], xv[ps][2], 0x05010400u);
        const unsigned hi23 = __builtin_amdgcn_perm(xv[ps][3], xv[ps][2], 0x07030602u);
        unsigned *dst = reinterpret_cast<unsigned *>(xt + (4 * g) * PITCH + 4 * q);
        dst[0 * PITCH / 4] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
        dst[1 * PITCH / 4] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        dst[2 * PITCH / 4] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        dst[3 * PITCH / 4] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
    }
    // The tile is this wave's alone and LDS serves a wave's accesses in order: no barrier, only the order kept.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
    const unsigned char *xrow = xt + l31 * PITCH + half * 16;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
        const v4i xf = *reinterpret_cast<const v4i *>(xrow + kk * 32);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[kk], xf, acc, 0, 0, 0);
    }

    // D block: column = lane%32 = pixel, row = 8*(v/4) + 4*(lane/32) + v%4 = channel.  red[wave][v/4][lane] = four rows.
    v4i *red = reinterpret_cast<v4i *>(smem + 4 * 32 * PITCH);
#pragma unroll
    for (int vg = 0; vg < 4; ++vg)
        red[(wave * 4 + vg) * 64 + lane] = v4i{acc[4 * vg], acc[4 * vg + 1], acc[4 * vg + 2], acc[4 * vg + 3]};
    __syncthreads();
    v4i sum = red[wave * 64 + lane];
#pragma unroll
    for (int o = 1; o < 4; ++o) {
        const v4i t = red[(o * 4 + wave) * 64 + lane];
        sum[0] += t[0];
        sum[1] += t[1];
        sum[2] += t[2];
        sum[3] += t[3];
    }
    const int p = px0 + l31, kr = k0 + 8 * wave + 4 * half;
    if (p < a.HW) {
        int32_t *base = a.out + ((size_t)n * a.K + kr) * a.HW + p;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kr + j < a.K) base[(size_t)j * a.HW] = sum[j];
    }
}

// ---- the split form on NHWC tensors -----------------------------------------------------------------
// Pixels x channels times the weight rows: both operands are depth-contiguous as they are, so a lane fetches its MFMA
// operands straight from memory (row lane%32 of either side, 16 bytes per 32-deep step) and LDS carries only the
// sum over the four waves' quarters of the depth.  The partial blocks are laid out so that after the barrier
// eight consecutive lanes hold the 32 output channels of a pixel: a store instruction writes eight 128-byte runs.
struct PointNhwcArgs {
    const int8_t *in;   // [M][C], M = N*H*W pixels
    const int8_t *wt;   // [K][C]
    int32_t *out;       // [M][K], K a multiple of 4, 16-byte aligned
    int M, K;
};
constexpr int NHWC_RED_PITCH = 33;   // 16-byte slots per (wave, four-row group): 32 pixels and one of padding

template <int NKK>  // C = 32 * NKK, NKK a multiple of 4
__global__ void __launch_bounds__(256) conv_pointwise_nhwc_split_kernel(const PointNhwcArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    static_assert(NKK % 4 == 0, "four waves share the depth");
    constexpr int C = 32 * NKK, CW = C / 4, NK = NKK / 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, half = lane >> 5;
    const int p0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int8_t *xrow = a.in + (size_t)min(p0 + l31, a.M - 1) * C + wave * CW + half * 16;
    const int8_t *wrow = a.wt + (size_t)min(k0 + l31, a.K - 1) * C + wave * CW + half * 16;
    v4i xf[NK], wf[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) xf[kk] = ld_v4(xrow + kk * 32);
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) wf[kk] = ld_v4(wrow + kk * 32);
    v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[kk], xf[kk], acc, 0, 0, 0);

    // D block: column = lane%32 = pixel, rows 8*vg + 4*half + (0..3) = four consecutive channels, group cg = 2*vg + half
    v4i *red = reinterpret_cast<v4i *>(smem);   // [wave][cg][NHWC_RED_PITCH]
#pragma unroll
    for (int vg = 0; vg < 4; ++vg)
        red[(wave * 8 + 2 * vg + half) * NHWC_RED_PITCH + l31] = v4i{acc[4 * vg], acc[4 * vg + 1], acc[4 * vg + 2], acc[4 * vg + 3]};
    __syncthreads();
    const int pix = 8 * wave + (lane >> 3), cg = lane & 7;   // wave w: pixels 8w .. 8w+7, a pixel's channels in eight lanes
    v4i sum = red[cg * NHWC_RED_PITCH + pix];
#pragma unroll
    for (int o = 1; o < 4; ++o) {
        const v4i t = red[(o * 8 + cg) * NHWC_RED_PITCH + pix];
        sum[0] += t[0];
        sum[1] += t[1];
        sum[2] += t[2];
        sum[3] += t[3];
    }
    const int p = p0 + pix, k = k0 + 4 * cg;
    if (p < a.M && k < a.K) *reinterpret_cast<v4i *>(a.out + (size_t)p * a.K + k) = sum;   // K % 4 == 0: k + 3 < K
}

// ---- the same layer for large batches: a workgroup owns up to 224 pixels of one image ---------------
// With 32-pixel tiles a workgroup uses 32 bytes of every 128-byte line of its C channel rows and the rest
// of each line is fetched again by whoever owns the neighbouring tile; at large batch the vector cache's
// miss traffic, not HBM, bounds the kernel.  Here a workgroup takes PXB = 7 column blocks (224 pixels: a
// whole 14x14 image, whose channel rows are then one contiguous block of memory) and walks the channels
// in chunks of 64: fetch chunk c+1 (pixels to registers, this wave's weight operands too), multiply chunk c
// out of LDS (7 x 2 MFMAs per wave), transpose chunk c+1 into the other LDS buffer, one barrier.
// Weight operands are re-read per chunk (64 KB in all, L2-resident) instead of living in 16 B x C/32 registers.
constexpr int IMG_PXB = 7, IMG_PX = 32 * IMG_PXB, IMG_CH = 64, IMG_PITCH = IMG_CH + 16;
constexpr int IMG_PASSES = (IMG_PX / 4 + 15) / 16;   // 16 quads x 16 pixel groups per pass of 256 threads

struct PointImageArgs {
    const int8_t *in;
    const int8_t *wt;
    int32_t *out;
    int C, HW, K, ptiles;   // ptiles = ranges of 224 pixels per image
    unsigned m_ptiles;
    int W;
    unsigned m_W;
    ActOut act;             // activation epilogue (act.out != null): `out` is not written
};

__global__ void __launch_bounds__(256) conv_pointwise_image_kernel(const PointImageArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // two buffers [IMG_PX][IMG_PITCH]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, half = lane >> 5;
    const int k0 = blockIdx.y * 128 + wave * 32;
    const int tile = xcd_contiguous(blockIdx.x, gridDim.x);
    const int n = fast_div_any(tile, a.ptiles, a.m_ptiles), px0 = (tile - n * a.ptiles) * IMG_PX;
    const int npx = min(IMG_PX, a.HW - px0);             // a multiple of 4
    const int nchunks = a.C / IMG_CH;

    // pixel fetch: thread = (pixel group gl + 8*gh + 16*pass, quad q) -> four channel rows x four pixels
    const int gl = tid & 7, q = (tid >> 3) & 15, gh = tid >> 7;
    const int8_t *img = a.in + (size_t)n * a.C * a.HW + px0;
    const int8_t *wrow = a.wt + (size_t)min(k0 + l31, a.K - 1) * a.C + half * 16;
    unsigned xv[IMG_PASSES][4];
    v4i wn[2];
    auto fetch = [&](int c) {
#pragma unroll
        for (int ps = 0; ps < IMG_PASSES; ++ps) {
            const int g = min(16 * ps + 8 * gh + gl, npx / 4 - 1);   // groups past the range re-read the last one
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[ps][j] = ld_u32(img + (size_t)(IMG_CH * c + 4 * q + j) * a.HW + 4 * g);
        }
        wn[0] = ld_v4(wrow + IMG_CH * c);
        wn[1] = ld_v4(wrow + IMG_CH * c + 32);
    };
    auto spill = [&](unsigned char *buf) {   // registers -> LDS, 4x4 bytes transposed: XT[pixel][channel]
#pragma unroll
        for (int ps = 0; ps < IMG_PASSES; ++ps) {
            const int g = 16 * ps + 8 * gh + gl;
            if (4 * g < IMG_PX) {
                const unsigned lo01 = __builtin_amdgcn_perm(xv[ps][1], xv[ps][0], 0x05010400u);
                const unsigned hi01 = __builtin_amdgcn_perm(xv[ps][1], xv[ps][0], 0x07030602u);
                const unsigned lo23 = __builtin_amdgcn_perm(xv[ps][3], xv[ps][2], 0x05010400u);
                const unsigned hi23 = __builtin_amdgcn_perm(xv[ps][3], xv[ps][2], 0x07030602u);
                unsigned *dst = reinterpret_cast<unsigned *>(buf + (4 * g) * IMG_PITCH + 4 * q);
                dst[0 * IMG_PITCH / 4] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
                dst[1 * IMG_PITCH / 4] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
                dst[2 * IMG_PITCH / 4] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
                dst[3 * IMG_PITCH / 4] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
            }
        }
    };

    v16i acc[IMG_PXB];
#pragma unroll
    for (int b = 0; b < IMG_PXB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0;

    fetch(0);
    spill(smem);
    v4i wf[2] = {wn[0], wn[1]};
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        unsigned char *cur = smem + (c & 1) * (IMG_PX * IMG_PITCH), *nxt = smem + ((c + 1) & 1) * (IMG_PX * IMG_PITCH);
        if (c + 1 < nchunks) fetch(c + 1);   // uniform
        const unsigned char *xrow = cur + l31 * IMG_PITCH + half * 16;
#pragma unroll
        for (int b = 0; b < IMG_PXB; ++b) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const v4i xf = *reinterpret_cast<const v4i *>(xrow + b * 32 * IMG_PITCH + kk * 32);
                acc[b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[kk], xf, acc[b], 0, 0, 0);
            }
        }
        if (c + 1 < nchunks) {
            spill(nxt);
            wf[0] = wn[0];
            wf[1] = wn[1];
        }
        __syncthreads();
    }

    // D block b: column = lane%32 = pixel px0 + 32 b + lane%32, row = 8*(v/4) + 4*(lane/32) + v%4 = channel
    if (a.act.out) {
#pragma unroll
        for (int b = 0; b < IMG_PXB; ++b) {
            if (32 * b + l31 < npx) {
                const int p = px0 + 32 * b + l31, py = fast_div_any(p, a.W, a.m_W), qx = p - py * a.W;
#pragma unroll
                for (int vg = 0; vg < 4; ++vg)
                    act_store4(a.act, n, py, qx, k0 + 8 * vg + 4 * half, a.K, acc[b][4 * vg], acc[b][4 * vg + 1],
                               acc[b][4 * vg + 2], acc[b][4 * vg + 3]);
            }
        }
        return;
    }
    int32_t *obase = a.out + ((size_t)n * a.K + k0 + 4 * half) * a.HW + px0 + l31;
#pragma unroll
    for (int b = 0; b < IMG_PXB; ++b) {
        if (32 * b + l31 < npx) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kr = 8 * (v >> 2) + (v & 3);
                if (k0 + 4 * half + kr < a.K) obase[(size_t)kr * a.HW + 32 * b] = acc[b][v];
            }
        }
    }
}

// The batch form pays when it has a workgroup for every compute unit and wastes little of its last pixel range
// (C4b: 448 images through the 32-pixel form 25.5 us, 512 images through this one 22.8 us).
static bool image_form_pays(const WindowProblem &g)
{
    const long long HW = (long long)g.H * g.W, pt = (HW + IMG_PX - 1) / IMG_PX, kgroups = (g.K + 127) / 128;
    if (g.C % IMG_CH != 0 || (long long)g.N * pt > 2147483647LL) return false;
    return (long long)g.N * pt * kgroups >= 256 && pt * IMG_PX * 100 <= HW * 115;
}

static hipError_t launch_pointwise_image(const WindowProblem &g, hipStream_t st)
{
    PointImageArgs a{};
    a.in = g.in;
    a.wt = g.wt;
    a.out = g.out;
    a.C = g.C;
    a.HW = g.H * g.W;
    a.K = g.K;
    a.ptiles = (a.HW + IMG_PX - 1) / IMG_PX;
    a.m_ptiles = magic_for(a.ptiles);
    a.W = g.W;
    a.m_W = magic_for(g.W);
    a.act = g.act;
    const dim3 grid((unsigned)(g.N * a.ptiles), (unsigned)((g.K + 127) / 128));
    hipLaunchKernelGGL(conv_pointwise_image_kernel, grid, dim3(256), (size_t)2 * IMG_PX * IMG_PITCH, st, a);
    return hipGetLastError();
}

template <int NKK>
hipError_t launch_nkk(const PointArgs &a, dim3 grid, hipStream_t st)
{
    if (a.act.out) hipLaunchKernelGGL((conv_pointwise_kernel<NKK, true>), grid, dim3(256), (size_t)32 * (32 * NKK + 16), st, a);
    else hipLaunchKernelGGL((conv_pointwise_kernel<NKK, false>), grid, dim3(256), (size_t)32 * (32 * NKK + 16), st, a);
    return hipGetLastError();
}

template <int NKK>
hipError_t launch_split(const PointArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)a.ntiles, (unsigned)((a.K + 31) / 32));
    hipLaunchKernelGGL((conv_pointwise_split_kernel<NKK>), grid, dim3(256), (size_t)4 * 32 * (8 * NKK + 16) + 4 * 4 * 64 * 16, st, a);
    return hipGetLastError();
}

template <int NKK>
hipError_t launch_nhwc_split(const PointNhwcArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.M + 31) / 32), (unsigned)((a.K + 31) / 32));
    hipLaunchKernelGGL((conv_pointwise_nhwc_split_kernel<NKK>), grid, dim3(256), (size_t)4 * 8 * NHWC_RED_PITCH * 16, st, a);
    return hipGetLastError();
}

}  // namespace

// The NHWC split form: whole 128-channel quarters, a result in 16-byte pieces, and a grid of at most two workgroups
// per compute unit -- it has no pixels to turn around, so it stays ahead of the general GEMM stage for twice as long
// as the NCHW split form (14x14 images: C = 512, K = 1024, two images 3.5 against 3.8 us, four 5.4 against 4.3;
// C = K = 256, eight images 2.6 against 3.2, sixteen level).  Pointers 16-byte aligned (the caller checks).
bool pointwise_nhwc_split_fits(long long M, int C, int K)
{
    return C % 128 == 0 && C <= 512 && K % 4 == 0 && M >= 1 && ((M + 31) / 32) * ((K + 31) / 32) <= 512;
}

hipError_t launch_pointwise_nhwc_split(const int8_t *in, const int8_t *wt, int32_t *out, long long M, int C, int K,
                                       hipStream_t st)
{
    if (!pointwise_nhwc_split_fits(M, C, K)) return hipErrorInvalidValue;
    const PointNhwcArgs a{in, wt, out, (int)M, K};
    switch (C / 128) {
        case 1: return launch_nhwc_split<4>(a, st);
        case 2: return launch_nhwc_split<8>(a, st);
        case 3: return launch_nhwc_split<12>(a, st);
        case 4: return launch_nhwc_split<16>(a, st);
    }
    return hipErrorInvalidValue;
}

bool pointwise_fits(const WindowProblem &g)
{
    if (g.R != 1 || g.S != 1 || g.stride != 1 || g.pad != 0) return false;
    if (g.C % 64 != 0 || g.C > 512) return false;
    const long long HW = (long long)g.H * g.W;
    if (HW % 4 != 0 || HW > 2147483647LL) return false;
    const long long tiles = (HW + 31) / 32;
    return (long long)g.N * tiles <= 2147483647LL && (g.K + 127) / 128 <= 65535;
}

hipError_t launch_pointwise_conv(const WindowProblem &g, hipStream_t st)
{
    if (!pointwise_fits(g)) return hipErrorInvalidValue;
    if (image_form_pays(g)) return launch_pointwise_image(g, st);
    PointArgs a{};
    a.in = g.in;
    a.wt = g.wt;
    a.out = g.out;
    a.C = g.C;
    a.HW = g.H * g.W;
    a.K = g.K;
    a.tiles = (a.HW + 31) / 32;
    a.m_tiles = magic_for(a.tiles);
    a.ntiles = g.N * a.tiles;
    a.W = g.W;
    a.m_W = magic_for(g.W);
    a.act = g.act;
    const int kgroups = (g.K + 127) / 128;
    // While the split form has at most one workgroup per compute unit it is the faster one (eight 14x14 images, C = 512,
    // K = 128: 2.9 against 3.8 us; C = K = 256, four images: 2.4 against 2.9); at about two per compute unit the two
    // are level, beyond that the form below, which turns a pixel tile around once for 128 output channels, wins.
    if (!a.act.out && g.C % 128 == 0 && (long long)a.ntiles * ((g.K + 31) / 32) <= 256) {
        switch (g.C / 128) {
            case 1: return launch_split<4>(a, st);
            case 2: return launch_split<8>(a, st);
            case 3: return launch_split<12>(a, st);
            case 4: return launch_split<16>(a, st);
        }
    }
    int wgs = 256 * 4 / kgroups;  // about four workgroups fit a CU
    if (wgs < 256) wgs = 256;
    const dim3 grid((unsigned)(a.ntiles < wgs ? a.ntiles : wgs), (unsigned)kgroups);
    switch (g.C / 32) {
        case 2: return launch_nkk<2>(a, grid, st);
        case 4: return launch_nkk<4>(a, grid, st);
        case 6: return launch_nkk<6>(a, grid, st);
        case 8: return launch_nkk<8>(a, grid, st);
        case 10: return launch_nkk<10>(a, grid, st);
        case 12: return launch_nkk<12>(a, grid, st);
        case 14: return launch_nkk<14>(a, grid, st);
        case 16: return launch_nkk<16>(a, grid, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace c2i8
