// Layout rewrites of Table 2 as bandwidth-bound copy kernels: every destination byte
// (zero padding included) is written exactly once, in 16-byte pieces, and source reads run
// along the contiguous W axis across the lanes of a wave.
#include "kernels.h"
#include "rewrite_bodies.h"

namespace c2i8 {

// ---- pack_layout: NCHW -> [N][Cb][Hp][Wp][cb] -------------------------------------------
// One thread produces VEC = min(cb,16) channel-contiguous bytes of one padded pixel.
// Lanes run along padded pixels, so each per-channel byte load of a wave is a contiguous
// run of the source row.
template <int VEC>
__global__ void __launch_bounds__(256)
pack_layout_kernel(const int8_t *__restrict__ src, int8_t *__restrict__ dst,
                   int C, int H, int W, int cb, int pad, int Hp, int Wp, int Cb,
                   long long pixels /* N*Cb*Hp*Wp */)
{
    const int groups = cb / VEC;  // VEC-byte groups per pixel
    const long long total = pixels * groups;
    const long long HW = (long long)H * W;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long long)gridDim.x * blockDim.x) {
        // t = (((n*Cb + b)*groups + g)*Hp + hp)*Wp + wp : pixel index fastest across lanes
        long long rest = t;
        const int wp = (int)(rest % Wp);
        rest /= Wp;
        const int hp = (int)(rest % Hp);
        rest /= Hp;
        const int g = (int)(rest % groups);
        rest /= groups;
        const int b = (int)(rest % Cb);
        const long long n = rest / Cb;
        const int h = hp - pad, w = wp - pad;
        const int c0 = b * cb + g * VEC;
        int v[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = 0;
        if (h >= 0 && h < H && w >= 0 && w < W) {
            const int8_t *s = src + ((n * C + c0) * H + h) * (long long)W + w;
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (c0 + i < C) v[i] = s[i * HW];
        }
        int8_t *d = dst + ((((n * Cb + b) * Hp + hp) * (long long)Wp + wp) * cb + g * VEC);
        if (VEC == 16) {
            v4i o;
            o[0] = pack4(v[0], v[1], v[2], v[3]);
            o[1] = pack4(v[4], v[5], v[6], v[7]);
            o[2] = pack4(v[8], v[9], v[10], v[11]);
            o[3] = pack4(v[12], v[13], v[14], v[15]);
            *reinterpret_cast<v4i *>(d) = o;
        } else {
#pragma unroll
            for (int i = 0; i < VEC; i += 4)
                *reinterpret_cast<unsigned *>(d + i) = pack4(v[i], v[i + 1], v[i + 2], v[i + 3]);
        }
    }
}


// Tiled version for cb % 16 == 0 and H*W % 4 == 0 (every channel plane starts dword-aligned).
// A workgroup owns TP consecutive padded pixels of one (image, channel block, 64-channel
// slice).  The interior pixels among them are one contiguous run of the source plane, so each
// channel contributes one contiguous run of <= TP bytes: it is fetched with dword loads into
// an LDS tile [channel][pixel], then read back channel-wise so that four lanes write the 64
// contiguous bytes of one pixel and a wave writes 1 KB of contiguous destination.
constexpr int PACK_TP = 256;            // padded pixels per workgroup
constexpr int PACK_CH = 64;             // channels per LDS tile
constexpr int PACK_PITCH = PACK_TP + 4; // bytes; pitch % 16 == 4 spreads the 16-channel groups over banks

// Number of interior (non-border) pixels with padded flat index < o.
__device__ __forceinline__ int interior_before(int o, int Wp, int pad, int H, int W)
{
    const int hp = o / Wp, wp = o - hp * Wp;
    const int rows = min(max(hp - pad, 0), H);
    int n = rows * W;
    if (hp >= pad && hp < pad + H) n += min(max(wp - pad, 0), W);
    return n;
}

struct PackArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, cb, pad, Hp, Wp, Cb, tiles_per_img, slices /* ceil(cb/64) */;
    int tp;  // padded pixels per workgroup: 256 for >= 64 channels per slice, 512 for 32, 1024 for 16
};

__device__ __forceinline__ void pack_layout_tiled_body(const PackArgs &a, int bid, unsigned char *tile)
{
    const int8_t *__restrict__ src = a.src;
    int8_t *__restrict__ dst = a.dst;
    const int C = a.C, H = a.H, W = a.W, cb = a.cb, pad = a.pad, Wp = a.Wp, Cb = a.Cb;
    const int HW = H * W, HpWp = a.Hp * Wp;
    const int t = bid % a.tiles_per_img;
    bid /= a.tiles_per_img;
    const int sl = bid % a.slices;
    bid /= a.slices;
    const int b = bid % Cb;
    const long long n = bid / Cb;
    const int TP = a.tp, pitch = TP + 4, tpq = TP >> 6;  // tpq threads share one channel row
    const int o0 = t * TP, o1 = min(o0 + TP, HpWp);
    const int i0 = interior_before(o0, Wp, pad, H, W), i1 = interior_before(o1, Wp, pad, H, W);
    const int a0 = i0 & ~3;                       // dword-aligned start of the source run
    const int c0 = b * cb + sl * PACK_CH;         // first channel of this slice
    const int nch = min(PACK_CH, cb - sl * PACK_CH);
    const int8_t *plane0 = src + (n * C + c0) * (long long)HW;

    if (i1 > i0) {
        // thread = (channel, 64-byte piece of the run): four 16-byte loads (+ the 4-byte tail)
        // are all in flight before the first LDS write, so one round trip covers the tile
        const int cl = threadIdx.x / tpq, qd = threadIdx.x - cl * tpq;
        const bool live = cl < nch && c0 + cl < C;
        v4i v[4] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}};
        unsigned tail = 0;
        if (live) {
            const int8_t *base = plane0 + (long long)cl * HW + a0;
            const int8_t *p = base + 64 * qd;
            if (a0 + pitch <= HW) {  // uniform: the whole window lies inside the plane
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const v4i_a4 *>(p + 16 * k);
                tail = *reinterpret_cast<const unsigned *>(base + TP);
            } else {  // last tile of a plane: dword by dword, guarded
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = a0 + 64 * qd + 16 * k + 4 * e;
                        if (i + 4 <= HW) v[k][e] = *reinterpret_cast<const int *>(p + 16 * k + 4 * e);
                    }
                if (a0 + TP + 4 <= HW) tail = *reinterpret_cast<const unsigned *>(base + TP);
            }
        }
        if (cl < nch) {
            unsigned *row = reinterpret_cast<unsigned *>(tile + cl * pitch + 64 * qd);
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int e = 0; e < 4; ++e) row[4 * k + e] = (unsigned)v[k][e];
            if (qd == tpq - 1) row[16] = tail;
        }
    }
    __syncthreads();

    const int G = nch / 16;  // 16-channel groups per pixel in this slice
    int8_t *out0 = dst + (((n * Cb + b) * (long long)HpWp) * cb + sl * PACK_CH);
    for (int idx = threadIdx.x; idx < (o1 - o0) * G; idx += 256) {
        const int pl = idx / G, g = idx - pl * G;
        const int o = o0 + pl;
        const int hp = o / Wp, wp = o - hp * Wp;
        v4i ov = {0, 0, 0, 0};
        if (hp >= pad && hp < pad + H && wp >= pad && wp < pad + W) {
            const int col = (hp - pad) * W + (wp - pad) - a0;
            const unsigned char *q = tile + (g * 16) * pitch + col;
            unsigned bytes[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) bytes[k] = q[k * pitch];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                ov[k] = (int)(bytes[4 * k] | (bytes[4 * k + 1] << 8) | (bytes[4 * k + 2] << 16) |
                              (bytes[4 * k + 3] << 24));
        }
        *reinterpret_cast<v4i *>(out0 + (long long)o * cb + g * 16) = ov;
    }
}

__global__ void __launch_bounds__(256) pack_layout_tiled_kernel(const PackArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char tile[PACK_CH * PACK_PITCH];
    pack_layout_tiled_body(a, xcd_contiguous(blockIdx.x, gridDim.x), tile);
}

__global__ void __launch_bounds__(256) pack_layout_wave_kernel(const PackWaveArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned tile[4 * PW_LDS / 4];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long wid = (long long)xcd_contiguous(blockIdx.x, gridDim.x) * 4 + wave;
    if (wid < a.waves) pack_layout_wave_body(a, wid, tile + wave * (PW_LDS / 4));
}

__global__ void __launch_bounds__(256) pack_layout_src_kernel(const PackSrcArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned tile[4 * PW_LDS / 4];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long wid = (long long)xcd_contiguous(blockIdx.x, gridDim.x) * 4 + wave;
    if (wid < a.waves) pack_layout_src_body(a, wid, tile + wave * (PW_LDS / 4));
}

static int grid_for(long long work_items, int block)
{
    long long g = (work_items + block - 1) / block;
    const long long cap = 256LL * 32;  // 32 workgroups per CU keeps every CU busy
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (int)g;
}

// Fills `a` and the workgroup count if the tiled kernel can run this problem.
static bool plan_pack_tiled(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst,
                            PackArgs *a, long long *blocks)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad, Cb = (C + cb - 1) / cb;
    const long long hpwp = (long long)Hp * Wp;
    if (!(cb % 16 == 0 && ((long long)H * W) % 4 == 0 && (reinterpret_cast<uintptr_t>(src) & 3) == 0 &&
          hpwp < (1LL << 30) && (long long)H * W < (1LL << 30)))
        return false;
    const int tp = cb == 16 ? 4 * PACK_TP : cb == 32 ? 2 * PACK_TP : PACK_TP;  // tp * channels <= 16 K
    const int tiles = (int)((hpwp + tp - 1) / tp), slices = (cb + PACK_CH - 1) / PACK_CH;
    *blocks = (long long)N * Cb * slices * tiles;
    if (*blocks >= (1LL << 31)) return false;
    *a = PackArgs{src, dst, C, H, W, cb, pad, Hp, Wp, Cb, tiles, slices, tp};
    return true;
}

hipError_t launch_pack_layout(int N, int C, int H, int W, int cb, int pad,
                              const int8_t *src, int8_t *dst, hipStream_t st)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad, Cb = (C + cb - 1) / cb;
    const long long pixels = (long long)N * Cb * Hp * Wp;
    {
        // 64-channel slices: destination order once there are enough units to fill the chip (whole-line stores,
        // 15 % faster there), source order below that (one round of LDS reads: a shorter dependent chain)
        PackWaveArgs a;
        PackSrcArgs as;
        long long blocks, blocks_s;
        const bool dst_ok = plan_pack_wave(N, C, H, W, cb, pad, src, dst, &a, &blocks);
        const bool src_ok = plan_pack_src(N, C, H, W, cb, pad, src, dst, &as, &blocks_s);
        if (src_ok && !(dst_ok && a.waves >= 256 * 16)) {
            hipLaunchKernelGGL(pack_layout_src_kernel, dim3((unsigned)blocks_s), dim3(256), 0, st, as);
            return hipGetLastError();
        }
        if (dst_ok) {
            hipLaunchKernelGGL(pack_layout_wave_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
            return hipGetLastError();
        }
    }
    {
        PackArgs a;
        long long blocks;
        if (plan_pack_tiled(N, C, H, W, cb, pad, src, dst, &a, &blocks)) {
            hipLaunchKernelGGL(pack_layout_tiled_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
            return hipGetLastError();
        }
    }
    if (cb % 16 == 0) {
        const long long items = pixels * (cb / 16);
        hipLaunchKernelGGL(pack_layout_kernel<16>, dim3(grid_for(items, 256)), dim3(256), 0, st,
                           src, dst, C, H, W, cb, pad, Hp, Wp, Cb, pixels);
    } else if (cb % 8 == 0) {
        const long long items = pixels * (cb / 8);
        hipLaunchKernelGGL(pack_layout_kernel<8>, dim3(grid_for(items, 256)), dim3(256), 0, st,
                           src, dst, C, H, W, cb, pad, Hp, Wp, Cb, pixels);
    } else {
        const long long items = pixels * (cb / 4);
        hipLaunchKernelGGL(pack_layout_kernel<4>, dim3(grid_for(items, 256)), dim3(256), 0, st,
                           src, dst, C, H, W, cb, pad, Hp, Wp, Cb, pixels);
    }
    return hipGetLastError();
}

// ---- pack_weights -----------------------------------------------------------------------
__global__ void __launch_bounds__(256) pack_weights_blocked_kernel(const WeightArgs a)
{
    pack_weights_blocked_body(a, blockIdx.x, gridDim.x, 256);
}

hipError_t launch_pack_weights_blocked(int K, int C, int R, int S, int cb, int depth,
                                       const int8_t *src, int8_t *dst, hipStream_t st)
{
    const long long items = (long long)K * (depth / 16);
    if (items >= (1LL << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_weights_blocked_kernel, dim3(grid_for(items, 256)), dim3(256), 0, st,
                       weight_args_blocked(K, C, R, S, cb, depth, src, dst));
    return hipGetLastError();
}

// Row-padded copy: dst[k][j] = j < CRS ? src[k][j] : 0 (the (c,r,s) order is KCRS itself).
__device__ __forceinline__ void pack_weights_rows_body(const WeightArgs &a, int vbid, int vgrid)
{
    const int8_t *__restrict__ src = a.src;
    int8_t *__restrict__ dst = a.dst;
    const int K = a.K, CRS = a.C * a.R * a.S, depth = a.depth;
    const int chunks = depth / 16;
    const int total = K * chunks;  // < 2^31 (launcher-checked)
    for (int t = vbid * 256 + (int)threadIdx.x; t < total; t += vgrid * 256) {
        const int k = fast_div_any(t, chunks, a.m_chunks), ch = t - k * chunks;
        const int8_t *s = src + (long long)k * CRS;
        int v[16];
        // sixteen loads with no branch between them (positions past the row re-read its last byte)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = s[min(ch * 16 + i, CRS - 1)];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = ch * 16 + i < CRS ? v[i] : 0;
        v4i o;
        o[0] = pack4(v[0], v[1], v[2], v[3]);
        o[1] = pack4(v[4], v[5], v[6], v[7]);
        o[2] = pack4(v[8], v[9], v[10], v[11]);
        o[3] = pack4(v[12], v[13], v[14], v[15]);
        *reinterpret_cast<v4i *>(dst + (long long)k * depth + (long long)ch * 16) = o;
    }
}

__global__ void __launch_bounds__(256) pack_weights_rows_kernel(const WeightArgs a)
{
    pack_weights_rows_body(a, blockIdx.x, gridDim.x);
}

hipError_t launch_pack_weights_rows(int K, int CRS, int depth, const int8_t *src, int8_t *dst,
                                    hipStream_t st)
{
    const long long items = (long long)K * (depth / 16);
    if (items >= (1LL << 31)) return hipErrorInvalidValue;
    // the row copy only needs the product C*R*S: pass it as C with R = S = 1
    hipLaunchKernelGGL(pack_weights_rows_kernel, dim3(grid_for(items, 256)), dim3(256), 0, st,
                       WeightArgs{src, dst, K, CRS, 1, 1, 0, depth, 0, magic_for(depth / 16), 0u, 0u});
    return hipGetLastError();
}

// ---- im2col -----------------------------------------------------------------------------
// dst[m][(c*R + r)*S + s] = in0[n][c][p*st+r-pad][q*st+s-pad]; one thread per 16-byte piece
// of a row, pieces of one row on consecutive lanes (contiguous stores).  Source indices are
// computed in closed form; there is no index list.
__global__ void __launch_bounds__(256)
im2col_kernel(const int8_t *__restrict__ src, int8_t *__restrict__ dst,
              int C, int H, int W, int R, int S, int stride, int pad, int P, int Q,
              int kg, int kg_pad, long long M)
{
    const int chunks = kg_pad / 16;
    const long long total = M * chunks;
    const int PQ = P * Q;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long long)gridDim.x * blockDim.x) {
        const int ch = (int)(t % chunks);
        const long long m = t / chunks;
        const long long n = m / PQ;
        const int pq = (int)(m - n * PQ);
        const int p = pq / Q, q = pq - p * Q;
        const int h0 = p * stride - pad, w0 = q * stride - pad;
        const int8_t *img = src + n * C * (long long)H * W;
        int j = ch * 16;
        int s = j % S, cr = j / S;
        int r = cr % R, c = cr / R;
        int v[16];
        bool in[16];
        // the sixteen loads first, from coordinates clamped into the image (no branch between them)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int h = h0 + r, w = w0 + s;
            in[i] = j + i < kg && h >= 0 && h < H && w >= 0 && w < W;
            v[i] = img[((long long)min(c, C - 1) * H + min(max(h, 0), H - 1)) * W + min(max(w, 0), W - 1)];
            if (++s == S) {
                s = 0;
                if (++r == R) {
                    r = 0;
                    ++c;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = in[i] ? v[i] : 0;
        v4i o;
        o[0] = pack4(v[0], v[1], v[2], v[3]);
        o[1] = pack4(v[4], v[5], v[6], v[7]);
        o[2] = pack4(v[8], v[9], v[10], v[11]);
        o[3] = pack4(v[12], v[13], v[14], v[15]);
        *reinterpret_cast<v4i *>(dst + m * kg_pad + (long long)ch * 16) = o;
    }
}


// Tiled version.  A workgroup owns TQ consecutive output pixels of one output row (n, p) and
// a slice of Cc channels.  The source patch those pixels touch -- rows p*st+r-pad for every
// r, columns q0*st-pad .. (q0+TQ-1)*st-pad+S-1 -- is staged in LDS with the out-of-image
// part zero-filled, so building a destination piece needs no bounds tests: walking (c,r,s)
// in depth order is "+1 byte" inside a kernel row and "+pitch-S+1" at the end of one.
// Index splits use multiply-high by a host-computed reciprocal (exact for the small ranges
// involved), and the patch loads are issued four at a time before any is consumed.  The patch
// pitch is an odd number of dwords: lanes of the second phase read the same columns of many
// different rows, and an even pitch puts those on a handful of LDS banks.
constexpr int I2C_LDS = 48 * 1024;

struct I2cArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, R, S, stride, pad, P, Q, kg, kg_pad;
    int TQ, qtiles, Cc, cslices, span, pitch;
    unsigned m_span, m_R, m_S;  // ceil(2^32 / d)
    int use_recipe;
    long long src_bytes;        // N*C*H*W
};
constexpr int I2C_PBASE = 16;   // slack in front of the patch: a run may start up to three bytes before a row
// Zero bytes behind the patch: what the zero tail of the depth reads, for every pixel of a tile (four pixels at a
// time, a window of up to 16 bytes plus the alignment slack each).
static __host__ __device__ inline int i2c_zero_run(int TQ, int stride) { return ((TQ + 3) * stride + 24) & ~3; }

// Four consecutive pixels of one 16-byte depth piece per thread (stride ST known at compile time).  A run of
// the recipe moves ST bytes per pixel, so the four pixels' runs lie in one window of 3*ST + 4 bytes: it is read
// once as aligned dwords, shifted to start at byte 0 (per-lane shift), and each pixel's dword is then a fixed
// byte-align of two of its dwords.
template <int ST>
__device__ __forceinline__ void i2c_produce4(const unsigned char *lds, const uint2 *rec, int8_t *out0, int nq, int chunks,
                                             unsigned m_chunks, int kg_pad)
{
    constexpr int NW = (3 * ST + 4 + 3) / 4;   // dwords of the shifted window
    const int groups = (nq + 3) >> 2;
    for (int idx = threadIdx.x; idx < groups * chunks; idx += 256) {
        const int gq = fast_div(idx, m_chunks), ch = idx - gq * chunks;
        const unsigned px = (unsigned)(4 * gq * ST);
        const uint4 *rp = reinterpret_cast<const uint4 *>(rec + ch * 4);
        const uint4 ra = rp[0], rb = rp[1];
        const unsigned ex[4] = {ra.x, ra.z, rb.x, rb.z}, em[4] = {ra.y, ra.w, rb.y, rb.w};
        v4i ov[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            unsigned run[2][4];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const unsigned at = (half ? ex[d] >> 16 : ex[d] & 0xFFFFu) + px;
                const unsigned *p = reinterpret_cast<const unsigned *>(lds + (at & ~3u));
                unsigned w[NW + 1], nrm[NW];
#pragma unroll
                for (int k = 0; k <= NW; ++k) w[k] = p[k];
#pragma unroll
                for (int k = 0; k < NW; ++k) nrm[k] = __builtin_amdgcn_alignbyte(w[k + 1], w[k], at & 3u);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int off = i * ST;
                    run[half][i] = (off & 3) == 0 ? nrm[off >> 2]
                                                  : __builtin_amdgcn_alignbyte(nrm[(off >> 2) + 1 < NW ? (off >> 2) + 1 : NW - 1],
                                                                               nrm[off >> 2], (unsigned)(off & 3));
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) ov[i][d] = (int)((run[0][i] & em[d]) | (run[1][i] & ~em[d]));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * gq + i < nq)
                __builtin_nontemporal_store(ov[i], reinterpret_cast<v4i *>(out0 + (long long)(4 * gq + i) * kg_pad + (ch << 4)));
    }
}

__device__ __forceinline__ void im2col_tiled_body(const I2cArgs &a, int bid, unsigned char *lds)
{
    const int8_t *__restrict__ src = a.src;
    int8_t *__restrict__ dst = a.dst;
    const int cs = bid % a.cslices;
    bid /= a.cslices;
    const int qt = bid % a.qtiles;
    bid /= a.qtiles;
    const int p = bid % a.P;
    const long long n = bid / a.P;
    const int q0 = qt * a.TQ, nq = min(a.TQ, a.Q - q0);
    const int c0 = cs * a.Cc, nc = min(a.Cc, a.C - c0);
    const int w_lo = q0 * a.stride - a.pad, h_lo = p * a.stride - a.pad;
    const int8_t *img = src + (n * a.C + c0) * (long long)a.H * a.W;

    // LDS: [slack][patch: nc*R rows x pitch][zero run][recipe table]
    constexpr int PBASE = I2C_PBASE;
    unsigned char *patch = lds + PBASE;
    const int rows = nc * a.R;
    const int zoff = PBASE + rows * a.pitch;

    if (a.W >= 16) {
        // stage the patch in 16-byte pieces: one load at any byte address
        // -- a piece that starts left of the image row or runs past its end reads the neighbouring row's bytes
        // -- and a byte mask that turns everything outside the row, and every row outside the image, to zero
        const int pcs = (a.pitch + 15) >> 4;   // (the last piece of a row may be cut short by the pitch)
        const int total = rows * pcs;
        const unsigned m_pcs = magic_for_device(pcs);
        const long long img_off = (n * a.C + c0) * (long long)a.H * a.W;
        for (int base = 0; base < total; base += 256 * 4) {
            v4i v[4];
            int hh[4], ww[4];
            long long want[4];
            bool moved[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = min(base + u * 256 + (int)threadIdx.x, total - 1);
                const int row = fast_div(idx, m_pcs), t = idx - row * pcs;
                const int cl = fast_div(row, a.m_R), r = row - cl * a.R;
                hh[u] = h_lo + r, ww[u] = w_lo + 16 * t;
                want[u] = img_off + ((long long)cl * a.H + min(max(hh[u], 0), a.H - 1)) * a.W + ww[u];
                const long long at = min(max(want[u], 0LL), a.src_bytes - 16);
                moved[u] = at != want[u];
                __builtin_memcpy(&v[u], src + at, 16);   // (nothing that needs the data between the loads)
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (moved[u]) {   // the tensor's first or last bytes: byte by byte
                    asm volatile("" ::: "memory");   // stays a branch
                    const long long at = min(max(want[u], 0LL), a.src_bytes - 16);
                    v[u] = at - want[u] > -16 && at - want[u] < 16 ? shift_piece(v[u], (int)(at - want[u])) : v4i{0, 0, 0, 0};
                }
                const bool rowok = hh[u] >= 0 && hh[u] < a.H;
                const int lo = min(max(-ww[u], 0), 16), hi = rowok ? min(max(a.W - ww[u], 0), 16) : 0;
                v4i x;
#pragma unroll
                for (int q = 0; q < 2; ++q) {   // eight bytes at a time
                    const int l = min(max(lo - 8 * q, 0), 8), h8 = min(max(hi - 8 * q, 0), 8);
                    const unsigned long long ml = l == 8 ? 0ull : ~0ull << (8 * l), mh = h8 == 0 ? 0ull : ~0ull >> (64 - 8 * h8);
                    x[2 * q] = (int)((unsigned)v[u][2 * q] & (unsigned)(ml & mh));
                    x[2 * q + 1] = (int)((unsigned)v[u][2 * q + 1] & (unsigned)((ml & mh) >> 32));
                }
                const int idx = base + u * 256 + (int)threadIdx.x;
                if (idx < total) {
                    // dword stores: the pitch is an odd number of dwords, which keeps the column-wise reads of the
                    // second phase off each other's banks
                    const int row = fast_div(idx, m_pcs), t = idx - row * pcs;
                    unsigned *o = reinterpret_cast<unsigned *>(patch + row * a.pitch + 16 * t);
#pragma unroll
                    for (int m = 0; m < 4; ++m)
                        if (16 * t + 4 * m < a.pitch) o[m] = (unsigned)x[m];
                }
            }
        }
    } else {
    // narrow images: four columns at a time, without branches: one (unaligned) dword load
    // from the column window clamped into the image row, shifted so that the bytes that fall
    // outside the row become the zero padding
    const int pd = a.pitch >> 2;  // dwords per patch row
    const int total = rows * pd;
    const unsigned m_pd = (unsigned)((0x100000000ULL + pd - 1) / pd);
    for (int base = 0; base < total; base += 256 * 4) {
        unsigned v[4];
        int at[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = min(base + u * 256 + (int)threadIdx.x, total - 1);
            const int row = fast_div(idx, m_pd), c4 = idx - row * pd;
            const int cl = fast_div(row, a.m_R), r = row - cl * a.R;
            const int h = h_lo + r, w = w_lo + 4 * c4;
            const int hc = min(max(h, 0), a.H - 1), wc = min(max(w, 0), a.W - 4);  // W >= 4 (host-checked)
            unsigned x;
            __builtin_memcpy(&x, img + ((long long)cl * a.H + hc) * a.W + wc, 4);
            const int d = wc - w;  // > 0: window starts left of the row, < 0: it runs past the end
            const unsigned sh = (unsigned)(d > 0 ? d : -d) * 8u;
            unsigned y = d >= 0 ? (x << (sh & 31u)) : (x >> (sh & 31u));
            if (sh >= 32u || h != hc) y = 0u;
            v[u] = y;
            at[u] = row * a.pitch + 4 * c4;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + u * 256 + (int)threadIdx.x < total) *reinterpret_cast<unsigned *>(patch + at[u]) = v[u];
    }
    }

    // destination pieces of this channel slice: depth range [c0*R*S, (c0+nc)*R*S), plus the
    // zero tail up to kg_pad for the last slice; slice boundaries are multiples of 16
    const int RS = a.R * a.S;
    const int j_begin = c0 * RS;
    const int j_end = (cs == a.cslices - 1) ? a.kg_pad : (c0 + nc) * RS;
    const int chunks = (j_end - j_begin) >> 4;
    const unsigned m_chunks = (unsigned)((0x100000000ULL + chunks - 1) / chunks);
    int8_t *out0 = dst + ((n * a.P + p) * (long long)a.Q + q0) * a.kg_pad + j_begin;

    if (a.use_recipe) {
        // Every destination dword is at most two byte runs of the patch (S >= 3: the first run gives
        // n0 >= 1 bytes, the next kernel row the other 4 - n0 <= 3 <= S): a run inside
        // one kernel row, then the start of the next row or the zero tail.  The recipe -- where
        // each run starts and how many bytes the first one gives -- depends on the depth only,
        // so it is tabulated once; a pixel adds q*stride.  A run is fetched as two aligned
        // dwords and one byte-align; the two runs are merged under a byte mask.
        const int zsz = i2c_zero_run(a.TQ, a.stride);
        for (int i = threadIdx.x; i < (zsz >> 2); i += 256) *reinterpret_cast<unsigned *>(lds + zoff + 4 * i) = 0u;
        if (threadIdx.x < PBASE / 4) *reinterpret_cast<unsigned *>(lds + 4 * threadIdx.x) = 0u;
        // per destination dword: {start of the first run | start of the second run minus n0 << 16, byte mask of the first run}
        uint2 *rec = reinterpret_cast<uint2 *>(lds + ((zoff + zsz + 15) & ~15));
        const int ndw = (j_end - j_begin) >> 2;
        for (int dd = threadIdx.x; dd < ndw; dd += 256) {
            const int j0 = dd << 2;
            unsigned o0 = (unsigned)zoff, n0 = 4, w1 = (unsigned)zoff;
            if (j_begin + j0 < a.kg) {
                const int cr = fast_div(j0, a.m_S), sx = j0 - cr * a.S;
                o0 = (unsigned)(PBASE + cr * a.pitch + sx);
                n0 = (unsigned)min(4, a.S - sx);
                w1 = o0;
                if (n0 < 4) {
                    const unsigned o1 = (j_begin + j0 + (int)n0 < a.kg) ? (unsigned)(PBASE + (cr + 1) * a.pitch)
                                                                        : (unsigned)zoff;
                    w1 = o1 - n0;
                }
            }
            rec[dd] = make_uint2(o0 | (w1 << 16), n0 >= 4 ? 0xFFFFFFFFu : ((1u << (8 * n0)) - 1u));
        }
        __syncthreads();
        if (a.stride == 1) return i2c_produce4<1>(lds, rec, out0, nq, chunks, m_chunks, a.kg_pad);
        if (a.stride == 2) return i2c_produce4<2>(lds, rec, out0, nq, chunks, m_chunks, a.kg_pad);
        for (int idx = threadIdx.x; idx < nq * chunks; idx += 256) {
            const int ql = fast_div(idx, m_chunks), ch = idx - ql * chunks;
            const unsigned px = (unsigned)(ql * a.stride);
            v4i ov;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint2 e = rec[ch * 4 + d];
                const unsigned a0 = (e.x & 0xFFFFu) + px, a1 = (e.x >> 16) + px;
                const unsigned *p0 = reinterpret_cast<const unsigned *>(lds + (a0 & ~3u));
                const unsigned *p1 = reinterpret_cast<const unsigned *>(lds + (a1 & ~3u));
                const unsigned v0 = __builtin_amdgcn_alignbyte(p0[1], p0[0], a0 & 3u);
                const unsigned v1 = __builtin_amdgcn_alignbyte(p1[1], p1[0], a1 & 3u);
                ov[d] = (int)((v0 & e.y) | (v1 & ~e.y));
            }
            __builtin_nontemporal_store(ov, reinterpret_cast<v4i *>(out0 + (long long)ql * a.kg_pad + (ch << 4)));
        }
        return;
    }

    __syncthreads();
    for (int idx = threadIdx.x; idx < nq * chunks; idx += 256) {
        const int ql = fast_div(idx, m_chunks), ch = idx - ql * chunks;
        const int jl = ch << 4;  // depth offset inside this slice
        const int cr = fast_div(jl, a.m_S);  // (c - c0)*R + r
        int sx = jl - cr * a.S;
        int addr = cr * a.pitch + ql * a.stride + sx;
        const int valid = a.kg - j_begin - jl;  // bytes of this piece that are real depth
        unsigned bytes[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            bytes[k] = k < valid ? patch[addr] : 0u;
            ++addr;
            if (++sx == a.S) {
                sx = 0;
                addr += a.pitch - a.S;
            }
        }
        v4i ov;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            ov[k] = (int)(bytes[4 * k] | (bytes[4 * k + 1] << 8) | (bytes[4 * k + 2] << 16) |
                          (bytes[4 * k + 3] << 24));
        *reinterpret_cast<v4i *>(out0 + (long long)ql * a.kg_pad + jl) = ov;
    }
}

__global__ void __launch_bounds__(256) im2col_tiled_kernel(const I2cArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char patch[];
    im2col_tiled_body(a, xcd_contiguous(blockIdx.x, gridDim.x), patch);
}

// Fills `a`, the workgroup count and the LDS bytes if the tiled kernel can run this problem.
static bool plan_im2col_tiled(int N, int C, int H, int W, int R, int S, int stride, int pad, int P, int Q,
                              int kg_pad, const int8_t *src, int8_t *dst, I2cArgs *out, long long *blocks,
                              size_t *lds)
{
    // tile width: enough pixels that a workgroup writes a few tens of KB, within one row
    int TQ = (32 * 1024 + kg_pad - 1) / kg_pad;
    if (TQ > Q) TQ = Q;
    if (TQ > 256) TQ = 256;
    // small problems: narrower tiles until there are about two workgroups per CU (measured:
    // narrower than that costs more in repeated patch staging than the extra workgroups gain)
    const long long rows = (long long)N * P;
    if (rows * ((Q + TQ - 1) / TQ) < 512) {
        const long long want = (512 + rows - 1) / rows;
        int narrow = (int)((Q + want - 1) / want);
        if (narrow < 32) narrow = 32;
        if (narrow < TQ) TQ = narrow;
    }
    if (TQ < 1) TQ = 1;
    const long long span64 = (long long)(TQ - 1) * stride + S;
    const int span = (int)span64, pitch = 4 * (((span + 3) / 4) | 1);   // an odd number of dwords
    // channels per slice: all of them if the patch fits, else a multiple of 16 that does
    int Cc = C;
    if ((long long)C * R * pitch > I2C_LDS) Cc = (int)(I2C_LDS / ((long long)R * pitch)) / 16 * 16;
    if (Cc <= 0) return false;
    if (W < 4) return false;  // the staging loads take 4 bytes of one image row
    if ((long long)C * H * W >= (1LL << 40)) return false;
    const int qtiles = (Q + TQ - 1) / TQ;
    const long long cslices = (C + Cc - 1) / Cc;
    *blocks = (long long)N * P * qtiles * cslices;
    // multiply-high index splits are exact while dividend * divisor < 2^32
    const bool small = span64 < 65536 && S < 1024 && R < 65536 && (long long)C * R * S < (1LL << 20) &&
                       kg_pad < (1 << 19);
    if (!small || *blocks >= (1LL << 31)) return false;
    // LDS: slack + patch + zero run + (recipe path) 8 B per destination dword of a slice
    const long long patch_bytes = I2C_PBASE + (long long)(Cc < C ? Cc : C) * R * pitch;
    const long long zsz = i2c_zero_run(TQ, stride);
    const long long slice_depth = cslices == 1 ? kg_pad : (long long)Cc * R * S + 64;
    const long long with_recipe = ((patch_bytes + zsz + 15) & ~15LL) + 2 * slice_depth;
    const bool recipe = S >= 3 && with_recipe <= 60 * 1024;
    I2cArgs a;
    a.src = src; a.dst = dst;
    a.C = C; a.H = H; a.W = W; a.R = R; a.S = S; a.stride = stride; a.pad = pad; a.P = P; a.Q = Q;
    a.kg = C * R * S; a.kg_pad = kg_pad; a.TQ = TQ; a.qtiles = qtiles; a.Cc = Cc;
    a.cslices = (int)cslices; a.span = span; a.pitch = pitch;
    a.m_span = (unsigned)((0x100000000ULL + span - 1) / span);
    a.m_R = (unsigned)((0x100000000ULL + R - 1) / R);
    a.m_S = (unsigned)((0x100000000ULL + S - 1) / S);
    a.use_recipe = recipe;
    a.src_bytes = (long long)N * C * H * W;
    *out = a;
    *lds = (size_t)(recipe ? with_recipe : patch_bytes + 8);
    return true;
}

hipError_t launch_im2col(int N, int C, int H, int W, int R, int S, int stride, int pad,
                         int P, int Q, int kg_pad, const int8_t *src, int8_t *dst, hipStream_t st)
{
    const long long M = (long long)N * P * Q;
    const long long items = M * (kg_pad / 16);
    {
        I2cArgs a;
        long long blocks;
        size_t lds;
        if (plan_im2col_tiled(N, C, H, W, R, S, stride, pad, P, Q, kg_pad, src, dst, &a, &blocks, &lds)) {
            hipLaunchKernelGGL(im2col_tiled_kernel, dim3((unsigned)blocks), dim3(256), lds, st, a);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL(im2col_kernel, dim3(grid_for(items, 256)), dim3(256), 0, st,
                       src, dst, C, H, W, R, S, stride, pad, P, Q, C * R * S, kg_pad, M);
    return hipGetLastError();
}

// ---- input rewrite + weight rewrite in one launch ----------------------------------------
// The two rewrites of a convolution are independent; for the small layers this library is
// measured on, a kernel launch costs more than either of them, so the one-shot path runs
// them as two workgroup ranges of a single grid.
struct FusedArgs {
    int in_blocks, w_blocks, in_is_im2col, w_is_blocked, in_is_wave;
    PackArgs pk;
    PackSrcArgs pw;
    I2cArgs ic;
    WeightArgs wt;
};

__global__ void __launch_bounds__(256) rewrite_fused_kernel(const FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int bid = blockIdx.x;
    if (bid < a.in_blocks) {
        const int lid = xcd_contiguous(bid, a.in_blocks);
        if (a.in_is_im2col) {
            im2col_tiled_body(a.ic, lid, lds);
        } else if (a.in_is_wave) {
            const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            const long long wid = (long long)lid * 4 + wave;
            if (wid < a.pw.waves)
                pack_layout_src_body(a.pw, wid, reinterpret_cast<unsigned *>(lds) + wave * (PW_LDS / 4));
        } else {
            pack_layout_tiled_body(a.pk, lid, lds);
        }
    } else {
        if (a.w_is_blocked) pack_weights_blocked_body(a.wt, bid - a.in_blocks, a.w_blocks, 256);
        else pack_weights_rows_body(a.wt, bid - a.in_blocks, a.w_blocks);
    }
}

// Returns hipErrorNotSupported when the tiled input kernels cannot take the problem; the
// caller then launches the two rewrites separately.
hipError_t launch_rewrite_fused(bool im2col, int N, int C, int H, int W, int K, int R, int S, int stride,
                                int pad, int P, int Q, int cb, int depth, const int8_t *in, int8_t *xq,
                                const int8_t *wt, int8_t *wq, hipStream_t st)
{
    FusedArgs a{};
    long long blocks = 0;
    size_t lds = PACK_CH * PACK_PITCH;
    if (im2col) {
        if (!plan_im2col_tiled(N, C, H, W, R, S, stride, pad, P, Q, depth, in, xq, &a.ic, &blocks, &lds))
            return hipErrorNotSupported;
        a.wt = WeightArgs{wt, wq, K, C * R * S, 1, 1, 0, depth, 0, magic_for(depth / 16), 0u, 0u};
    } else {
        if (plan_pack_src(N, C, H, W, cb, pad, in, xq, &a.pw, &blocks)) {
            a.in_is_wave = 1;
            lds = 4 * PW_LDS;
        } else if (!plan_pack_tiled(N, C, H, W, cb, pad, in, xq, &a.pk, &blocks)) {
            return hipErrorNotSupported;
        }
        a.wt = weight_args_blocked(K, C, R, S, cb, depth, wt, wq);
    }
    const long long w_items = (long long)K * (depth / 16);
    if (w_items >= (1LL << 31)) return hipErrorNotSupported;
    a.in_blocks = (int)blocks;
    a.w_blocks = grid_for(w_items, 256);
    a.in_is_im2col = im2col;
    a.w_is_blocked = !im2col;
    if (blocks + a.w_blocks >= (1LL << 31)) return hipErrorNotSupported;
    hipLaunchKernelGGL(rewrite_fused_kernel, dim3((unsigned)(blocks + a.w_blocks)), dim3(256), lds, st, a);
    return hipGetLastError();
}

// ---- channel blocking from an NHWC source (Sec. 5.2: source layouts other than NCHW) -------
// dst[n][c/cb][h+pad][w+pad][c%cb] = src[n][h][w][c]: the channels of a pixel are already
// contiguous, so a destination 16-byte piece is one 16-byte load (any alignment), the tail of a
// pixel's channels byte by byte, zero on the border and past C.  One thread per 16 bytes.
struct PackNhwcArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, cb, pad, Hp, Wp, Cb, g16;
    long long total;  // 16-byte pieces
    unsigned m_g16, m_Wp, m_Hp, m_Cb;
};

// (virtual workgroup vbid of vgrid: the one-shot path runs this as one workgroup range of a shared grid)
__device__ __forceinline__ void pack_layout_nhwc_body(const PackNhwcArgs &a, int vbid, int vgrid)
{
    for (long long t = (long long)vbid * 256 + threadIdx.x; t < a.total; t += (long long)vgrid * 256) {
        int c16, wp, hp, b;
        long long n;
        if (a.total < (1LL << 31)) {
            const int i0 = (int)t;
            const int i1 = fast_div_any(i0, a.g16, a.m_g16); c16 = i0 - i1 * a.g16;
            const int i2 = fast_div_any(i1, a.Wp, a.m_Wp); wp = i1 - i2 * a.Wp;
            const int i3 = fast_div_any(i2, a.Hp, a.m_Hp); hp = i2 - i3 * a.Hp;
            const int i4 = fast_div_any(i3, a.Cb, a.m_Cb); b = i3 - i4 * a.Cb;
            n = i4;
        } else {
            long long r = t;
            c16 = (int)(r % a.g16); r /= a.g16;
            wp = (int)(r % a.Wp); r /= a.Wp;
            hp = (int)(r % a.Hp); r /= a.Hp;
            b = (int)(r % a.Cb); n = r / a.Cb;
        }
        const int c0 = b * a.cb + c16 * 16, h = hp - a.pad, w = wp - a.pad;
        v4i v = {0, 0, 0, 0};
        if (h >= 0 && h < a.H && w >= 0 && w < a.W && c0 < a.C) {
            const int8_t *p = a.src + ((n * a.H + h) * a.W + w) * a.C + c0;
            if (c0 + 16 <= a.C) {
                __builtin_memcpy(&v, p, 16);
            } else {
                unsigned char bytes[16] = {0};
                for (int i = 0; c0 + i < a.C; ++i) bytes[i] = (unsigned char)p[i];
                __builtin_memcpy(&v, bytes, 16);
            }
        }
        __builtin_nontemporal_store(v, &reinterpret_cast<v4i *>(a.dst)[t]);   // whole lines, written once: streamed (+6 % at 0.85 GB)
    }
}

__global__ void __launch_bounds__(256) pack_layout_nhwc_kernel(const PackNhwcArgs a)
{
    pack_layout_nhwc_body(a, blockIdx.x, gridDim.x);
}

// channel blocking from NHWC and the blocked weight rewrite as two workgroup ranges of one grid
__global__ void __launch_bounds__(256) rewrite_fused_nhwc_kernel(const PackNhwcArgs a, const WeightArgs w, int in_blocks,
                                                                 int w_blocks)
{
    if ((int)blockIdx.x < in_blocks) pack_layout_nhwc_body(a, blockIdx.x, in_blocks);
    else pack_weights_blocked_body(w, blockIdx.x - in_blocks, w_blocks, 256);
}

static PackNhwcArgs pack_nhwc_args(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst)
{
    PackNhwcArgs a{};
    a.src = src; a.dst = dst;
    a.C = C; a.H = H; a.W = W; a.cb = cb; a.pad = pad;
    a.Hp = H + 2 * pad; a.Wp = W + 2 * pad;
    a.Cb = (C + cb - 1) / cb;
    a.g16 = cb / 16;
    a.total = (long long)N * a.Cb * a.Hp * a.Wp * a.g16;
    a.m_g16 = magic_for(a.g16); a.m_Wp = magic_for(a.Wp); a.m_Hp = magic_for(a.Hp); a.m_Cb = magic_for(a.Cb);
    return a;
}

hipError_t launch_pack_layout_nhwc(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst,
                                   hipStream_t st)
{
    const PackNhwcArgs a = pack_nhwc_args(N, C, H, W, cb, pad, src, dst);
    hipLaunchKernelGGL(pack_layout_nhwc_kernel, dim3(grid_for(a.total, 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// hipErrorNotSupported: more weight pieces than the blocked body indexes with 32 bits (the caller then
// launches the two rewrites separately)
hipError_t launch_rewrite_fused_nhwc(int N, int C, int H, int W, int K, int R, int S, int pad, int cb, int depth,
                                     const int8_t *in, int8_t *xq, const int8_t *wt, int8_t *wq, hipStream_t st)
{
    const PackNhwcArgs a = pack_nhwc_args(N, C, H, W, cb, pad, in, xq);
    const long long w_items = (long long)K * (depth / 16);
    if (w_items >= (1LL << 31)) return hipErrorNotSupported;
    const WeightArgs w = weight_args_blocked(K, C, R, S, cb, depth, wt, wq);
    const int in_blocks = grid_for(a.total, 256), w_blocks = grid_for(w_items, 256);
    hipLaunchKernelGGL(rewrite_fused_nhwc_kernel, dim3(in_blocks + w_blocks), dim3(256), 0, st, a, w, in_blocks, w_blocks);
    return hipGetLastError();
}

// ---- stencil unrolling from an NHWC source (Sec. 5.2) ------------------------------------------------
// dst[(n,p,q)][(r*S + s)*C + c] = in0[n][p*st+r-pad][q*st+s-pad][c], zero past C*R*S: the channels of a tap
// are contiguous in the source, so with C % 16 == 0 a destination 16-byte piece is one 16-byte load of one
// tap (or zeros); other channel counts go byte by byte.  One thread per 16 destination bytes; the load is
// issued from a clamped address and discarded where the tap lies outside the image.
struct I2cNhwcArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, R, S, stride, pad, P, Q, kg, kg_pad, chunks;
    long long total;   // pieces
    unsigned m_chunks, m_Q, m_P, m_C, m_S;
};

__global__ void __launch_bounds__(256) im2col_nhwc_kernel(const I2cNhwcArgs a)
{
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < a.total; t += (long long)gridDim.x * 256) {
        long long m, n;
        int ch, q, p;
        if (a.total < (1LL << 31)) {   // uniform: the usual case, 32-bit multiply-high splits
            const int mi = fast_div_any((int)t, a.chunks, a.m_chunks);
            ch = (int)t - mi * a.chunks;
            const int npi = fast_div_any(mi, a.Q, a.m_Q);
            q = mi - npi * a.Q;
            const int ni = fast_div_any(npi, a.P, a.m_P);
            p = npi - ni * a.P;
            m = mi, n = ni;
        } else {
            m = t / a.chunks;
            ch = (int)(t - m * a.chunks);
            const long long np_ = m / a.Q;
            q = (int)(m - np_ * a.Q);
            n = np_ / a.P;
            p = (int)(np_ - n * a.P);
        }
        const int j0 = 16 * ch;
        v4i o = {0, 0, 0, 0};
        if ((a.C & 15) == 0) {   // uniform
            const int tap = fast_div_any(min(j0, a.kg - 16), a.C, a.m_C), c0 = min(j0, a.kg - 16) - tap * a.C;
            const int r = fast_div_any(tap, a.S, a.m_S), s = tap - r * a.S;
            const int h = p * a.stride + r - a.pad, w = q * a.stride + s - a.pad;
            const int hc = min(max(h, 0), a.H - 1), wc = min(max(w, 0), a.W - 1);
            const v4i x = *reinterpret_cast<const v4i *>(a.src + ((n * a.H + hc) * a.W + wc) * a.C + c0);
            if (j0 < a.kg && h == hc && w == wc) o = x;
        } else {
            unsigned b[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {   // sixteen independent loads, then the selection
                const int j = min(j0 + i, a.kg - 1);
                const int tap = fast_div_any(j, a.C, a.m_C), c = j - tap * a.C;
                const int r = fast_div_any(tap, a.S, a.m_S), s = tap - r * a.S;
                const int h = p * a.stride + r - a.pad, w = q * a.stride + s - a.pad;
                const int hc = min(max(h, 0), a.H - 1), wc = min(max(w, 0), a.W - 1);
                const unsigned x = (unsigned char)a.src[((n * a.H + hc) * a.W + wc) * a.C + c];
                b[i] = (j0 + i < a.kg && h == hc && w == wc) ? x : 0u;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) o[k] = (int)(b[4 * k] | b[4 * k + 1] << 8 | b[4 * k + 2] << 16 | b[4 * k + 3] << 24);
        }
        // written once, whole lines per wave: streamed past the caches, which keep the re-read source
        __builtin_nontemporal_store(o, reinterpret_cast<v4i *>(a.dst + m * a.kg_pad + j0));
    }
}

// dst[k][(r*S + s)*C + c] = src[k][c][r][s], zero past C*R*S; one thread per destination byte (weights are small)
__global__ void __launch_bounds__(256) pack_weights_rsc_kernel(const int8_t *src, int8_t *dst, int K, int C, int R, int S,
                                                               int depth)
{
    const long long total = (long long)K * depth;
    const int kg = C * R * S;
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < total; t += (long long)gridDim.x * 256) {
        const long long k = t / depth;
        const int j = (int)(t - k * depth);
        const int jc = min(j, kg - 1), tap = jc / C, c = jc - tap * C;
        const int8_t x = src[(k * C + c) * (long long)(R * S) + tap];
        dst[t] = j < kg ? x : (int8_t)0;
    }
}

hipError_t launch_im2col_nhwc(int N, int C, int H, int W, int R, int S, int stride, int pad, int P, int Q, int kg_pad,
                              const int8_t *src, int8_t *dst, hipStream_t st)
{
    I2cNhwcArgs a{};
    a.src = src; a.dst = dst;
    a.C = C; a.H = H; a.W = W; a.R = R; a.S = S; a.stride = stride; a.pad = pad; a.P = P; a.Q = Q;
    a.kg = C * R * S; a.kg_pad = kg_pad; a.chunks = kg_pad / 16;
    a.total = (long long)N * P * Q * a.chunks;
    a.m_C = magic_for(C); a.m_S = magic_for(S);
    a.m_chunks = magic_for(a.chunks); a.m_Q = magic_for(Q); a.m_P = magic_for(P);
    hipLaunchKernelGGL(im2col_nhwc_kernel, dim3(grid_for(a.total, 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_pack_weights_rsc(int K, int C, int R, int S, int depth, const int8_t *src, int8_t *dst, hipStream_t st)
{
    hipLaunchKernelGGL(pack_weights_rsc_kernel, dim3(grid_for((long long)K * depth, 256)), dim3(256), 0, st, src, dst, K, C,
                       R, S, depth);
    return hipGetLastError();
}

// ---- unpacking for an NHWC consumer: [N][K][PQ] int32 -> [N][PQ][K] ---------------------------
// Tiles of 64 channels x 32 pixels through LDS (pitch 33: the pixel-wise writes and the
// channel-wise reads are both conflict-free); reads run along pixels in 128-byte runs, writes
// along channels in 256-byte runs.
__global__ void __launch_bounds__(256) unpack_nhwc_kernel(const int32_t *src, int32_t *dst, int K, int PQ,
                                                          int tiles_k, int tiles_p, long long ntiles)
{
    __shared__ int32_t tile[64][33];
    const int rx = threadIdx.x & 31, ry = threadIdx.x >> 5;  // read:  32 pixels x 8 channel rows per pass
    const int wx = threadIdx.x & 63, wy = threadIdx.x >> 6;  // write: 64 channels x 4 pixel rows per pass
    // neighbouring tiles share the cache lines at their common edge (a row of pixels is not a multiple of
    // a line): workgroups that run side by side in one XCD, behind one L2, take neighbouring tiles
    // (L2 fetches 1.13x the source instead of 2x; the time is the same, a plain copy's)
    for (long long t = xcd_contiguous(blockIdx.x, gridDim.x); t < ntiles; t += gridDim.x) {
        const int tp = (int)(t % tiles_p);
        const long long r = t / tiles_p;
        const int tk = (int)(r % tiles_k);
        const long long n = r / tiles_k;
        const int k0 = tk * 64, p0 = tp * 32;
        const int32_t *s = src + (size_t)n * K * PQ;
        int32_t *d = dst + (size_t)n * PQ * K;
        // all eight loads first (indices clamped into the plane: no branch between the loads); what the
        // clamped ones fetch lands in tile cells that are never written out
        int32_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = s[(size_t)min(k0 + ry + 8 * i, K - 1) * PQ + min(p0 + rx, PQ - 1)];
#pragma unroll
        for (int i = 0; i < 8; ++i) tile[ry + 8 * i][rx] = v[i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int p = p0 + wy + 4 * i, k = k0 + wx;
            if (k < K && p < PQ) __builtin_nontemporal_store(tile[wx][wy + 4 * i], &d[(size_t)p * K + k]);   // 256-byte runs, written once: streamed
        }
        __syncthreads();
    }
}

hipError_t launch_unpack_nhwc(int N, int K, long long PQ, const int32_t *src, int32_t *dst, hipStream_t st)
{
    const int tiles_k = (K + 63) / 64, tiles_p = (int)((PQ + 31) / 32);
    const long long ntiles = (long long)N * tiles_k * tiles_p;
    hipLaunchKernelGGL(unpack_nhwc_kernel, dim3(grid_for(ntiles * 256, 256)), dim3(256), 0, st, src, dst, K, (int)PQ,
                       tiles_k, tiles_p, ntiles);
    return hipGetLastError();
}

// ---- activation between two int8 layers (Sec. 5.1: the accelerator's ALU; the benchmark's step
// between convolution and unpacking): rounding right shift, optional max(., 0), clip to int8 -------

// same element order, int32 -> int8; one thread per 16 elements
__global__ void __launch_bounds__(256) requant_kernel(const int32_t *src, int8_t *dst, long long count, int shift, int relu)
{
    const long long n16 = (count + 15) / 16;
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < n16; t += (long long)gridDim.x * 256) {
        const long long e0 = 16 * t;
        if (e0 + 16 <= count) {
            v4i o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v4i x;
                __builtin_memcpy(&x, src + e0 + 4 * j, 16);
                o[j] = (int)pack4(act_requant(x[0], shift, relu), act_requant(x[1], shift, relu), act_requant(x[2], shift, relu),
                                  act_requant(x[3], shift, relu));
            }
            __builtin_memcpy(dst + e0, &o, 16);
        } else {
            for (long long e = e0; e < count; ++e) dst[e] = (int8_t)act_requant(src[e], shift, relu);
        }
    }
}

// activation and the next layer's channel blocking in one pass:
// dst[n][k/cb][p+pad][q+pad][k%cb] = requant(src[n][k][p][q]); zero where k >= K and on the border.
// One thread per 16 destination bytes (16 channels of one pixel: 16 loads a plane apart).
struct RequantPackArgs {
    const int32_t *src;
    int8_t *dst;
    int K, P, Q, cb, pad, Hp, Wp, Cb, g16, shift, relu;
    long long total;
    unsigned m_g16, m_Wp, m_Hp, m_Cb;
};

__global__ void __launch_bounds__(256) requant_pack_kernel(const RequantPackArgs a)
{
    const size_t PQ = (size_t)a.P * a.Q;
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < a.total; t += (long long)gridDim.x * 256) {
        int c16, wp, hp, b;
        long long n;
        if (a.total < (1LL << 31)) {
            const int i0 = (int)t;
            const int i1 = fast_div_any(i0, a.g16, a.m_g16); c16 = i0 - i1 * a.g16;
            const int i2 = fast_div_any(i1, a.Wp, a.m_Wp); wp = i1 - i2 * a.Wp;
            const int i3 = fast_div_any(i2, a.Hp, a.m_Hp); hp = i2 - i3 * a.Hp;
            const int i4 = fast_div_any(i3, a.Cb, a.m_Cb); b = i3 - i4 * a.Cb;
            n = i4;
        } else {
            long long r = t;
            c16 = (int)(r % a.g16); r /= a.g16;
            wp = (int)(r % a.Wp); r /= a.Wp;
            hp = (int)(r % a.Hp); r /= a.Hp;
            b = (int)(r % a.Cb); n = r / a.Cb;
        }
        const int k0 = b * a.cb + c16 * 16, p = hp - a.pad, q = wp - a.pad;
        v4i o = {0, 0, 0, 0};
        if (p >= 0 && p < a.P && q >= 0 && q < a.Q && k0 < a.K) {
            const int32_t *s = a.src + ((size_t)n * a.K + k0) * PQ + (size_t)p * a.Q + q;
            int x[16], v[16];
            // all sixteen loads first (channels past K re-read the last one: no branch between the loads)
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = s[(size_t)min(i, a.K - 1 - k0) * PQ];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = k0 + i < a.K ? act_requant(x[i], a.shift, a.relu) : 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (int)pack4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
        }
        reinterpret_cast<v4i *>(a.dst)[t] = o;
    }
}

hipError_t launch_requant(long long count, const int32_t *src, int8_t *dst, int shift, int relu, hipStream_t st)
{
    hipLaunchKernelGGL(requant_kernel, dim3(grid_for((count + 15) / 16, 256)), dim3(256), 0, st, src, dst, count, shift,
                       relu);
    return hipGetLastError();
}

hipError_t launch_requant_pack(int N, int K, int P, int Q, int cb, int pad, int shift, int relu, const int32_t *src,
                               int8_t *dst, hipStream_t st)
{
    RequantPackArgs a{};
    a.src = src; a.dst = dst;
    a.K = K; a.P = P; a.Q = Q; a.cb = cb; a.pad = pad; a.shift = shift; a.relu = relu;
    a.Hp = P + 2 * pad; a.Wp = Q + 2 * pad;
    a.Cb = (K + cb - 1) / cb;
    a.g16 = cb / 16;
    a.total = (long long)N * a.Cb * a.Hp * a.Wp * a.g16;
    a.m_g16 = magic_for(a.g16); a.m_Wp = magic_for(a.Wp); a.m_Hp = magic_for(a.Hp); a.m_Cb = magic_for(a.Cb);
    hipLaunchKernelGGL(requant_pack_kernel, dim3(grid_for(a.total, 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

static hipError_t launch_phase_split(int N, int C, int H, int W, int pad, int s, int H2, int W2, long long pn, long long pc,
                                     long long pa, long long pb, const int8_t *src, int8_t *dst, hipStream_t st);

// ---- Image Pack (Table 2, row 1: the stride phases of the padded image become channels) -----
// dst[n][(c*s + a)*s + b][i][j] = in0[n][c][s*i + a - pad][s*j + b - pad]; one thread per four
// consecutive destination bytes (any alignment of rows; the flat tail is written byte-wise)
struct ImagePackArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, s, pad, C2, H2, W2;
    long long total;  // N * C2 * H2 * W2
    unsigned m_W2, m_H2, m_C2;
};

// Stride 2, fewer than 2^31 destination bytes: a destination dword is every second byte of an
// 8-byte source window -- two dword loads at any byte address and one byte permute -- unless
// the window touches the border, a row end or the tensor's tail (then byte by byte).
__global__ void __launch_bounds__(256) image_pack_s2_kernel(const ImagePackArgs a)
{
    const int ndw = (int)((a.total + 3) / 4);
    for (int t = blockIdx.x * 256 + threadIdx.x; t < ndw; t += gridDim.x * 256) {
        const int e0 = 4 * t;
        const int row = fast_div_any(e0, a.W2, a.m_W2), j0 = e0 - row * a.W2;
        const int nc = fast_div_any(row, a.H2, a.m_H2), i = row - nc * a.H2;
        const int n = fast_div_any(nc, a.C2, a.m_C2), c2 = nc - n * a.C2;
        const int b = c2 & 1, aa = (c2 >> 1) & 1, c = c2 >> 2;
        const int h = 2 * i + aa - a.pad, w0 = 2 * j0 + b - a.pad;
        if (j0 + 4 <= a.W2 && h >= 0 && h < a.H && w0 >= 0 && w0 + 8 <= a.W) {
            const int8_t *p = a.src + (((size_t)n * a.C + c) * a.H + h) * a.W + w0;
            unsigned lo, hi;
            __builtin_memcpy(&lo, p, 4);
            __builtin_memcpy(&hi, p + 4, 4);
            *reinterpret_cast<unsigned *>(a.dst + e0) = __builtin_amdgcn_perm(hi, lo, 0x06040200u);
            continue;
        }
        // general path for this dword: it may run over a row end into the next row / channel / image
        int j = j0, ii = i, cc2 = c2;
        long long nn = n;
        unsigned v = 0;
        int nb = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if ((long long)e0 + u < a.total) {
                const int bb = cc2 & 1, a2 = (cc2 >> 1) & 1, c1 = cc2 >> 2;
                const int hh = 2 * ii + a2 - a.pad, ww = 2 * j + bb - a.pad;
                int x = 0;
                if (hh >= 0 && hh < a.H && ww >= 0 && ww < a.W) x = a.src[((nn * a.C + c1) * a.H + hh) * a.W + ww];
                v |= (unsigned)(x & 0xFF) << (8 * u);
                ++nb;
                if (++j == a.W2) {
                    j = 0;
                    if (++ii == a.H2) {
                        ii = 0;
                        if (++cc2 == a.C2) {
                            cc2 = 0;
                            ++nn;
                        }
                    }
                }
            }
        }
        if (nb == 4) *reinterpret_cast<unsigned *>(a.dst + e0) = v;
        else
            for (int u = 0; u < nb; ++u) a.dst[e0 + u] = (int8_t)(v >> (8 * u));
    }
}

// Any stride: one thread per four consecutive destination bytes of the flat tensor.
__global__ void __launch_bounds__(256) image_pack_kernel(const ImagePackArgs a)
{
    const long long ndw = (a.total + 3) / 4;
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < ndw; t += (long long)gridDim.x * 256) {
        const long long e0 = 4 * t;
        int j = (int)(e0 % a.W2);
        long long rest = e0 / a.W2;
        int i = (int)(rest % a.H2);
        rest /= a.H2;
        int c2 = (int)(rest % a.C2);
        long long n = rest / a.C2;
        unsigned v = 0;
        int nb = 0;
        // the four loads first, from coordinates clamped into the tensor (no branch between them)
        int x[4];
        bool in[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int b = c2 % a.s, ca = c2 / a.s, aa = ca % a.s, c = ca / a.s;
            const int h = a.s * i + aa - a.pad, w = a.s * j + b - a.pad;
            const bool live = e0 + u < a.total;
            in[u] = live && h >= 0 && h < a.H && w >= 0 && w < a.W;
            const long long nn = live ? n : 0;
            x[u] = a.src[((nn * a.C + (live ? c : 0)) * a.H + min(max(h, 0), a.H - 1)) * a.W + min(max(w, 0), a.W - 1)];
            nb += live;
            if (++j == a.W2) {
                j = 0;
                if (++i == a.H2) {
                    i = 0;
                    if (++c2 == a.C2) {
                        c2 = 0;
                        ++n;
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) v |= (unsigned)((in[u] ? x[u] : 0) & 0xFF) << (8 * u);
        if (nb == 4) *reinterpret_cast<unsigned *>(a.dst + e0) = v;
        else
            for (int u = 0; u < nb; ++u) a.dst[e0 + u] = (int8_t)(v >> (8 * u));
    }
}

// dst[k][(c*s + a)*s + b][r][t] = src[k][c][s*r + a][s*t + b] inside the kernel, else 0; one thread per byte
__global__ void __launch_bounds__(256) image_pack_weights_kernel(const int8_t *src, int8_t *dst, int K, int C, int R,
                                                                 int S, int s, int R2, int S2)
{
    const long long total = (long long)K * C * s * s * R2 * S2;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const int t = (int)(e % S2);
        long long rest = e / S2;
        const int r = (int)(rest % R2);
        rest /= R2;
        const int b = (int)(rest % s);
        rest /= s;
        const int aa = (int)(rest % s);
        rest /= s;
        const int c = (int)(rest % C);
        const long long k = rest / C;
        const int rr = s * r + aa, ss = s * t + b;
        dst[e] = (rr < R && ss < S) ? src[((k * C + c) * R + rr) * S + ss] : (int8_t)0;
    }
}

hipError_t launch_image_pack(int N, int C, int H, int W, int stride, int pad, int H2, int W2,
                             const int8_t *src, int8_t *dst, hipStream_t st)
{
    ImagePackArgs a{src, dst, C, H, W, stride, pad, C * stride * stride, H2, W2, 0, 0u, 0u, 0u};
    a.total = (long long)N * a.C2 * H2 * W2;
    a.m_W2 = magic_for(W2);
    a.m_H2 = magic_for(H2);
    a.m_C2 = magic_for(a.C2);
    const hipError_t e = launch_phase_split(N, C, H, W, pad, stride, H2, W2, (long long)C * stride * stride,
                                            (long long)stride * stride, stride, 1, src, dst, st);
    if (e != hipErrorNotSupported) return e;
    if (stride == 2 && a.total < (1LL << 31) - 4)
        hipLaunchKernelGGL(image_pack_s2_kernel, dim3(grid_for((a.total + 3) / 4, 256)), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(image_pack_kernel, dim3(grid_for((a.total + 3) / 4, 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_image_pack_weights(int K, int C, int R, int S, int stride, const int8_t *src, int8_t *dst,
                                     hipStream_t st)
{
    const int R2 = (R + stride - 1) / stride, S2 = (S + stride - 1) / stride;
    const long long total = (long long)K * C * stride * stride * R2 * S2;
    hipLaunchKernelGGL(image_pack_weights_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, K, C, R, S,
                       stride, R2, S2);
    return hipGetLastError();
}

// ---- dilation as Image Pack into the batch (Sec. 6.1; Table 2 row 1, [N, I] => [N*s, I/s]) --------
// A stride-1 convolution with dilation d reads, for one output pixel, only padded-input pixels whose
// row and column agree with the output pixel's modulo d.  The d*d phases are therefore independent
// dense convolutions on sub-images, which go into the batch:
//   dst[(n*d + a)*d + b][c][i][j] = x0[n][c][d*i + a][d*j + b]       (x0: zero-padded, continued by zeros)
// and their results are interleaved back:
//   out[n][k][d*i + a][d*j + b] = src[(n*d + a)*d + b][k][i][j].
struct DilationArgs {
    const void *src;
    void *dst;
    int C, H, W, pad, d, H2, W2;   // pack: source image and sub-image extents
    int K, P, Q, P2, Q2;           // unpack: output and sub-result extents
    int chunks;                    // blocks per plane
    long long planes;
    unsigned m_chunks, m_C, m_dd, m_d, m_W2, m_K, m_Q;
};

// One block = 1024 consecutive bytes of one sub-image plane (n2, c); a thread makes four of them.
__global__ void __launch_bounds__(256) dilation_pack_kernel(const DilationArgs a, const int words)
{
    const int8_t *src = static_cast<const int8_t *>(a.src);
    int8_t *dst = static_cast<int8_t *>(a.dst);
    const int plane_sz = a.H2 * a.W2;
    const int nblocks = (int)(a.planes * a.chunks);   // the launcher keeps this below 2^31
    for (int bid = blockIdx.x; bid < nblocks; bid += gridDim.x) {
        const int plane = fast_div_any(bid, a.chunks, a.m_chunks), chunk = bid - plane * a.chunks;
        const int n2 = fast_div_any(plane, a.C, a.m_C), c = plane - n2 * a.C;
        const int dd = a.d * a.d;
        const int n = fast_div_any(n2, dd, a.m_dd), ab = n2 - n * dd;
        const int pa = fast_div_any(ab, a.d, a.m_d), pb = ab - pa * a.d;
        const int8_t *img = src + ((long long)n * a.C + c) * a.H * a.W;
        const int e0 = chunk * 1024 + 4 * (int)threadIdx.x;
        int i = fast_div_any(min(e0, plane_sz - 1), a.W2, a.m_W2), j = min(e0, plane_sz - 1) - i * a.W2;
        // the four loads first, from coordinates clamped into the image
        int x[4];
        bool in[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int h = a.d * i + pa - a.pad, w = a.d * j + pb - a.pad;
            in[u] = e0 + u < plane_sz && h >= 0 && h < a.H && w >= 0 && w < a.W;
            x[u] = img[min(max(h, 0), a.H - 1) * a.W + min(max(w, 0), a.W - 1)];
            if (++j == a.W2) {
                j = 0;
                ++i;
            }
        }
        unsigned v = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) v |= (unsigned)((in[u] ? x[u] : 0) & 0xFF) << (8 * u);
        int8_t *o = dst + (long long)plane * plane_sz + e0;
        if (words && e0 + 3 < plane_sz) *reinterpret_cast<unsigned *>(o) = v;
        else
            for (int u = 0; u < 4; ++u)
                if (e0 + u < plane_sz) o[u] = (int8_t)(v >> (8 * u));
    }
}

// One block = 1024 consecutive elements of one output plane (n, k); a thread moves four of them, 256 apart.
__global__ void __launch_bounds__(256) dilation_unpack_kernel(const DilationArgs a)
{
    const int32_t *src = static_cast<const int32_t *>(a.src);
    int32_t *dst = static_cast<int32_t *>(a.dst);
    const int plane_sz = a.P * a.Q;
    const long long sub_sz = (long long)a.P2 * a.Q2;
    const int nblocks = (int)(a.planes * a.chunks);   // the launcher keeps this below 2^31
    for (int bid = blockIdx.x; bid < nblocks; bid += gridDim.x) {
        const int plane = fast_div_any(bid, a.chunks, a.m_chunks), chunk = bid - plane * a.chunks;
        const long long n = fast_div_any(plane, a.K, a.m_K);
        const int k = plane - (int)n * a.K;
        int32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = min(chunk * 1024 + 256 * u + (int)threadIdx.x, plane_sz - 1);
            const int p = fast_div_any(e, a.Q, a.m_Q), q = e - p * a.Q;
            const int i = fast_div_any(p, a.d, a.m_d), pa = p - i * a.d;
            const int j = fast_div_any(q, a.d, a.m_d), pb = q - j * a.d;
            v[u] = src[(((n * a.d + pa) * a.d + pb) * a.K + k) * sub_sz + (long long)i * a.Q2 + j];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = chunk * 1024 + 256 * u + (int)threadIdx.x;
            if (e < plane_sz) __builtin_nontemporal_store(v[u], &dst[(long long)plane * plane_sz + e]);
        }
    }
}

hipError_t launch_dilation_pack(int N, int C, int H, int W, int pad, int d, int H2, int W2, const int8_t *src,
                                int8_t *dst, hipStream_t st)
{
    const hipError_t e = launch_phase_split(N, C, H, W, pad, d, H2, W2, (long long)d * d * C, 1, (long long)d * C, C,
                                            src, dst, st);
    if (e != hipErrorNotSupported) return e;
    DilationArgs a{};
    a.src = src;
    a.dst = dst;
    a.C = C, a.H = H, a.W = W, a.pad = pad, a.d = d, a.H2 = H2, a.W2 = W2;
    a.planes = (long long)N * d * d * C;
    a.chunks = (int)(((long long)H2 * W2 + 1023) / 1024);
    if (a.planes * a.chunks > 2147483647LL) return hipErrorInvalidValue;
    a.m_chunks = magic_for(a.chunks);
    a.m_C = magic_for(C);
    a.m_dd = magic_for(d * d);
    a.m_d = magic_for(d);
    a.m_W2 = magic_for(W2);
    // dword stores when every plane starts on a dword
    const int words = ((long long)H2 * W2) % 4 == 0 && (reinterpret_cast<uintptr_t>(dst) & 3) == 0;
    hipLaunchKernelGGL(dilation_pack_kernel, dim3(grid_for(a.planes * a.chunks * 256, 256)), dim3(256), 0, st, a, words);
    return hipGetLastError();
}

// Dilation 2: output row p = 2i + a takes its even columns from row i of sub-result (a, 0) and its odd columns from
// row i of sub-result (a, 1).  A thread loads four consecutive values of each (16 bytes, dword-aligned) and stores
// the eight interleaved values as two 16-byte pieces; consecutive lanes take consecutive groups of a row, then the
// next row, so both sides move in contiguous runs.  Rows shorter than a group, an odd last column, and the very end
// of the tensor go value by value.
struct Unpack2Args {
    const int32_t *src;
    int32_t *dst;
    int K, P, Q, P2, Q2, ngrp;
    long long items, src_elems;   // N*K * P * ngrp; elements of the sub-results
    unsigned m_ngrp, m_P, m_K;
};
__global__ void __launch_bounds__(256) dilation_unpack2_kernel(const Unpack2Args a)
{
    const long long it = (long long)blockIdx.x * 256 + threadIdx.x;
    if (it >= a.items) return;
    const int row = fast_div_any((int)it, a.ngrp, a.m_ngrp), g = (int)it - row * a.ngrp;   // (items < 2^31: the launcher checks)
    const int plane = fast_div_any(row, a.P, a.m_P), p = row - plane * a.P;
    const int n = fast_div_any(plane, a.K, a.m_K), k = plane - n * a.K;
    // (the last group of a row is moved back to end with the row: it overlaps its neighbour, both write the same values)
    const int i = p >> 1, pa = p & 1, j0 = a.Q2 >= 4 ? min(4 * g, a.Q2 - 4) : 0;
    const long long sub_sz = (long long)a.P2 * a.Q2;
    const long long s0 = (((long long)(n * 2 + pa) * 2 + 0) * a.K + k) * sub_sz + (long long)i * a.Q2 + j0;
    const long long s1 = s0 + (long long)a.K * sub_sz;
    int32_t *o = a.dst + ((long long)plane * a.P + p) * a.Q + 2 * j0;
    if (j0 + 4 <= a.Q2 && 2 * j0 + 8 <= a.Q && s1 + 4 <= a.src_elems) {
        const v4i e = *reinterpret_cast<const v4i_a4 *>(a.src + s0), f = *reinterpret_cast<const v4i_a4 *>(a.src + s1);
        __builtin_nontemporal_store(v4i{e[0], f[0], e[1], f[1]}, reinterpret_cast<v4i_a4 *>(o));
        __builtin_nontemporal_store(v4i{e[2], f[2], e[3], f[3]}, reinterpret_cast<v4i_a4 *>(o + 4));
    } else {   // (every wave has such lanes when rows are not whole groups: the eight loads first, then the stores)
        int32_t e[4], f[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ju = min(j0 + u, a.Q2 - 1) - j0;
            e[u] = a.src[s0 + ju];
            f[u] = a.src[s1 + ju];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (j0 + u < a.Q2 && 2 * (j0 + u) < a.Q) o[2 * u] = e[u];
            if (j0 + u < a.Q2 && 2 * (j0 + u) + 1 < a.Q) o[2 * u + 1] = f[u];
        }
    }
}

hipError_t launch_dilation_unpack(int N, int K, int P, int Q, int d, int P2, int Q2, const int32_t *src, int32_t *dst,
                                  hipStream_t st)
{
    if (d == 2 && (long long)N * K * P <= 2147483647LL && (long long)N * 2 <= 1073741823LL) {
        Unpack2Args b{};
        b.src = src, b.dst = dst;
        b.K = K, b.P = P, b.Q = Q, b.P2 = P2, b.Q2 = Q2;
        b.ngrp = (Q2 + 3) / 4;
        b.items = (long long)N * K * P * b.ngrp;
        b.src_elems = 4LL * N * K * P2 * Q2;
        b.m_ngrp = magic_for(b.ngrp), b.m_P = magic_for(P), b.m_K = magic_for(K);
        const long long blocks = (b.items + 255) / 256;
        if (b.items <= 2147483647LL) {
            hipLaunchKernelGGL(dilation_unpack2_kernel, dim3((unsigned)blocks), dim3(256), 0, st, b);
            return hipGetLastError();
        }
    }
    DilationArgs a{};
    a.src = src;
    a.dst = dst;
    a.d = d, a.K = K, a.P = P, a.Q = Q, a.P2 = P2, a.Q2 = Q2;
    a.planes = (long long)N * K;
    a.chunks = (int)(((long long)P * Q + 1023) / 1024);
    if (a.planes * a.chunks > 2147483647LL) return hipErrorInvalidValue;
    a.m_chunks = magic_for(a.chunks);
    a.m_K = magic_for(K);
    a.m_Q = magic_for(Q);
    a.m_d = magic_for(d);
    hipLaunchKernelGGL(dilation_unpack_kernel, dim3(grid_for(a.planes * a.chunks * 256, 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---- Image Pack through LDS: both forms of Table 2 row 1 (phases to channels, phases to batch) ------
// dst plane (n, c, a, b) [H2][W2]:  dst[i][j] = in0[n][c][s*i + a - pad][s*j + b - pad], zero outside the image;
// the plane's index is n*pn + c*pc + a*pa + b*pb, which is all that differs between the stride form
// ([N][(c*s + a)*s + b]) and the dilation form ([(n*s + a)*s + b][c]).
// A workgroup owns destination rows [i0, i0 + RI) of the s*s planes of one (n, c): that is the
// contiguous source rows s*i0 - pad .. of one image plane.  It loads them with dword loads at any byte
// address into a zero-padded LDS tile (row r, byte x = padded row s*i0 + r, padded column x), then every
// thread gathers destination dwords from the tile, four bytes s apart, and stores them: the strided
// access happens in LDS, both sides of HBM see whole lines.
struct PhaseSplitArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, pad, s, H2, W2;
    long long pn, pc, pa, pb;   // destination plane index = n*pn + c*pc + a*pa + b*pb
    long long src_bytes;        // N*C*H*W
    int RI, chunks, TPd;        // destination rows per workgroup, workgroups per plane, tile pitch in dwords
    int G, planes;              // whole (n, c) planes per workgroup (1 when a plane is cut into chunks), N*C
    int nblocks;
    unsigned m_chunks, m_C, m_TPd, m_W2, m_ndw, m_rows, m_ss, m_s;
};

__global__ void __launch_bounds__(256) phase_split_kernel(const PhaseSplitArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    constexpr int U = 4;   // 16-byte loads in flight per thread
    const int TP = 4 * a.TPd, TC = a.TPd / 4;   // tile pitch in bytes (a multiple of 16), 16-byte pieces per row
    for (int bid = blockIdx.x; bid < a.nblocks; bid += gridDim.x) {
        const int grp = fast_div_any(bid, a.chunks, a.m_chunks), chunk = bid - grp * a.chunks;
        const int pl0 = grp * a.G, np = min(a.G, a.planes - pl0);
        const int i0 = chunk * a.RI, ri = min(a.RI, a.H2 - i0);
        const int rows = a.s * ri;            // tile rows per plane
        // 1. source rows to the tile: plane gp of the group, tile row r, 16-byte piece t
        const int ntile = np * rows * TC;
        const unsigned m_rows = ri == a.RI ? a.m_rows : magic_for_device(rows);
        for (int base = 0; base < ntile; base += U * 256) {
            v4i v[U];
            int hh[U], w0[U];
            long long want[U];
            bool moved[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {   // the loads first, from addresses clamped into the tensor
                const int idx = min(base + 256 * u + tid, ntile - 1);
                const int row = fast_div(idx, a.m_TPd), t = idx - row * TC;   // tile-sized operands: exact
                const int gp = fast_div(row, m_rows), r = row - gp * rows;
                hh[u] = a.s * i0 + r - a.pad;
                w0[u] = 16 * t - a.pad;
                want[u] = ((long long)(pl0 + gp) * a.H + min(max(hh[u], 0), a.H - 1)) * a.W + w0[u];
                const long long at = min(max(want[u], 0LL), a.src_bytes - 16);
                moved[u] = at != want[u];
                __builtin_memcpy(&v[u], a.src + at, 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = base + 256 * u + tid;
                if (moved[u]) {   // the tensor's first or last bytes: byte by byte
                    asm volatile("" ::: "memory");   // stays a branch: only the first and last workgroup come here
                    unsigned x[4] = {0u, 0u, 0u, 0u}, b[16];
#pragma unroll
                    for (int k = 0; k < 16; ++k)   // sixteen independent loads, then the selection
                        b[k] = (unsigned char)a.src[min(max(want[u] + k, 0LL), a.src_bytes - 1)];
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const long long p = want[u] + k;
                        x[k >> 2] |= (p >= 0 && p < a.src_bytes ? b[k] : 0u) << (8 * (k & 3));
                    }
                    v[u] = v4i{(int)x[0], (int)x[1], (int)x[2], (int)x[3]};
                }
                // bytes [lo, hi) of the piece lie inside the image row
                const int lo = min(max(-w0[u], 0), 16), hi = min(max(a.W - w0[u], 0), 16);
                const bool rowok = hh[u] >= 0 && hh[u] < a.H;
                v4i x;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int l = min(max(lo - 4 * m, 0), 4), h = min(max(hi - 4 * m, 0), 4);
                    const unsigned keep = (rowok && h > l) ? (0xFFFFFFFFu >> ((32 - 8 * h) & 31)) & (0xFFFFFFFFu << ((8 * l) & 31)) : 0u;
                    x[m] = (int)((unsigned)v[u][m] & keep);
                }
                if (idx < ntile) *reinterpret_cast<v4i *>(smem + (size_t)idx * 16) = x;
            }
        }
        __syncthreads();
        // 2. destination.  The rows [i0, i0 + ri) of one phase's plane are `flat` consecutive bytes; a thread
        // makes sixteen of them, a 16-byte piece aligned in memory (a plane may start at any byte: the first
        // and the last piece of the range can be partial, and are then written in smaller units).
        const int flat = ri * a.W2, npc = (flat + 15) / 16 + 1, ss = a.s * a.s, nitems = np * ss * npc;
        const unsigned m_npc = ri == a.RI ? a.m_ndw : magic_for_device(npc);
        for (int item = tid; item < nitems; item += 256) {
            const int q = fast_div(item, m_npc), g = item - q * npc;   // tile-sized operands: exact
            const int gp = fast_div(q, a.m_ss), ph = q - gp * ss;
            const int pa = fast_div(ph, a.m_s), pb = ph - pa * a.s;
            const int pl = pl0 + gp, n = fast_div_any(pl, a.C, a.m_C), c = pl - n * a.C;
            int8_t *o = a.dst + ((long long)n * a.pn + (long long)c * a.pc + pa * a.pa + pb * a.pb) * ((long long)a.H2 * a.W2) +
                        (long long)i0 * a.W2;
            const int f0 = 16 * g - (int)(reinterpret_cast<uintptr_t>(o) & 15);
            if (f0 >= flat) continue;
            const int fs = max(f0, 0);
            int il = fast_div(fs, a.m_W2), j = fs - il * a.W2;
            const unsigned char *sub = smem + (gp * rows) * TP + pb;
            unsigned v[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int fm = f0 + 4 * m;
                if (fm >= 0 && fm + 3 < flat && j + 3 < a.W2) {   // a whole dword inside one row: bytes s apart
                    const unsigned char *b = sub + (a.s * il + pa) * TP + a.s * j;
                    v[m] = (unsigned)b[0] | (unsigned)b[a.s] << 8 | (unsigned)b[2 * a.s] << 16 | (unsigned)b[3 * a.s] << 24;
                    j += 4;
                    if (j == a.W2) {
                        j = 0;
                        ++il;
                    }
                } else {
                    v[m] = 0;
                    for (int k = 0; k < 4; ++k) {
                        if (fm + k < 0 || fm + k >= flat) continue;
                        v[m] |= (unsigned)sub[(a.s * il + pa) * TP + a.s * j] << (8 * k);
                        if (++j == a.W2) {
                            j = 0;
                            ++il;
                        }
                    }
                }
            }
            if (f0 >= 0 && f0 + 15 < flat) __builtin_nontemporal_store(v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]}, reinterpret_cast<v4i *>(o + f0));
            else
                for (int m = 0; m < 4; ++m) {
                    const int fm = f0 + 4 * m;
                    if (fm >= 0 && fm + 3 < flat) *reinterpret_cast<unsigned *>(o + fm) = v[m];
                    else
                        for (int k = 0; k < 4; ++k)
                            if (fm + k >= 0 && fm + k < flat) o[fm + k] = (int8_t)(v[m] >> (8 * k));
                }
        }
        __syncthreads();  // the tile is reused
    }
}

// Phases of two (stride or dilation 2) need no tile: within a padded source row the two column phases are
// the even and the odd bytes.  A thread takes 32 consecutive padded bytes of one row (two 16-byte loads at any
// byte address), zeroes the bytes outside the image, separates even from odd bytes with one byte permute per
// dword, and stores 16 bytes of each of the row's two phase planes; destination rows start at any byte, so
// these are 16-byte stores at any address.  A workgroup is [row parity][destination rows][pieces of a row],
// the piece index in the low lane bits and the destination rows running on across planes: a wave writes
// consecutive rows of one phase plane, one contiguous run per store instruction.  The last piece of a row is
// moved back to end with the row (it overlaps its neighbour, both write the same values) instead of being
// cut short; rows shorter than 16 bytes go out in 8/4/2/1-byte units.  Every byte of HBM is touched once.
struct PhaseSplit2Args {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, pad, H2, W2, planes;
    long long pn, pc, pa, pb;
    int npr, lp2;               // 16-byte destination pieces per row; log2 of the lanes a row takes (>= npr)
    int slots, both;            // destination rows per workgroup; 1: a workgroup holds both row parities of them
    int total;                  // planes * H2: destination rows of one phase, over all planes
    unsigned m_H2, m_C;
};

// The first nb bytes (1..15) of v to o, any address.
__device__ __forceinline__ void store_head(int8_t *o, v4i v, int nb)
{
    typedef int v2i_a1 __attribute__((ext_vector_type(2), aligned(1)));
    typedef int i_a1 __attribute__((aligned(1)));
    typedef short s_a1 __attribute__((aligned(1)));
    if (nb & 8) *reinterpret_cast<v2i_a1 *>(o) = v2i_a1{v[0], v[1]};
    const int d2 = (nb & 8) ? v[2] : v[0], d3 = (nb & 8) ? v[3] : v[1];
    o += nb & 8;
    if (nb & 4) *reinterpret_cast<i_a1 *>(o) = d2;
    const unsigned d = (unsigned)((nb & 4) ? d3 : d2);
    o += nb & 4;
    if (nb & 2) *reinterpret_cast<s_a1 *>(o) = (short)d;
    if (nb & 1) o[nb & 2] = (int8_t)(d >> (8 * (nb & 2)));
}

__global__ void __launch_bounds__(256) phase_split2_kernel(const PhaseSplit2Args a)
{
    const int tid = threadIdx.x;
    const int t = tid & ((1 << a.lp2) - 1), rl = tid >> a.lp2;   // piece of the row; row of the workgroup
    const int pa = a.both ? (rl >= a.slots) : (int)(blockIdx.x & 1);
    const int g = a.both ? (int)blockIdx.x * a.slots + (rl - pa * a.slots) : (int)(blockIdx.x >> 1);
    if (t >= a.npr || g >= a.total) return;
    const int pl = fast_div_any(g, a.H2, a.m_H2), il = g - pl * a.H2;
    const int n = fast_div_any(pl, a.C, a.m_C), c = pl - n * a.C;
    const int col0 = a.W2 >= 16 ? min(16 * t, a.W2 - 16) : 0;   // first destination column of the piece
    const int w0 = 2 * col0 - a.pad;                            // image column of the first of its 32 source bytes
    const int h = 2 * il + pa - a.pad;
    const long long bytes = (long long)a.planes * a.H * a.W;
    const long long want = ((long long)pl * a.H + min(max(h, 0), a.H - 1)) * a.W + w0;
    const long long o1 = min(max(want, 0LL), bytes - 16), o2 = min(max(want + 16, 0LL), bytes - 16);
    v4i lo4, hi4;
    __builtin_memcpy(&lo4, a.src + o1, 16);
    __builtin_memcpy(&hi4, a.src + o2, 16);
    if (o1 != want || o2 != want + 16) {   // the tensor's first or last bytes: byte by byte
        asm volatile("" ::: "memory");     // stays a branch: only the first and the last rows come here
        lo4 = o1 - want > -16 && o1 - want < 16 ? shift_piece(lo4, (int)(o1 - want)) : v4i{0, 0, 0, 0};
        hi4 = o2 - want - 16 > -16 && o2 - want - 16 < 16 ? shift_piece(hi4, (int)(o2 - want - 16)) : v4i{0, 0, 0, 0};
    }
    // bytes [lo, hi) of the 32 lie inside the image row (none of them when the row itself is padding)
    unsigned x[8];
    {
        const bool rowok = h >= 0 && h < a.H;
        const int lo = min(max(-w0, 0), 32), hi = rowok ? min(max(a.W - w0, 0), 32) : 0;
#pragma unroll
        for (int p = 0; p < 4; ++p) {   // eight bytes at a time
            const int l = min(max(lo - 8 * p, 0), 8), hh = min(max(hi - 8 * p, 0), 8);
            const unsigned long long ml = l == 8 ? 0ull : ~0ull << (8 * l), mh = hh == 0 ? 0ull : ~0ull >> (64 - 8 * hh);
            const unsigned k0 = (unsigned)(ml & mh), k1 = (unsigned)((ml & mh) >> 32);
            x[2 * p] = (unsigned)(p < 2 ? lo4[2 * p] : hi4[2 * p - 4]) & k0;
            x[2 * p + 1] = (unsigned)(p < 2 ? lo4[2 * p + 1] : hi4[2 * p - 3]) & k1;
        }
    }
    v4i even, odd;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        even[m] = (int)__builtin_amdgcn_perm(x[2 * m + 1], x[2 * m], 0x06040200u);
        odd[m] = (int)__builtin_amdgcn_perm(x[2 * m + 1], x[2 * m], 0x07050301u);
    }
    const long long plane_bytes = (long long)a.H2 * a.W2;
    int8_t *o_even = a.dst + ((long long)n * a.pn + (long long)c * a.pc + pa * a.pa) * plane_bytes + (long long)il * a.W2 + col0;
    int8_t *o_odd = o_even + a.pb * plane_bytes;
    const int nb = a.W2 - col0;   // bytes of the destination row from this piece on (16 or more, or the whole short row)
    if (nb >= 16) {
        *reinterpret_cast<v4i_a1 *>(o_even) = even;
        *reinterpret_cast<v4i_a1 *>(o_odd) = odd;
    } else {
        store_head(o_even, even, nb);
        store_head(o_odd, odd, nb);
    }
}

// Returns hipErrorNotSupported when a tile of one destination row does not fit LDS (the callers then
// use their element-wise kernels).
static hipError_t launch_phase_split(int N, int C, int H, int W, int pad, int s, int H2, int W2, long long pn, long long pc,
                                     long long pa, long long pb, const int8_t *src, int8_t *dst, hipStream_t st)
{
    if (s == 2 && (long long)N * C * H * W >= 32 && (long long)N * C * H2 <= 2147483647LL && W2 <= 16 * 256) {
        PhaseSplit2Args b{};
        b.src = src, b.dst = dst;
        b.C = C, b.H = H, b.W = W, b.pad = pad, b.H2 = H2, b.W2 = W2, b.planes = N * C;
        b.pn = pn, b.pc = pc, b.pa = pa, b.pb = pb;
        b.npr = (W2 + 15) / 16;
        while ((1 << b.lp2) < b.npr) ++b.lp2;
        b.total = N * C * H2;
        b.both = b.lp2 < 8;
        b.slots = b.both ? 128 >> b.lp2 : 1;
        const long long nblocks = b.both ? ((long long)b.total + b.slots - 1) / b.slots : 2LL * b.total;
        if (nblocks <= 2147483647LL) {   // (larger tensors take the tile kernel below)
            b.m_H2 = magic_for(H2), b.m_C = magic_for(C);
            hipLaunchKernelGGL(phase_split2_kernel, dim3((unsigned)nblocks), dim3(256), 0, st, b);
            return hipGetLastError();
        }
    }
    PhaseSplitArgs a{};
    a.src = src, a.dst = dst;
    a.C = C, a.H = H, a.W = W, a.pad = pad, a.s = s, a.H2 = H2, a.W2 = W2;
    a.pn = pn, a.pc = pc, a.pa = pa, a.pb = pb;
    a.src_bytes = (long long)N * C * H * W;
    if (a.src_bytes < 16 || (long long)N * C > 2147483647LL) return hipErrorNotSupported;
    a.planes = N * C;
    const long long pitch = ((long long)s * W2 + 15) / 16 * 16;
    const long long budget = 16 * 1024;    // per workgroup: eight of them share a compute unit
    long long ri = budget / (pitch * s);   // destination rows whose s*ri source rows fit the budget
    if (ri < 1) return hipErrorNotSupported;
    a.G = 1;
    if (ri >= H2) {
        ri = H2;
        long long g = budget / (pitch * s * H2);
        // enough workgroups to fill the chip come first
        while (g > 1 && (a.planes + g - 1) / g < 256 * 8) g /= 2;
        a.G = (int)(g < 1 ? 1 : g > 64 ? 64 : g);
    }
    a.RI = (int)ri;
    a.chunks = (H2 + a.RI - 1) / a.RI;
    a.TPd = (int)(pitch / 4);
    const long long nblocks = (long long)((a.planes + a.G - 1) / a.G) * a.chunks;
    if (nblocks > 2147483647LL) return hipErrorNotSupported;
    a.nblocks = (int)nblocks;
    a.m_chunks = magic_for(a.chunks);
    a.m_C = magic_for(C);
    a.m_TPd = magic_for(a.TPd / 4);   // 16-byte pieces per tile row
    a.m_W2 = magic_for(W2);
    a.m_ndw = magic_for(((long long)a.RI * W2 + 15) / 16 + 1);   // 16-byte pieces per phase and chunk
    a.m_rows = magic_for((long long)s * a.RI);
    a.m_ss = magic_for((long long)s * s);
    a.m_s = magic_for(s);
    const size_t lds = (size_t)a.G * s * a.RI * pitch;
    const int grid = a.nblocks < 256 * 16 ? a.nblocks : 256 * 16;
    hipLaunchKernelGGL(phase_split_kernel, dim3(grid), dim3(256), lds, st, a);
    return hipGetLastError();
}

// ---- zero fill (a kernel, not a memset node, so that callers may capture it) --------------
__global__ void __launch_bounds__(256) fill_zero_kernel(v4i *dst, long long n16, int8_t *tail, int ntail)
{
    const v4i z = {0, 0, 0, 0};
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < n16;
         t += (long long)gridDim.x * blockDim.x)
        dst[t] = z;
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t st)
{
    // dst is 16-byte aligned for every buffer the library clears (hipMalloc'd int32 tensors).
    const long long n16 = (long long)(bytes / 16);
    const int ntail = (int)(bytes % 16);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(n16, 256)), dim3(256), 0, st,
                       reinterpret_cast<v4i *>(dst), n16, reinterpret_cast<int8_t *>(dst) + n16 * 16, ntail);
    return hipGetLastError();
}

}  // namespace c2i8
