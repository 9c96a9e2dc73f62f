// Layout rewrites of Table 2 as bandwidth-bound copy kernels: every destination byte
// (zero padding included) is written exactly once, in 16-byte pieces, and source reads run
// along the contiguous W axis across the lanes of a wave.
#include "kernels.h"

namespace c2i8 {

typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned pack4(int b0, int b1, int b2, int b3)
{
    return (unsigned)(b0 & 0xFF) | ((unsigned)(b1 & 0xFF) << 8) | ((unsigned)(b2 & 0xFF) << 16) |
           ((unsigned)(b3 & 0xFF) << 24);
}

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

static int grid_for(long long work_items, int block)
{
    long long g = (work_items + block - 1) / block;
    const long long cap = 256LL * 32;  // 32 workgroups per CU keeps every CU busy
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (int)g;
}

hipError_t launch_pack_layout(int N, int C, int H, int W, int cb, int pad,
                              const int8_t *src, int8_t *dst, hipStream_t st)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad, Cb = (C + cb - 1) / cb;
    const long long pixels = (long long)N * Cb * Hp * Wp;
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
// Blocked: dst[k][((b*R + r)*S + s)*cb + ci] = src[k][b*cb+ci][r][s]; one thread per 16 B.
__global__ void __launch_bounds__(256)
pack_weights_blocked_kernel(const int8_t *__restrict__ src, int8_t *__restrict__ dst,
                            int K, int C, int R, int S, int cb, int depth, int nreal)
{
    const int chunks = depth / 16;
    const long long total = (long long)K * chunks;
    const int g16 = cb / 16, RS = R * S;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long long)gridDim.x * blockDim.x) {
        const int ch = (int)(t % chunks);
        const long long k = t / chunks;
        int v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = 0;
        if (ch < nreal) {
            const int sub = ch % g16, tap = ch / g16;
            const int rs = tap % RS, b = tap / RS;
            const int c0 = b * cb + sub * 16;
            const int8_t *s = src + (k * C + c0) * RS + rs;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (c0 + i < C) v[i] = s[i * RS];
        }
        v4i o;
        o[0] = pack4(v[0], v[1], v[2], v[3]);
        o[1] = pack4(v[4], v[5], v[6], v[7]);
        o[2] = pack4(v[8], v[9], v[10], v[11]);
        o[3] = pack4(v[12], v[13], v[14], v[15]);
        *reinterpret_cast<v4i *>(dst + k * depth + (long long)ch * 16) = o;
    }
}

hipError_t launch_pack_weights_blocked(int K, int C, int R, int S, int cb, int depth,
                                       const int8_t *src, int8_t *dst, hipStream_t st)
{
    const int Cb = (C + cb - 1) / cb;
    const int nreal = Cb * R * S * (cb / 16);
    const long long items = (long long)K * (depth / 16);
    hipLaunchKernelGGL(pack_weights_blocked_kernel, dim3(grid_for(items, 256)), dim3(256), 0, st,
                       src, dst, K, C, R, S, cb, depth, nreal);
    return hipGetLastError();
}

// Row-padded copy: dst[k][j] = j < CRS ? src[k][j] : 0 (the (c,r,s) order is KCRS itself).
__global__ void __launch_bounds__(256)
pack_weights_rows_kernel(const int8_t *__restrict__ src, int8_t *__restrict__ dst,
                         int K, int CRS, int depth)
{
    const int chunks = depth / 16;
    const long long total = (long long)K * chunks;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long long)gridDim.x * blockDim.x) {
        const int ch = (int)(t % chunks);
        const long long k = t / chunks;
        const int8_t *s = src + k * CRS + ch * 16;
        int v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = (ch * 16 + i < CRS) ? s[i] : 0;
        v4i o;
        o[0] = pack4(v[0], v[1], v[2], v[3]);
        o[1] = pack4(v[4], v[5], v[6], v[7]);
        o[2] = pack4(v[8], v[9], v[10], v[11]);
        o[3] = pack4(v[12], v[13], v[14], v[15]);
        *reinterpret_cast<v4i *>(dst + k * depth + (long long)ch * 16) = o;
    }
}

hipError_t launch_pack_weights_rows(int K, int CRS, int depth, const int8_t *src, int8_t *dst,
                                    hipStream_t st)
{
    const long long items = (long long)K * (depth / 16);
    hipLaunchKernelGGL(pack_weights_rows_kernel, dim3(grid_for(items, 256)), dim3(256), 0, st,
                       src, dst, K, CRS, depth);
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
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int h = h0 + r, w = w0 + s;
            int x = 0;
            if (j + i < kg && h >= 0 && h < H && w >= 0 && w < W)
                x = img[((long long)c * H + h) * W + w];
            v[i] = x;
            if (++s == S) {
                s = 0;
                if (++r == R) {
                    r = 0;
                    ++c;
                }
            }
        }
        v4i o;
        o[0] = pack4(v[0], v[1], v[2], v[3]);
        o[1] = pack4(v[4], v[5], v[6], v[7]);
        o[2] = pack4(v[8], v[9], v[10], v[11]);
        o[3] = pack4(v[12], v[13], v[14], v[15]);
        *reinterpret_cast<v4i *>(dst + m * kg_pad + (long long)ch * 16) = o;
    }
}

hipError_t launch_im2col(int N, int C, int H, int W, int R, int S, int stride, int pad,
                         int P, int Q, int kg_pad, const int8_t *src, int8_t *dst, hipStream_t st)
{
    const long long M = (long long)N * P * Q;
    const long long items = M * (kg_pad / 16);
    hipLaunchKernelGGL(im2col_kernel, dim3(grid_for(items, 256)), dim3(256), 0, st,
                       src, dst, C, H, W, R, S, stride, pad, P, Q, C * R * S, kg_pad, M);
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
