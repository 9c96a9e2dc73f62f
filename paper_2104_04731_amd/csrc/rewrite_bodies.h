// Device bodies of the layout rewrites that more than one kernel uses (the stand-alone
// rewrite kernels, the two-rewrites-in-one-launch kernel, and the whole-convolution kernel),
// with the host helpers that fill their argument blocks.
#pragma once
#include "act_requant.h"
#include "kernels.h"

namespace c2i8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));  // 16 bytes at a dword-aligned address
typedef int v4i_a1 __attribute__((ext_vector_type(4), aligned(1)));  // 16 bytes at any address
// A 16-byte piece wanted from byte offset `want` of a tensor was fetched from `at` instead (`want` clamped into the
// tensor, |at - want| < 16): move the bytes to where they belong, zeros coming in -- the bytes that were outside the
// tensor.  Registers only: the workgroup that holds a tensor's first bytes sets the kernel's time at small sizes,
// and a second memory round trip there showed in it.
__device__ __forceinline__ v4i shift_piece(v4i v, int at_minus_want)
{
    unsigned __int128 x;
    __builtin_memcpy(&x, &v, 16);
    x = at_minus_want > 0 ? x << (8 * at_minus_want) : x >> (8 * -at_minus_want);
    __builtin_memcpy(&v, &x, 16);
    return v;
}

// Workgroups are dealt round-robin over the 8 XCDs (each with its own L2).  Mapping the
// hardware id to a logical id that is contiguous per XCD makes neighbouring tiles -- which
// share source cache lines (pack) or whole source rows (im2col) -- run behind the same L2.
__device__ __forceinline__ int xcd_contiguous(int id, int n)
{
    const int x = id & 7, q = n >> 3, rem = n & 7;
    return x * q + (x < rem ? x : rem) + (id >> 3);
}

__device__ __forceinline__ unsigned pack4(int b0, int b1, int b2, int b3)
{
    return (unsigned)(b0 & 0xFF) | ((unsigned)(b1 & 0xFF) << 8) | ((unsigned)(b2 & 0xFF) << 16) |
           ((unsigned)(b3 & 0xFF) << 24);
}

// n / d for magic = ceil(2^32 / d) truncated to 32 bits (0 encodes d == 1); exact while
// n * d < 2^32
__device__ __forceinline__ int fast_div(int n, unsigned magic)
{
    return magic ? (int)__umulhi((unsigned)n, magic) : n;
}
// The same for any 0 <= n < 2^31: the estimate is never low and at most one too high.
__device__ __forceinline__ int fast_div_any(int n, int d, unsigned magic)
{
    int q = fast_div(n, magic);
    if ((long long)q * d > n) --q;
    return q;
}
// Four consecutive output channels k .. k+3 of pixel (n, p, q) -- what one lane holds in v%4 of an MFMA
// result block -- activated and stored as one dword of the blocked tensor (bytes past channel K-1 are not written).
__device__ __forceinline__ void act_store4(const ActOut &e, int n, int p, int q, int k, int K, int x0, int x1, int x2, int x3)
{
    if (k >= K) return;
    const size_t pix = ((size_t)n * e.Cb + (k >> e.cb_log2)) * e.Hp * e.Wp + (size_t)(p + e.pad) * e.Wp + (q + e.pad);
    int8_t *dst = e.out + (pix << e.cb_log2) + (k & ((1 << e.cb_log2) - 1));
    const int y[4] = {act_requant(x0, e.shift, e.relu), act_requant(x1, e.shift, e.relu), act_requant(x2, e.shift, e.relu),
                      act_requant(x3, e.shift, e.relu)};
    if (k + 3 < K) *reinterpret_cast<unsigned *>(dst) = pack4(y[0], y[1], y[2], y[3]);
    else
        for (int t = 0; t < 4; ++t)
            if (k + t < K) dst[t] = (int8_t)y[t];
}

__device__ __forceinline__ unsigned magic_for_device(int d)  // the same constant, made on the device
{
    return d == 1 ? 0u : (unsigned)(0xFFFFFFFFu / (unsigned)d) + 1u;
}
static inline unsigned magic_for(long long d) { return (unsigned)((0x100000000ULL + (unsigned long long)d - 1) / (unsigned long long)d); }

// Wave-tiled version for 64-channel slices (cb % 64 == 0).  The unit of work is one wave and
// 64 consecutive DESTINATION pixels (records of 64 channels) of one padded plane slice: 4 KB out, written as
// four store instructions of 1 KB each -- whole lines, the zero border included, nothing left for a second
// store to complete.  No workgroup barrier anywhere: the four waves of a workgroup only share a launch.
//   source: the interior records of a unit are consecutive source pixels (image rows follow each other in
//        memory and the border exists in the destination only): at most 64 bytes of every channel plane from
//        the unit's first interior pixel on;
//   in:  lane = (16-byte piece of that run, channel l/4 + 16k): four loads per lane at any byte address, each
//        wave instruction covering the runs of 16 channels;
//   LDS: a private [64 channels][17 dwords] tile per wave (odd pitch: the row-wise writes and the column-wise
//        reads below are conflict-free);
//   out: lane = (16-channel group g = l%4, record l/4 + 16u): where the record is a border pixel, zeros; else
//        it reads the dword holding its source pixel from each of its 16 channel rows and picks that pixel's
//        byte out of each (three byte operations per destination dword); the four lanes of a record write its
//        64 bytes side by side, sixteen records per instruction one after the other in memory.
// (The form in source order below lets the lane that writes a row's last pixel zero the border behind it: its
// stores are runs broken at every image row plus a few-lane store for each border, which costs 15 % of the time once
// the chip is full.)
struct PackWaveArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, cb, pad, Hp, Wp, Cb, slices, chunks;  // chunks = ceil(Hp*Wp / 64)
    long long waves;
    unsigned m_Wp, m_chunks, m_slices, m_Cb;
};
constexpr int PW_PITCH = 17;                      // dwords per channel row
constexpr int PW_LDS = 64 * PW_PITCH * 4;         // bytes per wave

__device__ __forceinline__ void pack_layout_wave_body(const PackWaveArgs &a, long long wid, unsigned *tile)
{
    const int C = a.C, H = a.H, W = a.W, cb = a.cb, pad = a.pad, Wp = a.Wp;
    const int HW = H * W, HpWp = a.Hp * Wp;
    const int lane = threadIdx.x & 63;
    // wid = ((n*Cb + b)*slices + sl)*chunks + chunk
    const int id = (int)wid;
    const int q1 = fast_div_any(id, a.chunks, a.m_chunks), chunk = id - q1 * a.chunks;
    const int q2 = fast_div_any(q1, a.slices, a.m_slices), sl = q1 - q2 * a.slices;
    const int q3 = fast_div_any(q2, a.Cb, a.m_Cb), b = q2 - q3 * a.Cb;
    const long long n = q3;
    const int c0 = b * cb + sl * 64;
    const int T0 = chunk * 64, nrec = min(64, HpWp - T0);   // this unit's records [T0, T0 + nrec)
    int8_t *out0 = a.dst + ((n * a.Cb + b) * (long long)HpWp) * cb + sl * 64;

    // the first interior record at or after T0 (wave-uniform) and its source pixel
    int ha = fast_div_any(T0, Wp, a.m_Wp), wa = T0 - ha * Wp;
    if (ha < pad) ha = pad, wa = pad;
    else if (wa < pad) wa = pad;
    else if (wa >= pad + W) ++ha, wa = pad;
    const bool any = ha < pad + H && ha * Wp + wa < T0 + nrec;
    const int src_lo = any ? (ha - pad) * W + (wa - pad) : 0;

    if (any) {
        const int8_t *plane0 = a.src + (n * C + c0) * (long long)HW + src_lo;
        const int p = lane & 3, chq = lane >> 2;
        v4i v[4];
        // The loads of a lane are issued back to back, none under a per-lane condition (a load under a
        // condition makes the compiler wait for it before the next one): channels past C are read from a
        // clamped channel and zeroed after; in the unit that holds a plane's last pixels a piece that would run
        // past the plane is fetched lower and moved down in registers.
        if (src_lo + 64 <= HW) {   // uniform
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ch = min(chq + 16 * k, C - 1 - c0);
                v[k] = *reinterpret_cast<const v4i_a1 *>(plane0 + (long long)ch * HW + 16 * p);
            }
        } else {
            const int left = HW - src_lo;                    // bytes of the plane from src_lo on (1..63)
            const int at = max(min(16 * p, left - 16), -src_lo);   // (a plane holds at least 16 bytes: the launcher checks)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ch = min(chq + 16 * k, C - 1 - c0);
                const v4i x = *reinterpret_cast<const v4i_a1 *>(plane0 + (long long)ch * HW + at);
                v[k] = 16 * p - at < 16 ? shift_piece(x, at - 16 * p) : v4i{0, 0, 0, 0};   // (a piece wholly past the plane is not used)
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (c0 + chq + 16 * k >= C) v[k] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            unsigned *row = tile + (chq + 16 * k) * PW_PITCH + 4 * p;
#pragma unroll
            for (int e = 0; e < 4; ++e) row[e] = (unsigned)v[k][e];
        }
    }
    // same wave on both sides: the LDS executes a wave's accesses in order
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();

    const int g = lane & 3;
    const unsigned *rows = tile + (g * 16) * PW_PITCH;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int rec = (lane >> 2) + 16 * u, t = T0 + rec;
        const int hp = fast_div_any(t, Wp, a.m_Wp), wp = t - hp * Wp;
        const bool inside = any && hp >= pad && hp < pad + H && wp >= pad && wp < pad + W;
        const int li = inside ? (hp - pad) * W + (wp - pad) - src_lo : 0;   // 0 .. 63
        const unsigned sel = 0x0C0C0400u + (unsigned)(li & 3) * 0x0101u;    // byte li%4 of two dwords, into the low half
        const unsigned *col = rows + (li >> 2);
        unsigned d[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) d[c] = col[c * PW_PITCH];
        v4i o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned lo = __builtin_amdgcn_perm(d[4 * q + 1], d[4 * q], sel), hi = __builtin_amdgcn_perm(d[4 * q + 3], d[4 * q + 2], sel);
            o[q] = inside ? (int)(lo | (hi << 16)) : 0;
        }
        if (rec < nrec) __builtin_nontemporal_store(o, reinterpret_cast<v4i *>(out0 + (long long)t * cb + g * 16));
    }
}

// Fills `a` and the workgroup count if the wave-tiled kernel can run this problem.
static inline bool plan_pack_wave(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst,
                           PackWaveArgs *a, long long *blocks)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad, Cb = (C + cb - 1) / cb;
    const long long hw = (long long)H * W;
    if (!(cb % 64 == 0 && hw >= 16 && hw < (1LL << 30) && (long long)Hp * Wp < (1LL << 30))) return false;
    const int slices = cb / 64;
    const long long chunks = ((long long)Hp * Wp + 63) / 64;
    const long long waves = (long long)N * Cb * slices * chunks;
    if (waves >= (1LL << 31)) return false;
    *blocks = (waves + 3) / 4;
    *a = PackWaveArgs{src, dst, C, H, W, cb, pad, Hp, Wp, Cb, slices, (int)chunks, waves,
                      magic_for(Wp), magic_for(chunks), magic_for(slices), magic_for(Cb)};
    return true;
}

// The same in SOURCE order, for problems too small to fill the chip (there the time is the length of a wave's
// dependent chain, and this form has one round of LDS reads where the destination-ordered form has four).
// The unit of work is one wave:
// 64 consecutive SOURCE pixels of the 64 channel planes of a slice (4 KB in, 4 KB out), with
// no workgroup barrier anywhere -- the four waves of a workgroup only share a launch.
//   in:  lane = (16-byte piece of the 64-byte run, channel l/4 + 16k): four loads per lane,
//        each wave instruction covering whole 64-byte runs of 16 channels;
//   LDS: a private [64 channels][17 dwords] tile per wave (odd pitch: the row-wise writes
//        and the column-wise reads below are conflict-free);
//   out: lane = (16-channel group g = l%4, dword column l/4): the dwords of four consecutive
//        pixels from 16 channels, transposed with byte permutes into the four pixels' 16
//        channel-contiguous bytes; the four lanes of a pixel write its 64 bytes side by side;
//   border: the lane that writes the last pixel of an image row also zeroes the 2*pad border
//        pixels that follow it in the padded order (right border + next row's left border);
//        the waves holding the first and the last pixel of a plane zero the top and bottom rows.
// Working in source order means there is no mapping from padded index back to the image.
struct PackSrcArgs {
    const int8_t *src;
    int8_t *dst;
    int C, H, W, cb, pad, Hp, Wp, Cb, slices, chunks;  // chunks = ceil(H*W / 64)
    long long waves;
    unsigned m_W, m_chunks, m_slices, m_Cb;
};

__device__ __forceinline__ void pack_layout_src_body(const PackSrcArgs &a, long long wid, unsigned *tile)
{
    const int C = a.C, H = a.H, W = a.W, cb = a.cb, pad = a.pad, Wp = a.Wp;
    const int HW = H * W, HpWp = a.Hp * Wp;
    const int lane = threadIdx.x & 63;
    // wid = ((n*Cb + b)*slices + sl)*chunks + chunk
    const int id = (int)wid;
    const int q1 = fast_div_any(id, a.chunks, a.m_chunks), chunk = id - q1 * a.chunks;
    const int q2 = fast_div_any(q1, a.slices, a.m_slices), sl = q1 - q2 * a.slices;
    const int q3 = fast_div_any(q2, a.Cb, a.m_Cb), b = q2 - q3 * a.Cb;
    const long long n = q3;
    const int c0 = b * cb + sl * 64;
    const int s0 = chunk * 64;  // first source pixel
    const int8_t *plane0 = a.src + (n * C + c0) * (long long)HW + s0;
    int8_t *out0 = a.dst + ((n * a.Cb + b) * (long long)HpWp) * cb + sl * 64;

    {
        const int p = lane & 3, chq = lane >> 2;
        const bool whole = s0 + 64 <= HW;  // uniform
        v4i v[4];
        // The loads of a lane are issued back to back, none under a per-lane condition (a load under a
        // condition makes the compiler wait for it before the next one): channels past C and, in the
        // last chunk of a plane, dwords past the plane are read from a clamped address and zeroed after.
        if (whole) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ch = min(chq + 16 * k, C - 1 - c0);
                v[k] = *reinterpret_cast<const v4i_a4 *>(plane0 + (long long)ch * HW + 16 * p);
            }
        } else {
            const int last = HW - s0 - 4;   // >= 0: a chunk holds at least one dword of the plane
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ch = min(chq + 16 * k, C - 1 - c0);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[k][e] = *reinterpret_cast<const int *>(plane0 + (long long)ch * HW + min(16 * p + 4 * e, last));
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (16 * p + 4 * e > last) v[k][e] = 0;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (c0 + chq + 16 * k >= C) v[k] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            unsigned *row = tile + (chq + 16 * k) * PW_PITCH + 4 * p;
#pragma unroll
            for (int e = 0; e < 4; ++e) row[e] = (unsigned)v[k][e];
        }
    }
    // same wave on both sides: the LDS executes a wave's accesses in order
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();

    const v4i zero = {0, 0, 0, 0};
    {
        const int g = lane & 3, cq = lane >> 2;
        const unsigned *col = tile + (g * 16) * PW_PITCH + cq;
        unsigned d[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) d[c] = col[c * PW_PITCH];
        // o[j][q] = byte j of d[4q .. 4q+3]: pixel j, channels 4q .. 4q+3
        v4i o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned t0 = __builtin_amdgcn_perm(d[4 * q + 1], d[4 * q], 0x05010400u);
            const unsigned t1 = __builtin_amdgcn_perm(d[4 * q + 1], d[4 * q], 0x07030602u);
            const unsigned t2 = __builtin_amdgcn_perm(d[4 * q + 3], d[4 * q + 2], 0x05010400u);
            const unsigned t3 = __builtin_amdgcn_perm(d[4 * q + 3], d[4 * q + 2], 0x07030602u);
            o[0][q] = (int)__builtin_amdgcn_perm(t2, t0, 0x05040100u);
            o[1][q] = (int)__builtin_amdgcn_perm(t2, t0, 0x07060302u);
            o[2][q] = (int)__builtin_amdgcn_perm(t3, t1, 0x05040100u);
            o[3][q] = (int)__builtin_amdgcn_perm(t3, t1, 0x07060302u);
        }
        const int i = s0 + 4 * cq;
        const int h = fast_div(i, a.m_W), w = i - h * W;
        int8_t *row_end = nullptr;  // W >= 4: at most one of the four pixels ends an image row
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i + j < HW) {
                int wj = w + j, hj = h;
                if (wj >= W) {
                    wj -= W;
                    ++hj;
                }
                int8_t *dp = out0 + ((long long)(hj + pad) * Wp + wj + pad) * cb + g * 16;
                *reinterpret_cast<v4i *>(dp) = o[j];
                if (wj == W - 1 && hj < H - 1) row_end = dp;
            }
        }
        if (row_end)  // the border pixels up to the next image row
            for (int z = 1; z <= 2 * pad; ++z) *reinterpret_cast<v4i *>(row_end + (long long)z * cb) = zero;
    }
    if (pad > 0) {
        // border rows above the first and below the last pixel of the plane: four lanes per pixel
        const int top = pad * Wp + pad, bottom0 = (pad + H - 1) * Wp + pad + W;
        if (chunk == 0)
            for (int idx = lane; idx < top * 4; idx += 64)
                *reinterpret_cast<v4i *>(out0 + (long long)(idx >> 2) * cb + (idx & 3) * 16) = zero;
        if (chunk == a.chunks - 1)
            for (int idx = lane; idx < (HpWp - bottom0) * 4; idx += 64)
                *reinterpret_cast<v4i *>(out0 + (long long)(bottom0 + (idx >> 2)) * cb + (idx & 3) * 16) = zero;
    }
}

// Fills `a` and the workgroup count if the wave-tiled kernel can run this problem.
static inline bool plan_pack_src(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst,
                           PackSrcArgs *a, long long *blocks)
{
    const int Hp = H + 2 * pad, Wp = W + 2 * pad, Cb = (C + cb - 1) / cb;
    const long long hw = (long long)H * W;
    if (!(cb % 64 == 0 && hw % 4 == 0 && (reinterpret_cast<uintptr_t>(src) & 3) == 0 && W >= 4 &&
          hw * W < (1LL << 32) && (long long)Hp * Wp < (1LL << 30)))  // multiply-high split by W stays exact
        return false;
    const int slices = cb / 64;
    const long long chunks = (hw + 63) / 64;
    const long long waves = (long long)N * Cb * slices * chunks;
    if (waves >= (1LL << 31)) return false;
    *blocks = (waves + 3) / 4;
    *a = PackSrcArgs{src, dst, C, H, W, cb, pad, Hp, Wp, Cb, slices, (int)chunks, waves,
                      magic_for(W), magic_for(chunks), magic_for(slices), magic_for(Cb)};
    return true;
}

// ---- pack_weights -----------------------------------------------------------------------
// Blocked: dst[k][((b*R + r)*S + s)*cb + ci] = src[k][b*cb+ci][r][s]; one thread per 16 B.
struct WeightArgs {
    const int8_t *src;
    int8_t *dst;
    int K, C, R, S, cb, depth, nreal;  // cb == 0: row-padded copy (depth order of KCRS itself)
    unsigned m_chunks, m_g16, m_RS;    // ceil(2^32 / d) for depth/16, cb/16, R*S
};

// One thread per 16 destination bytes, `nthreads` threads per (virtual) workgroup; K*depth/16 < 2^31.
__device__ __forceinline__ void pack_weights_blocked_body(const WeightArgs &a, int vbid, int vgrid, int nthreads)
{
    const int8_t *__restrict__ src = a.src;
    int8_t *__restrict__ dst = a.dst;
    const int K = a.K, C = a.C, cb = a.cb, depth = a.depth, nreal = a.nreal;
    const int chunks = depth / 16;
    const int total = K * chunks;
    const int g16 = cb / 16, RS = a.R * a.S;
    for (int t = vbid * nthreads + (int)threadIdx.x; t < total; t += vgrid * nthreads) {
        const int k = fast_div_any(t, chunks, a.m_chunks), ch = t - k * chunks;
        // sixteen loads issued back to back, none under a condition: a piece past the real depth and the
        // channels past C read a clamped address and are zeroed afterwards
        int v[16];
        const int chr = min(ch, nreal - 1);
        const int tap = fast_div_any(chr, g16, a.m_g16), sub = chr - tap * g16;
        const int b = fast_div_any(tap, RS, a.m_RS), rs = tap - b * RS;
        const int c0 = b * cb + sub * 16;
        const int8_t *s = src + (long long)k * C * RS + rs;
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = s[(long long)min(c0 + i, C - 1) * RS];
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (ch >= nreal || c0 + i >= C) v[i] = 0;
        v4i o;
        o[0] = pack4(v[0], v[1], v[2], v[3]);
        o[1] = pack4(v[4], v[5], v[6], v[7]);
        o[2] = pack4(v[8], v[9], v[10], v[11]);
        o[3] = pack4(v[12], v[13], v[14], v[15]);
        *reinterpret_cast<v4i *>(dst + (long long)k * depth + (long long)ch * 16) = o;
    }
}

static inline WeightArgs weight_args_blocked(int K, int C, int R, int S, int cb, int depth,
                                             const int8_t *src, int8_t *dst)
{
    const int Cb = (C + cb - 1) / cb;
    return WeightArgs{src, dst, K, C, R, S, cb, depth, Cb * R * S * (cb / 16),
                      magic_for(depth / 16), magic_for(cb / 16), magic_for((long long)R * S)};
}

}  // namespace c2i8
