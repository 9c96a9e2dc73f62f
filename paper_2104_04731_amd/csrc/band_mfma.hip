// GEMM stage for small many-channel layers: the reduction depth is split over the waves of a
// workgroup, and the activations a workgroup needs stay resident in LDS.
//
// The general GEMM stage (igemm_mfma.hip) streams a TK x 64 B weight tile and a TM x 64 B
// activation tile per depth step through LDS.  On a layer like 8 x 256 x 14 x 14 -> 512, 3 x 3
// that is 288 KB per 64 x 64 tile for 0.6 us of multiplying, nine tenths of it the same pixels
// fetched once per kernel tap.  Here (channel blocks of 64 only) one workgroup owns a band of
// PT output rows of one image x 32 output channels:
//   * window: the (PT-1)*stride + (R-1)*dil + 1 rows of the zero-padded blocked image the band
//     touches, all channel blocks, copied into LDS ONCE (global_load_lds_dwordx4, whole rows:
//     a contiguous range of the blocked tensor).  A kernel tap is an address offset into it --
//     the weight/data-buffer residency argument of Sec. 6.1 applied to LDS;
//   * depth split: wave w multiplies depth steps [w*kpw, (w+1)*kpw) (a step = 64 channels of
//     one tap) for ALL the band's pixels.  Its weights -- 32 rows x 64 B per step -- are fetched by
//     that wave alone into its own LDS region and read from there exactly once, so no wave waits
//     for another in the main loop: one barrier after the window has landed, one before the
//     partial sums are added up;
//   * v_mfma_i32_16x16x64_i8: D[channel][pixel] += W[channel][64] . X[pixel][64], 16 pixels per
//     block, so a 14-pixel image row wastes 2 columns, not 18.  A weight fragment (16 rows) is
//     used for every pixel block, an activation fragment for both row blocks;
//   * shifted fragments (stride 1, three taps per kernel row): a pixel block is 16 consecutive INPUT
//     columns of one window row, holding 14 output columns.  Tap s of a kernel row needs, for output column q,
//     input column q + s: the fragment of tap 0 moved s lanes within its 16-lane rows (DPP row shift, a
//     register move).  LDS then serves one activation fragment per six MFMAs instead of per two;
//   * the four waves' partial sums meet in LDS (each wave's region is its spent weight region);
//     wave w adds up and stores every fourth 16 x 16 block, straight to NKPQ.
// Both LDS operands are XOR-swizzled per 64-byte row ((row/4)%4 on the 16-byte chunk index), done
// by the lanes' choice of source chunk, so the column-wise fragment reads spread over all banks.
#include "kernels.h"
#include "rewrite_bodies.h"

#include <type_traits>

namespace c2i8 {

namespace {

constexpr int BAND_WAVES = 4, BAND_TK = 32;
constexpr size_t BAND_LDS_LIMIT = 160 * 1024;

constexpr int BAND_KPW_MAX = 12;
constexpr int BAND_MAP = 512;

struct BandArgs {
    const int8_t *act;  // [N][Cb][Hp][Wp][64]
    const int8_t *wq;   // [K][depth], depth index ((b*R + r)*S + s)*64 + c
    int32_t *out;       // [N][K][P][Q], or [N][P][Q][K] (out_nhwc)
    int out_nhwc, out_wide_k;    // NHWC result; K % 4 == 0 and out on 16 bytes: a lane's four channels go out as one piece
    ActOut aout;                 // activation epilogue (aout.out != null): `out` is not written
    int K, P, Q, Wp, stride;
    int depth, ksteps, kpw;      // bytes per weight row; 64-byte steps in all and per wave
    int PT, bands;               // output rows per band, bands per image
    int npix;                    // PT * Q
    int tiled, CT, CTN;          // shifted-fragment form: output columns per block, blocks per output row
    int wmax;                    // last pixel of a channel block's window
    int win_pieces, win_total;   // 1 KB pieces (16 pixels) of one channel block's window; of all blocks
    int win_per_wave;            // ceil(win_total / 4)
    int wave_region;             // LDS bytes per wave: weights, later partial sums
    int tiles_k, tiles_m, m_fastest;
    int xk, bk, bm;              // 2-D split over the XCDs: xk XCD columns, an XCD's block is bk x bm tiles (0: off)
    unsigned mg_bk, mg_per;
    int blk_bytes;               // one channel block of one image
    long long img_bytes;         // one image
    long long out_img;           // K*P*Q
    unsigned mg_Q, mg_bands, mg_tiles_k, mg_tiles_m, mg_CTN, mg_win_pieces;
    // window pixel offset of the wave's u-th group of depth steps (a group = the steps that share their
    // activation fragments: one step, or in the shifted-fragment form the taps of one kernel row):
    // its channel block's window + its kernel tap (row)
    int toff[BAND_WAVES][BAND_KPW_MAX];
    // grids of up to BAND_MAP workgroups: block -> (tk | tm << 16), made on the host (one scalar load instead of
    // the index arithmetic below; the kernel is short enough for that to show)
    int use_map;
    unsigned tmap[BAND_MAP];
};

// n / d for 0 <= n < 2^31 with magic = ceil(2^32 / d) truncated to 32 bits (0 encodes d == 1).
__device__ __forceinline__ int bdiv(int n, int d, unsigned magic)
{
    int q = magic ? (int)__umulhi((unsigned)n, magic) : n;
    if ((long long)q * d > n) --q;
    return q;
}
// The same without the correction step: exact while n * d < 2^32 (pixel indices of a tile).
__device__ __forceinline__ int bdiv_small(int n, unsigned magic)
{
    return magic ? (int)__umulhi((unsigned)n, magic) : n;
}

__device__ __forceinline__ int band_xcd_id(int id, int n)
{
    const int x = id & 7, q = n >> 3, rem = n & 7;
    return x * q + (x < rem ? x : rem) + (id >> 3);
}

// 16 bytes per lane from base + off (base wave-uniform, off a per-lane byte offset below 2^32) to LDS byte
// address lds_base + 16*lane (lds_base wave-uniform).  Completion is counted by vmcnt.
__device__ __forceinline__ void band_dma16(const int8_t *base, unsigned off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(off), "s"(base)
                 : "memory");
}
template <int N>
__device__ __forceinline__ void band_wait_dma()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ void band_barrier()
{
    asm volatile("" : : : "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's LDS accesses are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" : : : "memory");
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// One wave per SIMD: a wave issues at most one instruction every four cycles, so every instruction in the
// main loop competes with the MFMAs for issue slots.  Hence: every LDS address the loop uses is computed
// before it (one register per group of depth steps and pixel block -- registers are plentiful at this
// occupancy), index arithmetic is 32-bit with wave-uniform bases kept in scalar registers, and per-wave
// tables come from the host.
//
// SROW: depth steps that share their activation fragments (1, or 3 = the taps of a kernel row in the
// shifted-fragment form); GPW: such groups per wave; PB: pixel blocks per workgroup;
// FULL: every wave multiplies exactly GPW groups (no test around a group).
template <int SROW, int GPW, int PB, bool FULL>
__global__ void __launch_bounds__(BAND_WAVES * 64, 1) conv_band_kernel(const BandArgs a)
{
    constexpr int KPW = SROW * GPW;  // depth steps per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned tmap_e = a.tmap[min(blockIdx.x, (unsigned)BAND_MAP - 1)];   // (asked for with the rest, used if use_map)
    // Ask for every scalar argument now, in one batch: fetched one by one where first used, each costs a
    // scalar-cache miss of a few hundred cycles on a kernel that runs for a few thousand.
    asm volatile("" : : "s"(tmap_e), "s"(a.use_map), "s"(a.act), "s"(a.wq), "s"(a.out), "s"(a.K), "s"(a.P), "s"(a.Q), "s"(a.Wp), "s"(a.stride), "s"(a.depth),
                 "s"(a.ksteps), "s"(a.kpw), "s"(a.PT), "s"(a.bands), "s"(a.npix), "s"(a.CT), "s"(a.CTN), "s"(a.wmax));
    asm volatile("" : : "s"(a.win_pieces), "s"(a.win_total), "s"(a.win_per_wave), "s"(a.wave_region), "s"(a.tiles_k),
                 "s"(a.tiles_m), "s"(a.m_fastest), "s"(a.xk), "s"(a.bk), "s"(a.bm), "s"(a.mg_bk), "s"(a.mg_per), "s"(a.blk_bytes), "s"(a.img_bytes), "s"(a.out_img), "s"(a.mg_Q),
                 "s"(a.mg_bands), "s"(a.mg_tiles_k), "s"(a.mg_tiles_m), "s"(a.mg_CTN), "s"(a.mg_win_pieces));

    // workgroup -> (32 output channels, image, band)
    const int lid = band_xcd_id(blockIdx.x, gridDim.x);
    int tk, tm;
    if (a.use_map) {
        tk = (int)(tmap_e & 0xFFFFu), tm = (int)(tmap_e >> 16);
    } else if (a.bk) {   // XCD x = (x % xk, x / xk) owns the bk x bm block of tiles at that position
        const int per = a.bk * a.bm, x = bdiv(lid, per, a.mg_per), j = lid - x * per;
        const int jm = bdiv_small(j, a.mg_bk), jk = j - jm * a.bk;
        const int xr = x / a.xk;
        tk = (x - xr * a.xk) * a.bk + jk;
        tm = xr * a.bm + jm;
    } else if (a.m_fastest) {
        tk = bdiv(lid, a.tiles_m, a.mg_tiles_m);
        tm = lid - tk * a.tiles_m;
    } else {
        tm = bdiv(lid, a.tiles_k, a.mg_tiles_k);
        tk = lid - tm * a.tiles_k;
    }
    const int n = bdiv(tm, a.bands, a.mg_bands), band = tm - n * a.bands;
    const int p0 = band * a.PT, k0 = tk * BAND_TK;
    const int js = wave * a.kpw;
    const int nks = max(0, min(a.kpw, a.ksteps - js));  // depth steps of this wave
    const int ng = nks / SROW;                          // groups of them (whole groups by construction)

    const int wave_off = wave * a.wave_region, win_off = BAND_WAVES * a.wave_region;  // LDS byte offsets

    // A transfer moves 16 rows x 64 B; lane l lands at row l/4, position l%4 and fetches the chunk that
    // belongs there after the swizzle.
    const int lrow = lane >> 2;
    const int lane_part = lrow * 64 + (((lane & 3) ^ ((lane >> 4) & 3)) << 4);

    // ---- window: every wave fetches a contiguous quarter of the pieces of all channel blocks' windows ----
    {
        const int last = a.blk_bytes - 16;  // rows past the padded image (a short last band) read this
        const int per = a.win_per_wave, g0 = wave * per, g1 = min(g0 + per, a.win_total);
        int b = bdiv_small(g0, a.mg_win_pieces), i = g0 - b * a.win_pieces;  // channel block, piece of its window
        const int8_t *blk = a.act + (size_t)n * a.img_bytes + (size_t)b * a.blk_bytes;
        const int row0 = p0 * a.stride * a.Wp * 64 + lane_part;
        unsigned dst = lds0 + (unsigned)win_off + (unsigned)g0 * 1024u;
        for (int g = g0; g < g1;) {
            const int cnt = min(a.win_pieces - i, g1 - g);  // pieces left in this channel block's window
            int off = row0 + i * 1024;
            for (int c = 0; c < cnt; ++c) {  // (kept short: a transfer already holds the wave for ~60 cycles)
                band_dma16(blk, (unsigned)min(off, last), dst);
                dst += 1024u;
                off += 1024;
            }
            g += cnt;
            i = 0;
            blk += a.blk_bytes;
        }
    }
    // ---- where the lane's pixel of every block sits in a window (tap (0, 0)) ---------------------------
    const int col = lane & 15, grp = lane >> 4;  // pixel within a block / 16-byte chunk of a depth step
    int wbase[PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        if (SROW > 1) {  // block = 16 consecutive input columns of one window row
            const int pr = bdiv_small(pb, a.mg_CTN), ct = pb - pr * a.CTN;
            wbase[pb] = min(pr * a.Wp + ct * a.CT + col, a.wmax);
        } else {        // block = 16 consecutive output pixels of the band, row-major
            const int i = pb * 16 + col;
            const int pr = bdiv_small(i, a.mg_Q), q = i - pr * a.Q;
            const bool valid = i < a.npix && p0 + pr < a.P;
            wbase[pb] = valid ? (pr * a.stride) * a.Wp + q * a.stride : 0;
        }
    }
    // ---- this wave's weights: exactly 2*KPW transfers (steps past the last repeat it), and in between
    // the LDS addresses of the main loop: one register per group and pixel block ---------------------------
    int baddr[GPW][PB];
    {
        const unsigned row_lo = (unsigned)(min(k0 + lrow, a.K - 1) * a.depth) + (unsigned)(lane_part & 63);
        const unsigned row_hi = (unsigned)(min(k0 + 16 + lrow, a.K - 1) * a.depth) + (unsigned)(lane_part & 63);
        const unsigned dst = lds0 + (unsigned)wave_off;
#pragma unroll
        for (int t = 0; t < KPW; ++t) {
            const int8_t *step = a.wq + (size_t)min(js + t, a.ksteps - 1) * 64;
            band_dma16(step, row_lo, dst + (unsigned)(t * 2) * 1024u);
            band_dma16(step, row_hi, dst + (unsigned)(t * 2 + 1) * 1024u);
            if (t % SROW == 0) {
                const int tap = a.toff[wave][t / SROW];
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
                    const int w = wbase[pb] + tap;
                    baddr[t / SROW][pb] = win_off + (w << 6) + ((grp ^ ((w >> 2) & 3)) << 4);
                    asm volatile("" : "+v"(baddr[t / SROW][pb]));  // keep it in its register: recomputing it in the loop costs issue slots
                }
            }
        }
    }
    const int afrag = wave_off + col * 64 + ((grp ^ ((col >> 2) & 3)) << 4);  // weight fragment: row col, chunk grp
    // (every address is a multiple of 16: say so, or the reads are split into dword pairs)
    auto read_a = [&](int t, int rb) -> v4i {
        return *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + afrag + (t * 2 + rb) * 1024, 16));
    };
    auto read_b = [&](int u, int pb) -> v4i {
        return *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + baddr[u][pb], 16));
    };

    v4i acc[2][PB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[rb][pb] = v4i{0, 0, 0, 0};

    band_wait_dma<2 * KPW>();  // every window piece this wave asked for has landed ...
    band_barrier();            // ... and everyone else's

    // ---- main loop: no barrier.  All activation fragments of group u+1 are requested before group u
    // multiplies; the weight fragments of step t+1 half-way through step t (once their transfers have landed).
    v4i af[2][2], bq[2][PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) bq[0][pb] = read_b(0, pb);
    band_wait_dma<2 * (KPW - 1)>();
    af[0][0] = read_a(0, 0);
    af[0][1] = read_a(0, 1);
    static_for<0, GPW>([&](auto uc) {
        constexpr int u = decltype(uc)::value;
        if (FULL || u < ng) {
            if constexpr (u + 1 < GPW) {
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) bq[(u + 1) & 1][pb] = read_b(u + 1, pb);  // (unused past the last group)
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<0, SROW>([&](auto sc) {
                constexpr int s = decltype(sc)::value, t = u * SROW + s;
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
                    // tap s of the kernel row reads the input column s places to the right: the same fragment,
                    // shifted s lanes down within its 16-lane row (row_shl: a lane takes the value of the lane
                    // s places up; lanes that would reach past the row get 0 and hold no output column)
                    v4i bf = bq[u & 1][pb];
                    if constexpr (s > 0) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) bf[v] = __builtin_amdgcn_update_dpp(0, bf[v], 0x100 + s, 0xF, 0xF, true);
                    }
                    acc[0][pb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[t & 1][0], bf, acc[0][pb], 0, 0, 0);
                    acc[1][pb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[t & 1][1], bf, acc[1][pb], 0, 0, 0);
                    if constexpr (t + 1 < KPW) {
                        if (pb == PB / 2) {
                            __builtin_amdgcn_sched_barrier(0);  // the MFMAs above stay above the wait
                            band_wait_dma<2 * (KPW - 2 - t)>();
                            af[(t + 1) & 1][0] = read_a(t + 1, 0);
                            af[(t + 1) & 1][1] = read_a(t + 1, 1);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
            });
        }
    });

    // ---- add the four waves' partial sums.  Every wave leaves all its 2*PB blocks in its own region (its
    // spent weights); block i = rb*PB + pb is then summed and stored by wave i%4, which finds it by address --
    // no test on a register index anywhere. ------------------------------------------------------------------
    band_wait_dma<0>();  // transfers of steps this wave did not multiply must not land on partial sums
    {
        v4i *const mine = reinterpret_cast<v4i *>(__builtin_assume_aligned(smem + wave_off, 16));
#pragma unroll
        for (int i = 0; i < 2 * PB; ++i) mine[i * 64 + lane] = acc[i / PB][i % PB];
    }
    band_barrier();
    // D block: column = pixel = lane%16, row = channel = 4*(lane/16) + v.  Output offset = a wave-uniform part
    // (image, row block, pixel block) + a per-lane part computed once; four planes = four scalar bases.
    // Every wave walks the same number of slots (a slot past the last block stores nothing), so the loop has
    // no exits: with one wave per SIMD every branch and every scalar instruction costs an issue slot.
    const int plane = a.P * a.Q;
    int32_t *const out0 = a.out + (size_t)n * a.out_img + (size_t)k0 * plane;
    int32_t *const out1 = out0 + plane, *const out2 = out1 + plane, *const out3 = out2 + plane;
    const int lane_off = 4 * grp * plane + col;
    const int kleft = a.K - k0 - 4 * grp;   // output channels from this lane's first one to the last
    const bool k_whole = k0 + BAND_TK <= a.K;  // wave-uniform: no channel of the tile lies past the last
    constexpr int SLOTS = (2 * PB + BAND_WAVES - 1) / BAND_WAVES;
    if (SROW > 1 && k_whole && a.out_nhwc && a.out_wide_k && a.aout.out == nullptr) {
        // The same for an NHWC result whose pixels take 16-byte pieces: a lane's four sums are channels k .. k+3 of
        // one pixel; 32-bit byte offsets against the image's base.
        v4i sums[SLOTS];
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int i = wave + BAND_WAVES * m;
            sums[m] = *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + i * 1024 + lane * 16, 16));
#pragma unroll
            for (int o = 1; o < BAND_WAVES; ++o)
                sums[m] += *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + o * a.wave_region + i * 1024 + lane * 16, 16));
        }
        const char *const img = reinterpret_cast<const char *>(a.out + (size_t)n * a.out_img);
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int i = wave + BAND_WAVES * m;
            const int rb = i >= PB ? 1 : 0, pb = i - rb * PB;
            const int pr = bdiv_small(pb, a.mg_CTN), q0 = (pb - pr * a.CTN) * a.CT;  // wave-uniform
            const int cols = (i < 2 * PB && pr < a.PT && p0 + pr < a.P) ? min(a.CT, a.Q - q0) : 0;
            const unsigned offb = (unsigned)(((p0 + pr) * a.Q + q0 + col) * a.K + k0 + rb * 16 + 4 * grp) * 4u;
            if (col < cols) *reinterpret_cast<v4i *>(const_cast<char *>(img) + offb) = sums[m];
        }
        return;
    }
    if (SROW > 1 && k_whole && !(a.out_nhwc | (a.aout.out != nullptr))) {
        // The common case -- int32 NKPQ result, whole channel tile, shifted-fragment form -- on a path of its own:
        // every sum is read before the first store (one LDS round trip for the wave, not one per slot), no test of
        // the result's form inside the loop, and 32-bit byte offsets against four scalar plane bases (the host
        // refuses results of 2^30 elements per image and more).
        v4i sums[SLOTS];
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int i = wave + BAND_WAVES * m;
            sums[m] = *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + i * 1024 + lane * 16, 16));
#pragma unroll
            for (int o = 1; o < BAND_WAVES; ++o)
                sums[m] += *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + o * a.wave_region + i * 1024 + lane * 16, 16));
        }
        const char *const b0 = reinterpret_cast<const char *>(out0), *const b1 = reinterpret_cast<const char *>(out1);
        const char *const b2 = reinterpret_cast<const char *>(out2), *const b3 = reinterpret_cast<const char *>(out3);
#pragma unroll
        for (int m = 0; m < SLOTS; ++m) {
            const int i = wave + BAND_WAVES * m;
            const int rb = i >= PB ? 1 : 0, pb = i - rb * PB;
            const int pr = bdiv_small(pb, a.mg_CTN), q0 = (pb - pr * a.CTN) * a.CT;  // wave-uniform
            const int cols = (i < 2 * PB && pr < a.PT && p0 + pr < a.P) ? min(a.CT, a.Q - q0) : 0;
            const unsigned offb = (unsigned)(rb * 16 * plane + (p0 + pr) * a.Q + q0 + lane_off) * 4u;
            if (col < cols) {
                *reinterpret_cast<int32_t *>(const_cast<char *>(b0) + offb) = sums[m][0];
                *reinterpret_cast<int32_t *>(const_cast<char *>(b1) + offb) = sums[m][1];
                *reinterpret_cast<int32_t *>(const_cast<char *>(b2) + offb) = sums[m][2];
                *reinterpret_cast<int32_t *>(const_cast<char *>(b3) + offb) = sums[m][3];
            }
        }
        return;
    }
#pragma unroll
    for (int m = 0; m < SLOTS; ++m) {
        const int i = wave + BAND_WAVES * m;  // wave-uniform; the regions hold SLOTS*4 blocks
        const int rb = i >= PB ? 1 : 0, pb = i - rb * PB;
        v4i sum = *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + i * 1024 + lane * 16, 16));
#pragma unroll
        for (int o = 1; o < BAND_WAVES; ++o)
            sum += *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + o * a.wave_region + i * 1024 + lane * 16, 16));
        unsigned off;
        bool valid;
        if (SROW > 1) {
            const int pr = bdiv_small(pb, a.mg_CTN), q0 = (pb - pr * a.CTN) * a.CT;  // wave-uniform
            const int cols = (i < 2 * PB && pr < a.PT && p0 + pr < a.P) ? min(a.CT, a.Q - q0) : 0;
            valid = col < cols;
            off = (unsigned)(rb * 16 * plane + (p0 + pr) * a.Q + q0 + lane_off);
        } else {
            const int px = pb * 16 + col;
            const int pr = bdiv_small(px, a.mg_Q), q = px - pr * a.Q;
            valid = i < 2 * PB && px < a.npix && p0 + pr < a.P;
            off = (unsigned)(rb * 16 * plane + (p0 + pr) * a.Q + q + lane_off - col);
        }
        // A lane's four values are channels k .. k+3 of one pixel: one piece of an NHWC result, one dword of the
        // next layer's blocked input after the activation.  (Wave-uniform tests: one of the three forms runs.)
        if (a.out_nhwc | (a.aout.out != nullptr)) {
            int pp, qq;
            if (SROW > 1) {
                const int pr = bdiv_small(pb, a.mg_CTN);
                pp = p0 + pr, qq = (pb - pr * a.CTN) * a.CT + col;
            } else {
                const int px = pb * 16 + col, pr = bdiv_small(px, a.mg_Q);
                pp = p0 + pr, qq = px - pr * a.Q;
            }
            const int k = k0 + rb * 16 + 4 * grp;
            if (valid && k < a.K) {
                if (a.aout.out) {
                    act_store4(a.aout, n, pp, qq, k, a.K, sum[0], sum[1], sum[2], sum[3]);
                } else {
                    int32_t *px = a.out + (((size_t)n * a.P + pp) * a.Q + qq) * a.K + k;
                    if (a.out_wide_k) *reinterpret_cast<v4i *>(px) = sum;
                    else {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (k + v < a.K) px[v] = sum[v];
                    }
                }
            }
        } else if (k_whole) {
            if (valid) {
                out0[off] = sum[0];
                out1[off] = sum[1];
                out2[off] = sum[2];
                out3[off] = sum[3];
            }
        } else {
            const int kl = kleft - rb * 16;
            if (valid && kl > 0) out0[off] = sum[0];
            if (valid && kl > 1) out1[off] = sum[1];
            if (valid && kl > 2) out2[off] = sum[2];
            if (valid && kl > 3) out3[off] = sum[3];
        }
    }
}

constexpr int kBandPB[] = {4, 7, 8};
constexpr int kBandGroups1[] = {3, 6, 9, 12};  // groups per wave, one step per group
constexpr int kBandGroups3[] = {1, 2, 3, 4};   // groups per wave, three steps per group

struct BandPlan {
    BandArgs a;
    int srow, gpw, pb;  // template arguments to launch
    bool full;
    size_t lds;
    int grid;
};

unsigned magic_of(long long d) { return d <= 1 ? 0u : (unsigned)((0x100000000ULL + (unsigned long long)d - 1) / (unsigned long long)d); }

// Fills the plan; false where the kernel does not apply.
bool band_plan(const GemmProblem &g, BandPlan *bp)
{
    if (g.mode != ACT_BLOCKED || g.cb != 64 || g.il_d) return false;
    if (g.act_out && (g.o_cb < 4 || (g.o_cb & (g.o_cb - 1)))) return false;
    if (g.Q <= 0 || g.PQ % g.Q) return false;
    const int P = g.PQ / g.Q, Q = g.Q, dil = g.dil > 0 ? g.dil : 1;
    const long long ksteps = (long long)g.Cb * g.R * g.S;
    if (ksteps * 64 != g.depth) return false;
    if (g.M % g.PQ) return false;
    const int N = g.M / g.PQ;
    // Shifted fragments: stride 1, dense taps, three of them per kernel row; a block is then 16 input
    // columns that hold CT = 14 output columns.
    const bool tiled = g.stride == 1 && dil == 1 && g.S == 3;
    const int srow = tiled ? 3 : 1;
    const int CT = tiled ? 16 - (g.S - 1) : 16, CTN = tiled ? (Q + CT - 1) / CT : 1;
    const long long groups = ksteps / srow;  // groups of steps that share their activation fragments
    const int gpw = (int)((groups + BAND_WAVES - 1) / BAND_WAVES);
    int GPW = 0;
    for (int c : tiled ? kBandGroups3 : kBandGroups1)
        if (!GPW && c >= gpw) GPW = c;
    if (!GPW) return false;
    const int KPW = GPW * srow, kpw = gpw * srow;
    // pixel blocks: the choice that pads an image's pixels least (ties: fewer blocks)
    int PB = 0, PT = 0;
    long long best = 0;
    for (int c : kBandPB) {
        int pt = tiled ? c / CTN : c * 16 / Q;
        if (pt < 1) continue;
        if (pt > P) pt = P;
        const long long padded = (long long)((P + pt - 1) / pt) * c;
        if (!PB || padded < best) {
            PB = c;
            PT = pt;
            best = padded;
        }
    }
    if (!PB) return false;  // an output row wider than the largest pixel tile
    PT = (P + (P + PT - 1) / PT - 1) / ((P + PT - 1) / PT);  // same number of bands, of even height
    const long long WR = (long long)(PT - 1) * g.stride + (long long)(g.R - 1) * dil + 1;
    const long long win_pieces = (WR * g.Wp + 15) / 16;
    const long long red = (2LL * PB + BAND_WAVES - 1) / BAND_WAVES * BAND_WAVES * 1024, wbytes = (long long)KPW * 2048;  // whole slots
    const long long wave_region = red > wbytes ? red : wbytes;
    const long long lds = BAND_WAVES * wave_region + g.Cb * win_pieces * 1024;
    if (lds > (long long)BAND_LDS_LIMIT) return false;
    const long long bands = (P + PT - 1) / PT;
    const long long tiles_k = (g.K + BAND_TK - 1) / BAND_TK, tiles_m = (long long)N * bands;
    if (tiles_k * tiles_m > 0x7FFFFFFFLL) return false;
    if ((long long)g.Hp * g.Wp * 64 > 0x7FFFFFFFLL || (long long)(g.Cb * win_pieces + 1) * 16 + WR * g.Wp > 0x7FFFFFFFLL)
        return false;
    if ((long long)g.K * g.depth > 0x7FFFFFFFLL || (long long)g.K * P * Q > 0x3FFFFFFFLL) return false;  // 32-bit offsets

    BandArgs &a = bp->a;
    a.act = g.act;
    a.wq = g.wq;
    a.out = g.out;
    a.out_nhwc = g.out_nhwc;
    a.out_wide_k = g.K % 4 == 0 && (reinterpret_cast<uintptr_t>(g.out) & 15) == 0;
    a.aout = ActOut{};
    if (g.act_out) {
        int lg = 0;
        while ((1 << lg) < g.o_cb) ++lg;
        a.aout = ActOut{g.act_out, g.act_shift, g.act_relu, lg, g.o_pad, P + 2 * g.o_pad, Q + 2 * g.o_pad, (g.K + g.o_cb - 1) / g.o_cb};
    }
    a.K = g.K;
    a.P = P;
    a.Q = Q;
    a.Wp = g.Wp;
    a.stride = g.stride;
    a.depth = g.depth;
    a.ksteps = (int)ksteps;
    a.kpw = kpw;
    a.PT = PT;
    a.bands = (int)bands;
    a.npix = PT * Q;
    a.tiled = tiled;
    a.CT = CT;
    a.CTN = CTN;
    a.wmax = PT * g.Wp - 1;  // a clamped pixel plus any tap row stays inside the window
    a.win_pieces = (int)win_pieces;
    a.win_total = (int)(g.Cb * win_pieces);
    a.win_per_wave = (a.win_total + BAND_WAVES - 1) / BAND_WAVES;
    a.wave_region = (int)wave_region;
    a.tiles_k = (int)tiles_k;
    a.tiles_m = (int)tiles_m;
    a.blk_bytes = g.Hp * g.Wp * 64;
    a.img_bytes = (long long)a.blk_bytes * g.Cb;
    a.out_img = (long long)g.K * P * Q;
    for (int w = 0; w < BAND_WAVES; ++w)
        for (int u = 0; u < BAND_KPW_MAX; ++u) {
            long long j = ((long long)w * gpw + u) * srow;  // first step of the group
            if (j > ksteps - 1) j = ksteps - 1;
            const int b = (int)(j / (g.R * g.S)), rs = (int)(j % (g.R * g.S));
            a.toff[w][u] = b * (int)win_pieces * 16 + ((rs / g.S) * g.Wp + (tiled ? 0 : rs % g.S)) * dil;
        }
    {
        // each XCD (own L2) runs a contiguous eighth of the list: order it so that what one XCD pulls in
        // (windows of its bands + weight rows of its channel tiles) is least
        const long long per = (tiles_k * tiles_m + 7) / 8;
        const double wbytes_k = (double)BAND_TK * g.depth, win_bytes = (double)g.Cb * win_pieces * 1024;
        auto cost = [&](long long fast, long long slow, double fb, double sb) {
            const long long nf = per < fast ? per : fast;
            long long ns = (per + fast - 1) / fast + 1;
            if (ns > slow) ns = slow;
            return nf * fb + ns * sb;
        };
        a.m_fastest = cost(tiles_m, tiles_k, win_bytes, wbytes_k) < cost(tiles_k, tiles_m, wbytes_k, win_bytes);
        // ... or, where both tile counts divide, a 2-D split: XCD columns x XCD rows = 8, every XCD a block of tiles
        // (what it pulls in: its block's weight rows + its block's windows)
        double best = a.m_fastest ? cost(tiles_m, tiles_k, win_bytes, wbytes_k) : cost(tiles_k, tiles_m, wbytes_k, win_bytes);
        a.xk = a.bk = a.bm = 0;
        for (int xk = 2; xk <= 4; xk *= 2) {
            const int xm = 8 / xk;
            if (tiles_k % xk || tiles_m % xm) continue;
            const double c = (double)(tiles_k / xk) * wbytes_k + (double)(tiles_m / xm) * win_bytes;
            if (c < best) {
                best = c;
                a.xk = xk, a.bk = (int)(tiles_k / xk), a.bm = (int)(tiles_m / xm);
            }
        }
        a.mg_bk = magic_of(a.bk);
        a.mg_per = magic_of((long long)a.bk * a.bm);
        // the same mapping as a table, where it fits
        const long long grid = tiles_k * tiles_m;
        a.use_map = grid <= BAND_MAP && tiles_k < 65536 && tiles_m < 65536;
        if (a.use_map)
            for (int i = 0; i < (int)grid; ++i) {
                const int x = i & 7, q = (int)grid >> 3, rem = (int)grid & 7;
                const int lid = x * q + (x < rem ? x : rem) + (i >> 3);   // (band_xcd_id)
                int tk, tm;
                if (a.bk) {
                    const int per = a.bk * a.bm, xx = lid / per, j = lid - xx * per, jm = j / a.bk, jk = j - jm * a.bk;
                    tk = (xx % a.xk) * a.bk + jk;
                    tm = (xx / a.xk) * a.bm + jm;
                } else if (a.m_fastest) {
                    tk = lid / (int)tiles_m, tm = lid - tk * (int)tiles_m;
                } else {
                    tm = lid / (int)tiles_k, tk = lid - tm * (int)tiles_k;
                }
                a.tmap[i] = (unsigned)tk | ((unsigned)tm << 16);
            }
    }
    a.mg_Q = magic_of(Q);
    a.mg_bands = magic_of(bands);
    a.mg_tiles_k = magic_of(tiles_k);
    a.mg_tiles_m = magic_of(tiles_m);
    a.mg_CTN = magic_of(CTN);
    a.mg_win_pieces = magic_of(win_pieces);
    bp->srow = srow;
    bp->gpw = GPW;
    bp->pb = PB;
    bp->full = groups == (long long)BAND_WAVES * GPW;
    bp->lds = (size_t)lds;
    bp->grid = (int)(tiles_k * tiles_m);
    return true;
}

template <int SROW, int GPW, int PB, bool FULL>
hipError_t launch_band(const BandPlan &bp, hipStream_t st)
{
    auto kern = conv_band_kernel<SROW, GPW, PB, FULL>;
    static bool raised = false;  // dynamic-LDS ceiling granted, per instantiation
    if (bp.lds > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)BAND_LDS_LIMIT);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL(kern, dim3(bp.grid), dim3(BAND_WAVES * 64), bp.lds, st, bp.a);
    return hipGetLastError();
}

}  // namespace

bool band_applies(const GemmProblem &g)
{
    BandPlan bp;
    return band_plan(g, &bp);
}

size_t band_lds_bytes(const GemmProblem &g)
{
    BandPlan bp;
    return band_plan(g, &bp) ? bp.lds : 0;
}

TileInfo band_tile_info(const GemmProblem &g)
{
    BandPlan bp;
    if (!band_plan(g, &bp)) return TileInfo{0, 0, 0, 0};
    return TileInfo{BAND_TK, bp.pb * 16, BAND_WAVES * 64, 1};
}

// The picker's estimate (core cycles, same scale as gemm_pick's).  Measured: the kernel wins where one round of
// workgroups covers the problem and -- in the form without shifted fragments -- the reduction is deep enough to
// pay for its fixed parts (address set-up, summing the waves' partial results); with more rounds the general
// kernel's large tiles move fewer bytes per MAC.
double band_cost(const GemmProblem &g)
{
    BandPlan bp;
    if (!band_plan(g, &bp)) return 1e300;
    const BandArgs &a = bp.a;
    if (bp.grid > 256 || (bp.srow == 1 && a.ksteps < 18)) return 1e300;
    const double bytes = (double)a.win_total * 1024 + (double)BAND_TK * a.depth;
    const double mfma = (double)a.kpw * bp.pb * 2 * 25.0;
    return 1800.0 + (bytes / 40.0 > mfma ? bytes / 40.0 : mfma) + 1800.0;
}

hipError_t launch_band_conv(const GemmProblem &g, hipStream_t st)
{
    BandPlan bp;
    if (!band_plan(g, &bp)) return hipErrorInvalidValue;
#define C2I8_BAND_CASE(SROW, GPW, PB)                       \
    if (bp.srow == SROW && bp.gpw == GPW && bp.pb == PB)    \
        return bp.full ? launch_band<SROW, GPW, PB, true>(bp, st) : launch_band<SROW, GPW, PB, false>(bp, st);
#define C2I8_BAND_PBS(SROW, GPW) C2I8_BAND_CASE(SROW, GPW, 4) C2I8_BAND_CASE(SROW, GPW, 7) C2I8_BAND_CASE(SROW, GPW, 8)
    C2I8_BAND_PBS(1, 3) C2I8_BAND_PBS(1, 6) C2I8_BAND_PBS(1, 9) C2I8_BAND_PBS(1, 12)
    C2I8_BAND_PBS(3, 1) C2I8_BAND_PBS(3, 2) C2I8_BAND_PBS(3, 3) C2I8_BAND_PBS(3, 4)
#undef C2I8_BAND_PBS
#undef C2I8_BAND_CASE
    return hipErrorInvalidValue;
}

}  // namespace c2i8
