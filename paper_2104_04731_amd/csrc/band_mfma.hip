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
//     used for every pixel block, an activation fragment for both row blocks: 1 KB of LDS reads
//     per 2 MFMAs;
//   * the four waves' partial sums meet in LDS (each wave's region is its spent weight region);
//     wave w adds up and stores every fourth 16 x 16 block, straight to NKPQ.
// Both LDS operands are XOR-swizzled per 64-byte row ((row/4)%4 on the 16-byte chunk index), done
// by the lanes' choice of source chunk, so the column-wise fragment reads spread over all banks.
#include "kernels.h"

#include <type_traits>

namespace c2i8 {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int BAND_WAVES = 4, BAND_TK = 32;
constexpr size_t BAND_LDS_LIMIT = 160 * 1024;

constexpr int BAND_KPW_MAX = 12;

struct BandArgs {
    const int8_t *act;  // [N][Cb][Hp][Wp][64]
    const int8_t *wq;   // [K][depth], depth index ((b*R + r)*S + s)*64 + c
    int32_t *out;       // [N][K][P][Q]
    int K, P, Q, Wp, stride;
    int depth, ksteps, kpw;      // bytes per weight row; 64-byte steps in all and per wave
    int PT, bands;               // output rows per band, bands per image
    int npix;                    // PT * Q
    int win_pieces, win_total;   // 1 KB pieces (16 pixels) of one channel block's window; of all blocks
    int wave_region;             // LDS bytes per wave: weights, later partial sums
    int tiles_k, tiles_m, m_fastest;
    int blk_bytes;               // one channel block of one image
    long long img_bytes;         // one image
    long long out_img;           // K*P*Q
    unsigned mg_Q, mg_bands, mg_tiles_k, mg_tiles_m;
    // window pixel offset of depth step w*kpw + t: its channel block's window + its kernel tap
    int toff[BAND_WAVES][BAND_KPW_MAX];
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
// before it (one register per depth step and pixel block -- registers are plentiful at this occupancy),
// index arithmetic is 32-bit with wave-uniform bases kept in scalar registers, and per-wave tables come
// from the host.
// FULL: every wave multiplies exactly KPW steps (the depth is 4*KPW steps): no test around a step.
template <int KPW, int PB, bool FULL>
__global__ void __launch_bounds__(BAND_WAVES * 64, 1) conv_band_kernel(const BandArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // workgroup -> (32 output channels, image, band)
    const int lid = band_xcd_id(blockIdx.x, gridDim.x);
    int tk, tm;
    if (a.m_fastest) {
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

    const int wave_off = wave * a.wave_region, win_off = BAND_WAVES * a.wave_region;  // LDS byte offsets

    // A transfer moves 16 rows x 64 B; lane l lands at row l/4, position l%4 and fetches the chunk that
    // belongs there after the swizzle.
    const int lrow = lane >> 2;
    const int lane_part = lrow * 64 + (((lane & 3) ^ ((lane >> 4) & 3)) << 4);

    // ---- window: pieces wave, wave+4, ... of all channel blocks' windows ------------------------------
    {
        const int last = a.blk_bytes - 16;  // rows past the padded image (a short last band) read this
        const int row0 = p0 * a.stride * a.Wp * 64 + lane_part;
        const int8_t *blk = a.act + (size_t)n * a.img_bytes;  // channel block of the next piece
        int i = wave;                                        // its piece within that block's window
        while (i >= a.win_pieces) {
            i -= a.win_pieces;
            blk += a.blk_bytes;
        }
        unsigned dst = lds0 + (unsigned)win_off + (unsigned)wave * 1024u;
        for (int g = wave; g < a.win_total; g += BAND_WAVES) {
            band_dma16(blk, (unsigned)min(row0 + i * 1024, last), dst);
            dst += BAND_WAVES * 1024u;
            i += BAND_WAVES;
            while (i >= a.win_pieces) {
                i -= a.win_pieces;
                blk += a.blk_bytes;
            }
        }
    }
    // ---- this wave's weights: exactly 2*KPW transfers (steps past the last repeat it).  A transfer
    // occupies the memory pipe for some 60 cycles during which the wave can issue other work, so the LDS
    // addresses the main loop will use are computed in between: one register per depth step and pixel block.
    const int col = lane & 15, grp = lane >> 4;  // pixel within a block / 16-byte chunk of a depth step
    int wbase[PB];  // byte address of the lane's pixel in the window at tap (0, 0); swizzle bits clear
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        const int i = pb * 16 + col;
        const int pr = bdiv_small(i, a.mg_Q), q = i - pr * a.Q;
        const bool valid = i < a.npix && p0 + pr < a.P;
        wbase[pb] = valid ? (pr * a.stride) * a.Wp + q * a.stride : 0;
    }
    int baddr[KPW][PB];  // activation fragment of pixel block pb at depth step t
    {
        const unsigned row_lo = (unsigned)(min(k0 + lrow, a.K - 1) * a.depth) + (unsigned)(lane_part & 63);
        const unsigned row_hi = (unsigned)(min(k0 + 16 + lrow, a.K - 1) * a.depth) + (unsigned)(lane_part & 63);
        const unsigned dst = lds0 + (unsigned)wave_off;
#pragma unroll
        for (int t = 0; t < KPW; ++t) {
            const int8_t *step = a.wq + (size_t)min(js + t, a.ksteps - 1) * 64;
            band_dma16(step, row_lo, dst + (unsigned)(t * 2) * 1024u);
            band_dma16(step, row_hi, dst + (unsigned)(t * 2 + 1) * 1024u);
            const int tap = a.toff[wave][t];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int w = wbase[pb] + tap;
                baddr[t][pb] = win_off + (w << 6) + ((grp ^ ((w >> 2) & 3)) << 4);
                asm volatile("" : "+v"(baddr[t][pb]));  // keep it in its register: recomputing it in the loop costs issue slots
            }
        }
    }
    const int afrag = wave_off + col * 64 + ((grp ^ ((col >> 2) & 3)) << 4);  // weight fragment: row col, chunk grp
    // (every address is a multiple of 16: say so, or the reads are split into dword pairs)
    auto read_a = [&](int t, int rb) -> v4i {
        return *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + afrag + (t * 2 + rb) * 1024, 16));
    };
    auto read_b = [&](int t, int pb) -> v4i {
        return *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + baddr[t][pb], 16));
    };

    v4i acc[2][PB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[rb][pb] = v4i{0, 0, 0, 0};

    band_wait_dma<2 * KPW>();  // every window piece this wave asked for has landed ...
    band_barrier();            // ... and everyone else's

    // ---- main loop: no barrier.  All activation fragments of step t+1 are requested before step t
    // multiplies, its weight fragments half-way through (once their transfers have landed). -----------------
    v4i af[2][2], bq[2][PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) bq[0][pb] = read_b(0, pb);
    band_wait_dma<2 * (KPW - 1)>();
    af[0][0] = read_a(0, 0);
    af[0][1] = read_a(0, 1);
    static_for<0, KPW>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        if (FULL || t < nks) {
            if constexpr (t + 1 < KPW) {
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) bq[(t + 1) & 1][pb] = read_b(t + 1, pb);  // (unused past the last step)
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                acc[0][pb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[t & 1][0], bq[t & 1][pb], acc[0][pb], 0, 0, 0);
                acc[1][pb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[t & 1][1], bq[t & 1][pb], acc[1][pb], 0, 0, 0);
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
    int32_t *const out_n = a.out + (size_t)n * a.out_img;
    const int plane = a.P * a.Q;
#pragma unroll
    for (int m = 0; m < (2 * PB + BAND_WAVES - 1) / BAND_WAVES; ++m) {
        const int i = wave + BAND_WAVES * m;  // wave-uniform
        if (i >= 2 * PB) break;
        const int rb = i >= PB ? 1 : 0, pb = i - rb * PB;
        const v4i *part = reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + i * 1024 + lane * 16, 16));
        v4i sum = part[0];
#pragma unroll
        for (int o = 1; o < BAND_WAVES; ++o)
            sum += *reinterpret_cast<const v4i *>(__builtin_assume_aligned(smem + o * a.wave_region + i * 1024 + lane * 16, 16));
        // D block: column = pixel = lane%16, row = channel = 4*(lane/16) + v
        const int px = pb * 16 + col;
        const int pr = bdiv_small(px, a.mg_Q), q = px - pr * a.Q;
        if (px >= a.npix || p0 + pr >= a.P) continue;
        const int k = k0 + rb * 16 + 4 * grp;
        const unsigned off = (unsigned)(k * plane + (p0 + pr) * a.Q + q);
        if (k + 3 < a.K) {
            out_n[off] = sum[0];
            out_n[off + (unsigned)plane] = sum[1];
            out_n[off + 2u * (unsigned)plane] = sum[2];
            out_n[off + 3u * (unsigned)plane] = sum[3];
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (k + v < a.K) out_n[off + (unsigned)(v * plane)] = sum[v];
        }
    }
}

constexpr int kBandPB[] = {4, 7, 8};
constexpr int kBandKPW[] = {3, 6, 9, 12};

struct BandPlan {
    BandArgs a;
    int pb, kpw_slot;  // template arguments to launch
    size_t lds;
    int grid;
};

unsigned magic_of(long long d) { return d <= 1 ? 0u : (unsigned)((0x100000000ULL + (unsigned long long)d - 1) / (unsigned long long)d); }

// Fills the plan; false where the kernel does not apply.
bool band_plan(const GemmProblem &g, BandPlan *bp)
{
    if (g.mode != ACT_BLOCKED || g.cb != 64 || g.act_out || g.il_d || g.out_nhwc) return false;
    if (g.Q <= 0 || g.PQ % g.Q) return false;
    const int P = g.PQ / g.Q, Q = g.Q, dil = g.dil > 0 ? g.dil : 1;
    const long long ksteps = (long long)g.Cb * g.R * g.S;
    if (ksteps * 64 != g.depth) return false;
    const int kpw = (int)((ksteps + BAND_WAVES - 1) / BAND_WAVES);
    int KPW = 0;
    for (int c : kBandKPW)
        if (!KPW && c >= kpw) KPW = c;
    if (!KPW) return false;
    if (g.M % g.PQ) return false;
    const int N = g.M / g.PQ;
    // pixel blocks: the choice that pads an image's pixels least (ties: fewer blocks)
    int PB = 0, PT = 0;
    long long best = 0;
    for (int c : kBandPB) {
        int pt = c * 16 / Q;
        if (pt < 1) continue;
        if (pt > P) pt = P;
        const long long padded = (long long)((P + pt - 1) / pt) * c * 16;
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
    const long long red = 2LL * PB * 1024, wbytes = (long long)KPW * 2048;
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
    a.win_pieces = (int)win_pieces;
    a.win_total = (int)(g.Cb * win_pieces);
    a.wave_region = (int)wave_region;
    a.tiles_k = (int)tiles_k;
    a.tiles_m = (int)tiles_m;
    a.blk_bytes = g.Hp * g.Wp * 64;
    a.img_bytes = (long long)a.blk_bytes * g.Cb;
    a.out_img = (long long)g.K * P * Q;
    for (int w = 0; w < BAND_WAVES; ++w)
        for (int t = 0; t < BAND_KPW_MAX; ++t) {
            long long j = (long long)w * kpw + t;
            if (j > ksteps - 1) j = ksteps - 1;
            const int b = (int)(j / (g.R * g.S)), rs = (int)(j % (g.R * g.S));
            a.toff[w][t] = b * (int)win_pieces * 16 + ((rs / g.S) * g.Wp + rs % g.S) * dil;
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
    }
    a.mg_Q = magic_of(Q);
    a.mg_bands = magic_of(bands);
    a.mg_tiles_k = magic_of(tiles_k);
    a.mg_tiles_m = magic_of(tiles_m);
    bp->pb = PB;
    bp->kpw_slot = KPW;
    bp->lds = (size_t)lds;
    bp->grid = (int)(tiles_k * tiles_m);
    return true;
}

template <int KPW, int PB, bool FULL>
hipError_t launch_band(const BandPlan &bp, hipStream_t st)
{
    auto kern = conv_band_kernel<KPW, PB, FULL>;
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
// workgroups covers the problem and the reduction is deep enough to pay for its fixed parts (address set-up,
// summing the waves' partial results); with more rounds the general kernel's large tiles move fewer bytes.
double band_cost(const GemmProblem &g)
{
    BandPlan bp;
    if (!band_plan(g, &bp)) return 1e300;
    const BandArgs &a = bp.a;
    if (bp.grid > 256 || a.ksteps < 18) return 1e300;
    const double bytes = (double)a.win_total * 1024 + (double)BAND_TK * a.depth;
    const double mfma = (double)a.kpw * bp.pb * 2 * 16 * 1.8;
    return 5000.0 + (bytes / 25.0 > mfma ? bytes / 25.0 : mfma) + 4000.0;
}

hipError_t launch_band_conv(const GemmProblem &g, hipStream_t st)
{
    BandPlan bp;
    if (!band_plan(g, &bp)) return hipErrorInvalidValue;
    const bool full = bp.a.ksteps == BAND_WAVES * bp.kpw_slot;
#define C2I8_BAND_CASE(KPW, PB) \
    if (bp.kpw_slot == KPW && bp.pb == PB) return full ? launch_band<KPW, PB, true>(bp, st) : launch_band<KPW, PB, false>(bp, st);
    C2I8_BAND_CASE(3, 4) C2I8_BAND_CASE(3, 7) C2I8_BAND_CASE(3, 8)
    C2I8_BAND_CASE(6, 4) C2I8_BAND_CASE(6, 7) C2I8_BAND_CASE(6, 8)
    C2I8_BAND_CASE(9, 4) C2I8_BAND_CASE(9, 7) C2I8_BAND_CASE(9, 8)
    C2I8_BAND_CASE(12, 4) C2I8_BAND_CASE(12, 7) C2I8_BAND_CASE(12, 8)
#undef C2I8_BAND_CASE
    return hipErrorInvalidValue;
}

}  // namespace c2i8
