// GEMM stage of the convolution: out[k][m] = sum_j wq[k][j] * act(m)[j] on the CDNA4 int8
// MFMA (v_mfma_i32_32x32x32_i8), the counterpart of the paper's VTA GEMM core
// C[x][y] += A[x][z] * B[y][z] (Sec. 5.1) with x = output channel, y = output pixel,
// z = fused reduction depth.  Both operands are depth-contiguous, which is exactly what
// the layout rewrites (Table 2) produce.
//
// Workgroup = TK output channels x TM output pixels; depth is walked in 64-byte steps.
// Per step the TK x 64 B weight tile and TM x 64 B activation tile are staged in LDS as
// four planes of 16-byte chunks ([chunk][row][16 B]), so both the staging writes and the
// MFMA operand reads (32 consecutive rows of one plane per half-wave) are contiguous
// 16-byte accesses.  Global loads for step i+1 are in flight while step i is multiplied
// (register prefetch, two LDS stages, one barrier per step).
//
// The activation row of pixel m is addressed as rowbase(m) + koff[chunk]: for the blocked
// layout koff walks (channel block, r, s) over the zero-padded image (implicit GEMM, no
// unrolled matrix in memory); for a row-major matrix (im2col output) it is 16*chunk.
#include "kernels.h"

namespace c2i8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const int8_t *act;
    const int8_t *wq;
    int32_t *out;
    int K, M, depth, PQ, Q;
    int stride, cb, g16, R, S, Hp, Wp, nreal;
    long long img_bytes;
    int tiles_k, tiles_m;
    int ksteps_total, ksteps_per_split, split_k;
};

// Workgroups are dealt round-robin over the 8 XCDs (each with its own L2); give every XCD
// a contiguous range of logical tile ids so that neighbours in tile order share an L2.
__device__ __forceinline__ int xcd_contiguous_id(int id, int n)
{
    const int x = id & 7, q = n >> 3, rem = n & 7;
    return x * q + (x < rem ? x : rem) + (id >> 3);
}

template <int TK, int TM, int WK, int WM, int MODE>
__global__ void __launch_bounds__(WK *WM * 64) igemm_i8_kernel(const GemmArgs a)
{
    constexpr int NT = WK * WM * 64;
    constexpr int WTK = TK / WK, WTM = TM / WM;
    constexpr int FK = WTK / 32, FM = WTM / 32;
    constexpr int LW = (TK * 4 + NT - 1) / NT, LA = (TM * 4 + NT - 1) / NT;
    constexpr int PW = TK * 16, PA = TM * 16;  // bytes per chunk plane
    constexpr int STAGE = 4 * (PW + PA);
    static_assert(WTK % 32 == 0 && WTM % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
    static_assert((TK & (TK - 1)) == 0 && (TM & (TM - 1)) == 0, "tile extents are powers of two");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int *koff = reinterpret_cast<int *>(smem + 2 * STAGE);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wm = wave / WK;

    int lid = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int tk = lid % a.tiles_k;
    lid /= a.tiles_k;
    const int tm = lid % a.tiles_m;
    const int split = lid / a.tiles_m;
    const int k0 = tk * TK, m0 = tm * TM;
    const int ks_begin = split * a.ksteps_per_split;
    const int nks = min(a.ksteps_total - ks_begin, a.ksteps_per_split);

    if (MODE == ACT_BLOCKED) {
        for (int t = tid; t < nks * 4; t += NT) {
            const int gt = ks_begin * 4 + t;
            int off = 0;  // chunks past the real depth meet zero weights: any valid address will do
            if (gt < a.nreal) {
                const int sub = gt % a.g16, tap = gt / a.g16;
                const int s = tap % a.S, rb = tap / a.S;
                const int r = rb % a.R, b = rb / a.R;
                off = ((b * a.Hp + r) * a.Wp + s) * a.cb + sub * 16;
            }
            koff[t] = off;
        }
    }

    // Per-thread staging slots: (row, chunk) pairs, row fastest across lanes.
    const int8_t *wsrc[LW];
    int wdst[LW];
    const int8_t *asrc[LA];
    int adst[LA], achunk[LA];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int idx = tid + i * NT, row = idx % TK, chunk = (idx / TK) & 3;
        const int kk = min(k0 + row, a.K - 1);
        wsrc[i] = a.wq + (size_t)kk * a.depth + (size_t)(ks_begin * 4 + chunk) * 16;
        wdst[i] = chunk * PW + row * 16;
    }
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int idx = tid + i * NT, row = idx % TM, chunk = (idx / TM) & 3;
        const int m = min(m0 + row, a.M - 1);
        if (MODE == ACT_MATRIX) {
            asrc[i] = a.act + (size_t)m * a.depth + (size_t)(ks_begin * 4 + chunk) * 16;
        } else {
            const int n = m / a.PQ, pq = m - n * a.PQ;
            const int p = pq / a.Q, q = pq - p * a.Q;
            asrc[i] = a.act + (size_t)n * a.img_bytes +
                      ((size_t)(p * a.stride) * a.Wp + (size_t)q * a.stride) * a.cb;
        }
        achunk[i] = chunk;
        adst[i] = 4 * PW + chunk * PA + row * 16;
    }
    constexpr bool WFULL = (TK * 4) % NT == 0, AFULL = (TM * 4) % NT == 0;
    const bool wlast = WFULL || (tid + (LW - 1) * NT < TK * 4);
    const bool alast = AFULL || (tid + (LA - 1) * NT < TM * 4);

    v4i wreg[LW], areg[LA];
    auto fetch = [&](int j) {  // j = step relative to ks_begin
#pragma unroll
        for (int i = 0; i < LW; ++i)
            if (i < LW - 1 || wlast) wreg[i] = *reinterpret_cast<const v4i *>(wsrc[i] + (size_t)j * 64);
#pragma unroll
        for (int i = 0; i < LA; ++i)
            if (i < LA - 1 || alast) {
                if (MODE == ACT_MATRIX)
                    areg[i] = *reinterpret_cast<const v4i *>(asrc[i] + (size_t)j * 64);
                else
                    areg[i] = *reinterpret_cast<const v4i *>(asrc[i] + koff[j * 4 + achunk[i]]);
            }
    };
    auto stash = [&](unsigned char *st) {
#pragma unroll
        for (int i = 0; i < LW; ++i)
            if (i < LW - 1 || wlast) *reinterpret_cast<v4i *>(st + wdst[i]) = wreg[i];
#pragma unroll
        for (int i = 0; i < LA; ++i)
            if (i < LA - 1 || alast) *reinterpret_cast<v4i *>(st + adst[i]) = areg[i];
    };

    v16i acc[FK][FM];
#pragma unroll
    for (int i = 0; i < FK; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    if (MODE == ACT_BLOCKED) __syncthreads();  // koff visible
    fetch(0);
    stash(smem);
    __syncthreads();

    const int wrow = (wk * WTK + (lane & 31)) * 16;
    const int arow = 4 * PW + (wm * WTM + (lane & 31)) * 16;
    for (int j = 0; j < nks; ++j) {
        unsigned char *cur = smem + (j & 1) * STAGE;
        unsigned char *nxt = smem + ((j & 1) ^ 1) * STAGE;
        const bool more = j + 1 < nks;
        if (more) fetch(j + 1);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int plane = 2 * h + (lane >> 5);
            v4i wf[FK], af[FM];
#pragma unroll
            for (int i = 0; i < FK; ++i)
                wf[i] = *reinterpret_cast<const v4i *>(cur + plane * PW + wrow + i * 512);
#pragma unroll
            for (int i = 0; i < FM; ++i)
                af[i] = *reinterpret_cast<const v4i *>(cur + plane * PA + arow + i * 512);
#pragma unroll
            for (int i = 0; i < FK; ++i)
#pragma unroll
                for (int jm = 0; jm < FM; ++jm)
                    acc[i][jm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[i], af[jm], acc[i][jm], 0, 0, 0);
        }
        if (more) stash(nxt);
        __syncthreads();
    }

    // Epilogue: D block (i, jm): column = lane%32 (pixel), row = 8*(v/4) + 4*(lane/32) + v%4.
    // Consecutive lanes write consecutive pixels of one output plane: 128-byte runs in NKPQ.
#pragma unroll
    for (int jm = 0; jm < FM; ++jm) {
        const int m = m0 + wm * WTM + jm * 32 + (lane & 31);
        if (m >= a.M) continue;
        const int n = m / a.PQ, pq = m - n * a.PQ;
        int32_t *base = a.out + (size_t)n * a.K * a.PQ + pq;
#pragma unroll
        for (int i = 0; i < FK; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + wk * WTK + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (k < a.K) {
                    int32_t *dst = base + (size_t)k * a.PQ;
                    if (a.split_k > 1)
                        __hip_atomic_fetch_add(dst, acc[i][jm][v], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                    else
                        *dst = acc[i][jm][v];
                }
            }
        }
    }
}

// ---- tile table -----------------------------------------------------------------------
struct TileDef {
    int tk, tm, wk, wm;
};
static const TileDef kTiles[] = {
    {32, 32, 1, 1},    // 0  tiny problems
    {64, 64, 2, 2},    // 1
    {128, 128, 2, 2},  // 2
    {32, 128, 1, 4},   // 3  few output channels
    {64, 128, 2, 2},   // 4
    {64, 256, 1, 4},   // 5
    {128, 64, 2, 2},   // 6
    {256, 128, 4, 2},  // 7
    {128, 256, 2, 4},  // 8
    {256, 256, 2, 4},  // 9  steady state
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

int gemm_num_tiles() { return kNumTiles; }
TileInfo gemm_tile_info(int t)
{
    return TileInfo{kTiles[t].tk, kTiles[t].tm, kTiles[t].wk * kTiles[t].wm * 64};
}

template <int TK, int TM, int WK, int WM>
static hipError_t launch_tile(const GemmArgs &a, int mode, hipStream_t st)
{
    constexpr int NT = WK * WM * 64;
    constexpr int STAGE = 4 * (TK + TM) * 16;
    const size_t lds = 2 * (size_t)STAGE + (mode == ACT_BLOCKED ? (size_t)a.ksteps_per_split * 16 : 0);
    const int grid = a.tiles_k * a.tiles_m * a.split_k;
    auto kb = igemm_i8_kernel<TK, TM, WK, WM, ACT_BLOCKED>;
    auto km = igemm_i8_kernel<TK, TM, WK, WM, ACT_MATRIX>;
    auto kern = mode == ACT_BLOCKED ? kb : km;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, a);
    return hipGetLastError();
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Rough per-launch time model (cycles) used to pick a tile and a depth split:
// every CU runs one workgroup at a time; a workgroup's step costs the larger of its MFMA
// time and its operand-fetch time; split-K adds the atomic traffic of one more output tile.
void gemm_pick(const GemmProblem &g, int *tile, int *split_k)
{
    const int ksteps = g.depth / 64;
    static const int splits[] = {1, 2, 3, 4, 6, 8, 9, 12, 16};
    double best = 1e300;
    int bt = *tile >= 0 ? *tile : 0, bs = *split_k > 0 ? *split_k : 1;
    for (int t = 0; t < kNumTiles; ++t) {
        if (*tile >= 0 && t != *tile) continue;
        const TileDef &d = kTiles[t];
        const int waves = d.wk * d.wm;
        const double tiles = (double)ceil_div(g.K, d.tk) * ceil_div(g.M, d.tm);
        const double mfma = (double)d.tk * d.tm * 64 / (1024.0 * (waves < 4 ? waves : 4));
        const double fetch = (double)(d.tk + d.tm) * 64 / 40.0;
        const double step = mfma > fetch ? mfma : fetch;
        for (int s : splits) {
            if (*split_k > 0 && s != *split_k) continue;
            if (s > ksteps) continue;
            const int per = ceil_div(ksteps, s);
            if (ceil_div(ksteps, per) != s) continue;  // no empty slices
            const double rounds = (double)(long long)((tiles * s + 255) / 256);
            const double store = (double)d.tk * d.tm * 4 / (s > 1 ? 24.0 : 64.0);
            const double wg = 3000.0 + per * step + store;
            const double total = rounds * wg + (s > 1 ? 4000.0 : 0.0);
            if (total < best) {
                best = total;
                bt = t;
                bs = s;
            }
        }
    }
    *tile = bt;
    *split_k = bs;
}

hipError_t launch_gemm(const GemmProblem &g, int tile, int split_k, hipStream_t st)
{
    const TileDef &d = kTiles[tile];
    GemmArgs a;
    a.act = g.act;
    a.wq = g.wq;
    a.out = g.out;
    a.K = g.K;
    a.M = g.M;
    a.depth = g.depth;
    a.PQ = g.PQ;
    a.Q = g.Q;
    a.stride = g.stride;
    a.cb = g.cb;
    a.g16 = g.cb / 16;
    a.R = g.R;
    a.S = g.S;
    a.Hp = g.Hp;
    a.Wp = g.Wp;
    a.nreal = g.mode == ACT_BLOCKED ? g.Cb * g.R * g.S * (g.cb / 16) : g.depth / 16;
    a.img_bytes = (long long)g.Cb * g.Hp * g.Wp * g.cb;
    a.tiles_k = ceil_div(g.K, d.tk);
    a.tiles_m = ceil_div(g.M, d.tm);
    a.ksteps_total = g.depth / 64;
    if (split_k < 1) split_k = 1;
    if (split_k > a.ksteps_total) split_k = a.ksteps_total;
    a.ksteps_per_split = ceil_div(a.ksteps_total, split_k);
    a.split_k = ceil_div(a.ksteps_total, a.ksteps_per_split);
    if (a.split_k > 1) {
        hipError_t e = launch_fill_zero(g.out, (size_t)g.M * g.K * sizeof(int32_t), st);
        if (e != hipSuccess) return e;
    }
    switch (tile) {
        case 0: return launch_tile<32, 32, 1, 1>(a, g.mode, st);
        case 1: return launch_tile<64, 64, 2, 2>(a, g.mode, st);
        case 2: return launch_tile<128, 128, 2, 2>(a, g.mode, st);
        case 3: return launch_tile<32, 128, 1, 4>(a, g.mode, st);
        case 4: return launch_tile<64, 128, 2, 2>(a, g.mode, st);
        case 5: return launch_tile<64, 256, 1, 4>(a, g.mode, st);
        case 6: return launch_tile<128, 64, 2, 2>(a, g.mode, st);
        case 7: return launch_tile<256, 128, 4, 2>(a, g.mode, st);
        case 8: return launch_tile<128, 256, 2, 4>(a, g.mode, st);
        case 9: return launch_tile<256, 256, 2, 4>(a, g.mode, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace c2i8
