// GEMM stage of the convolution: out[k][m] = sum_j wq[k][j] * act(m)[j] on the CDNA4 int8
// MFMA (v_mfma_i32_32x32x32_i8), the counterpart of the paper's VTA GEMM core
// C[x][y] += A[x][z] * B[y][z] (Sec. 5.1) with x = output channel, y = output pixel,
// z = fused reduction depth.  Both operands are depth-contiguous, which is exactly what
// the layout rewrites (Table 2) produce.
//
// Workgroup = TK output channels x TM output pixels; depth is walked in 64-byte steps.
// Each step's TK x 64 B weight tile and TM x 64 B activation tile travel global -> LDS
// directly (global_load_lds_dwordx4: no register staging) into a ring of NSTAGE stages, so
// NSTAGE-1 steps of operand traffic are in flight while one step is multiplied; that depth,
// not occupancy, is what hides the L2/HBM latency of these small problems.  One wave
// instruction moves 16 rows x 64 B: four lanes fetch one row's 64 contiguous bytes and the
// data lands lane-contiguous in LDS.  Which 16-byte chunk of the row a lane fetches is
// XOR-swizzled with the row index, so the MFMA operand reads (32 consecutive rows of one
// chunk per half-wave, 16 bytes per lane) touch every LDS bank group equally.
//
// The activation row of pixel m is addressed as rowbase(m) + koff[chunk]: for the blocked
// layout koff walks (channel block, r, s) over the zero-padded image (implicit GEMM, no
// unrolled matrix in memory); for a row-major matrix (im2col output) it is 16*chunk.
#include "act_requant.h"
#include "kernels.h"

#include <type_traits>

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
    int out_fits_32bit;  // every output byte offset is below 2^32
    int m_fastest;       // tile order inside an XCD
    unsigned mg_g16, mg_S, mg_R, mg_PQ, mg_Q, mg_tiles_k, mg_tiles_m;  // ceil(2^32 / d), 0 for d == 1
    // Activation fused into the epilogue (null: the int32 result goes to `out`): the next layer's
    // channel-blocked input [N][o_Cb][o_Hp][o_Wp][1 << o_cb_log2], int8.
    int8_t *act_out;
    int act_shift, act_relu, o_cb_log2, o_pad, o_Hp, o_Wp, o_Cb;
    // Interleaving epilogue (il_d >= 2): the problem is the dense convolution on the il_d^2 sub-images of a
    // dilated layer (image n2 = (n*il_d + a)*il_d + b); result pixel (i, j) of it is pixel
    // (il_d*i + a, il_d*j + b) of image n in `out` [.][K][il_P][il_Q], or nothing if that lies outside.
    int il_d, il_P, il_Q;
    unsigned mg_il_dd, mg_il_d;
    int dil;  // ACT_BLOCKED: distance between kernel taps in the padded image (1 = dense kernel)
    int out_nhwc;  // `out` is [N][P][Q][K] instead of [N][K][P][Q]
    int grp_m;     // > 0: tile order in groups of grp_m pixel tiles (below); 0: one of the two row-major orders
    unsigned mg_grp_sz, mg_grp_m, mg_tiles_km;  // ceil(2^32 / d) for grp_m * tiles_k, grp_m, tiles_k * tiles_m
    int stagger;   // start offsets of the first round of workgroups: this many 64-cycle units per phase step (0: none)
};

// n / d for 0 <= n < 2^31 with magic = ceil(2^32 / d) truncated to 32 bits (0 encodes d == 1):
// the multiply-high estimate is never low and at most one too high.
__device__ __forceinline__ int div_magic(int n, int d, unsigned magic)
{
    int q = magic ? (int)__umulhi((unsigned)n, magic) : n;
    if ((long long)q * d > n) --q;
    return q;
}

// Workgroups are dealt round-robin over the 8 XCDs (each with its own L2); give every XCD
// a contiguous range of logical tile ids so that neighbours in tile order share an L2.
__device__ __forceinline__ int xcd_contiguous_id(int id, int n)
{
    const int x = id & 7, q = n >> 3, rem = n & 7;
    return x * q + (x < rem ? x : rem) + (id >> 3);
}

// 16 bytes per lane from `src` (per-lane address) to LDS byte address lds_base + 16*lane
// (lds_base wave-uniform).  Completion is tracked by vmcnt; the compiler does not see the
// LDS write, hence the explicit waits below.
__device__ __forceinline__ void dma16(const int8_t *src, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_base), "v"(src)
                 : "memory");
}
template <int N>
__device__ __forceinline__ void wait_dma_outstanding()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
// All LDS reads of this wave have returned, then the workgroup barrier.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" : : : "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0), vmcnt and expcnt untouched
    __builtin_amdgcn_s_barrier();
    asm volatile("" : : : "memory");
}

// How many of the transfer slots u*nq/l + off (u < l) come before slot qb.
constexpr int slots_before(int l, int nq, int off, int qb)
{
    int n = 0;
    for (int u = 0; u < l; ++u) n += (u * nq / l + off < qb) ? 1 : 0;
    return n;
}

// HELP extra waves per workgroup only move operands (they issue their share of the transfers
// and keep the barriers, no MFMA): a wave moves about 1 KB per 140-180 cycles through the
// global->LDS path whatever the queue depth, so small tiles, whose four MFMA waves would be
// starved at ~25 B/clk per CU, are fed by eight issuing waves instead.
//
// DS = 2 (small wave tiles only) runs two groups of WK x WM multiplying waves on the same
// output tile, each on its half of every stage's depth; the second group's accumulators are
// added to the first's through LDS before the epilogue.  A 32x32 wave tile reads 4 KB of LDS
// per 64 MFMA cycles, and four waves alone reach only ~100 B/clk of LDS bandwidth where eight
// reach ~190: the second group doubles what a small tile can multiply per cycle.
//
// WPC > 1 caps the registers so that WPC workgroups fit one CU: while one of them waits at a
// barrier or drains its output tile, the matrix pipe works for the other.
//
// The body is a device function of (logical workgroup id, workgroup count, LDS base).
template <int TK, int TM, int WK, int WM, int KS, int NSTAGE, int HELP, int DS, int MODE>
__device__ __forceinline__ void igemm_body(const GemmArgs &a, int block_id, int nblocks, unsigned char *smem)
{
    constexpr int NWM = WK * WM;           // waves of one multiplying group
    constexpr int NWC = NWM * DS;          // waves that multiply
    constexpr int NW = NWC + HELP, NT = NW * 64;  // waves that transfer (all of them)
    constexpr int WTK = TK / WK, WTM = TM / WM;
    constexpr int FK = WTK / 32, FM = WTM / 32;
    // A ring stage holds KS depth steps: RP bytes of every row.  One transfer instruction
    // moves RPI rows x RP bytes (LPR lanes per row); with KS = 2 a row piece is one whole
    // 128-byte cache line.
    constexpr int RP = 64 * KS, LPR = 4 * KS, RPI = 64 / LPR;
    constexpr int LW = TK / RPI / NW, LA = TM / RPI / NW;  // transfers per wave and stage
    constexpr int L = LW + LA;
    constexpr int WBYTES = TK * RP, STAGE = (TK + TM) * RP;
    constexpr int NH = 2 * KS;  // 32-deep halves per stage
    static_assert(KS == 1 || KS == 2 || KS == 4, "64, 128 or 256 bytes of depth per stage");
    static_assert(DS == 1 || (DS == 2 && (TK / WK / 32) * (TM / WM / 32) <= 2), "depth groups: small wave tiles only");
    static_assert(WTK % 32 == 0 && WTM % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
    static_assert((TK / RPI) % NW == 0 && (TM / RPI) % NW == 0, "transfers divide evenly over waves");
    static_assert(KS == 1 || (KS == 2 && NW % 2 == 0) || (KS == 4 && NW % 4 == 0),
                  "row swizzle of a transfer must not depend on its slot");
    static_assert(NSTAGE >= 2 && (NSTAGE - 1) * L <= 63, "vmcnt is a 6-bit counter");

    int *koff = reinterpret_cast<int *>(smem + NSTAGE * STAGE);
    const unsigned lds0 =
        (unsigned)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = DS == 1 ? 0 : wave / NWM;  // depth group of this wave
    const int wk = (wave % NWM) % WK, wm = (wave % NWM) / WK;

    // The workgroups of one round finish together, and so do their output tiles: every compute unit then
    // writes at once, the memory system takes the tiles in turn and the matrix pipes idle meanwhile.  In a
    // launch of many rounds the first round therefore starts at 32 different offsets (one per compute unit
    // of an XCD; ids are dealt round-robin over the XCDs), which spreads the writes of every later round too.
    if (a.stagger && block_id < 256)
        for (int z = ((block_id >> 3) & 31) * a.stagger; z >= 16; z -= 16) __builtin_amdgcn_s_sleep(16);

    int lid = xcd_contiguous_id(block_id, nblocks);
    int tk, tm;
    if (a.grp_m) {
        // Groups of grp_m pixel tiles, each crossed with every channel tile; inside a group the pixel tiles run
        // fastest.  The 32 tiles an XCD works on at a time then form a grp_m x 32/grp_m block of the tile grid and
        // share grp_m + 32/grp_m operand panels instead of 33 (a row of the grid): what its L2 must hold and pull in.
        const int per = a.tiles_k * a.tiles_m, split_id = div_magic(lid, per, a.mg_tiles_km), r = lid - split_id * per;
        const int gsz = a.grp_m * a.tiles_k, g = div_magic(r, gsz, a.mg_grp_sz), j = r - g * gsz;
        const int gm = min(a.grp_m, a.tiles_m - g * a.grp_m);   // the last group may be narrower
        tk = gm == a.grp_m ? div_magic(j, a.grp_m, a.mg_grp_m) : j / gm;
        tm = g * a.grp_m + j - tk * gm;
        lid = split_id;
    } else if (a.m_fastest) {  // consecutive tiles share a weight tile (few output channels per XCD)
        const int q1 = div_magic(lid, a.tiles_m, a.mg_tiles_m);
        tm = lid - q1 * a.tiles_m;
        lid = div_magic(q1, a.tiles_k, a.mg_tiles_k);
        tk = q1 - lid * a.tiles_k;
    } else {            // consecutive tiles share an activation tile
        const int q1 = div_magic(lid, a.tiles_k, a.mg_tiles_k);
        tk = lid - q1 * a.tiles_k;
        lid = div_magic(q1, a.tiles_m, a.mg_tiles_m);
        tm = q1 - lid * a.tiles_m;
    }
    const int split = lid;
    const int k0 = tk * TK, m0 = tm * TM;
    const int ks_begin = split * a.ksteps_per_split;
    const int nks = min(a.ksteps_total - ks_begin, a.ksteps_per_split);
    const int ns = nks / KS;  // stages; the host only picks KS = 2 for an even step count

    if (MODE == ACT_BLOCKED) {
        for (int t = tid; t < nks * 4; t += NT) {
            const int gt = ks_begin * 4 + t;
            int off = 0;  // chunks past the real depth meet zero weights: any valid address will do
            if (gt < a.nreal) {
                const int tap = div_magic(gt, a.g16, a.mg_g16), sub = gt - tap * a.g16;
                const int rb = div_magic(tap, a.S, a.mg_S), s = tap - rb * a.S;
                const int b = div_magic(rb, a.R, a.mg_R), r = rb - b * a.R;
                off = ((b * a.Hp + r * a.dil) * a.Wp + s * a.dil) * a.cb + sub * 16;  // tap (r, s), taps dil apart
            }
            koff[t] = off;
        }
    }

    // Transfer slots.  Slot i of this wave moves rows g*RPI .. g*RPI+RPI-1 (g = i*NW + wave)
    // of the weight (or activation) tile.  Lane l fetches row g*RPI + l/LPR and lands at 16-byte
    // position l%LPR of that row in LDS; the chunk it fetches is that position XOR a few row
    // bits (KS = 1: (row/4)%4, KS = 2: (row/2)%8, KS = 4: row%16), which is what spreads the later
    // column-wise MFMA operand reads over all LDS banks.
    const int lrow = lane / LPR;
    const int x = KS == 1   ? ((lane & 3) ^ ((lane >> 4) & 3))
                  : KS == 2 ? ((lane & 7) ^ (((wave & 1) << 2) | (lane >> 4)))
                            : ((lane & 15) ^ (((wave & 3) << 2) | (lane >> 4)));
    const int8_t *wsrc[LW];
    const int8_t *asrc[LA];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int row = (i * NW + wave) * RPI + lrow;
        const int kk = min(k0 + row, a.K - 1);
        wsrc[i] = a.wq + (size_t)kk * a.depth + (size_t)ks_begin * 64 + x * 16;
    }
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = (i * NW + wave) * RPI + lrow;
        const int m = min(m0 + row, a.M - 1);
        if (MODE == ACT_MATRIX) {
            asrc[i] = a.act + (size_t)m * a.depth + (size_t)ks_begin * 64 + x * 16;
        } else {
            const int n = div_magic(m, a.PQ, a.mg_PQ), pq = m - n * a.PQ;
            const int p = div_magic(pq, a.Q, a.mg_Q), q = pq - p * a.Q;
            asrc[i] = a.act + (size_t)n * a.img_bytes +
                      ((size_t)(p * a.stride) * a.Wp + (size_t)q * a.stride) * a.cb;
        }
    }
    // One transfer of stage j (t < LW: weight rows, else activation rows) into ring slot `st`.
    auto dma_item = [&](int t, int j, unsigned st, size_t aoff) {
        if (t < LW) dma16(wsrc[t] + (size_t)j * RP, st + t * NW * 1024);
        else dma16(asrc[t - LW] + aoff, st + WBYTES + (t - LW) * NW * 1024);
    };
    auto stage_aoff = [&](int j) -> size_t {
        if (MODE == ACT_BLOCKED) return (size_t)koff[j * LPR + x];
        return (size_t)j * RP;
    };

    v16i acc[FK][FM];
#pragma unroll
    for (int i = 0; i < FK; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // Transfers issued back to back stall the issuing wave (one instruction occupies it for
    // well over a hundred cycles), and with them its MFMAs.  Large wave tiles therefore spread
    // the transfers of one stage over all the MFMAs of a stage (SPREAD): stage j+NSTAGE-1 is
    // fetched, one transfer every few MFMAs, while stage j is multiplied, into the ring slot
    // that stage j-1 left; the prologue then fills only NSTAGE-1 slots.
    constexpr bool SPREAD = NSTAGE >= 3 && HELP == 0 && (WTK / 32) * (WTM / 32) > 2;
    constexpr int PRO = SPREAD ? NSTAGE - 1 : NSTAGE;  // stages fetched before the loop

    if (MODE == ACT_BLOCKED) __syncthreads();  // koff visible
#pragma unroll
    for (int j = 0; j < PRO; ++j)
        if (j < ns) {
            const unsigned st = lds0 + (unsigned)j * STAGE + (unsigned)wave * 1024u;
            const size_t aoff = stage_aoff(j);
#pragma unroll
            for (int t = 0; t < L; ++t) dma_item(t, j, st, aoff);
        }

    if (HELP > 0 && wave >= NWC) {
        // transfer-only wave: same waits, barriers and refills as the multiplying waves
        if (NSTAGE <= ns) wait_dma_outstanding<(NSTAGE - 1) * L>();
        else wait_dma_outstanding<0>();
        lds_barrier();
        for (int j = 0; j < ns; ++j) {
            const int jn = j + NSTAGE;
            const bool refill = jn < ns;
            if (refill) wait_dma_outstanding<(NSTAGE - 2) * L>();
            else wait_dma_outstanding<0>();
            lds_barrier();
            if (refill) {
                const unsigned st = lds0 + (unsigned)(j % NSTAGE) * STAGE + (unsigned)wave * 1024u;
                const size_t aoff = stage_aoff(jn);
#pragma unroll
                for (int t = 0; t < L; ++t) dma_item(t, jn, st, aoff);
            }
        }
        return;
    }

    // MFMA operand reads: lane l takes row (l%32) of a 32-row block; half h of a stage is
    // chunk 4*(h/2) + 2*(h%2) + l/32 of that row, at its swizzled position.
    const int rswz = KS == 1 ? ((lane >> 2) & 3) : KS == 2 ? ((lane >> 1) & 7) : (lane & 15);
    const int wrow = (wk * WTK + (lane & 31)) * RP;
    const int arow = WBYTES + (wm * WTM + (lane & 31)) * RP;
    int coff[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) coff[h] = (((h >> 1) * 4 + 2 * (h & 1) + (lane >> 5)) ^ rswz) << 4;
    // One fragment read, in the order the MFMAs of a half (g = i*FM + j) first need them:
    // weight block 0, every activation block, then the remaining weight blocks.
    auto read_item = [&](int t, const unsigned char *st, int co, v4i(&wf)[FK], v4i(&af)[FM]) {
        if (t == 0) wf[0] = *reinterpret_cast<const v4i *>(st + wrow + co);
        else if (t <= FM) af[t - 1] = *reinterpret_cast<const v4i *>(st + arow + (t - 1) * 32 * RP + co);
        else wf[t - FM] = *reinterpret_cast<const v4i *>(st + wrow + (t - FM) * 32 * RP + co);
    };
    constexpr int NM = FK * FM, NR = FK + FM;
    // Read t of the next half is issued right after MFMA read_slot(t) of this one: as early as
    // the MFMA count allows, so that the last of them has landed when the next half begins.
    auto read_slot = [](int t) constexpr { return NR > NM ? (t > NR - NM ? t - (NR - NM) : 0) : t; };

    if constexpr (FK * FM <= 2) {
        // Small wave tiles: one or two MFMAs per 32-deep half cannot cover an LDS read, so the
        // fragments of a whole stage are read one stage ahead (two register sets), and the
        // halves alternate between two accumulators to halve the dependent MFMA chain.
        constexpr int NHG = NH / DS;   // halves of a stage this wave multiplies
        const int h0 = grp * NHG;      // ... starting at this one
        v4i wq[2][NHG][FK], aq[2][NHG][FM];
        v16i acc2[FK][FM];
#pragma unroll
        for (int i = 0; i < FK; ++i)
#pragma unroll
            for (int j = 0; j < FM; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[i][j][v] = 0;
        int co[NHG];
#pragma unroll
        for (int h = 0; h < NHG; ++h) co[h] = DS == 1 ? coff[h] : (grp ? coff[(NHG + h) % NH] : coff[h]);
        (void)h0;
        if (NSTAGE <= ns) wait_dma_outstanding<(NSTAGE - 1) * L>();
        else wait_dma_outstanding<0>();
        lds_barrier();
#pragma unroll
        for (int h = 0; h < NHG; ++h)
#pragma unroll
            for (int t = 0; t < NR; ++t) read_item(t, smem, co[h], wq[0][h], aq[0][h]);
        for (int j = 0; j < ns; j += 2) {
#pragma unroll
            for (int par = 0; par < 2; ++par) {  // stage j + par multiplies set `par`
                const int jj = j + par;
                if (jj < ns) {
                    const int jn = jj + NSTAGE;
                    const bool refill = jn < ns;
                    if (refill) wait_dma_outstanding<(NSTAGE - 2) * L>();
                    else wait_dma_outstanding<0>();
                    lds_barrier();  // stage jj+1 has landed; everyone holds stage jj in registers
                    if (refill) {
                        const unsigned st = lds0 + (unsigned)(jj % NSTAGE) * STAGE + (unsigned)wave * 1024u;
                        const size_t aoff = stage_aoff(jn);
#pragma unroll
                        for (int t = 0; t < L; ++t) dma_item(t, jn, st, aoff);
                    }
                    // (after the last stage this reads a stale slot; the values are never used)
                    const unsigned char *nxt = smem + ((jj + 1) % NSTAGE) * STAGE;
#pragma unroll
                    for (int h = 0; h < NHG; ++h)
#pragma unroll
                        for (int t = 0; t < NR; ++t) read_item(t, nxt, co[h], wq[par ^ 1][h], aq[par ^ 1][h]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int h = 0; h < NHG; ++h)
#pragma unroll
                        for (int g = 0; g < NM; ++g) {
                            if (h & 1)
                                acc2[g / FM][g % FM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                    wq[par][h][g / FM], aq[par][h][g % FM], acc2[g / FM][g % FM], 0, 0, 0);
                            else
                                acc[g / FM][g % FM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                    wq[par][h][g / FM], aq[par][h][g % FM], acc[g / FM][g % FM], 0, 0, 0);
                        }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < FK; ++i)
#pragma unroll
            for (int j = 0; j < FM; ++j) acc[i][j] += acc2[i][j];
        if constexpr (DS == 2) {
            // second group -> LDS -> first group (the ring is idle: every transfer has landed
            // and, after this barrier, every fragment read has returned)
            lds_barrier();
            v4i *xch = reinterpret_cast<v4i *>(smem) + (wave % NWM) * NM * 256;
            if (grp == 1) {
#pragma unroll
                for (int g = 0; g < NM; ++g)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        v4i t;
#pragma unroll
                        for (int e = 0; e < 4; ++e) t[e] = acc[g / FM][g % FM][4 * q4 + e];
                        xch[(g * 4 + q4) * 64 + lane] = t;
                    }
            }
            lds_barrier();
            if (grp == 1) return;
#pragma unroll
            for (int g = 0; g < NM; ++g)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const v4i t = xch[(g * 4 + q4) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[g / FM][g % FM][4 * q4 + e] += t[e];
                }
        }
    } else if constexpr (SPREAD) {
        // Software pipeline, transfers spread.  Slot q = h*NM + g of a stage is one MFMA plus its
        // side work: a share of the fragment reads of the next half, and transfer u of stage
        // j+NSTAGE-1 when u*NQ/L == q.  The barrier sits after the first MFMA of the last half:
        // by then every wave holds the last fragments of stage j in registers (its ring slot is
        // free for iteration j+1 to refill) and stage j+1 has landed.
        // The two waves that share a SIMD (w and w + 4) take their transfer slots half a
        // spacing apart, so that one of them can always feed the matrix pipe.
        constexpr int NQ = NH * NM, QB = (NH - 1) * NM;
        constexpr int OFF = NW > 4 ? NQ / L / 2 : 0;
        constexpr int DB = slots_before(L, NQ, 0, QB);  // transfers of an iteration issued before its barrier
        static_assert(slots_before(L, NQ, OFF, QB) == DB, "both wave groups issue the same count before the barrier");
        const bool late = OFF > 0 && ((wave >> 2) & 1);
        v4i wf[2][FK], af[2][FM];
        if (PRO <= ns) wait_dma_outstanding<(PRO - 1) * L>();
        else wait_dma_outstanding<0>();
        lds_barrier();
#pragma unroll
        for (int t = 0; t < NR; ++t) read_item(t, smem, coff[0], wf[0], af[0]);

        for (int j = 0; j < ns; ++j) {
            const unsigned char *cur = smem + (j % NSTAGE) * STAGE;
            const unsigned char *nxt = smem + ((j + 1) % NSTAGE) * STAGE;
            const int jn = j + NSTAGE - 1;
            const bool refill = jn < ns;  // uniform
            const unsigned st = lds0 + (unsigned)(jn % NSTAGE) * STAGE + (unsigned)wave * 1024u;
            size_t aoff = 0;
            if (refill) aoff = stage_aoff(jn);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
#pragma unroll
                for (int g = 0; g < NM; ++g) {
                    const int q = h * NM + g;
                    acc[g / FM][g % FM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                        wf[h & 1][g / FM], af[h & 1][g % FM], acc[g / FM][g % FM], 0, 0, 0);
                    if (q == QB) {
                        // stage j+1 landed: everything issued after it may still be in flight
                        if (refill) wait_dma_outstanding<(NSTAGE - 3) * L + DB>();
                        else wait_dma_outstanding<0>();
                        lds_barrier();
                    }
#pragma unroll
                    for (int u = 0; u < L; ++u) {
                        if (u * NQ / L == q && refill && !late) dma_item(u, jn, st, aoff);
                        if (OFF > 0 && u * NQ / L + OFF == q && refill && late) dma_item(u, jn, st, aoff);
                    }
                    // (after the last stage the reads hit a stale slot; the values are never used)
#pragma unroll
                    for (int u = 0; u < NR; ++u)
                        if (read_slot(u) == g)
                            read_item(u, h == NH - 1 ? nxt : cur, coff[(h + 1) % NH], wf[(h + 1) & 1], af[(h + 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    } else {
        // Software pipeline.  The matrix pipe idles whenever a wave does anything else for long,
        // so every LDS fragment read, every transfer and every address update is slotted between
        // two MFMAs (an MFMA runs for 32 cycles after issue; the side work issues underneath it),
        // and the order is pinned.  Fragment sets alternate: half h multiplies set h%2 while the
        // reads of half h+1 fill the other set.  The last half of a stage also holds the barrier
        // (everyone has read the stage: its ring slot is free; the next stage has landed), the
        // transfers of stage j+NSTAGE into the freed slot, and the first reads of stage j+1.
        v4i wf[2][FK], af[2][FM];
        if (NSTAGE <= ns) wait_dma_outstanding<(NSTAGE - 1) * L>();
        else wait_dma_outstanding<0>();
        lds_barrier();
    #pragma unroll
        for (int t = 0; t < NR; ++t) read_item(t, smem, coff[0], wf[0], af[0]);

        for (int j = 0; j < ns; ++j) {
            const unsigned char *cur = smem + (j % NSTAGE) * STAGE;
    #pragma unroll
            for (int h = 0; h < NH - 1; ++h) {
    #pragma unroll
                for (int g = 0; g < NM; ++g) {
                    acc[g / FM][g % FM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                        wf[h & 1][g / FM], af[h & 1][g % FM], acc[g / FM][g % FM], 0, 0, 0);
    #pragma unroll
                    for (int u = 0; u < NR; ++u)
                        if (read_slot(u) == g) read_item(u, cur, coff[h + 1], wf[(h + 1) & 1], af[(h + 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }

            const int jn = j + NSTAGE;
            const bool refill = jn < ns;  // uniform
            const unsigned st = lds0 + (unsigned)(j % NSTAGE) * STAGE + (unsigned)wave * 1024u;
            const unsigned char *nxt = smem + ((j + 1) % NSTAGE) * STAGE;
            size_t aoff = 0;
            if (refill) aoff = stage_aoff(jn);
    #pragma unroll
            for (int g = 0; g < NM; ++g) {
                acc[g / FM][g % FM] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                    wf[1][g / FM], af[1][g % FM], acc[g / FM][g % FM], 0, 0, 0);
                if (g == 0) {
                    if (refill) wait_dma_outstanding<(NSTAGE - 2) * L>();
                    else wait_dma_outstanding<0>();
                    lds_barrier();
                }
                // side items of the last half: the first reads of stage j+1 (after the last stage
                // they hit a stale slot; the values are never used) and the transfers
    #pragma unroll
                for (int u = 0; u < NR; ++u)
                    if (read_slot(u) == g) read_item(u, nxt, coff[0], wf[0], af[0]);
    #pragma unroll
                for (int u = g * L / NM; u < (g + 1) * L / NM; ++u)
                    if (refill) dma_item(u, jn, st, aoff);
                __builtin_amdgcn_sched_barrier(0);
            }
        }

    }

    // Epilogue: D block (i, jm): column = lane%32 (pixel), row = 8*(v/4) + 4*(lane/32) + v%4.
    // Consecutive lanes write consecutive pixels of one output plane: 128-byte runs in NKPQ.
    if (a.act_out) {
        // Fused activation: the four values v%4 of a lane are four consecutive output channels of one
        // pixel -- one dword of that pixel's channel-contiguous run in the next layer's blocked input.
        const int o_cb = 1 << a.o_cb_log2;
#pragma unroll
        for (int jm = 0; jm < FM; ++jm) {
            const int m = m0 + wm * WTM + jm * 32 + (lane & 31);
            if (m >= a.M) continue;
            const int n = div_magic(m, a.PQ, a.mg_PQ), pq = m - n * a.PQ;
            const int p = div_magic(pq, a.Q, a.mg_Q), q = pq - p * a.Q;
            const size_t pix = (size_t)(p + a.o_pad) * a.o_Wp + q + a.o_pad;
            const size_t plane = (size_t)a.o_Hp * a.o_Wp;
#pragma unroll
            for (int i = 0; i < FK; ++i) {
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int k = k0 + wk * WTK + i * 32 + 8 * vg + 4 * (lane >> 5);
                    if (k >= a.K) continue;
                    int y[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) y[t] = act_requant(acc[i][jm][4 * vg + t], a.act_shift, a.act_relu);
                    int8_t *dst = a.act_out + ((((size_t)n * a.o_Cb + (k >> a.o_cb_log2)) * plane + pix) << a.o_cb_log2) +
                                  (k & (o_cb - 1));
                    if (k + 3 < a.K)
                        *reinterpret_cast<unsigned *>(dst) = (unsigned)(y[0] & 0xFF) | (unsigned)(y[1] & 0xFF) << 8 |
                                                             (unsigned)(y[2] & 0xFF) << 16 | (unsigned)(y[3] & 0xFF) << 24;
                    else
                        for (int t = 0; t < 4; ++t)
                            if (k + t < a.K) dst[t] = (int8_t)y[t];
                }
            }
        }
        return;
    }
    if (a.out_nhwc) {
        // NHWC result: the four values v%4 of a lane are four consecutive channels of one pixel, 16 bytes of
        // that pixel's channel run (aligned when K % 4 == 0; a depth split adds them one by one)
#pragma unroll
        for (int jm = 0; jm < FM; ++jm) {
            const int m = m0 + wm * WTM + jm * 32 + (lane & 31);
            if (m >= a.M) continue;
            int32_t *pix = a.out + (size_t)m * a.K;
#pragma unroll
            for (int i = 0; i < FK; ++i) {
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int k = k0 + wk * WTK + i * 32 + 8 * vg + 4 * (lane >> 5);
                    if (k >= a.K) continue;
                    if (a.split_k > 1) {
                        for (int t = 0; t < 4; ++t)
                            if (k + t < a.K)
                                __hip_atomic_fetch_add(pix + k + t, acc[i][jm][4 * vg + t], __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                    } else if (k + 3 < a.K && (a.K & 3) == 0) {
                        *reinterpret_cast<v4i *>(pix + k) =
                            v4i{acc[i][jm][4 * vg], acc[i][jm][4 * vg + 1], acc[i][jm][4 * vg + 2], acc[i][jm][4 * vg + 3]};
                    } else {
                        for (int t = 0; t < 4; ++t)
                            if (k + t < a.K) pix[k + t] = acc[i][jm][4 * vg + t];
                    }
                }
            }
        }
        return;
    }
    if (a.il_d) {
        const size_t il_PQ = (size_t)a.il_P * a.il_Q;
#pragma unroll
        for (int jm = 0; jm < FM; ++jm) {
            const int m = m0 + wm * WTM + jm * 32 + (lane & 31);
            if (m >= a.M) continue;
            const int n2 = div_magic(m, a.PQ, a.mg_PQ), pq = m - n2 * a.PQ;
            const int si = div_magic(pq, a.Q, a.mg_Q), sj = pq - si * a.Q;
            const int dd = a.il_d * a.il_d;
            const int n = div_magic(n2, dd, a.mg_il_dd), ab = n2 - n * dd;
            const int pa = div_magic(ab, a.il_d, a.mg_il_d), pb = ab - pa * a.il_d;
            const int p = a.il_d * si + pa, q = a.il_d * sj + pb;
            if (p >= a.il_P || q >= a.il_Q) continue;   // a sub-image row or column past the real output
            int32_t *base = a.out + (size_t)n * a.K * il_PQ + (size_t)p * a.il_Q + q;
#pragma unroll
            for (int i = 0; i < FK; ++i) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = k0 + wk * WTK + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    if (k < a.K) base[(size_t)k * il_PQ] = acc[i][jm][v];
                }
            }
        }
        return;
    }
    const bool interior = a.out_fits_32bit && k0 + TK <= a.K && m0 + TM <= a.M;
    if (interior) {
        // Whole tile in range: address = uniform row base (scalar registers, advanced by whole
        // output rows) + one 32-bit per-lane offset per column block; no per-element tests.
        const size_t rowbytes = (size_t)a.PQ * sizeof(int32_t);
        char *const obase = reinterpret_cast<char *>(a.out);
        auto write_tile = [&](auto atomic) {
#pragma unroll
            for (int jm = 0; jm < FM; ++jm) {
                const int m = m0 + wm * WTM + jm * 32 + (lane & 31);
                const int n = div_magic(m, a.PQ, a.mg_PQ), pq = m - n * a.PQ;
                const unsigned lane_off =
                    ((unsigned)n * a.K * a.PQ + pq + (unsigned)(k0 + wk * WTK + 4 * (lane >> 5)) * a.PQ) * 4u;
#pragma unroll
                for (int i = 0; i < FK; ++i) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        char *urow = obase + (size_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * rowbytes;
                        int32_t *dst = reinterpret_cast<int32_t *>(urow + lane_off);
                        if (decltype(atomic)::value)
                            __hip_atomic_fetch_add(dst, acc[i][jm][v], __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                        else
                            *dst = acc[i][jm][v];
                    }
                }
            }
        };
        if (a.split_k > 1) write_tile(std::true_type{});
        else write_tile(std::false_type{});
        return;
    }
#pragma unroll
    for (int jm = 0; jm < FM; ++jm) {
        const int m = m0 + wm * WTM + jm * 32 + (lane & 31);
        if (m >= a.M) continue;
        const int n = div_magic(m, a.PQ, a.mg_PQ), pq = m - n * a.PQ;
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

template <int TK, int TM, int WK, int WM, int KS, int NSTAGE, int HELP, int DS, int WPC, int MODE>
__global__ void __launch_bounds__((WK * WM * DS + HELP) * 64, (WK * WM * DS + HELP + 3) / 4 * WPC)
    igemm_i8_kernel(const GemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    igemm_body<TK, TM, WK, WM, KS, NSTAGE, HELP, DS, MODE>(a, blockIdx.x, gridDim.x, smem);
}

// ---- tile table -----------------------------------------------------------------------
struct TileDef {
    int tk, tm, wk, wm, ks, nstage, help, ds, wpc;
};
// One row per kernel instantiation: TK, TM, WK, WM, KS, NSTAGE, HELP, DS, WPC.  The table the picker reads and
// the launch switch are both generated from this list, so a tile index means the same thing in both.
#define C2I8_TILE_LIST(X) \
    X(32, 32, 1, 1, 1, 8, 0, 1, 1) /* 0 */ \
    X(64, 64, 2, 2, 1, 8, 0, 1, 1) /* 1 */ \
    X(128, 128, 2, 2, 1, 6, 0, 1, 1) /* 2 */ \
    X(32, 128, 1, 2, 1, 8, 0, 1, 1) /* 3 */ \
    X(64, 128, 2, 2, 1, 8, 0, 1, 1) /* 4 */ \
    X(64, 256, 1, 4, 1, 6, 0, 1, 1) /* 5 */ \
    X(128, 64, 2, 2, 1, 8, 0, 1, 1) /* 6 */ \
    X(256, 128, 2, 2, 1, 5, 0, 1, 1) /* 7 */ \
    X(128, 256, 2, 2, 1, 5, 0, 1, 1) /* 8 */ \
    X(256, 256, 2, 2, 1, 4, 0, 1, 1) /* 9 */ \
    X(256, 128, 2, 2, 1, 3, 0, 1, 1) /* 10 */ \
    X(128, 256, 2, 2, 1, 3, 0, 1, 1) /* 11 */ \
    X(128, 128, 2, 2, 1, 4, 0, 1, 1) /* 12 */ \
    X(256, 256, 2, 4, 2, 2, 0, 1, 1) /* 13 */ \
    X(256, 256, 2, 2, 2, 2, 0, 1, 1) /* 14 */ \
    X(256, 128, 2, 2, 2, 3, 0, 1, 1) /* 15 */ \
    X(128, 128, 2, 2, 2, 4, 0, 1, 1) /* 16 */ \
    X(64, 64, 2, 2, 2, 4, 0, 1, 1) /* 17 */ \
    X(64, 64, 2, 2, 2, 6, 0, 1, 1) /* 18 */ \
    X(32, 64, 1, 2, 2, 6, 0, 1, 1) /* 19 */ \
    X(64, 128, 2, 2, 2, 4, 0, 1, 1) /* 20 */ \
    X(64, 64, 2, 2, 2, 4, 4, 1, 1) /* 21 */ \
    X(64, 64, 2, 2, 2, 8, 4, 1, 1) /* 22 */ \
    X(128, 128, 2, 2, 2, 4, 4, 1, 1) /* 23 */ \
    X(64, 128, 2, 2, 2, 4, 4, 1, 1) /* 24 */ \
    X(128, 64, 2, 2, 2, 4, 4, 1, 1) /* 25 */ \
    X(256, 128, 2, 2, 2, 3, 4, 1, 1) /* 26 */ \
    X(128, 256, 2, 2, 2, 3, 4, 1, 1) /* 27 */ \
    X(64, 64, 2, 2, 2, 4, 0, 2, 1) /* 28 */ \
    X(64, 64, 2, 2, 2, 6, 0, 2, 1) /* 29 */ \
    X(64, 128, 2, 2, 2, 4, 0, 2, 1) /* 30 */ \
    X(128, 64, 2, 2, 2, 4, 0, 2, 1) /* 31 */ \
    X(32, 64, 1, 2, 2, 6, 0, 2, 1) /* 32 */ \
    X(32, 32, 1, 1, 2, 8, 0, 2, 1) /* 33 */ \
    X(128, 256, 2, 4, 1, 3, 0, 1, 2) /* 34 */ \
    X(256, 128, 4, 2, 1, 3, 0, 1, 2) /* 35 */ \
    X(128, 128, 2, 2, 1, 4, 0, 1, 2) /* 36 */ \
    X(128, 128, 2, 2, 2, 2, 0, 1, 2) /* 37 */ \
    X(256, 256, 2, 4, 1, 4, 0, 1, 1) /* 38 */ \
    X(256, 256, 4, 2, 1, 4, 0, 1, 1) /* 39 */ \
    X(256, 256, 2, 4, 1, 3, 0, 1, 1) /* 40 */ \
    X(64, 64, 2, 2, 4, 4, 4, 1, 1) /* 41 */ \
    X(64, 64, 2, 2, 4, 4, 0, 2, 1) /* 42 */ \
    X(64, 64, 2, 2, 4, 3, 4, 1, 1) /* 43 */ \
    X(64, 64, 2, 2, 4, 4, 0, 1, 1) /* 44 */

static const TileDef kTiles[] = {
#define C2I8_ROW(...) {__VA_ARGS__},
    C2I8_TILE_LIST(C2I8_ROW)
#undef C2I8_ROW
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

int gemm_num_tiles() { return kNumTiles; }
size_t gemm_tile_lds_bytes(int t, int mode, int steps_per_slice);
TileInfo gemm_tile_info(int t)
{
    return TileInfo{kTiles[t].tk, kTiles[t].tm, (kTiles[t].wk * kTiles[t].wm * kTiles[t].ds + kTiles[t].help) * 64, kTiles[t].ks};
}

// LDS a launch of tile `d` asks for: the operand ring plus, for the blocked layout, one offset per 16-byte
// depth chunk of a slice (`per` 64-byte steps).  The picker and the launcher use the same figure.
constexpr size_t kLdsLimit = 160 * 1024;
static size_t tile_lds_bytes(const TileDef &d, int mode, int per)
{
    return (size_t)d.nstage * (d.tk + d.tm) * 64 * d.ks + (mode == ACT_BLOCKED ? (size_t)per * 16 : 0);
}

template <int TK, int TM, int WK, int WM, int KS, int NSTAGE, int HELP, int DS, int WPC = 1>
static hipError_t launch_tile(const GemmArgs &a, int mode, hipStream_t st)
{
    constexpr int NT = (WK * WM * DS + HELP) * 64;
    const size_t lds = tile_lds_bytes(TileDef{TK, TM, WK, WM, KS, NSTAGE, HELP, DS, WPC}, mode, a.ksteps_per_split);
    const int grid = a.tiles_k * a.tiles_m * a.split_k;
    auto kb = igemm_i8_kernel<TK, TM, WK, WM, KS, NSTAGE, HELP, DS, WPC, ACT_BLOCKED>;
    auto km = igemm_i8_kernel<TK, TM, WK, WM, KS, NSTAGE, HELP, DS, WPC, ACT_MATRIX>;
    auto kern = mode == ACT_BLOCKED ? kb : km;
    if (lds > kLdsLimit) return hipErrorInvalidValue;  // the picker never offers such a pair
    static size_t raised[2] = {0, 0};  // dynamic-LDS ceiling already granted, per kernel
    if (lds > 64 * 1024 && lds > raised[mode]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised[mode] = 160 * 1024;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, a);
    return hipGetLastError();
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

size_t gemm_tile_lds_bytes(int t, int mode, int steps_per_slice) { return tile_lds_bytes(kTiles[t], mode, steps_per_slice); }

// A tile with 128- or 256-byte stages walks the depth two or four steps at a time: every slice
// must be a whole number of stages.
static bool tile_fits(const TileDef &d, int ksteps, int per)
{
    return d.ks == 1 || (ksteps % d.ks == 0 && per % d.ks == 0);
}

// Per-launch time model (core cycles) used to pick a tile and a depth split.  Its constants
// were fitted to a table of measured launch times (every tile on the five benchmark shapes
// and on batch-scaled versions of them, both layouts) so that the tile it ranks first loses
// as little as possible against the measured best; they are rates and latencies in spirit --
// bytes per cycle a wave and a CU move global->LDS, the latency chain of a lone workgroup's
// depth step, the sustained share of the MFMA issue rate, output bytes per cycle and CU,
// the cost of starting a workgroup and each of its waves -- but only the ranking is used.
bool gemm_pick(const GemmProblem &g, int *tile, int *split_k, double *cost)
{
    const int ksteps = g.depth / 64;
    bool found = false;
    static const int splits[] = {1, 2, 3, 4, 6, 8, 9, 12, 16};
    double best = 1e300;
    int bt = *tile >= 0 ? *tile : 0, bs = *split_k > 0 ? *split_k : 1;
    for (int t = 0; t < kNumTiles; ++t) {
        if (*tile >= 0 && t != *tile) continue;
        const TileDef &d = kTiles[t];
        const int mwaves = d.wk * d.wm, waves = mwaves * d.ds + d.help;
        const double tiles = (double)ceil_div(g.K, d.tk) * ceil_div(g.M, d.tm);
        const double lds = (double)d.nstage * (d.tk + d.tm) * 64 * d.ks + 2048;
        const int acc = d.tk * d.tm / (mwaves * 64);  // accumulator registers per lane
        int cap = (int)(160.0 * 1024 / lds);
        const int reg_cap = acc > 128 ? 1 : acc > 64 ? 2 : 4;  // 512 registers per lane and SIMD
        const int wave_cap = waves >= 8 ? reg_cap / 2 : reg_cap;
        if (cap > wave_cap) cap = wave_cap;
        if (cap < 1) cap = 1;
        const double mfma = (double)d.tk * d.tm * 64 / 4096.0 / 0.6;
        const double bytes = (double)(d.tk + d.tm) * 64;
        const double lat = d.ks == 1 ? 350.0 : 360.0 / d.ks;  // barrier-to-barrier chain, per 64-deep step
        const int forced[] = {*split_k > ksteps ? ksteps : *split_k};
        const int *cand = *split_k > 0 ? forced : splits;
        const int ncand = *split_k > 0 ? 1 : (int)(sizeof(splits) / sizeof(splits[0]));
        for (int ci = 0; ci < ncand; ++ci) {
            int s = cand[ci];
            if (s > ksteps) continue;
            s = ceil_div(ksteps, ceil_div(ksteps, s));  // drop slices that would be empty
            const int per = ceil_div(ksteps, s);
            if (!tile_fits(d, ksteps, per)) continue;
            if (tile_lds_bytes(d, g.mode, per) > kLdsLimit) continue;  // ring + offset table must fit one CU's LDS
            const double wgs = tiles * s;
            int res = (int)((wgs + 255) / 256);  // workgroups sharing a CU
            if (res > cap) res = cap;
            double dma = (d.ks >= 2 ? 5.5 : 6.5) * waves * res;
            const double dma_max = d.ks >= 2 ? 44.0 : 38.0;
            if (dma > dma_max) dma = dma_max;
            double step = lat;
            if (res * mfma > step) step = res * mfma;
            if (res * bytes / dma > step) step = res * bytes / dma;
            const double store = res * (double)d.tk * d.tm * 4 / (s > 1 ? 2.2 : 4.0);
            const double start = 5000.0 + 5.0 * (d.tk + d.tm) / waves + (d.ds == 2 ? 1000.0 : 0.0) + 400.0 * waves * res;
            const double wg = start + per * step + store;
            const double rounds = (double)(long long)((wgs + 256.0 * res - 1) / (256.0 * res));
            double total = rounds * wg + (s > 1 ? 6000.0 : 0.0);
            // measured on two machines at N = 2048: among the 256 x 256 tiles the eight-wave one with 128-byte
            // stages is 5-15 % ahead of the four-wave one, which the cycle model above ranks level
            if (d.tk * d.tm >= 65536 && waves >= 8 && d.ks >= 2) total *= 0.95;
            if (total < best) {
                best = total;
                bt = t;
                bs = s;
                found = true;
            }
        }
    }
    *tile = bt;
    *split_k = bs;
    if (cost) *cost = best;
    return found;
}

// Fills the kernel's argument block; false if the tile cannot walk this depth in whole stages.
static bool make_gemm_args(const GemmProblem &g, int tile, int split_k, GemmArgs *out)
{
    const TileDef &d = kTiles[tile];
    GemmArgs a;
    a.act = g.act;
    a.wq = g.wq;
    a.out = g.out;
    a.act_out = g.act_out;
    a.act_shift = g.act_shift;
    a.act_relu = g.act_relu;
    a.o_cb_log2 = 0;
    while ((1 << a.o_cb_log2) < g.o_cb) ++a.o_cb_log2;
    a.o_pad = g.o_pad;
    a.o_Hp = g.PQ / g.Q + 2 * g.o_pad;
    a.o_Wp = g.Q + 2 * g.o_pad;
    a.o_Cb = g.o_cb > 0 ? (g.K + g.o_cb - 1) / g.o_cb : 0;
    a.dil = g.dil > 0 ? g.dil : 1;
    a.out_nhwc = g.out_nhwc;
    a.il_d = g.il_d;
    a.il_P = g.il_P;
    a.il_Q = g.il_Q;

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
    if (!tile_fits(d, a.ksteps_total, a.ksteps_per_split)) return false;
    a.out_fits_32bit = (unsigned long long)g.M * g.K * sizeof(int32_t) < (1ULL << 32);
    {
        // Start offsets of the first round (see the kernel): worth their idle time where the launch runs several
        // rounds and a large output tile is a sizeable part of a workgroup's life (small tiles drift apart by
        // themselves: measured level or slightly worse with offsets).  Estimates in core cycles: 60 per
        // MFMA and SIMD in the main loop (measured at steady state), 8 output bytes per cycle as a compute unit's
        // share of the memory system.  The offsets span about twice the time an output tile takes (measured best).
        const double mfma_per_simd = (double)(d.tk / 32) * (d.tm / 32) * 2 / 4;  // per 64-byte depth step
        const double main_clk = (double)a.ksteps_per_split * mfma_per_simd * 60.0;
        const double epi_clk = (double)d.tk * d.tm * (g.act_out ? 1 : 4) / 8.0;
        const long long grid = (long long)a.tiles_k * a.tiles_m * a.split_k;
        a.stagger = 0;
        if (grid >= 2 * 256 && a.split_k == 1 && epi_clk >= 16000 && epi_clk >= 0.15 * (main_clk + epi_clk)) {
            a.stagger = (int)(2.0 * epi_clk / (32 * 64) + 0.5);
        }
    }
    {
        // Each XCD has its own L2 and gets a contiguous eighth of the tile list: order the
        // list so that the operand rows one XCD has to pull in are as few as possible.
        const long long per_xcd = ((long long)a.tiles_k * a.tiles_m + 7) / 8;
        auto rows = [&](long long fast, long long slow, double fast_rows, double slow_rows) {
            const long long nf = per_xcd < fast ? per_xcd : fast;
            long long nsl = (per_xcd + fast - 1) / fast + 1;
            if (nsl > slow) nsl = slow;
            return nf * fast_rows + nsl * slow_rows;
        };
        // an implicit-GEMM pixel row re-reads each input byte R*S/stride^2 times: its unique
        // bytes are that much smaller than a weight row's
        double reuse = 1.0;
        if (g.mode == ACT_BLOCKED) {
            reuse = (double)g.R * g.S / ((double)g.stride * g.stride);
            if (reuse < 1.0) reuse = 1.0;
        }
        const double k_fast = rows(a.tiles_k, a.tiles_m, d.tk, d.tm / reuse);
        const double m_fast = rows(a.tiles_m, a.tiles_k, d.tm / reuse, d.tk);
        a.m_fastest = m_fast < k_fast;
        // ... or a blocked order, judged by the panels the 32 tiles that an XCD runs at a time share (the
        // row-major orders are the blockings 1 x 32 and min(32, tiles_k)-wide)
        a.grp_m = 0;
        if (a.tiles_k >= 4 && a.tiles_m >= 4) {
            auto panels = [&](long long gm_, long long gk_) { return gm_ * (d.tm / reuse) + gk_ * d.tk; };
            const long long kk = a.tiles_k < 32 ? a.tiles_k : 32, mm = a.tiles_m < 32 ? a.tiles_m : 32;
            double best = a.m_fastest ? panels(mm, (32 + mm - 1) / mm) : panels((32 + kk - 1) / kk, kk);
            for (int gmc = 2; gmc <= 16; gmc *= 2) {
                const long long gk_ = (32 + gmc - 1) / gmc;
                if (gmc > a.tiles_m || gk_ > a.tiles_k) continue;
                const double c = panels(gmc, gk_);
                if (c < 0.9 * best) {
                    best = c;
                    a.grp_m = gmc;
                }
            }
        }
    }
    auto magic = [](long long d) { return d <= 1 ? 0u : (unsigned)((0x100000000ULL + (unsigned long long)d - 1) / (unsigned long long)d); };
    a.mg_g16 = magic(a.g16);
    a.mg_S = magic(g.S);
    a.mg_R = magic(g.R);
    a.mg_PQ = magic(g.PQ);
    a.mg_Q = magic(g.Q);
    a.mg_il_dd = g.il_d ? magic(g.il_d * g.il_d) : 0;
    a.mg_il_d = g.il_d ? magic(g.il_d) : 0;
    a.mg_tiles_k = magic(a.tiles_k);
    a.mg_tiles_m = magic(a.tiles_m);
    a.mg_grp_sz = magic((long long)a.grp_m * a.tiles_k);
    a.mg_grp_m = magic(a.grp_m);
    a.mg_tiles_km = magic((long long)a.tiles_k * a.tiles_m);
    *out = a;
    return true;
}

hipError_t launch_gemm(const GemmProblem &g, int tile, int split_k, hipStream_t st)
{
    GemmArgs a;
    if (!make_gemm_args(g, tile, split_k, &a)) return hipErrorInvalidValue;
    if (a.act_out && a.split_k > 1) return hipErrorInvalidValue;  // the activation needs the whole sum
    if (a.il_d && a.split_k > 1) return hipErrorInvalidValue;     // `out` has another shape than the clear assumes
    if (a.split_k > 1) {
        hipError_t e = launch_fill_zero(g.out, (size_t)g.M * g.K * sizeof(int32_t), st);
        if (e != hipSuccess) return e;
    }
    int index = 0;
#define C2I8_CASE(tk, tm, wk, wm, ks, nstage, help, ds, wpc) \
    if (tile == index++) return launch_tile<tk, tm, wk, wm, ks, nstage, help, ds, wpc>(a, g.mode, st);
    C2I8_TILE_LIST(C2I8_CASE)
#undef C2I8_CASE
    return hipErrorInvalidValue;
}

// ---- MFMA-only probe: what the matrix cores sustain with nothing else in the way ---------------------
// Every wave keeps four independent 32x32 accumulators and issues v_mfma_i32_32x32x32_i8 back to back
// on register-resident operands (four pseudo-random fragment pairs made from the lane id).  Consecutive
// instructions take different fragments, as the blocks of a GEMM's wave tile do: with one constant pair the
// multiplier inputs would never toggle, and on a power-managed part that understates what real operands
// cost.  No LDS, no global loads; one store per lane at the end keeps the work alive.
__global__ void __launch_bounds__(256) mfma_probe_kernel(int iters, int32_t *out)
{
    const unsigned id = blockIdx.x * 256u + threadIdx.x;
    v4i a[4], b[4];
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            unsigned x = (id * 16u + (unsigned)(f * 4 + t)) * 2654435761u;
            x ^= x >> 15;
            x *= 2246822519u;
            x ^= x >> 13;
            a[f][t] = (int)x;
            b[f][t] = (int)(x * 3266489917u + 374761393u);
        }
    v16i acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[g][v] = 0;
    int it = 0;
    for (; it + 4 <= iters; it += 4) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                acc[g] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[(g + r) & 3], b[g], acc[g], 0, 0, 0);
    }
    for (; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[g] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[g], b[g], acc[g], 0, 0, 0);
    }
    int sum = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[g][v];
    out[id] = sum;
}

hipError_t launch_mfma_probe(int blocks, int iters, int32_t *out, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, iters, out);
    return hipGetLastError();
}

}  // namespace c2i8
