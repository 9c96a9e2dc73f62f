// GEMM stage that unrolls the stencil itself: the input stays NCHW and no rewritten copy of
// it is ever stored (Stencil Unroll + Fuse of Table 2 applied on the fly, for the layers whose
// unrolled matrix is many times the input -- the data growth Sec. 6.2 reports for it).
//
// Depth order.  The fused reduction index is j = (c*R + r)*S4 + s with S4 = ceil(S, 4): a kernel
// row is padded to whole dwords (the extra taps meet zero weights), the depth to a multiple of
// 64.  A dword of depth is then four horizontally adjacent input bytes of one (c, r) row, which
// in NCHW are contiguous in memory -- no byte gathering anywhere.
//
// One workgroup (4 waves) computes PT x QT output pixels of one image for up to 64 output
// channels:
//   1. window: the C * ((PT-1)*stride + R) input rows the tile touches, as wide as the tile's
//      pixels reach, are copied into LDS with the zero border filled in (dword loads from a
//      column clamped into the image row, shifted so that what falls outside becomes zero);
//   2. weights: the tile's rows of the weight operand -- KCRS itself, or the output of the weight
//      rewrite for this layout -- are copied into LDS in the padded depth order (a dword load at
//      any byte address, cut off at the end of its kernel row);
//   3. a table, one entry per depth dword: its offset in the window;
//   4. each wave owns 32 pixels of one output row: its MFMA activation operand for a 32-deep
//      step is four dwords at pixel*stride + table offset (any byte alignment: an aligned pair
//      and a byte-align each), its weight operand 16 bytes of weight row lane%32.
//      v_mfma_i32_32x32x32_i8, channels x pixels;
//   5. the D block (column = pixel = lane%32) goes straight to NKPQ: 128-byte runs per channel.
//
// NHWC source (Sec. 5.2).  A row of an NHWC image is W*C bytes in which the S*C bytes of a kernel row's taps
// and channels are one run: the same kernel computes it as a one-channel image of W*C columns with a kernel
// row of S*C bytes, a horizontal stride of stride*C and pad*C bytes of horizontal padding.  The depth order
// is then (r, s, c); the KCRS weight rows are copied into LDS as they are and brought into that order there.
// A lane's four results are four consecutive channels of a pixel, which is what an NHWC result stores.
#include "kernels.h"
#include "rewrite_bodies.h"

namespace c2i8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

struct WindowArgs {
    const int8_t *in;
    const int8_t *wt;
    int32_t *out;
    int C, H, W, K, P, Q, R, stride, pad;   // (NHWC source: C = 1, W in bytes; stride and pad are the vertical ones)
    int stride_w, pad_w;   // horizontal stride and padding in bytes of an image row
    int gC, gS, gRS;       // NHWC source: the real channel count, S and R*S of the KCRS weights
    int nhwc;              // NHWC source
    int out_nhwc, out_wide_k;  // result [N][P][Q][K]; K % 4 == 0 and out 16-byte aligned
    int PT, qshift;        // output rows per tile; tile columns QT = 32 << qshift, PT << qshift = 4
    int RW;                // window rows per channel: (PT-1)*stride + R
    int pitch;             // bytes per window row, a multiple of 4
    int tiles_q, tiles_p;  // tiles per image
    int CR, nd;            // C*R; dwords per kernel row: ceil(S, 4) / 4
    int w_S, w_row;        // weight operand: bytes per kernel row (S, or 4*nd once rewritten) and per channel
    int w_pitch;           // bytes per channel in LDS: depth + 16 (the 32 rows a wave reads start in different banks)
    int win_bytes, wl_bytes;  // LDS bytes of the window and of the weight rows (multiples of 16)
    int out_small;         // 4*K*P*Q < 2^32
    int in_small;          // C*H*W < 2^31
    int wt16;              // the weights are rewritten rows of `depth` bytes at a 16-byte aligned address: copied in 16-byte pieces
    int rpp;               // window fill by columns (0: not): window rows per pass of 256 threads, 256 / (pitch/4)
    int wide_out;          // Q % 4 == 0 and out 16-byte aligned: 16-byte stores
    ActOut act;            // activation epilogue (act.out != null): `out` is not written
    unsigned m_wd, m_RW, m_nd, m_R, m_tiles_q, m_tiles_p, m_gC;
};

__device__ __forceinline__ unsigned load_u32(const void *p)  // any alignment
{
    unsigned x;
    __builtin_memcpy(&x, p, 4);
    return x;
}

template <int NKK, int NKB, bool ACT, bool NHWC>  // ACT: the activation epilogue, a kernel of its own; NHWC: the source
// (four workgroups per compute unit asked for, i.e. up to 128 registers: the deep instantiations use 86 -- five
// fit -- and under a bound of 85 the compiler spilled their weight loads one by one, a wait behind each)
__global__ void __launch_bounds__(256, 4) conv_window_kernel(const WindowArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *win = smem;
    unsigned char *wl = smem + a.win_bytes;
    int *tab = reinterpret_cast<int *>(smem + a.win_bytes + a.wl_bytes);  // [NKK*8]
    constexpr int ND = NKK * 8;  // depth dwords
    constexpr int KB = 32 * NKB;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, half = lane >> 5;

    const int lid = xcd_contiguous(blockIdx.x, gridDim.x);
    const int t1 = fast_div_any(lid, a.tiles_q, a.m_tiles_q), tq = lid - t1 * a.tiles_q;
    const int n = fast_div_any(t1, a.tiles_p, a.m_tiles_p), tp = t1 - n * a.tiles_p;
    const int p0 = tp * a.PT, q0 = tq << (5 + a.qshift), k0 = blockIdx.y * KB;
    const int h_lo = p0 * a.stride - a.pad;
    const int w_first = q0 * a.stride_w - a.pad_w;
    const int w_lo = (w_first >> 2) << 2;  // rounded down, also when negative
    const int delta = w_first - w_lo;

    // Every global load of a thread is issued before the first LDS store, so that a workgroup
    // pays one memory round trip for both operands.
    // 2. weight rows k0 .. k0+KB-1 (those below K), brought into the padded depth order on the way:
    //    LDS dword d of a row holds the (up to) four taps s0 .. s0+3 of kernel row cr = d / nd.
    //    A thread keeps one d and walks down the rows.
    constexpr int RPP = 256 / ND;                  // rows per pass
    constexpr int WMAX = (KB + RPP - 1) / RPP;     // passes
    const int rows = min(KB, a.K - k0);
    const int8_t *wsrc = a.wt + (size_t)k0 * a.w_row;
    const int last = rows * a.w_row - 4;  // offset of the last whole dword of these rows
    const int r0 = tid / ND, d = tid - r0 * ND;
    const int wcr = fast_div(d, a.m_nd), ws0 = 4 * (d - wcr * a.nd);
    const int left = a.w_S - ws0;  // weight bytes of this kernel row from s0 on
    const bool real = wcr < a.CR && left > 0;
    const unsigned mask = !real ? 0u : left >= 4 ? 0xFFFFFFFFu : (1u << (8 * (left & 3))) - 1u;
    const int coff = wcr * a.w_S + ws0;
    unsigned wv[WMAX];
    // NHWC: the rows as they are, whole dwords of the run of `rows` rows (the last one fetched lower and shifted)
    constexpr int WRAW = NHWC ? KB / 4 : 1;   // rows of at most 256 bytes: 64 * KB dwords over 256 threads
    unsigned wraw[WRAW];
    const int raw_dw = (rows * a.w_row + 3) >> 2;
    // rewritten weights (rows of exactly the padded depth, zeros included): the tile's rows are one contiguous block,
    // fetched in 16-byte pieces -- three loads and three stores per thread for 64 rows of 192 bytes, no masks
    constexpr int PPR = ND / 4, WP16 = (KB * PPR + 255) / 256;   // pieces per row; pieces per thread
    v4i wp16[WP16];
    if (!NHWC && a.wt16) {
#pragma unroll
        for (int u = 0; u < WP16; ++u)
            wp16[u] = *reinterpret_cast<const v4i *>(wsrc + 16 * (unsigned)min(tid + u * 256, rows * PPR - 1));
    } else if (NHWC) {
        if (last >= 0) {
#pragma unroll
            for (int u = 0; u < WRAW; ++u) wraw[u] = load_u32(wsrc + (unsigned)min(4 * min(tid + u * 256, raw_dw - 1), last));
        }
    } else if (r0 < RPP && last >= 0) {
#pragma unroll
        for (int u = 0; u < WMAX; ++u) {
            const int row = min(r0 + u * RPP, rows - 1);
            const int off = real ? row * a.w_row + coff : 0;
            wv[u] = load_u32(wsrc + (unsigned)min(off, last));  // a dword that would run past the rows is fetched lower
        }
    }
    // 1. window
    {
        const int8_t *img = a.in + (size_t)n * a.C * a.H * a.W;
        const int wd = a.pitch >> 2, total = a.C * a.RW * wd;
        auto stage_pass = [&](int base) {
            // the loads of a pass first, nothing that needs their data in between (a use right after each
            // load makes the compiler wait for it: eight memory round trips in a row instead of one)
            // (all eight always: past the window's end they re-read its last dword -- a load under a
            // condition, even a uniform one, is waited for where the branches join)
            unsigned x[8], fix[8];  // fix: bits 0-4 left shift, 8-12 right shift, bit 16 = all zero
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = min(base + u * 256 + tid, total - 1);
                // exact: idx, row < 10240 and wd, RW <= 40960 keep n*d below 2^32
                const int row = (int)__umulhi((unsigned)idx, a.m_wd), c4 = idx - row * wd;  // wd >= 2
                const unsigned chi = __umulhi((unsigned)row, a.m_RW);
                const int c = a.RW == 1 ? row : (int)chi, rr = row - c * a.RW;
                const int h = h_lo + rr, w = w_lo + 4 * c4;
                const int hc = min(max(h, 0), a.H - 1), wc = min(max(w, 0), a.W - 4);  // W >= 4
                x[u] = load_u32(img + (unsigned)((c * a.H + hc) * a.W + wc));   // an image is below 2^31 bytes (host check)
                const int dd = wc - w;  // > 0: the dword starts left of the row, < 0: it runs past its end
                const unsigned sh = (unsigned)(dd > 0 ? dd : -dd) * 8u;
                fix[u] = (dd > 0 ? (sh & 31u) : 0u) | ((dd < 0 ? (sh & 31u) : 0u) << 8) |
                         ((sh >= 32u || h != hc) ? 0x10000u : 0u);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (base + u * 256 + tid < total) {
                    const unsigned y = (x[u] << (fix[u] & 31u)) >> ((fix[u] >> 8) & 31u);
                    *reinterpret_cast<unsigned *>(win + 4 * (base + u * 256 + tid)) = (fix[u] & 0x10000u) ? 0u : y;
                }
        };
        // Narrow windows (a row of at most 256 dwords, at most eight passes of rows): a thread keeps its column --
        // everything that depends on the column only (clamp, shifts, zero flag) is made once -- and walks down
        // the rows, one division per element instead of two and no multiply for the column.
        auto stage_columns = [&]() {
            const int r0 = (int)__umulhi((unsigned)tid, a.m_wd), c4 = tid - r0 * wd;   // wd >= 2
            const int rows_all = a.C * a.RW;
            const int w = w_lo + 4 * c4, wc = min(max(w, 0), a.W - 4);
            const int dd = wc - w;
            const unsigned sh = (unsigned)(dd > 0 ? dd : -dd) * 8u;
            const unsigned lsh = dd > 0 ? (sh & 31u) : 0u, rsh = dd < 0 ? (sh & 31u) : 0u;
            const bool col_zero = sh >= 32u;
            unsigned x[8];
            bool zero[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int row = min(r0 + u * a.rpp, rows_all - 1);
                const int c = a.RW == 1 ? row : (int)__umulhi((unsigned)row, a.m_RW), rr = row - c * a.RW;
                const int h = h_lo + rr, hc = min(max(h, 0), a.H - 1);
                x[u] = load_u32(img + (unsigned)((c * a.H + hc) * a.W + wc));
                zero[u] = col_zero || h != hc;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int row = r0 + u * a.rpp;
                if (r0 < a.rpp && row < rows_all)
                    *reinterpret_cast<unsigned *>(win + 4 * (row * wd + c4)) = zero[u] ? 0u : (x[u] << lsh) >> rsh;
            }
        };
        // windows of up to 8 KB -- the usual case -- in straight-line code: a loop header would make the
        // compiler drain the weight loads above before the first window load
        if (a.rpp) stage_columns();
        else if (total <= 256 * 8) stage_pass(0);
        else
            for (int base = 0; base < total; base += 256 * 8) stage_pass(base);
    }
    unsigned char *wr = smem + a.win_bytes + a.wl_bytes + 4 * ND;   // NHWC: the weight rows as they came
    if (NHWC) {
        if (last >= 0) {
#pragma unroll
            for (int u = 0; u < WRAW; ++u) {
                const int i = tid + u * 256;
                if (i < raw_dw) *reinterpret_cast<unsigned *>(wr + 4 * i) = wraw[u] >> (8 * (unsigned)max(4 * i - last, 0));
            }
        } else {
            for (int i = tid; i < rows * a.w_row; i += 256) wr[i] = (unsigned char)wsrc[i];
        }
        __syncthreads();
        // LDS dword d of a row: bytes s' = ws0 .. ws0+3 of kernel row wcr, s' = s*C + c, from KCRS byte (c*R + wcr)*S + s
        if (r0 < RPP) {
            int src_off[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int sp = ws0 + b, sx = fast_div(sp, a.m_gC), c = sp - sx * a.gC;
                src_off[b] = real && sp < a.w_S ? c * a.gRS + wcr * a.gS + sx : 0;   // (`mask` clears the bytes that are not there)
            }
            // all the byte reads first, straight-line: one LDS round trip for a thread's rows, not one per row
            unsigned wb[WMAX][4];
#pragma unroll
            for (int u = 0; u < WMAX; ++u) {
                const int row = min(r0 + u * RPP, rows - 1);
#pragma unroll
                for (int b = 0; b < 4; ++b) wb[u][b] = wr[row * a.w_row + src_off[b]];
            }
#pragma unroll
            for (int u = 0; u < WMAX; ++u) {
                const int row = r0 + u * RPP;
                if (row < rows)
                    *reinterpret_cast<unsigned *>(wl + row * a.w_pitch + 4 * d) =
                        (wb[u][0] | (wb[u][1] << 8) | (wb[u][2] << 16) | (wb[u][3] << 24)) & mask;
            }
        }
    } else if (a.wt16) {
#pragma unroll
        for (int u = 0; u < WP16; ++u) {
            const int i = tid + u * 256, row = i / PPR, col = i - row * PPR;
            if (i < rows * PPR) *reinterpret_cast<v4i *>(wl + row * a.w_pitch + col * 16) = wp16[u];
        }
    } else if (r0 < RPP) {
        if (last >= 0) {
#pragma unroll
            for (int u = 0; u < WMAX; ++u) {
                const int row = r0 + u * RPP;
                if (row < rows) {
                    const int over = row * a.w_row + coff - last;  // > 0 only at the very end of the rows
                    const unsigned x = (wv[u] >> (8 * (unsigned)max(over, 0))) & mask;
                    *reinterpret_cast<unsigned *>(wl + row * a.w_pitch + 4 * d) = x;
                }
            }
        } else {  // fewer than four weight bytes in all
            for (int row = r0; row < rows; row += RPP) {
                unsigned x = 0;
                const int off = row * a.w_row + coff;
                if (real)
                    for (int b = 0; off + b < rows * a.w_row; ++b) x |= (unsigned)(unsigned char)wsrc[off + b] << (8 * b);
                *reinterpret_cast<unsigned *>(wl + row * a.w_pitch + 4 * d) = x & mask;
            }
        }
    }
    // 3. table: where depth dword d starts in the window, relative to a pixel's first byte
    if (tid < ND) {
        const int cr = fast_div(tid, a.m_nd), s0 = 4 * (tid - cr * a.nd);
        const int c = fast_div(cr, a.m_R), r = cr - c * a.R;
        tab[tid] = cr < a.CR ? (c * a.RW + r) * a.pitch + s0 : 0;
    }
    __syncthreads();

    // 4. MFMA.  A pixel's four bytes start at any byte of the window: two aligned dwords and a
    //    byte-align (unaligned LDS reads are served one lane at a time).
    const int pw = wave >> a.qshift, qw = wave & ((1 << a.qshift) - 1);
    const int abyte = (pw * a.stride) * a.pitch + delta + (qw * 32 + l31) * a.stride_w;
    const unsigned char *a4 = win + (abyte & ~3);  // table offsets are multiples of 4: the byte shift is the lane's own
    const unsigned ash = (unsigned)abyte & 3u;
    const unsigned char *wbase = wl + l31 * a.w_pitch + half * 16;
    v16i acc[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[kb][v] = 0;
    // Every step's table entries first, then the dword pairs one step ahead of their use: written step by step, each
    // step was two dependent LDS round trips (table, then pairs) in front of its MFMAs.
    v4i ta[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) ta[kk] = *reinterpret_cast<const v4i *>(tab + kk * 8 + half * 4);
    unsigned plo[2][4], phi[2][4];
    auto fetch_pairs = [&](int kk) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned *pp = reinterpret_cast<const unsigned *>(a4 + ta[kk][i]);
            plo[kk & 1][i] = pp[0];
            phi[kk & 1][i] = pp[1];
        }
    };
    fetch_pairs(0);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
        if (kk + 1 < NKK) fetch_pairs(kk + 1);
        v4i af;
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = (int)__builtin_amdgcn_alignbyte(phi[kk & 1][i], plo[kk & 1][i], ash);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const v4i wf = *reinterpret_cast<const v4i *>(wbase + kb * 32 * a.w_pitch + kk * 32);
            acc[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, af, acc[kb], 0, 0, 0);
        }
    }

    // 5. D block: column = lane%32 = pixel, row = 8*(v/4) + 4*(lane/32) + v%4 = channel
    if (ACT) {
        const int p = p0 + pw, q = q0 + qw * 32 + l31;
        if (p < a.P && q < a.Q) {
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg)
                    act_store4(a.act, n, p, q, k0 + kb * 32 + 8 * vg + 4 * half, a.K, acc[kb][4 * vg], acc[kb][4 * vg + 1],
                               acc[kb][4 * vg + 2], acc[kb][4 * vg + 3]);
        }
        return;
    }
    const size_t PQ = (size_t)a.P * a.Q;
    int32_t *outn = a.out + (size_t)n * a.K * PQ;
    if (a.out_nhwc && a.out_wide_k) {
        // a lane's v%4 are channels k .. k+3 of its pixel: each wave lays its 32 pixels x KB channels out in LDS
        // as the result has them ([pixel][channel], rows of KB + 4 dwords) and stores 16-byte pieces with the
        // pieces of a pixel in consecutive lanes -- the channel runs of consecutive pixels follow each other in
        // the result, so a store instruction writes whole runs instead of 32-byte pairs
        __syncthreads();  // every wave is done with the window and the weights
        constexpr int TPITCH = KB + 4, CPP = KB / 4;   // dwords per pixel row; 16-byte pieces per pixel
        int *T = reinterpret_cast<int *>(smem) + wave * (32 * TPITCH);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg)
                *reinterpret_cast<v4i *>(T + l31 * TPITCH + kb * 32 + 8 * vg + 4 * half) =
                    v4i{acc[kb][4 * vg], acc[kb][4 * vg + 1], acc[kb][4 * vg + 2], acc[kb][4 * vg + 3]};
        __builtin_amdgcn_wave_barrier();  // LDS serves a wave's accesses in order
        const int p = p0 + pw, pc = lane % CPP, pr0 = lane / CPP;
        if (p >= a.P || k0 + 4 * pc >= a.K) return;
        int32_t *row = outn + ((size_t)p * a.Q) * a.K + k0 + 4 * pc;
#pragma unroll
        for (int j = 0; j < CPP / 2; ++j) {
            const int pr = pr0 + j * (64 / CPP), q = q0 + qw * 32 + pr;
            const v4i t = *reinterpret_cast<const v4i *>(T + pr * TPITCH + 4 * pc);
            if (q < a.Q) *reinterpret_cast<v4i *>(row + (size_t)q * a.K) = t;
        }
        return;
    }
    if (a.out_nhwc) {   // results that do not start on 16 bytes, or K % 4 != 0: one by one
        const int p = p0 + pw, q = q0 + qw * 32 + l31;
        if (p >= a.P || q >= a.Q) return;
        int32_t *px = outn + ((size_t)p * a.Q + q) * a.K;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int k = k0 + kb * 32 + 8 * vg + 4 * half;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (k + j < a.K) px[k + j] = acc[kb][4 * vg + j];
            }
        return;
    }
    if (a.wide_out) {
        // Q a multiple of 4 and `out` 16-byte aligned: each wave turns its 32x32 block around in LDS
        // (rows of 36 dwords) so that a lane stores four consecutive pixels of one channel -- 16-byte
        // stores, eight 128-byte runs per instruction instead of two
        __syncthreads();  // every wave is done with the window and the weights
        int *T = reinterpret_cast<int *>(smem) + wave * (32 * 36);
        const int tr = lane >> 3, tg = lane & 7;
        const int pp = p0 + pw, qq = q0 + qw * 32 + 4 * tg;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) T[(8 * (v >> 2) + 4 * half + (v & 3)) * 36 + l31] = acc[kb][v];
            __builtin_amdgcn_wave_barrier();  // LDS serves a wave's accesses in order: no wait beyond the compiler's own
            int32_t *dst = outn + (size_t)(k0 + kb * 32 + tr) * PQ + (size_t)pp * a.Q + qq;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v4i t = *reinterpret_cast<const v4i *>(T + (tr + 8 * j) * 36 + 4 * tg);
                if (pp < a.P && qq < a.Q && k0 + kb * 32 + tr + 8 * j < a.K)
                    *reinterpret_cast<v4i *>(dst + (size_t)(8 * j) * PQ) = t;
            }
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }
    const int p = p0 + pw, q = q0 + qw * 32 + l31;
    if (p >= a.P || q >= a.Q) return;
    if (a.out_small) {  // byte offsets inside an image's planes fit 32 bits: one add per store
        const unsigned PQ4 = (unsigned)PQ * 4u;
        const unsigned o = (unsigned)(k0 + 4 * half) * PQ4 + ((unsigned)p * a.Q + q) * 4u;
        char *ob = reinterpret_cast<char *>(outn);
        const bool full = k0 + KB <= a.K;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kr = kb * 32 + 8 * (v >> 2) + (v & 3);
                if (full || k0 + 4 * half + kr < a.K)
                    *reinterpret_cast<int32_t *>(ob + (o + (unsigned)kr * PQ4)) = acc[kb][v];
            }
        return;
    }
    int32_t *base = outn + (size_t)p * a.Q + q;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + kb * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (k < a.K) base[(size_t)k * PQ] = acc[kb][v];
        }
}

// dst[k][(cr*nd + d)*4 + b] = src[k][cr*S + 4*d + b] inside the kernel row, else 0; one thread per dword
__global__ void __launch_bounds__(256) pack_weights_window_kernel(const int8_t *src, int8_t *dst, int K, int CR,
                                                                  int S, int nd, int depth, unsigned m_nd)
{
    const int dd = depth >> 2;
    const long long total = (long long)K * dd;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        const int k = (int)(i / dd), d = (int)(i - (long long)k * dd);
        const int cr = fast_div(d, m_nd), s0 = 4 * (d - cr * nd);
        unsigned x = 0;
        if (cr < CR)
            for (int b = 0; b < 4 && s0 + b < S; ++b)
                x |= (unsigned)(unsigned char)src[((size_t)k * CR + cr) * S + s0 + b] << (8 * b);
        reinterpret_cast<unsigned *>(dst)[i] = x;
    }
}

}  // namespace

int window_depth(int C, int R, int S)
{
    const long long real = (long long)C * R * ((S + 3) / 4 * 4);
    if (real > 256) return 0;
    return (int)((real + 63) / 64 * 64);
}

constexpr long long WINDOW_LIMIT = 40 * 1024;  // bytes of LDS the input window of a tile may take

// Tile shape by output width, window geometry and the LDS it needs.
static bool window_plan(const WindowProblem &g, WindowArgs *a)
{
    if (g.nhwc_in && (g.wt_rewritten || (long long)g.S * g.C > 4096 || (long long)g.W * g.C > 2147483647LL ||
                      (long long)g.stride * g.C > 65536 || (long long)g.pad * g.C > 2147483647LL))
        return false;
    // an NHWC source is computed as one channel of W*C columns under a kernel row of S*C bytes
    const int C = g.nhwc_in ? 1 : g.C, W = g.nhwc_in ? g.W * g.C : g.W, S = g.nhwc_in ? g.S * g.C : g.S;
    const long long stride_w = g.nhwc_in ? (long long)g.stride * g.C : g.stride;
    const int depth = window_depth(C, g.R, S);
    if (depth == 0 || W < 4 || (long long)C * g.H * W > 0x7FFFFFFFLL) return false;  // (32-bit offsets inside an image)
    WindowArgs w{};
    w.in = g.in;
    w.wt = g.wt;
    w.out = g.out;
    w.C = C; w.H = g.H; w.W = W; w.K = g.K; w.P = g.P; w.Q = g.Q; w.R = g.R;
    w.stride = g.stride; w.pad = g.pad;
    w.stride_w = (int)stride_w; w.pad_w = g.nhwc_in ? g.pad * g.C : g.pad;
    w.gC = g.C; w.gS = g.S; w.gRS = g.R * g.S;
    w.m_gC = magic_for(g.C);
    w.nhwc = g.nhwc_in;
    w.out_nhwc = g.out_nhwc;
    w.out_wide_k = g.K % 4 == 0 && (reinterpret_cast<uintptr_t>(g.out) & 15) == 0;
    w.qshift = g.Q > 64 ? 2 : g.Q > 32 ? 1 : 0;
    w.PT = 4 >> w.qshift;
    const int QT = 32 << w.qshift;
    const int S4 = (S + 3) / 4 * 4;
    const long long RW = (long long)(w.PT - 1) * g.stride + g.R;
    const long long pitch = (((long long)(QT - 1) * stride_w + S4 + 3) + 3) / 4 * 4;
    if (RW > WINDOW_LIMIT || pitch > WINDOW_LIMIT || C * RW * pitch > WINDOW_LIMIT) return false;
    w.RW = (int)RW;
    const long long win = (C * RW * pitch + 4 + 15) / 16 * 16;  // + the dword after the last one (read, never used)
    w.CR = C * g.R;
    w.nd = S4 / 4;
    w.w_S = g.wt_rewritten ? S4 : S;
    w.w_row = g.wt_rewritten ? depth : C * g.R * S;
    w.wt16 = g.wt_rewritten && (reinterpret_cast<uintptr_t>(g.wt) & 15) == 0;
    w.w_pitch = depth + 16;
    const int kb = g.K > 32 ? 64 : 32;
    const long long wlb = (long long)kb * w.w_pitch;
    const long long raw = g.nhwc_in ? ((long long)kb * w.w_row + 3) / 4 * 4 : 0;   // the weight rows as they came
    if (win + 8 + wlb + depth + raw > 64 * 1024) return false;  // cannot happen within the limits above
    w.pitch = (int)pitch;
    w.win_bytes = (int)win;
    w.wl_bytes = (int)wlb;
    w.tiles_q = (g.Q + QT - 1) / QT;
    w.tiles_p = (g.P + w.PT - 1) / w.PT;
    if ((long long)g.N * w.tiles_p * w.tiles_q > 2147483647LL || (g.K + kb - 1) / kb > 65535) return false;
    w.m_wd = magic_for(pitch / 4);
    w.rpp = (pitch / 4 <= 256 && (long long)C * RW <= 8 * (256 / (pitch / 4))) ? (int)(256 / (pitch / 4)) : 0;
    w.m_RW = magic_for(w.RW);
    w.m_nd = magic_for(w.nd);
    w.m_R = magic_for(g.R);
    w.m_tiles_q = magic_for(w.tiles_q);
    w.m_tiles_p = magic_for(w.tiles_p);
    w.out_small = 4LL * g.K * g.P * g.Q < (1LL << 32);
    w.in_small = (long long)C * g.H * W < (1LL << 31);
    w.wide_out = g.Q % 4 == 0 && (reinterpret_cast<uintptr_t>(g.out) & 15) == 0;
    w.act = g.act;
    if (a) *a = w;
    return true;
}

bool window_fits(const WindowProblem &g) { return window_plan(g, nullptr); }

template <int NKK>
static hipError_t launch_window_nkk(const WindowArgs &a, dim3 grid, size_t lds, hipStream_t st)
{
    if (a.nhwc) {
        if (a.act.out) {
            if (a.K > 32) hipLaunchKernelGGL((conv_window_kernel<NKK, 2, true, true>), grid, dim3(256), lds, st, a);
            else hipLaunchKernelGGL((conv_window_kernel<NKK, 1, true, true>), grid, dim3(256), lds, st, a);
        } else if (a.K > 32) hipLaunchKernelGGL((conv_window_kernel<NKK, 2, false, true>), grid, dim3(256), lds, st, a);
        else hipLaunchKernelGGL((conv_window_kernel<NKK, 1, false, true>), grid, dim3(256), lds, st, a);
        return hipGetLastError();
    }
    if (a.act.out) {
        if (a.K > 32) hipLaunchKernelGGL((conv_window_kernel<NKK, 2, true, false>), grid, dim3(256), lds, st, a);
        else hipLaunchKernelGGL((conv_window_kernel<NKK, 1, true, false>), grid, dim3(256), lds, st, a);
    } else if (a.K > 32) hipLaunchKernelGGL((conv_window_kernel<NKK, 2, false, false>), grid, dim3(256), lds, st, a);
    else hipLaunchKernelGGL((conv_window_kernel<NKK, 1, false, false>), grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_window_conv(const WindowProblem &g, hipStream_t st)
{
    WindowArgs a;
    if (!window_plan(g, &a)) return hipErrorInvalidValue;
    const int depth = a.w_pitch - 16;
    const int kb = g.K > 32 ? 64 : 32;
    const dim3 grid((unsigned)(g.N * a.tiles_p * a.tiles_q), (unsigned)((g.K + kb - 1) / kb));
    size_t lds = (size_t)a.win_bytes + a.wl_bytes + (size_t)depth + (g.nhwc_in ? ((size_t)kb * a.w_row + 3) / 4 * 4 : 0);
    if (lds < 4 * 32 * 36 * 4) lds = 4 * 32 * 36 * 4;  // the output blocks of the four waves, turned around
    if (g.out_nhwc && lds < (size_t)4 * 32 * (kb + 4) * 4) lds = (size_t)4 * 32 * (kb + 4) * 4;
    switch (depth / 32) {
        case 2: return launch_window_nkk<2>(a, grid, lds, st);
        case 4: return launch_window_nkk<4>(a, grid, lds, st);
        case 6: return launch_window_nkk<6>(a, grid, lds, st);
        case 8: return launch_window_nkk<8>(a, grid, lds, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_pack_weights_window(int K, int C, int R, int S, const int8_t *src, int8_t *dst, hipStream_t st)
{
    const int depth = window_depth(C, R, S);
    if (depth == 0) return hipErrorInvalidValue;
    const int nd = (S + 3) / 4;
    const long long total = (long long)K * (depth / 4);
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(pack_weights_window_kernel, dim3(blocks), dim3(256), 0, st, src, dst, K, C * R, S, nd, depth,
                       magic_for(nd));
    return hipGetLastError();
}

}  // namespace c2i8
