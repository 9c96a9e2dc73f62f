// Internal launcher interface between the C-ABI glue and the HIP kernels.
// Launchers validate nothing: the glue has already checked every argument.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace c2i8 {

// How the GEMM stage finds the depth-contiguous activation row of output pixel m.
enum ActMode : int {
    ACT_BLOCKED = 0,  // [N][Cb][Hp][Wp][cb] produced by pack_layout
    ACT_MATRIX = 1    // [M][depth] produced by im2col (or any row-major matrix)
};

struct GemmProblem {
    const int8_t *act;  // activations
    const int8_t *wq;   // weights [K][depth]
    int32_t *out;       // [N][K][PQ]
    int K;              // output channels (GEMM rows)
    int M;              // output pixels N*P*Q (GEMM columns)
    int depth;          // fused reduction length, multiple of 64
    int PQ, Q;          // pixels per image, output width
    int mode;           // ActMode
    // ACT_BLOCKED only:
    int stride, cb, Cb, R, S, Hp, Wp;
    // Fused activation (act_out != null; split_k must be 1): instead of the int32 result, the GEMM stage
    // writes requant(result) as the next layer's blocked input [N][ceil(K/o_cb)][P+2 o_pad][Q+2 o_pad][o_cb],
    // o_cb a power of two >= 4; borders and channel padding are not written (the caller clears them).
    int8_t *act_out;
    int act_shift, act_relu, o_cb, o_pad;
    // Interleaving epilogue (il_d >= 2; split_k must be 1): this problem is the dense convolution on the
    // il_d^2 sub-images per image of a dilated layer, and `out` is that layer's own [N][K][il_P][il_Q].
    int il_d, il_P, il_Q;
    // ACT_BLOCKED: kernel taps `dil` pixels apart (0 or 1: dense); PQ and Q are then the dilated layer's own
    int dil;
    int out_nhwc;  // `out` is [N][PQ][K] (channels innermost) instead of [N][K][PQ]; a depth split clears the same bytes
};

struct TileInfo {
    int rows, cols, threads, steps;
};

int gemm_num_tiles();
TileInfo gemm_tile_info(int tile);
// Dynamic LDS a launch of `tile` asks for when a depth slice holds `steps_per_slice` 64-byte steps.
size_t gemm_tile_lds_bytes(int tile, int mode, int steps_per_slice);
// Chooses tile / split when tile < 0 / split_k <= 0; false if a forced choice cannot run
// this problem (a tile with 128-byte stages needs an even number of depth steps per slice).
bool gemm_pick(const GemmProblem &g, int *tile, int *split_k, double *cost = nullptr);
// The band kernel (band_mfma.hip): a GEMM stage for channel blocks of 64 that keeps a band of output rows'
// input window resident in LDS and splits the depth over its waves.  band_cost: the same cycle scale as
// the cost gemm_pick reports (1e300 where the kernel does not apply).
bool band_applies(const GemmProblem &g);
double band_cost(const GemmProblem &g);
TileInfo band_tile_info(const GemmProblem &g);
size_t band_lds_bytes(const GemmProblem &g);
hipError_t launch_band_conv(const GemmProblem &g, hipStream_t st);
// split_k > 1 clears `out` first and accumulates with atomics.
hipError_t launch_gemm(const GemmProblem &g, int tile, int split_k, hipStream_t st);

// blocks x 4 waves x iters x 4 MFMA 32x32x32 i8 on register operands; out: blocks * 256 int32
hipError_t launch_mfma_probe(int blocks, int iters, int32_t *out, hipStream_t st);

hipError_t launch_pack_layout(int N, int C, int H, int W, int cb, int pad,
                              const int8_t *src, int8_t *dst, hipStream_t st);
hipError_t launch_pack_layout_nhwc(int N, int C, int H, int W, int cb, int pad,
                                   const int8_t *src, int8_t *dst, hipStream_t st);  // cb % 16 == 0
hipError_t launch_rewrite_fused_nhwc(int N, int C, int H, int W, int K, int R, int S, int pad, int cb, int depth,
                                     const int8_t *in, int8_t *xq, const int8_t *wt, int8_t *wq, hipStream_t st);
hipError_t launch_im2col_nhwc(int N, int C, int H, int W, int R, int S, int stride, int pad, int P, int Q, int kg_pad,
                              const int8_t *src, int8_t *dst, hipStream_t st);  // src 16-byte aligned if C % 16 == 0
hipError_t launch_pack_weights_rsc(int K, int C, int R, int S, int depth, const int8_t *src, int8_t *dst, hipStream_t st);
hipError_t launch_requant(long long count, const int32_t *src, int8_t *dst, int shift, int relu, hipStream_t st);
hipError_t launch_requant_pack(int N, int K, int P, int Q, int cb, int pad, int shift, int relu, const int32_t *src,
                               int8_t *dst, hipStream_t st);
hipError_t launch_unpack_nhwc(int N, int K, long long PQ, const int32_t *src, int32_t *dst, hipStream_t st);
hipError_t launch_pack_weights_blocked(int K, int C, int R, int S, int cb, int depth,
                                       const int8_t *src, int8_t *dst, hipStream_t st);
hipError_t launch_pack_weights_rows(int K, int CRS, int depth,
                                    const int8_t *src, int8_t *dst, hipStream_t st);
hipError_t launch_im2col(int N, int C, int H, int W, int R, int S, int stride, int pad,
                         int P, int Q, int kg_pad,
                         const int8_t *src, int8_t *dst, hipStream_t st);
// Input rewrite (pack_layout or im2col) and weight rewrite as one grid; hipErrorNotSupported
// if the problem needs the general (separately launched) kernels.
hipError_t launch_rewrite_fused(bool im2col, int N, int C, int H, int W, int K, int R, int S, int stride,
                                int pad, int P, int Q, int cb, int depth, const int8_t *in, int8_t *xq,
                                const int8_t *wt, int8_t *wq, hipStream_t st);
hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t st);
// Image Pack: the stride phases of the zero-padded image (and of the kernel) become channels.
hipError_t launch_image_pack(int N, int C, int H, int W, int stride, int pad, int H2, int W2,
                             const int8_t *src, int8_t *dst, hipStream_t st);
// Dilation as Image Pack into the batch (Sec. 6.1): the d*d phases of the zero-padded image become
// sub-images [N*d*d][C][H2][W2]; their results [N*d*d][K][P2][Q2] are interleaved back into [N][K][P][Q].
hipError_t launch_dilation_pack(int N, int C, int H, int W, int pad, int d, int H2, int W2, const int8_t *src,
                                int8_t *dst, hipStream_t st);
hipError_t launch_dilation_unpack(int N, int K, int P, int Q, int d, int P2, int Q2, const int32_t *src, int32_t *dst,
                                  hipStream_t st);
hipError_t launch_image_pack_weights(int K, int C, int R, int S, int stride, const int8_t *src, int8_t *dst,
                                     hipStream_t st);

// GEMM stage that unrolls the stencil itself from the NCHW input (no rewritten activations).
// Activation in a kernel's epilogue: instead of the int32 result, requant(result) goes out as the next
// layer's channel-blocked int8 input [N][Cb][Hp][Wp][1 << cb_log2] (interior pixels and real channels only;
// the caller clears the rest).  out == nullptr: off.
struct ActOut {
    int8_t *out;
    int shift, relu, cb_log2, pad, Hp, Wp, Cb;
};

struct WindowProblem {
    const int8_t *in;   // [N][C][H][W]
    const int8_t *wt;   // KCRS, or (wt_rewritten) [K][depth] with depth index (c*R + r)*ceil(S,4) + s
    int32_t *out;       // [N][K][P][Q]
    int N, C, H, W, K, P, Q, R, S, stride, pad;
    int wt_rewritten;
    ActOut act;
    // NHWC source: in is [N][H][W][C] and the depth order is (r, s, c) -- a kernel row's S*C bytes are one run
    // of an image row -- with the KCRS weights brought into that order on their way into LDS; not with wt_rewritten
    int nhwc_in;
    int out_nhwc;       // out is [N][P][Q][K]
};
int window_depth(int C, int R, int S);          // 0 if the padded depth exceeds what the kernel unrolls
bool window_fits(const WindowProblem &g);       // depth, image width and LDS window within the kernel's limits
hipError_t launch_window_conv(const WindowProblem &g, hipStream_t st);
hipError_t launch_pack_weights_window(int K, int C, int R, int S, const int8_t *src, int8_t *dst, hipStream_t st);
// The same for 1x1 convolutions over whole 64-channel multiples: a workgroup turns its pixels
// around in LDS; the weights are used as they are ([K][C]).
inline bool pointwise_shape(int C, int R, int S) { return R == 1 && S == 1 && C % 64 == 0; }
bool pointwise_fits(const WindowProblem &g);    // stride 1, no padding, C <= 512, H*W a multiple of 4
hipError_t launch_pointwise_conv(const WindowProblem &g, hipStream_t st);
// 1x1, stride 1, no padding on NHWC tensors ([M][C] pixels, [K][C] weights, [M][K] result), small grids only
bool pointwise_nhwc_split_fits(long long M, int C, int K);
hipError_t launch_pointwise_nhwc_split(const int8_t *in, const int8_t *wt, int32_t *out, long long M, int C, int K,
                                       hipStream_t st);

}  // namespace c2i8
