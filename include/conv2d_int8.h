/* conv2d_int8 -- int8 2-D convolution on MI355X (gfx950) executed the way
 * arXiv 2104.04731 frames it: a data-layout rewrite (zero padding, channel
 * blocking, or stencil unrolling) followed by a tiled int8 x int8 -> int32
 * matrix-multiply intrinsic (there VTA's GEMM core, here the CDNA4 int8 MFMA).
 *
 * C ABI.  Plain pointers and sizes only.
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *     never frees or keeps it.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  All work is enqueued on `stream`; no call
 *     synchronises with the host.
 *   - Tensors are dense and contiguous:
 *       input   in  [N][C][H][W]      int8   (NCHW)
 *       weights wt  [K][C][R][S]      int8   (KCRS)
 *       output  out [N][K][P][Q]      int32  (NKPQ)
 *       P = floor((H + 2 pad - R)/stride) + 1,  Q likewise from W and S.
 *   - Every function returns a conv_status_t (size queries return bytes, 0 on
 *     invalid arguments).  Arguments are validated before anything is enqueued,
 *     so a non-zero status leaves all buffers untouched.  Nothing throws.
 *   - Calls on different host threads must use different streams AND, for the
 *     one-shot conv2d_int8 / conv2d_int8_nhwc, are serialised on the library's cached
 *     workspace: two such calls on one device must not run concurrently (one stream,
 *     or streams ordered by events).
 *
 * Operation computed (Sec. 3 tensor expression / Fig. 5 step 1; access [n, i+k]
 * of Table 2 => cross-correlation; 8-bit operands, 32-bit accumulation, Sec. 5.1):
 *   out[n][k][p][q] = sum_{c,r,s} in0[n][c][p*stride+r-pad][q*stride+s-pad] * wt[k][c][r][s]
 * with in0 = in inside the image and 0 outside; operands signed.
 */
#ifndef CONV2D_INT8_H
#define CONV2D_INT8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CONV_OK = 0,
    CONV_ERR_INVALID_ARG = 1,   /* null pointer, non-positive extent, kernel larger than padded image */
    CONV_ERR_UNSUPPORTED = 2,   /* valid problem the library has no path for (e.g. block size) */
    CONV_ERR_OVERFLOW_RISK = 3, /* C*R*S > 131072: an int32 accumulator could wrap */
    CONV_ERR_WORKSPACE = 4,     /* caller workspace too small / internal allocation failed */
    CONV_ERR_DEVICE = 5         /* a HIP call or launch reported an error */
} conv_status_t;

/* Which rewrite feeds the matrix intrinsic (Table 2; reference mapping of Sec. 5.1). */
typedef enum {
    CONV_LAYOUT_AUTO = 0,     /* let select_layout decide */
    CONV_LAYOUT_PACKED = 1,   /* Pad + Split + Reorder: [N][ceil(C/cb)][H+2pad][W+2pad][cb] */
    CONV_LAYOUT_IM2COL = 2,   /* Stencil Unroll + Fuse: [N*P*Q][depth], depth index (c,r,s) */
    CONV_LAYOUT_PAD_ONLY = 3, /* Pad only: one block cb = ceil(C,16), i.e. [N][H+2pad][W+2pad][cb] */
    CONV_LAYOUT_IMPLICIT = 4, /* Stencil Unroll + Fuse applied inside the GEMM stage: the input stays NCHW,
                                 nothing rewritten is stored.  Exists for the low-channel layers whose
                                 unrolled matrix is many times the input (Sec. 6.2), and for 1x1 kernels,
                                 whose weights need no rewrite at all.  Which problems it takes is a
                                 property of the kernels behind it, not of this interface: ask
                                 layout_overheads(desc, CONV_LAYOUT_IMPLICIT, 0, ...), which returns
                                 CONV_ERR_UNSUPPORTED outside the domain, exactly where every other entry
                                 point does.  Weight order of pack_weights for it: see pack_weights. */
    CONV_LAYOUT_IMAGE_PACK = 5 /* Image Pack (Table 2 row 1, for strides s > 1): the s*s stride phases of the
                                 zero-padded image become channels, the kernel is split the same way, and the
                                 convolution becomes the stride-1, pad-0 problem of image_pack_desc, which
                                 then runs in an inner layout: cb = 0 -> IMPLICIT, cb = 16/32/64 -> PACKED
                                 with that block.  Accepted by conv2d_int8_ex, conv2d_int8_workspace_bytes,
                                 layout_overheads and the selectors only (two rewrites in a row are not one
                                 GEMM-stage operand); stride 1 or an inner layout that does not apply:
                                 CONV_ERR_UNSUPPORTED. */
} conv_layout_t;

typedef struct {
    int N, C, H, W;   /* input  */
    int K, R, S;      /* filter */
    int stride, pad;  /* same in both spatial directions */
} conv_desc_t;

#define CONV_DEPTH_ALIGN 64 /* fused reduction depth is zero-padded to this (one MFMA k-step, bytes) */

/* ---- one-shot convolution (layout rewrite of input and weights + GEMM stage) ---------
 * Picks the layout with select_layout, uses a workspace the library caches per device.
 * Workspace rule: when a problem needs more than the cached block, a larger block is allocated
 * (hipMalloc, no synchronisation) and the superseded block is kept allocated until the process
 * ends, so work already enqueued and HIP graphs captured earlier stay valid.  Allocation is
 * impossible while `stream` is being captured: a call that would have to grow the block then
 * returns CONV_ERR_WORKSPACE with nothing enqueued -- make the first call for a problem size
 * outside capture (or use conv2d_int8_ex with a workspace of your own).
 * Two launches: both rewrites, then the GEMM stage; one launch and no workspace when the choice
 * is IMPLICIT -- except for large batches of a non-1x1 layer (2^21 output pixels and more), where the
 * weights are first rewritten into the cached workspace by a small kernel (if that block cannot be had,
 * e.g. under capture, the single launch runs instead: never an error from this). */
int conv2d_int8(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                const int8_t *in, const int8_t *wt, int32_t *out, void *stream);

/* conv2d_int8 for callers that cannot allocate: code under HIP graph capture, serving loops and harnesses
 * that forbid hipMalloc.  Same arguments, same result; the rewritten operands go to a fixed device array of
 * CONV_STATIC_WORKSPACE_BYTES that is part of the library's code object (every GPU the library is used on
 * holds its own copy from the first call there until the process ends).  The call itself never allocates or
 * frees and never synchronises.  A problem whose rewritten input + weights
 * (conv2d_int8_workspace_bytes(desc, CONV_LAYOUT_AUTO, 0, 0)) exceed the array: CONV_ERR_WORKSPACE, nothing
 * enqueued.  All calls on one GPU share the array and nothing orders them but the streams they are given:
 * two calls that may overlap on one GPU race on it (use one stream, or order the streams with events).
 * Nothing is assumed about what an earlier call left there: every byte the GEMM stage reads is written by
 * this call's own rewrites. */
#define CONV_STATIC_WORKSPACE_BYTES ((size_t)8 << 20)
int conv2d_int8_static(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       const int8_t *in, const int8_t *wt, int32_t *out, void *stream);

/* The same for NHWC tensors (Sec. 5.2): in [N][H][W][C], wt KCRS, out [N][P][Q][K] int32.  Channel
 * blocking straight from the NHWC source (pack_layout_nhwc) and the weight rewrite in one launch, then a
 * GEMM stage whose epilogue writes NHWC itself: two launches.  (An `out` that does not start on 16 bytes goes
 * through an NKPQ staging tensor in the cached workspace and unpack_nhwc_int32: three.)  Same workspace rules as conv2d_int8.
 * When select_layout's choice for the shape is IMPLICIT (not the 1x1 form) and R * ceil(S*C, 4) <= 256, the
 * kernel that unrolls the stencil itself reads the NHWC source directly -- depth order (r, s, c), a kernel row's
 * S*C bytes being one run of an image row -- and writes the NHWC result: one launch, no workspace.  A 1x1 layer
 * (stride 1, no padding, C a multiple of 64, all three tensors on 16 bytes) is a plain matrix product of the NHWC
 * input and the weight rows as they are: one launch of the GEMM stage (for a grid too small to fill the chip, of a
 * kernel whose waves share the depth), no rewrite, no workspace. */
int conv2d_int8_nhwc(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     const int8_t *in, const int8_t *wt, int32_t *out, void *stream);

/* ---- explicit form --------------------------------------------------------------------
 * layout: a conv_layout_t (AUTO allowed).  cb: channel block for PACKED (16, 32 or 64;
 * 0 = library's choice); the inner layout's block for IMAGE_PACK; ignored for the other layouts.
 * wt: KCRS weights, or -- if wt_is_packed != 0 -- the output of pack_weights for the
 * same layout/cb.  workspace: device memory of at least
 * conv2d_int8_workspace_bytes(desc, layout, cb, wt_is_packed) bytes, 256-byte aligned,
 * caller-owned, free to reuse once the stream has passed this call (may be NULL when that
 * size is 0, as it is for IMPLICIT, which reads `in` and either form of `wt` directly). */
int conv2d_int8_ex(const conv_desc_t *desc, int layout, int cb,
                   const int8_t *in, const int8_t *wt, int wt_is_packed, int32_t *out,
                   void *workspace, size_t workspace_bytes, void *stream);
size_t conv2d_int8_workspace_bytes(const conv_desc_t *desc, int layout, int cb, int wt_is_packed);

/* ---- GEMM stage alone (operands already rewritten; the "Op." column of Table 3) -------
 * in_packed: output of pack_layout (PACKED / PAD_ONLY) or im2col_int8 (IM2COL), or the NCHW
 * input itself (IMPLICIT); wt_packed: output of pack_weights.  layout must not be AUTO; cb as above (0 = 64 if
 * C >= 64 else ceil(C,16) rounded to 16/32/64).
 * tile: -1 = automatic, else an index < conv2d_int8_num_tiles() (for tuning sweeps), or CONV_TILE_BAND:
 * the second GEMM-stage kernel, for channel blocks of 64 (PACKED with cb = 64, or PAD_ONLY over 64 channels):
 * it keeps the input rows a band of output rows touches resident in LDS (each activation byte is fetched
 * once per workgroup, not once per kernel tap -- the buffer-residency argument of Sec. 6.1) and splits the
 * reduction depth over its waves; picked automatically for small many-channel layers;
 * split_k: 0 = automatic, else the number of depth slices (>= 2 accumulates with int32
 * atomics after clearing `out`; exact, because integer addition is associative; CONV_TILE_BAND: 0 or 1).
 * IMPLICIT has one kernel shape per problem: tile must be -1 and split_k 0 or 1. */
#define CONV_TILE_BAND (-2)
int conv2d_int8_packed(const conv_desc_t *desc, int layout, int cb,
                       const int8_t *in_packed, const int8_t *wt_packed, int32_t *out,
                       int tile, int split_k, void *stream);
/* The tile (an index, or CONV_TILE_BAND) and depth split the library would pick for this problem (host only);
 * tile = -1, split_k = 1 for IMPLICIT. */
int conv2d_int8_query_tiling(const conv_desc_t *desc, int layout, int cb, int *tile, int *split_k);
int conv2d_int8_num_tiles(void);
/* Describes tile `tile`: rows = output channels, cols = output pixels per workgroup;
 * steps = 64-byte depth steps per pipeline stage (a tile only runs problems whose depth
 * slices hold a whole number of stages; otherwise CONV_ERR_UNSUPPORTED). */
int conv2d_int8_tile_info(int tile, int *rows, int *cols, int *threads, int *steps);
/* Would conv2d_int8_packed accept this forced tile (>= 0, or CONV_TILE_BAND) and split_k (>= 1) for this
 * problem?  CONV_OK or CONV_ERR_UNSUPPORTED (host only). */
int conv2d_int8_tile_applies(const conv_desc_t *desc, int layout, int cb, int tile, int split_k);
/* LDS bytes per workgroup that this tile and split would ask for on this problem (operand ring plus, for
 * the blocked layouts, one offset per 16-byte depth chunk of a slice); 0 where the pair does not apply.
 * Never above 160 KB, one compute unit's LDS (host only). */
size_t conv2d_int8_tile_lds_bytes(const conv_desc_t *desc, int layout, int cb, int tile, int split_k);

/* ---- layout rewrites, individually callable (the "Transf." column of Table 3) ---------
 * pack_layout (Table 2 rows 2-4 on the input, plus the convolution's zero border):
 *   dst[n][c/cb][h+pad][w+pad][c%cb] = src[n][c][h][w]; zero where c >= C and on the border.
 *   cb: a multiple of 4, 4 <= cb <= 1024.  dst holds pack_layout_bytes(...) bytes. */
int pack_layout(int N, int C, int H, int W, int cb, int pad,
                const int8_t *src, int8_t *dst, void *stream);
size_t pack_layout_bytes(int N, int C, int H, int W, int cb, int pad);
/* The same rewrite from an NHWC source (Sec. 5.2: the dimensions the embedding leaves free may be in
 * any order in the source): dst as above, dst[n][c/cb][h+pad][w+pad][c%cb] = src[n][h][w][c];
 * cb a multiple of 16.  The GEMM stage and the NKPQ result are unchanged. */
int pack_layout_nhwc(int N, int C, int H, int W, int cb, int pad,
                     const int8_t *src, int8_t *dst, void *stream);

/* Activation between two int8 layers -- the step between convolution and unpacking in the benchmark
 * of Sec. 5.1, done there by the accelerator's ALU (shift, min, max).  The paper gives no formula; here
 *   y = clip(relu ? max(r, 0) : r, -128, 127),  r = floor(x / 2^shift + 1/2)   (0 <= shift <= 31)
 * requant_int8: same element order, int32 -> int8, `count` elements.
 * requant_pack_layout: the activation and the next layer's channel blocking in one pass -- from an NKPQ
 *   int32 result straight to what pack_layout would make of its int8 image:
 *   dst[n][k/cb][p+pad][q+pad][k%cb] = y(src[n][k][p][q]), zero where k >= K and on the border;
 *   cb a multiple of 16; dst holds pack_layout_bytes(N, K, P, Q, cb, pad) bytes, 16-byte aligned.
 *   Its output feeds conv2d_int8_packed (PACKED, cb) of the next layer directly. */
int requant_int8(long long count, const int32_t *src, int8_t *dst, int shift, int relu, void *stream);
int requant_pack_layout(int N, int K, int P, int Q, int cb, int pad, int shift, int relu,
                        const int32_t *src, int8_t *dst, void *stream);

/* Stencil Unroll + Fuse from an NHWC source (Sec. 5.2): src int8 [N][H][W][C] -> dst [N*P*Q][kg_pad] with depth
 * index (r*S + s)*C + c -- a tap's channels stay contiguous, so with C % 16 == 0 every destination 16-byte piece
 * is one load (src must then be 16-byte aligned); kg_pad >= C*R*S, a multiple of 16; dst 16-byte aligned, of
 * im2col_bytes(...) bytes.  pack_weights_rsc writes the weights in the same depth order:
 * dst[k][(r*S + s)*C + c] = wt[k][c][r][s], rows zero-padded to ceil(C*R*S, 64) bytes (the size pack_weights_bytes
 * gives for IM2COL).  The pair feeds the GEMM stage as an IM2COL operand (conv2d_int8_packed, _packed_nhwc,
 * _packed_requant with layout IM2COL and kg_pad = ceil(C*R*S, 64)). */
int im2col_nhwc_int8(int N, int C, int H, int W, int R, int S, int stride, int pad, int kg_pad,
                     const int8_t *src, int8_t *dst, void *stream);
int pack_weights_rsc(int K, int C, int R, int S, const int8_t *src, int8_t *dst, void *stream);

/* The GEMM stage with an NHWC result (Sec. 5.2): as conv2d_int8_packed, but out_nhwc is int32 [N][P][Q][K],
 * written by the epilogue itself (a lane of the MFMA result holds four consecutive channels of a pixel:
 * 16-byte stores when K % 4 == 0).  PACKED, PAD_ONLY or IM2COL (IMPLICIT: CONV_ERR_UNSUPPORTED); all three
 * pointers 16-byte aligned. */
int conv2d_int8_packed_nhwc(const conv_desc_t *desc, int layout, int cb,
                            const int8_t *in_packed, const int8_t *wt_packed, int32_t *out_nhwc,
                            int tile, int split_k, void *stream);

/* The same activation fused into the GEMM stage's epilogue (the ALU step behind the GEMM core, Sec. 5.1):
 * out_blocked = requant_pack_layout(conv2d_int8_packed(...)) without the int32 tensor ever being stored --
 * int8 [N][ceil(K/out_cb)][P + 2 out_pad][Q + 2 out_pad][out_cb], the next layer's PACKED input with its
 * spatial padding out_pad.  in_packed, wt_packed, layout, cb as for conv2d_int8_packed (with IMPLICIT:
 * the NCHW input itself and the output of pack_weights); out_cb 16, 32 or 64; shift 0..31; all three
 * pointers 16-byte aligned (IMPLICIT: out_blocked only).  One launch; a second one before it (a clear of out_blocked) when out_pad > 0 or K % out_cb != 0.
 * The whole depth is summed before the activation (no depth split). */
int conv2d_int8_packed_requant(const conv_desc_t *desc, int layout, int cb,
                               const int8_t *in_packed, const int8_t *wt_packed, int8_t *out_blocked,
                               int out_cb, int out_pad, int shift, int relu, void *stream);

/* Tensor unpacking for an NHWC consumer (the last step of the benchmark of Sec. 5.1 in the layout
 * of Sec. 5.2): dst[n][p][q][k] = src[n][k][p][q], int32. */
int unpack_nhwc_int32(int N, int K, int P, int Q, const int32_t *src, int32_t *dst, void *stream);

/* pack_weights (same rewrites on the weights, then Fuse of the reduction dimensions):
 *   dst[k][j], row length depth = pack_weights_depth(...), zero where no weight maps.
 *   PACKED / PAD_ONLY: j = ((c/cb * R + r) * S + s) * cb + c%cb   (cb a multiple of 16;
 *                      PAD_ONLY forces cb = ceil(C,16))
 *   IM2COL:            j = (c*R + r)*S + s
 *   IMPLICIT:          j = (c*R + r)*S4 + s,  S4 = ceil(S,4); for R = S = 1 and C % 64 == 0: j = c, depth = C */
int pack_weights(int K, int C, int R, int S, int layout, int cb,
                 const int8_t *src, int8_t *dst, void *stream);
int pack_weights_depth(int C, int R, int S, int layout, int cb);
size_t pack_weights_bytes(int K, int C, int R, int S, int layout, int cb);

/* im2col_int8 (Table 2 rows 1 and 5; "im2col" of Sec. 6.2):
 *   dst[(n*P + p)*Q + q][(c*R + r)*S + s] = in0[n][c][p*stride+r-pad][q*stride+s-pad],
 *   row length kg_pad >= C*R*S (a multiple of 16), zero-filled beyond C*R*S. */
int im2col_int8(int N, int C, int H, int W, int R, int S, int stride, int pad, int kg_pad,
                const int8_t *src, int8_t *dst, void *stream);
size_t im2col_bytes(int N, int C, int H, int W, int R, int S, int stride, int pad, int kg_pad);

/* image_pack_int8 / image_pack_weights (Table 2 row 1, Image Pack: [N, I] => [N*s, I/s]):
 *   packed problem (image_pack_desc): N, C2 = C*s*s, H2 = P + R2 - 1, W2 = Q + S2 - 1, K,
 *   R2 = ceil(R/s), S2 = ceil(S/s), stride 1, pad 0 -- its output is the output of `desc`.
 *   dst[n][(c*s + a)*s + b][i][j] = in0[n][c][s*i + a - pad][s*j + b - pad]      (a, b < s; 0 outside the image)
 *   wdst[k][(c*s + a)*s + b][r][t] = wt[k][c][s*r + a][s*t + b]                   (0 where s*r + a >= R or s*t + b >= S)
 *   stride 1: CONV_ERR_UNSUPPORTED.  dst must be 4-byte aligned. */
int image_pack_desc(const conv_desc_t *desc, conv_desc_t *packed);
size_t image_pack_bytes(const conv_desc_t *desc);
size_t image_pack_weights_bytes(const conv_desc_t *desc);
int image_pack_int8(const conv_desc_t *desc, const int8_t *src, int8_t *dst, void *stream);
int image_pack_weights(const conv_desc_t *desc, const int8_t *src, int8_t *dst, void *stream);

/* ---- dilated convolution (Sec. 6.1: packed into independent dense convolutions, then interleaved back)
 * Operation (stride 1, dilation d >= 2; desc->stride must be 1):
 *   out[n][k][p][q] = sum_{c,r,s} in0[n][c][p + r*d - pad][q + s*d - pad] * wt[k][c][r][s],
 *   P = H + 2 pad - d*(R-1), Q likewise; in0 as above.
 * One output pixel reads only padded-input pixels whose row and column agree with its own modulo d, so
 * the d*d phases are dense convolutions of their own: Image Pack (Table 2 row 1, [N, I] => [N*s, I/s])
 * applied to both image axes moves them into the batch,
 *   dilation_pack_int8:    dst[(n*d + a)*d + b][c][i][j] = in0[n][c][d*i + a - pad][d*j + b - pad],
 *                          dst int8 [N*d*d][C][H2][W2], H2 = ceil((H + 2 pad)/d), W2 likewise
 *                          (dilation_pack_bytes bytes; zeros where the padded image ends),
 *   dilated_desc:          the dense problem on it: N*d*d, C, H2, W2, K, R, S, stride 1, pad 0
 *                          (weights unchanged -- nothing is inflated, the point made in Sec. 6.1),
 *   dilation_unpack_int32: dst[n][k][d*i + a][d*j + b] = src[(n*d + a)*d + b][k][i][j] for d*i + a < P,
 *                          d*j + b < Q; src int32 [N*d*d][K][H2-R+1][W2-S+1], dst int32 [N][K][P][Q].
 * conv2d_int8_dilated runs the three steps: layout / cb choose how the dense problem runs (any
 * conv_layout_t that applies to it, AUTO allowed); workspace as for conv2d_int8_ex, of at least
 * conv2d_int8_dilated_workspace_bytes(desc, dilation, layout, cb) bytes (sub-images and the dense problem's
 * own workspace; with PACKED, PAD_ONLY and IM2COL the GEMM stage's epilogue writes the interleaved positions
 * itself -- three launches -- and only IMPLICIT stores the sub-images' results and interleaves in a pass of its own).  Errors: a spread kernel larger than the padded image is
 * CONV_ERR_INVALID_ARG; stride != 1, d < 2 or d > 64 are CONV_ERR_UNSUPPORTED; size queries return 0. */
int dilated_desc(const conv_desc_t *desc, int dilation, conv_desc_t *inner);
size_t dilation_pack_bytes(const conv_desc_t *desc, int dilation);
int dilation_pack_int8(const conv_desc_t *desc, int dilation, const int8_t *src, int8_t *dst, void *stream);
int dilation_unpack_int32(const conv_desc_t *desc, int dilation, const int32_t *src, int32_t *dst, void *stream);
size_t conv2d_int8_dilated_workspace_bytes(const conv_desc_t *desc, int dilation, int layout, int cb);
int conv2d_int8_dilated(const conv_desc_t *desc, int dilation, int layout, int cb,
                        const int8_t *in, const int8_t *wt, int32_t *out,
                        void *workspace, size_t workspace_bytes, void *stream);

/* The same operation without Image Pack: channel blocking of the image as it is (PACKED, block cb: 16, 32, 64
 * or 0 = library's choice) and a GEMM stage whose kernel taps are read `dilation` pixels apart -- on a machine
 * whose GEMM stage computes its operand addresses itself, a dilation is an address multiplier like a stride
 * (not the paper's route: there the intrinsic's operand must be a dense box, Sec. 4.2).  Any stride >= 1 and
 * dilation >= 1: out[n][k][p][q] = sum in0[n][c][p*stride + r*dilation - pad][q*stride + s*dilation - pad] * wt[k][c][r][s],
 * P = floor((H + 2 pad - dilation*(R-1) - 1)/stride) + 1.  Workspace as for conv2d_int8_ex, at least
 * conv2d_int8_dilated_direct_workspace_bytes(desc, dilation, cb) bytes.  Two launches. */
size_t conv2d_int8_dilated_direct_workspace_bytes(const conv_desc_t *desc, int dilation, int cb);
int conv2d_int8_dilated_direct(const conv_desc_t *desc, int dilation, int cb,
                               const int8_t *in, const int8_t *wt, int32_t *out,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Measurement aid: the int8 MFMA rate the chip sustains with nothing else in the way.  blocks workgroups of
 * four waves each issue iters x 4 v_mfma_i32_32x32x32_i8 (the GEMM unit of Sec. 5.1, 32 x 32 x 32 per
 * instruction) on register-resident pseudo-random operands that change from one instruction to the next: 2 * 32768 * 16 * iters * blocks operations in all.
 * out: blocks * 256 int32 (one checksum per lane, device memory).  blocks in 1..2^20, iters >= 1. */
int mfma_probe_int8(int blocks, int iters, int32_t *out, void *stream);

/* ---- the matrix intrinsic on its own (Sec. 5.1: C[x][y] += sum_z A[x][z] * B[y][z]) ----
 * A [X][Z], B [Y][Z] int8 row-major (both depth-contiguous, i.e. B is used transposed),
 * Cout [X][Y] int32, overwritten.  Z must be a multiple of 64. */
int gemm_int8_nt(int X, int Y, int Z, const int8_t *A, const int8_t *B, int32_t *Cout,
                 void *stream);

/* ---- per-shape layout selection (Sec. 4.4), host only, no device work ------------------
 * score = w_mac * O_MAC + w_data * O_Data, O_MAC = MAC_total - MAC_min (MACs issued after
 * padding every mapped dimension to the intrinsic minus the MACs of the definition),
 * O_Data = elements moved by rewrites and GEMM stage minus |in| + |wt| + |out|.
 * Candidates: PACKED with cb in {64,32,16}, IM2COL, PAD_ONLY, and IMPLICIT where it applies
 * (no rewritten elements, O_Data = 0; MAC_total = the MACs its kernels issue for the problem, as
 * layout_overheads reports them), and for strides above one IMAGE_PACK with inner
 * cb in {0,16,32,64} (the inner layout's terms on the packed problem, measured against the MACs
 * of the original definition, plus 2*(|X2| + |W2|) moved elements for the pack itself).  Ties: fewer rewritten
 * elements, then lower layout code, then larger cb.  select_layout uses the library's
 * MI355X weights (seconds per MAC and per byte); the paper's case studies use w = [1,1]. */
int select_layout(const conv_desc_t *desc, int *layout, int *cb, double *score);
int select_layout_weighted(const conv_desc_t *desc, double w_mac, double w_data,
                           int *layout, int *cb, double *score);
int layout_overheads(const conv_desc_t *desc, int layout, int cb,
                     int64_t *o_mac, int64_t *o_data, int64_t *rewritten_elems);

const char *conv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CONV2D_INT8_H */
