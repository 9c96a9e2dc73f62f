// C-ABI glue: argument validation, layout resolution, workspace carving, launch order.
// Every step of the path runs in the HIP kernels; nothing here touches tensor data.
#include "../../include/conv2d_int8.h"
#include "desc_check.h"
#include "kernels.h"

#include <mutex>

using namespace c2i8;

// Workspace of conv2d_int8_static, the entry point that allocates nothing (see there).
constexpr size_t STATIC_WS_BYTES = CONV_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_WS_BYTES];

namespace {

constexpr size_t WS_ALIGN = 256;
constexpr long long INT_LIMIT = 2147483647LL;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
int round_up_i(int x, int m) { return (x + m - 1) / m * m; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check_desc(const conv_desc_t *d) { return check_conv_desc(d); }

struct Plan {
    int layout, cb, Cb, depth, P, Q, Hp, Wp;
    int pointwise;  // IMPLICIT only: the 1x1 kernel takes it (else the window kernel)
    long long M;
    size_t x_bytes, w_bytes;
};

WindowProblem window_problem(const conv_desc_t *d, const Plan &pl, const int8_t *x, const int8_t *w,
                             int32_t *out, int wt_rewritten)
{
    return WindowProblem{x, w, out, d->N, d->C, d->H, d->W, d->K, pl.P, pl.Q, d->R, d->S, d->stride, d->pad,
                         wt_rewritten, ActOut{}, 0, 0};
}

int run_implicit(const Plan &pl, const WindowProblem &g, hipStream_t st)
{
    const hipError_t e = pl.pointwise ? launch_pointwise_conv(g, st) : launch_window_conv(g, st);
    return e == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int default_block(int C)
{
    if (C >= 64) return 64;
    if (C > 32) return 64;
    if (C > 16) return 32;
    return 16;
}

// Resolves AUTO / default block and sizes the rewritten operands.
int make_plan(const conv_desc_t *d, int layout, int cb, Plan *pl)
{
    int rc = check_desc(d);
    if (rc != CONV_OK) return rc;
    if (layout == CONV_LAYOUT_AUTO) {
        rc = select_layout(d, &layout, &cb, nullptr);
        if (rc != CONV_OK) return rc;
    }
    if (layout == CONV_LAYOUT_IMAGE_PACK) return CONV_ERR_UNSUPPORTED;  // two stages: not a single plan
    if (layout == CONV_LAYOUT_PAD_ONLY) cb = round_up_i(d->C, 16);
    else if (layout == CONV_LAYOUT_PACKED) {
        if (cb == 0) cb = default_block(d->C);
        if (cb < 16 || cb > 1024 || cb % 16) return CONV_ERR_UNSUPPORTED;
    } else if (layout == CONV_LAYOUT_IM2COL || layout == CONV_LAYOUT_IMPLICIT) cb = 0;
    else return CONV_ERR_INVALID_ARG;

    pl->layout = layout;
    pl->pointwise = 0;
    pl->cb = cb;
    pl->Hp = d->H + 2 * d->pad;
    pl->Wp = d->W + 2 * d->pad;
    pl->P = (pl->Hp - d->R) / d->stride + 1;
    pl->Q = (pl->Wp - d->S) / d->stride + 1;
    pl->M = (long long)d->N * pl->P * pl->Q;
    if (layout == CONV_LAYOUT_IMPLICIT) {
        pl->Cb = 0;
        pl->pointwise = pointwise_shape(d->C, d->R, d->S);
        pl->depth = pl->pointwise ? d->C : window_depth(d->C, d->R, d->S);
        const WindowProblem wp = window_problem(d, *pl, nullptr, nullptr, nullptr, 0);
        if (!(pl->pointwise ? pointwise_fits(wp) : window_fits(wp))) return CONV_ERR_UNSUPPORTED;
        pl->x_bytes = 0;  // nothing is rewritten: the GEMM stage reads the input and either weight form
        pl->w_bytes = 0;
        return CONV_OK;
    }
    if (layout == CONV_LAYOUT_IM2COL) {
        pl->Cb = 0;
        pl->depth = round_up_i(d->C * d->R * d->S, CONV_DEPTH_ALIGN);
        pl->x_bytes = (size_t)pl->M * pl->depth;
    } else {
        pl->Cb = (d->C + cb - 1) / cb;
        const long long real = (long long)pl->Cb * cb * d->R * d->S;
        if (real > (1LL << 24)) return CONV_ERR_UNSUPPORTED;
        pl->depth = round_up_i((int)real, CONV_DEPTH_ALIGN);
        const long long img = (long long)pl->Cb * pl->Hp * pl->Wp * cb;
        if (img > INT_LIMIT) return CONV_ERR_UNSUPPORTED;  // per-image offsets are 32-bit
        pl->x_bytes = (size_t)d->N * (size_t)img;
    }
    pl->w_bytes = (size_t)d->K * pl->depth;
    return CONV_OK;
}

// Image Pack: the equivalent stride-1, pad-0 problem, the sizes of its two rewritten operands, and
// the layout the stride-1 convolution then runs in (cb = 0: IMPLICIT, else PACKED with that block).
struct PackedProblem {
    conv_desc_t d2;
    size_t x2_bytes, w2_bytes;
    int inner_layout, inner_cb;
};

int image_pack_problem(const conv_desc_t *d, int cb, PackedProblem *pp, bool with_inner = true)
{
    int rc = check_desc(d);
    if (rc != CONV_OK) return rc;
    if (d->stride < 2) return CONV_ERR_UNSUPPORTED;  // nothing to pack
    const long long s = d->stride;
    const long long C2 = (long long)d->C * s * s;
    const long long R2 = (d->R + s - 1) / s, S2 = (d->S + s - 1) / s;
    const long long P = ((long long)d->H + 2LL * d->pad - d->R) / s + 1, Q = ((long long)d->W + 2LL * d->pad - d->S) / s + 1;
    const long long H2 = P + R2 - 1, W2 = Q + S2 - 1;
    if (C2 > INT_LIMIT || H2 > INT_LIMIT || W2 > INT_LIMIT || C2 * R2 * S2 > 131072LL) return CONV_ERR_UNSUPPORTED;
    pp->d2 = conv_desc_t{d->N, (int)C2, (int)H2, (int)W2, d->K, (int)R2, (int)S2, 1, 0};
    pp->x2_bytes = (size_t)d->N * (size_t)C2 * (size_t)H2 * (size_t)W2;
    pp->w2_bytes = (size_t)d->K * (size_t)C2 * (size_t)R2 * (size_t)S2;
    pp->inner_layout = cb == 0 ? CONV_LAYOUT_IMPLICIT : CONV_LAYOUT_PACKED;
    pp->inner_cb = cb;
    if (!with_inner) return CONV_OK;  // the pack alone: whatever runs on its output is the caller's choice
    Plan inner;
    return make_plan(&pp->d2, pp->inner_layout, pp->inner_cb, &inner);
}

// Dilation (stride 1) as Image Pack into the batch: the dense stride-1, pad-0 problem on the d*d
// sub-images of every padded image, and the sizes of the sub-image tensor and of its result.
struct DilatedProblem {
    conv_desc_t d2;
    int P, Q;  // extents of the dilated convolution's own output
    size_t x2_bytes, o2_bytes;
};

int dilated_problem(const conv_desc_t *d, int dilation, DilatedProblem *dp)
{
    if (!d) return CONV_ERR_INVALID_ARG;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride <= 0 ||
        d->pad < 0 || dilation <= 0)
        return CONV_ERR_INVALID_ARG;
    const long long dl = dilation;
    const long long Hp = (long long)d->H + 2LL * d->pad, Wp = (long long)d->W + 2LL * d->pad;
    const long long Re = dl * (d->R - 1) + 1, Se = dl * (d->S - 1) + 1;  // extent of the spread kernel
    if (Re > Hp || Se > Wp) return CONV_ERR_INVALID_ARG;
    if (d->stride != 1 || dilation < 2 || dilation > 64) return CONV_ERR_UNSUPPORTED;  // 1: nothing to pack
    if (Hp > INT_LIMIT || Wp > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    const long long N2 = (long long)d->N * dl * dl;
    const long long H2 = (Hp + dl - 1) / dl, W2 = (Wp + dl - 1) / dl;
    if (N2 > INT_LIMIT || H2 * W2 > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    dp->d2 = conv_desc_t{(int)N2, d->C, (int)H2, (int)W2, d->K, d->R, d->S, 1, 0};
    int rc = check_desc(&dp->d2);
    if (rc != CONV_OK) return rc;
    dp->P = (int)(Hp - Re + 1);
    dp->Q = (int)(Wp - Se + 1);
    if ((long long)dp->P * dp->Q > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    const long long P2 = H2 - d->R + 1, Q2 = W2 - d->S + 1;
    dp->x2_bytes = (size_t)N2 * d->C * (size_t)(H2 * W2);
    dp->o2_bytes = (size_t)N2 * d->K * (size_t)(P2 * Q2) * sizeof(int32_t);
    return CONV_OK;
}

// AUTO -> the selector's choice (which may be IMAGE_PACK with its inner block in *cb).
int resolve_layout(const conv_desc_t *d, int *layout, int *cb)
{
    if (*layout != CONV_LAYOUT_AUTO) return CONV_OK;
    int rc = check_desc(d);
    if (rc != CONV_OK) return rc;
    return select_layout(d, layout, cb, nullptr);
}

GemmProblem gemm_problem(const conv_desc_t *d, const Plan &pl, const int8_t *x, const int8_t *w,
                         int32_t *out)
{
    GemmProblem g{};
    g.act = x;
    g.wq = w;
    g.out = out;
    g.K = d->K;
    g.M = (int)pl.M;
    g.depth = pl.depth;
    g.PQ = pl.P * pl.Q;
    g.Q = pl.Q;
    g.mode = pl.layout == CONV_LAYOUT_IM2COL ? ACT_MATRIX : ACT_BLOCKED;
    g.stride = d->stride;
    g.cb = pl.cb;
    g.Cb = pl.Cb;
    g.R = d->R;
    g.S = d->S;
    g.Hp = pl.Hp;
    g.Wp = pl.Wp;
    return g;
}

// hipErrorInvalidValue comes from the launcher's own guards (a tile / split pair the picker would not
// offer); nothing was enqueued then.
int gemm_status(hipError_t e)
{
    return e == hipSuccess ? CONV_OK : e == hipErrorInvalidValue ? CONV_ERR_UNSUPPORTED : CONV_ERR_DEVICE;
}

// Which kernel runs the GEMM stage: a tile of the general kernel with a depth split, or the band kernel.
struct GemmChoice {
    int tile, split_k;  // tile == CONV_TILE_BAND: the band kernel (split_k 1)
};

int choose_gemm(const GemmProblem &g, int tile, int split_k, GemmChoice *c)
{
    if (tile == CONV_TILE_BAND) {
        if (split_k < 0 || split_k > 1 || !band_applies(g)) return split_k < 0 ? CONV_ERR_INVALID_ARG : CONV_ERR_UNSUPPORTED;
        *c = GemmChoice{CONV_TILE_BAND, 1};
        return CONV_OK;
    }
    if (tile < -1 || tile >= gemm_num_tiles()) return CONV_ERR_INVALID_ARG;
    if (split_k < 0) return CONV_ERR_INVALID_ARG;
    const bool free_choice = tile == -1 && split_k == 0;
    int t = tile, s = split_k;
    if (g.out && !aligned16(g.out) && s == 0) s = 1;  // the clear before a depth split writes 16-byte pieces
    if (g.out && !aligned16(g.out) && s > 1) return CONV_ERR_INVALID_ARG;
    double cost = 0;
    if (!gemm_pick(g, &t, &s, &cost)) {
        if (free_choice && band_applies(g)) {
            *c = GemmChoice{CONV_TILE_BAND, 1};
            return CONV_OK;
        }
        return CONV_ERR_UNSUPPORTED;
    }
    if (free_choice && band_cost(g) < cost) {
        *c = GemmChoice{CONV_TILE_BAND, 1};
        return CONV_OK;
    }
    *c = GemmChoice{t, s};
    return CONV_OK;
}

int run_gemm(const GemmProblem &g, int tile, int split_k, hipStream_t st)
{
    GemmChoice c;
    const int rc = choose_gemm(g, tile, split_k, &c);
    if (rc != CONV_OK) return rc;
    if (c.tile == CONV_TILE_BAND) return gemm_status(launch_band_conv(g, st));
    return gemm_status(launch_gemm(g, c.tile, c.split_k, st));
}

int rewrite_weights(const conv_desc_t *d, const Plan &pl, const int8_t *wt, int8_t *dst, hipStream_t st)
{
    hipError_t e;
    if (pl.layout == CONV_LAYOUT_IM2COL)
        e = launch_pack_weights_rows(d->K, d->C * d->R * d->S, pl.depth, wt, dst, st);
    else
        e = launch_pack_weights_blocked(d->K, d->C, d->R, d->S, pl.cb, pl.depth, wt, dst, st);
    return e == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int rewrite_input(const conv_desc_t *d, const Plan &pl, const int8_t *in, int8_t *dst, hipStream_t st)
{
    hipError_t e;
    if (pl.layout == CONV_LAYOUT_IM2COL)
        e = launch_im2col(d->N, d->C, d->H, d->W, d->R, d->S, d->stride, d->pad, pl.P, pl.Q, pl.depth,
                          in, dst, st);
    else
        e = launch_pack_layout(d->N, d->C, d->H, d->W, pl.cb, d->pad, in, dst, st);
    return e == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

// Cached workspace of the one-shot entry points, one per device, grown on demand.  A block that a larger
// problem supersedes is never freed: work already enqueued, or a HIP graph captured earlier, may still
// reference it, so it stays allocated until the process ends (blocks grow geometrically, so all superseded
// blocks together are smaller than the current one).
struct DeviceCache {
    void *ptr = nullptr;
    size_t bytes = 0;
};
std::mutex g_cache_mutex;
DeviceCache g_cache[64];

// The current device's block of at least `need` bytes.  Growing allocates, which a stream under capture
// must not do: then CONV_ERR_WORKSPACE, with no device call made.
int cached_workspace(size_t need, hipStream_t st, void **ptr, size_t *bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CONV_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    DeviceCache &c = g_cache[dev];
    if (c.bytes < need) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cs) != hipSuccess) return CONV_ERR_DEVICE;
        if (cs != hipStreamCaptureStatusNone) return CONV_ERR_WORKSPACE;
        const size_t least = align_up(need, 1 << 20);
        size_t want = align_up(need + need / 4, 1 << 20);
        if (want < 2 * c.bytes) want = 2 * c.bytes;
        void *p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess || !p) {
            (void)hipGetLastError();  // the generous size did not fit: try what this problem needs
            p = nullptr;
            want = least;
            if (hipMalloc(&p, want) != hipSuccess || !p) {
                (void)hipGetLastError();
                return CONV_ERR_WORKSPACE;
            }
        }
        c.ptr = p;  // the superseded block stays allocated (see above)
        c.bytes = want;
    }
    *ptr = c.ptr;
    *bytes = c.bytes;
    return CONV_OK;
}

// ---- workspace of the entry point that allocates nothing -----------------------------------------
// A file-scope device array stands in for the cached workspace.  Every GPU the library runs on holds
// its own copy of it, at its own address, from the moment the code object is loaded there until the
// process ends.  In host code the array's NAME is only a handle for the runtime: the address kernels
// can use is what hipGetSymbolAddress returns for the device that is current, asked once per device.
std::mutex g_static_ws_mutex;
void *g_static_ws[64] = {};  // per device: device address of `scratch` there

int static_workspace(void **ptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CONV_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_static_ws_mutex);
    if (!g_static_ws[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return CONV_ERR_DEVICE;
        }
        if (reinterpret_cast<uintptr_t>(p) % WS_ALIGN) return CONV_ERR_DEVICE;
        g_static_ws[dev] = p;
    }
    *ptr = g_static_ws[dev];
    return CONV_OK;
}

}  // namespace

extern "C" {

const char *conv_status_string(int s)
{
    switch (s) {
        case CONV_OK: return "ok";
        case CONV_ERR_INVALID_ARG: return "invalid argument";
        case CONV_ERR_UNSUPPORTED: return "unsupported problem";
        case CONV_ERR_OVERFLOW_RISK: return "reduction too deep for an int32 accumulator";
        case CONV_ERR_WORKSPACE: return "workspace too small or allocation failed";
        case CONV_ERR_DEVICE: return "HIP error";
    }
    return "unknown status";
}

size_t pack_layout_bytes(int N, int C, int H, int W, int cb, int pad)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || pad < 0 || cb < 4 || cb > 1024 || cb % 4) return 0;
    return (size_t)N * ((C + cb - 1) / cb) * cb * ((size_t)H + 2 * pad) * ((size_t)W + 2 * pad);
}

int pack_layout(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst,
                void *stream)
{
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0 || pad < 0) return CONV_ERR_INVALID_ARG;
    if (cb < 4 || cb > 1024 || cb % 4) return CONV_ERR_UNSUPPORTED;
    if (!aligned16(dst)) return CONV_ERR_INVALID_ARG;
    if ((long long)H + 2LL * pad > INT_LIMIT || (long long)W + 2LL * pad > INT_LIMIT)
        return CONV_ERR_UNSUPPORTED;
    return launch_pack_layout(N, C, H, W, cb, pad, src, dst, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ERR_DEVICE;
}

int pack_layout_nhwc(int N, int C, int H, int W, int cb, int pad, const int8_t *src, int8_t *dst, void *stream)
{
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0 || pad < 0) return CONV_ERR_INVALID_ARG;
    if (cb < 16 || cb > 1024 || cb % 16) return CONV_ERR_UNSUPPORTED;
    if (!aligned16(dst)) return CONV_ERR_INVALID_ARG;
    if ((long long)H + 2LL * pad > INT_LIMIT || (long long)W + 2LL * pad > INT_LIMIT)
        return CONV_ERR_UNSUPPORTED;
    return launch_pack_layout_nhwc(N, C, H, W, cb, pad, src, dst, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ERR_DEVICE;
}

int requant_int8(long long count, const int32_t *src, int8_t *dst, int shift, int relu, void *stream)
{
    if (!src || !dst || count <= 0 || shift < 0 || shift > 31) return CONV_ERR_INVALID_ARG;
    return launch_requant(count, src, dst, shift, relu != 0, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int requant_pack_layout(int N, int K, int P, int Q, int cb, int pad, int shift, int relu, const int32_t *src,
                        int8_t *dst, void *stream)
{
    if (!src || !dst || N <= 0 || K <= 0 || P <= 0 || Q <= 0 || pad < 0 || shift < 0 || shift > 31)
        return CONV_ERR_INVALID_ARG;
    if (cb < 16 || cb > 1024 || cb % 16) return CONV_ERR_UNSUPPORTED;
    if (!aligned16(dst)) return CONV_ERR_INVALID_ARG;
    if ((long long)P + 2LL * pad > INT_LIMIT || (long long)Q + 2LL * pad > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    return launch_requant_pack(N, K, P, Q, cb, pad, shift, relu != 0, src, dst, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ERR_DEVICE;
}

int unpack_nhwc_int32(int N, int K, int P, int Q, const int32_t *src, int32_t *dst, void *stream)
{
    if (!src || !dst || N <= 0 || K <= 0 || P <= 0 || Q <= 0) return CONV_ERR_INVALID_ARG;
    if ((long long)P * Q > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    return launch_unpack_nhwc(N, K, (long long)P * Q, src, dst, (hipStream_t)stream) == hipSuccess ? CONV_OK
                                                                                                  : CONV_ERR_DEVICE;
}

int pack_weights_depth(int C, int R, int S, int layout, int cb)
{
    if (C <= 0 || R <= 0 || S <= 0) return 0;
    long long real;
    if (layout == CONV_LAYOUT_IMPLICIT) return pointwise_shape(C, R, S) ? (C <= 512 ? C : 0) : window_depth(C, R, S);
    if (layout == CONV_LAYOUT_IM2COL) real = (long long)C * R * S;
    else if (layout == CONV_LAYOUT_PACKED || layout == CONV_LAYOUT_PAD_ONLY) {
        if (layout == CONV_LAYOUT_PAD_ONLY) cb = round_up_i(C, 16);
        if (cb < 16 || cb > 1024 || cb % 16) return 0;
        real = (long long)((C + cb - 1) / cb) * cb * R * S;
    } else return 0;
    if (real > (1LL << 24)) return 0;
    return round_up_i((int)real, CONV_DEPTH_ALIGN);
}

size_t pack_weights_bytes(int K, int C, int R, int S, int layout, int cb)
{
    if (K <= 0) return 0;
    return (size_t)K * (size_t)pack_weights_depth(C, R, S, layout, cb);
}

int pack_weights(int K, int C, int R, int S, int layout, int cb, const int8_t *src, int8_t *dst,
                 void *stream)
{
    if (!src || !dst || K <= 0 || C <= 0 || R <= 0 || S <= 0) return CONV_ERR_INVALID_ARG;
    if (layout != CONV_LAYOUT_IM2COL && layout != CONV_LAYOUT_PACKED && layout != CONV_LAYOUT_PAD_ONLY &&
        layout != CONV_LAYOUT_IMPLICIT)
        return CONV_ERR_INVALID_ARG;
    if (!aligned16(dst)) return CONV_ERR_INVALID_ARG;
    if (layout == CONV_LAYOUT_PAD_ONLY) cb = round_up_i(C, 16);
    const int depth = pack_weights_depth(C, R, S, layout, cb);
    if (depth == 0) return CONV_ERR_UNSUPPORTED;
    hipError_t e;
    if (layout == CONV_LAYOUT_IMPLICIT && pointwise_shape(C, R, S))
        e = launch_pack_weights_rows(K, C, depth, src, dst, (hipStream_t)stream);  // [K][C] as it is
    else if (layout == CONV_LAYOUT_IMPLICIT)
        e = launch_pack_weights_window(K, C, R, S, src, dst, (hipStream_t)stream);
    else if (layout == CONV_LAYOUT_IM2COL)
        e = launch_pack_weights_rows(K, C * R * S, depth, src, dst, (hipStream_t)stream);
    else
        e = launch_pack_weights_blocked(K, C, R, S, cb, depth, src, dst, (hipStream_t)stream);
    return e == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

size_t im2col_bytes(int N, int C, int H, int W, int R, int S, int stride, int pad, int kg_pad)
{
    conv_desc_t d{N, C, H, W, 1, R, S, stride, pad};
    if (check_desc(&d) != CONV_OK || kg_pad < C * R * S || kg_pad % 16) return 0;
    const long long P = (H + 2LL * pad - R) / stride + 1, Q = (W + 2LL * pad - S) / stride + 1;
    return (size_t)N * P * Q * kg_pad;
}

int im2col_int8(int N, int C, int H, int W, int R, int S, int stride, int pad, int kg_pad,
                const int8_t *src, int8_t *dst, void *stream)
{
    conv_desc_t d{N, C, H, W, 1, R, S, stride, pad};
    int rc = check_desc(&d);
    if (rc != CONV_OK) return rc;
    if (!src || !dst || !aligned16(dst)) return CONV_ERR_INVALID_ARG;
    if (kg_pad < C * R * S || kg_pad % 16) return CONV_ERR_INVALID_ARG;
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    return launch_im2col(N, C, H, W, R, S, stride, pad, P, Q, kg_pad, src, dst, (hipStream_t)stream) ==
                   hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int im2col_nhwc_int8(int N, int C, int H, int W, int R, int S, int stride, int pad, int kg_pad,
                     const int8_t *src, int8_t *dst, void *stream)
{
    conv_desc_t d{N, C, H, W, 1, R, S, stride, pad};
    int rc = check_desc(&d);
    if (rc != CONV_OK) return rc;
    if (!src || !dst || !aligned16(dst)) return CONV_ERR_INVALID_ARG;
    if (C % 16 == 0 && !aligned16(src)) return CONV_ERR_INVALID_ARG;  // 16-byte loads of a tap's channels
    if (kg_pad < C * R * S || kg_pad % 16) return CONV_ERR_INVALID_ARG;
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    return launch_im2col_nhwc(N, C, H, W, R, S, stride, pad, P, Q, kg_pad, src, dst, (hipStream_t)stream) == hipSuccess
               ? CONV_OK : CONV_ERR_DEVICE;
}

int pack_weights_rsc(int K, int C, int R, int S, const int8_t *src, int8_t *dst, void *stream)
{
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0 || !src || !dst) return CONV_ERR_INVALID_ARG;
    if ((long long)C * R * S > 131072LL) return CONV_ERR_OVERFLOW_RISK;
    const int depth = round_up_i(C * R * S, CONV_DEPTH_ALIGN);
    return launch_pack_weights_rsc(K, C, R, S, depth, src, dst, (hipStream_t)stream) == hipSuccess ? CONV_OK
                                                                                                  : CONV_ERR_DEVICE;
}

int image_pack_desc(const conv_desc_t *desc, conv_desc_t *packed)
{
    if (!packed) return CONV_ERR_INVALID_ARG;
    PackedProblem pp;
    int rc = image_pack_problem(desc, 16, &pp, false);
    if (rc != CONV_OK) return rc;
    *packed = pp.d2;
    return CONV_OK;
}

size_t image_pack_bytes(const conv_desc_t *desc)
{
    PackedProblem pp;
    return image_pack_problem(desc, 16, &pp, false) == CONV_OK ? pp.x2_bytes : 0;
}

size_t image_pack_weights_bytes(const conv_desc_t *desc)
{
    PackedProblem pp;
    return image_pack_problem(desc, 16, &pp, false) == CONV_OK ? pp.w2_bytes : 0;
}

int image_pack_int8(const conv_desc_t *desc, const int8_t *src, int8_t *dst, void *stream)
{
    PackedProblem pp;
    int rc = image_pack_problem(desc, 16, &pp, false);
    if (rc != CONV_OK) return rc;
    if (!src || !dst || (reinterpret_cast<uintptr_t>(dst) & 3)) return CONV_ERR_INVALID_ARG;
    return launch_image_pack(desc->N, desc->C, desc->H, desc->W, desc->stride, desc->pad, pp.d2.H, pp.d2.W, src, dst,
                             (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int image_pack_weights(const conv_desc_t *desc, const int8_t *src, int8_t *dst, void *stream)
{
    PackedProblem pp;
    int rc = image_pack_problem(desc, 16, &pp, false);
    if (rc != CONV_OK) return rc;
    if (!src || !dst) return CONV_ERR_INVALID_ARG;
    return launch_image_pack_weights(desc->K, desc->C, desc->R, desc->S, desc->stride, src, dst,
                                     (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int dilated_desc(const conv_desc_t *desc, int dilation, conv_desc_t *inner)
{
    if (!inner) return CONV_ERR_INVALID_ARG;
    DilatedProblem dp;
    int rc = dilated_problem(desc, dilation, &dp);
    if (rc != CONV_OK) return rc;
    *inner = dp.d2;
    return CONV_OK;
}

size_t dilation_pack_bytes(const conv_desc_t *desc, int dilation)
{
    DilatedProblem dp;
    return dilated_problem(desc, dilation, &dp) == CONV_OK ? dp.x2_bytes : 0;
}

int dilation_pack_int8(const conv_desc_t *desc, int dilation, const int8_t *src, int8_t *dst, void *stream)
{
    DilatedProblem dp;
    int rc = dilated_problem(desc, dilation, &dp);
    if (rc != CONV_OK) return rc;
    if (!src || !dst) return CONV_ERR_INVALID_ARG;
    const hipError_t e = launch_dilation_pack(desc->N, desc->C, desc->H, desc->W, desc->pad, dilation, dp.d2.H, dp.d2.W,
                                              src, dst, (hipStream_t)stream);
    return e == hipSuccess ? CONV_OK : e == hipErrorInvalidValue ? CONV_ERR_UNSUPPORTED : CONV_ERR_DEVICE;
}

int dilation_unpack_int32(const conv_desc_t *desc, int dilation, const int32_t *src, int32_t *dst, void *stream)
{
    DilatedProblem dp;
    int rc = dilated_problem(desc, dilation, &dp);
    if (rc != CONV_OK) return rc;
    if (!src || !dst) return CONV_ERR_INVALID_ARG;
    const hipError_t e = launch_dilation_unpack(desc->N, desc->K, dp.P, dp.Q, dilation, dp.d2.H - desc->R + 1,
                                                dp.d2.W - desc->S + 1, src, dst, (hipStream_t)stream);
    return e == hipSuccess ? CONV_OK : e == hipErrorInvalidValue ? CONV_ERR_UNSUPPORTED : CONV_ERR_DEVICE;
}

size_t conv2d_int8_dilated_workspace_bytes(const conv_desc_t *desc, int dilation, int layout, int cb)
{
    DilatedProblem dp;
    if (dilated_problem(desc, dilation, &dp) != CONV_OK) return 0;
    if (resolve_layout(&dp.d2, &layout, &cb) != CONV_OK) return 0;
    Plan pl;
    if (make_plan(&dp.d2, layout, cb, &pl) != CONV_OK) return 0;
    const size_t inner = conv2d_int8_workspace_bytes(&dp.d2, layout, cb, 0);
    // the GEMM stage interleaves in its epilogue; only IMPLICIT stores the sub-images' results
    const size_t ob = pl.layout == CONV_LAYOUT_IMPLICIT ? align_up(dp.o2_bytes, WS_ALIGN) : 0;
    return align_up(dp.x2_bytes, WS_ALIGN) + ob + inner;
}

int conv2d_int8_dilated(const conv_desc_t *desc, int dilation, int layout, int cb, const int8_t *in, const int8_t *wt,
                        int32_t *out, void *workspace, size_t workspace_bytes, void *stream)
{
    DilatedProblem dp;
    int rc = dilated_problem(desc, dilation, &dp);
    if (rc != CONV_OK) return rc;
    rc = resolve_layout(&dp.d2, &layout, &cb);
    if (rc != CONV_OK) return rc;
    if (!in || !wt || !out || !workspace || (reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)))
        return CONV_ERR_INVALID_ARG;
    Plan pl;
    rc = make_plan(&dp.d2, layout, cb, &pl);  // the dense problem runs in one single-stage layout
    if (rc != CONV_OK) return rc;
    const size_t inner = conv2d_int8_workspace_bytes(&dp.d2, layout, cb, 0);
    const bool stored = pl.layout == CONV_LAYOUT_IMPLICIT;  // else the GEMM stage's epilogue interleaves
    const size_t xb = align_up(dp.x2_bytes, WS_ALIGN), ob = stored ? align_up(dp.o2_bytes, WS_ALIGN) : 0;
    if (workspace_bytes < xb + ob + inner) return CONV_ERR_WORKSPACE;
    int8_t *x2 = static_cast<int8_t *>(workspace);
    void *ws = inner ? static_cast<void *>(x2 + xb + ob) : nullptr;
    rc = dilation_pack_int8(desc, dilation, in, x2, stream);
    if (rc != CONV_OK) return rc;
    if (stored) {
        int32_t *o2 = reinterpret_cast<int32_t *>(x2 + xb);
        rc = conv2d_int8_ex(&dp.d2, layout, cb, x2, wt, 0, o2, ws, inner, stream);
        if (rc != CONV_OK) return rc;
        return dilation_unpack_int32(desc, dilation, o2, out, stream);
    }
    // both rewrites of the dense problem, then its GEMM stage writing the dilated layer's own output
    hipStream_t st = (hipStream_t)stream;
    int8_t *xq = static_cast<int8_t *>(ws), *wq = xq + align_up(pl.x_bytes, WS_ALIGN);
    const conv_desc_t &e2 = dp.d2;
    const hipError_t e = launch_rewrite_fused(pl.layout == CONV_LAYOUT_IM2COL, e2.N, e2.C, e2.H, e2.W, e2.K, e2.R, e2.S,
                                              e2.stride, e2.pad, pl.P, pl.Q, pl.cb, pl.depth, x2, xq, wt, wq, st);
    if (e == hipErrorNotSupported) {
        rc = rewrite_weights(&dp.d2, pl, wt, wq, st);
        if (rc != CONV_OK) return rc;
        rc = rewrite_input(&dp.d2, pl, x2, xq, st);
        if (rc != CONV_OK) return rc;
    } else if (e != hipSuccess) return CONV_ERR_DEVICE;
    GemmProblem g = gemm_problem(&dp.d2, pl, xq, wq, out);
    g.il_d = dilation;
    g.il_P = dp.P;
    g.il_Q = dp.Q;
    // no depth split (the activation needs the whole sum): the band kernel, or the best tile of the general one
    int t = -1, s = 1;
    double cost = 0;
    const bool tiled = gemm_pick(g, &t, &s, &cost);
    if (band_applies(g) && (!tiled || band_cost(g) < cost)) return gemm_status(launch_band_conv(g, st));
    if (!tiled) return CONV_ERR_UNSUPPORTED;
    return gemm_status(launch_gemm(g, t, 1, st));
}

// Dilation as an address multiplier: the plan of the undilated problem with the dilated layer's output extents.
static int direct_dilated_plan(const conv_desc_t *desc, int dilation, int cb, Plan *pl)
{
    if (!desc || dilation <= 0) return CONV_ERR_INVALID_ARG;
    int rc = make_plan(desc, CONV_LAYOUT_PACKED, cb, pl);
    if (rc != CONV_OK) return rc;
    const long long Re = (long long)dilation * (desc->R - 1) + 1, Se = (long long)dilation * (desc->S - 1) + 1;
    if (Re > pl->Hp || Se > pl->Wp) return CONV_ERR_INVALID_ARG;
    pl->P = (int)((pl->Hp - Re) / desc->stride + 1);
    pl->Q = (int)((pl->Wp - Se) / desc->stride + 1);
    pl->M = (long long)desc->N * pl->P * pl->Q;
    return CONV_OK;
}

size_t conv2d_int8_dilated_direct_workspace_bytes(const conv_desc_t *desc, int dilation, int cb)
{
    Plan pl;
    if (direct_dilated_plan(desc, dilation, cb, &pl) != CONV_OK) return 0;
    return align_up(pl.x_bytes, WS_ALIGN) + align_up(pl.w_bytes, WS_ALIGN);
}

int conv2d_int8_dilated_direct(const conv_desc_t *desc, int dilation, int cb, const int8_t *in, const int8_t *wt,
                               int32_t *out, void *workspace, size_t workspace_bytes, void *stream)
{
    Plan pl;
    int rc = direct_dilated_plan(desc, dilation, cb, &pl);
    if (rc != CONV_OK) return rc;
    if (!in || !wt || !out || !workspace || (reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)))
        return CONV_ERR_INVALID_ARG;
    const size_t xb = align_up(pl.x_bytes, WS_ALIGN);
    if (workspace_bytes < xb + align_up(pl.w_bytes, WS_ALIGN)) return CONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int8_t *xq = static_cast<int8_t *>(workspace), *wq = xq + xb;
    const hipError_t e = launch_rewrite_fused(false, desc->N, desc->C, desc->H, desc->W, desc->K, desc->R, desc->S,
                                              desc->stride, desc->pad, pl.P, pl.Q, pl.cb, pl.depth, in, xq, wt, wq, st);
    if (e == hipErrorNotSupported) {
        rc = rewrite_weights(desc, pl, wt, wq, st);
        if (rc != CONV_OK) return rc;
        rc = rewrite_input(desc, pl, in, xq, st);
        if (rc != CONV_OK) return rc;
    } else if (e != hipSuccess) return CONV_ERR_DEVICE;
    GemmProblem g = gemm_problem(desc, pl, xq, wq, out);
    g.dil = dilation;
    return run_gemm(g, -1, 0, st);
}

int mfma_probe_int8(int blocks, int iters, int32_t *out, void *stream)
{
    if (blocks <= 0 || blocks > (1 << 20) || iters <= 0 || !out) return CONV_ERR_INVALID_ARG;
    return launch_mfma_probe(blocks, iters, out, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

int gemm_int8_nt(int X, int Y, int Z, const int8_t *A, const int8_t *B, int32_t *Cout, void *stream)
{
    if (X <= 0 || Y <= 0 || Z <= 0 || !A || !B || !Cout) return CONV_ERR_INVALID_ARG;
    if (Z % CONV_DEPTH_ALIGN) return CONV_ERR_UNSUPPORTED;
    if (Z > 131072) return CONV_ERR_OVERFLOW_RISK;
    if (!aligned16(A) || !aligned16(B)) return CONV_ERR_INVALID_ARG;
    GemmProblem g{};
    g.act = B;
    g.wq = A;
    g.out = Cout;
    g.K = X;
    g.M = Y;
    g.depth = Z;
    g.PQ = Y;
    g.Q = Y;
    g.mode = ACT_MATRIX;
    return run_gemm(g, -1, 0, (hipStream_t)stream);
}

int conv2d_int8_num_tiles(void) { return gemm_num_tiles(); }

int conv2d_int8_tile_info(int tile, int *rows, int *cols, int *threads, int *steps)
{
    if (tile < 0 || tile >= gemm_num_tiles()) return CONV_ERR_INVALID_ARG;
    TileInfo t = gemm_tile_info(tile);
    if (rows) *rows = t.rows;
    if (cols) *cols = t.cols;
    if (threads) *threads = t.threads;
    if (steps) *steps = t.steps;
    return CONV_OK;
}

int conv2d_int8_packed(const conv_desc_t *desc, int layout, int cb, const int8_t *in_packed,
                       const int8_t *wt_packed, int32_t *out, int tile, int split_k, void *stream)
{
    if (layout == CONV_LAYOUT_AUTO) return CONV_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(desc, layout, cb, &pl);
    if (rc != CONV_OK) return rc;
    if (pl.layout == CONV_LAYOUT_IMPLICIT) {
        if (!in_packed || !wt_packed || !out) return CONV_ERR_INVALID_ARG;
        if (tile != -1 || (split_k != 0 && split_k != 1)) return CONV_ERR_UNSUPPORTED;
        return run_implicit(pl, window_problem(desc, pl, in_packed, wt_packed, out, 1), (hipStream_t)stream);
    }
    if (!in_packed || !wt_packed || !out || !aligned16(in_packed) || !aligned16(wt_packed))
        return CONV_ERR_INVALID_ARG;
    return run_gemm(gemm_problem(desc, pl, in_packed, wt_packed, out), tile, split_k,
                    (hipStream_t)stream);
}

int conv2d_int8_packed_nhwc(const conv_desc_t *desc, int layout, int cb, const int8_t *in_packed,
                            const int8_t *wt_packed, int32_t *out_nhwc, int tile, int split_k, void *stream)
{
    if (layout == CONV_LAYOUT_AUTO) return CONV_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(desc, layout, cb, &pl);
    if (rc != CONV_OK) return rc;
    if (pl.layout == CONV_LAYOUT_IMPLICIT) return CONV_ERR_UNSUPPORTED;  // those kernels write NKPQ
    if (!in_packed || !wt_packed || !out_nhwc || !aligned16(in_packed) || !aligned16(wt_packed) || !aligned16(out_nhwc))
        return CONV_ERR_INVALID_ARG;
    GemmProblem g = gemm_problem(desc, pl, in_packed, wt_packed, out_nhwc);
    g.out_nhwc = 1;
    return run_gemm(g, tile, split_k, (hipStream_t)stream);
}

int conv2d_int8_packed_requant(const conv_desc_t *desc, int layout, int cb, const int8_t *in_packed,
                               const int8_t *wt_packed, int8_t *out_blocked, int out_cb, int out_pad, int shift, int relu,
                               void *stream)
{
    if (layout == CONV_LAYOUT_AUTO) return CONV_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(desc, layout, cb, &pl);
    if (rc != CONV_OK) return rc;
    if (!in_packed || !wt_packed || !out_blocked || out_pad < 0 || shift < 0 || shift > 31) return CONV_ERR_INVALID_ARG;
    const bool implicit = pl.layout == CONV_LAYOUT_IMPLICIT;  // reads the NCHW input and either weight form as they are
    if ((!implicit && (!aligned16(in_packed) || !aligned16(wt_packed))) || !aligned16(out_blocked)) return CONV_ERR_INVALID_ARG;
    if (out_cb != 16 && out_cb != 32 && out_cb != 64) return CONV_ERR_UNSUPPORTED;
    const long long Hq = (long long)pl.P + 2LL * out_pad, Wq = (long long)pl.Q + 2LL * out_pad;
    const long long Cbq = (desc->K + out_cb - 1) / out_cb;
    if (Hq > INT_LIMIT || Wq > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    // the kernel writes the real channels of the interior pixels; whatever else the blocked tensor has is zero
    if (out_pad > 0 || desc->K % out_cb != 0) {
        const size_t bytes = (size_t)desc->N * (size_t)Cbq * (size_t)Hq * (size_t)Wq * (size_t)out_cb;
        if (launch_fill_zero(out_blocked, bytes, st) != hipSuccess) return CONV_ERR_DEVICE;
    }
    if (implicit) {
        WindowProblem wp = window_problem(desc, pl, in_packed, wt_packed, nullptr, 1);
        int lg = 0;
        while ((1 << lg) < out_cb) ++lg;
        wp.act = ActOut{out_blocked, shift, relu != 0, lg, out_pad, (int)Hq, (int)Wq, (int)Cbq};
        return run_implicit(pl, wp, st);
    }
    GemmProblem g = gemm_problem(desc, pl, in_packed, wt_packed, nullptr);
    g.act_out = out_blocked;
    g.act_shift = shift;
    g.act_relu = relu != 0;
    g.o_cb = out_cb;
    g.o_pad = out_pad;
    // no depth split (the activation needs the whole sum): the band kernel, or the best tile of the general one
    int t = -1, s = 1;
    double cost = 0;
    const bool tiled = gemm_pick(g, &t, &s, &cost);
    if (band_applies(g) && (!tiled || band_cost(g) < cost)) return gemm_status(launch_band_conv(g, st));
    if (!tiled) return CONV_ERR_UNSUPPORTED;
    return gemm_status(launch_gemm(g, t, 1, st));
}

int conv2d_int8_query_tiling(const conv_desc_t *desc, int layout, int cb, int *tile, int *split_k)
{
    if (layout == CONV_LAYOUT_AUTO || !tile || !split_k) return CONV_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(desc, layout, cb, &pl);
    if (rc != CONV_OK) return rc;
    *tile = -1;
    *split_k = 1;
    if (pl.layout == CONV_LAYOUT_IMPLICIT) return CONV_OK;
    GemmChoice c;
    rc = choose_gemm(gemm_problem(desc, pl, nullptr, nullptr, nullptr), -1, 0, &c);
    if (rc != CONV_OK) return rc;
    *tile = c.tile;
    *split_k = c.split_k;
    return CONV_OK;
}

int conv2d_int8_tile_applies(const conv_desc_t *desc, int layout, int cb, int tile, int split_k)
{
    if (layout == CONV_LAYOUT_AUTO || (tile < 0 && tile != CONV_TILE_BAND) || tile >= gemm_num_tiles() || split_k < 1)
        return CONV_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(desc, layout, cb, &pl);
    if (rc != CONV_OK) return rc;
    if (pl.layout == CONV_LAYOUT_IMPLICIT) return CONV_ERR_UNSUPPORTED;
    GemmChoice c;
    return choose_gemm(gemm_problem(desc, pl, nullptr, nullptr, nullptr), tile, split_k, &c);
}

size_t conv2d_int8_tile_lds_bytes(const conv_desc_t *desc, int layout, int cb, int tile, int split_k)
{
    if (conv2d_int8_tile_applies(desc, layout, cb, tile, split_k) != CONV_OK) return 0;
    Plan pl;
    if (make_plan(desc, layout, cb, &pl) != CONV_OK) return 0;
    if (tile == CONV_TILE_BAND) return band_lds_bytes(gemm_problem(desc, pl, nullptr, nullptr, nullptr));
    const int steps = pl.depth / 64, slices = split_k > steps ? steps : split_k;
    const int per = (steps + slices - 1) / slices;
    return gemm_tile_lds_bytes(tile, pl.layout == CONV_LAYOUT_IM2COL ? ACT_MATRIX : ACT_BLOCKED, per);
}

size_t conv2d_int8_workspace_bytes(const conv_desc_t *desc, int layout, int cb, int wt_is_packed)
{
    if (resolve_layout(desc, &layout, &cb) != CONV_OK) return 0;
    if (layout == CONV_LAYOUT_IMAGE_PACK) {
        PackedProblem pp;
        if (wt_is_packed || image_pack_problem(desc, cb, &pp) != CONV_OK) return 0;
        return align_up(pp.x2_bytes, WS_ALIGN) + align_up(pp.w2_bytes, WS_ALIGN) +
               conv2d_int8_workspace_bytes(&pp.d2, pp.inner_layout, pp.inner_cb, 0);
    }
    Plan pl;
    if (make_plan(desc, layout, cb, &pl) != CONV_OK) return 0;
    return align_up(pl.x_bytes, WS_ALIGN) + (wt_is_packed ? 0 : align_up(pl.w_bytes, WS_ALIGN));
}

int conv2d_int8_ex(const conv_desc_t *desc, int layout, int cb, const int8_t *in, const int8_t *wt,
                   int wt_is_packed, int32_t *out, void *workspace, size_t workspace_bytes,
                   void *stream)
{
    int rc = resolve_layout(desc, &layout, &cb);
    if (rc != CONV_OK) return rc;
    if (layout == CONV_LAYOUT_IMAGE_PACK) {
        // rewrite both operands into the stride-1 problem, then run that problem in its inner layout
        PackedProblem pp;
        rc = image_pack_problem(desc, cb, &pp);
        if (rc != CONV_OK) return rc;
        if (wt_is_packed) return CONV_ERR_UNSUPPORTED;
        if (!in || !wt || !out || !workspace) return CONV_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(workspace) % WS_ALIGN) return CONV_ERR_INVALID_ARG;
        const size_t xb = align_up(pp.x2_bytes, WS_ALIGN), wb = align_up(pp.w2_bytes, WS_ALIGN);
        const size_t inner = conv2d_int8_workspace_bytes(&pp.d2, pp.inner_layout, pp.inner_cb, 0);
        if (workspace_bytes < xb + wb + inner) return CONV_ERR_WORKSPACE;
        int8_t *x2 = static_cast<int8_t *>(workspace), *w2 = x2 + xb;
        hipStream_t st = (hipStream_t)stream;
        if (launch_image_pack(desc->N, desc->C, desc->H, desc->W, desc->stride, desc->pad, pp.d2.H, pp.d2.W, in, x2,
                              st) != hipSuccess ||
            launch_image_pack_weights(desc->K, desc->C, desc->R, desc->S, desc->stride, wt, w2, st) != hipSuccess)
            return CONV_ERR_DEVICE;
        return conv2d_int8_ex(&pp.d2, pp.inner_layout, pp.inner_cb, x2, w2, 0, out, inner ? w2 + wb : nullptr, inner,
                              stream);
    }
    Plan pl;
    rc = make_plan(desc, layout, cb, &pl);
    if (rc != CONV_OK) return rc;
    if (!in || !wt || !out) return CONV_ERR_INVALID_ARG;
    if (pl.layout == CONV_LAYOUT_IMPLICIT)
        return run_implicit(pl, window_problem(desc, pl, in, wt, out, wt_is_packed ? 1 : 0), (hipStream_t)stream);
    if (!workspace) return CONV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) % WS_ALIGN) return CONV_ERR_INVALID_ARG;
    if (wt_is_packed && !aligned16(wt)) return CONV_ERR_INVALID_ARG;
    const size_t xb = align_up(pl.x_bytes, WS_ALIGN);
    const size_t need = xb + (wt_is_packed ? 0 : align_up(pl.w_bytes, WS_ALIGN));
    if (workspace_bytes < need) return CONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int8_t *xq = static_cast<int8_t *>(workspace);
    const int8_t *wq = wt;
    bool rewritten = false;
    if (!wt_is_packed) {
        int8_t *wdst = xq + xb;
        wq = wdst;
        // both rewrites in one launch when the tiled input kernels apply
        hipError_t e = launch_rewrite_fused(pl.layout == CONV_LAYOUT_IM2COL, desc->N, desc->C, desc->H,
                                            desc->W, desc->K, desc->R, desc->S, desc->stride, desc->pad,
                                            pl.P, pl.Q, pl.cb, pl.depth, in, xq, wt, wdst, st);
        if (e == hipSuccess) rewritten = true;
        else if (e != hipErrorNotSupported) return CONV_ERR_DEVICE;
        else {
            rc = rewrite_weights(desc, pl, wt, wdst, st);
            if (rc != CONV_OK) return rc;
        }
    }
    if (!rewritten) {
        rc = rewrite_input(desc, pl, in, xq, st);
        if (rc != CONV_OK) return rc;
    }
    return run_gemm(gemm_problem(desc, pl, xq, wq, out), -1, 0, st);
}

int conv2d_int8(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                const int8_t *in, const int8_t *wt, int32_t *out, void *stream)
{
    conv_desc_t d{N, C, H, W, K, R, S, stride, pad};
    int layout = CONV_LAYOUT_AUTO, cb = 0;
    int rc = resolve_layout(&d, &layout, &cb);
    if (rc != CONV_OK) return rc;
    if (!in || !wt || !out) return CONV_ERR_INVALID_ARG;
    const size_t need = conv2d_int8_workspace_bytes(&d, layout, cb, 0);
    if (need == 0) {  // IMPLICIT: nothing to stage (any other layout reports its problem here)
        if (layout != CONV_LAYOUT_IMPLICIT) return CONV_ERR_UNSUPPORTED;
        // Large batches: every workgroup of the stencil-unrolling kernel brings the tile's weight rows into the
        // padded depth order on its way into LDS, dword by dword; rows rewritten once by a small kernel are copied
        // in 16-byte pieces instead (a tenth of a workgroup's instructions).  Worth its launch from a few thousand
        // workgroups on (C3 at N=512: 495 -> 405 us); below that the single launch stays.
        const int depth = pack_weights_depth(C, R, S, CONV_LAYOUT_IMPLICIT, 0);
        const long long P = ((long long)H + 2 * pad - R) / stride + 1, Q = ((long long)W + 2 * pad - S) / stride + 1;
        if (!pointwise_shape(C, R, S) && depth > 0 && (long long)N * P * Q >= (1LL << 21)) {
            void *ws = nullptr;
            size_t ws_bytes = 0;
            if (cached_workspace(align_up((size_t)K * depth, WS_ALIGN), (hipStream_t)stream, &ws, &ws_bytes) == CONV_OK &&
                launch_pack_weights_window(K, C, R, S, wt, static_cast<int8_t *>(ws), (hipStream_t)stream) == hipSuccess)
                return conv2d_int8_ex(&d, layout, 0, in, static_cast<const int8_t *>(ws), 1, out, nullptr, 0, stream);
        }
        return conv2d_int8_ex(&d, layout, 0, in, wt, 0, out, nullptr, 0, stream);
    }
    void *ws = nullptr;
    size_t ws_bytes = 0;
    rc = cached_workspace(need, (hipStream_t)stream, &ws, &ws_bytes);
    if (rc != CONV_OK) return rc;
    return conv2d_int8_ex(&d, layout, cb, in, wt, 0, out, ws, ws_bytes, stream);
}

int conv2d_int8_static(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       const int8_t *in, const int8_t *wt, int32_t *out, void *stream)
{
    conv_desc_t d{N, C, H, W, K, R, S, stride, pad};
    int layout = CONV_LAYOUT_AUTO, cb = 0;
    int rc = resolve_layout(&d, &layout, &cb);
    if (rc != CONV_OK) return rc;
    if (!in || !wt || !out) return CONV_ERR_INVALID_ARG;
    const size_t need = conv2d_int8_workspace_bytes(&d, layout, cb, 0);
    if (need == 0) {  // IMPLICIT: nothing to stage (any other layout reports its problem here)
        if (layout != CONV_LAYOUT_IMPLICIT) return CONV_ERR_UNSUPPORTED;
        return conv2d_int8_ex(&d, layout, 0, in, wt, 0, out, nullptr, 0, stream);
    }
    if (need > STATIC_WS_BYTES) return CONV_ERR_WORKSPACE;  // the rewritten operands do not fit the fixed array
    void *ws = nullptr;
    rc = static_workspace(&ws);
    if (rc != CONV_OK) return rc;
    // Both rewrites write every byte of what the GEMM stage reads (zero borders and padding included), and a
    // depth split clears `out` with a kernel of its own: nothing is assumed about what the last call left.
    return conv2d_int8_ex(&d, layout, cb, in, wt, 0, out, ws, STATIC_WS_BYTES, stream);
}

int conv2d_int8_nhwc(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     const int8_t *in, const int8_t *wt, int32_t *out, void *stream)
{
    // channel blocking straight from the NHWC source, the usual GEMM stage into an NKPQ staging
    // tensor in the workspace, then unpacking to NHWC
    conv_desc_t d{N, C, H, W, K, R, S, stride, pad};
    Plan pl;
    int rc = make_plan(&d, CONV_LAYOUT_PACKED, 0, &pl);
    if (rc != CONV_OK) return rc;
    if (!in || !wt || !out) return CONV_ERR_INVALID_ARG;
    {   // the selector's choice is the kernel that unrolls the stencil itself, and its NHWC form takes the shape: one launch
        int layout = CONV_LAYOUT_AUTO, cb = 0;
        if (resolve_layout(&d, &layout, &cb) == CONV_OK && layout == CONV_LAYOUT_IMPLICIT && !pointwise_shape(C, R, S)) {
            WindowProblem wp{in, wt, out, N, C, H, W, K, pl.P, pl.Q, R, S, stride, pad, 0, ActOut{}, 1, 1};
            if (window_fits(wp))
                return launch_window_conv(wp, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
        }
    }
    if (R == 1 && S == 1 && stride == 1 && pad == 0 && C % CONV_DEPTH_ALIGN == 0 && aligned16(in) && aligned16(wt) && aligned16(out)) {
        // A 1x1 layer on NHWC tensors is a plain matrix product of operands that are depth-contiguous as they are:
        // pixels x channels times the weight rows, into pixels x output channels.  No rewrite, one launch.
        if (pointwise_nhwc_split_fits(pl.M, C, K))   // a grid that leaves most of the chip idle: the depth split over a workgroup's waves
            return launch_pointwise_nhwc_split(in, wt, out, pl.M, C, K, (hipStream_t)stream) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
        GemmProblem g{};
        g.act = in;
        g.wq = wt;
        g.out = out;
        g.K = K;
        g.M = (int)pl.M;
        g.depth = C;
        g.PQ = pl.P * pl.Q;
        g.Q = pl.Q;
        g.mode = ACT_MATRIX;
        g.out_nhwc = 1;
        return run_gemm(g, -1, 0, (hipStream_t)stream);
    }
    // The GEMM stage's epilogue writes NHWC itself (a lane's four values are four consecutive channels of a
    // pixel); only a result that does not start on 16 bytes goes through an NKPQ staging tensor and a pass.
    const bool direct = aligned16(out);
    const size_t xb = align_up(pl.x_bytes, WS_ALIGN), wb = align_up(pl.w_bytes, WS_ALIGN);
    const size_t ob = direct ? 0 : align_up((size_t)pl.M * d.K * sizeof(int32_t), WS_ALIGN);
    const size_t need = xb + wb + ob;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    rc = cached_workspace(need, (hipStream_t)stream, &ws, &ws_bytes);
    if (rc != CONV_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    int8_t *xq = static_cast<int8_t *>(ws), *wq = xq + xb;
    int32_t *nkpq = reinterpret_cast<int32_t *>(wq + wb);
    const hipError_t e = launch_rewrite_fused_nhwc(N, C, H, W, K, R, S, pad, pl.cb, pl.depth, in, xq, wt, wq, st);
    if (e == hipErrorNotSupported) {
        if (launch_pack_layout_nhwc(N, C, H, W, pl.cb, pad, in, xq, st) != hipSuccess) return CONV_ERR_DEVICE;
        rc = rewrite_weights(&d, pl, wt, wq, st);
        if (rc != CONV_OK) return rc;
    } else if (e != hipSuccess) return CONV_ERR_DEVICE;
    if (direct) {
        GemmProblem g = gemm_problem(&d, pl, xq, wq, out);
        g.out_nhwc = 1;
        return run_gemm(g, -1, 0, st);
    }
    rc = run_gemm(gemm_problem(&d, pl, xq, wq, nkpq), -1, 0, st);
    if (rc != CONV_OK) return rc;
    return launch_unpack_nhwc(N, K, (long long)pl.P * pl.Q, nkpq, out, st) == hipSuccess ? CONV_OK : CONV_ERR_DEVICE;
}

}  // extern "C"
