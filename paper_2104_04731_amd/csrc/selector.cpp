// Per-shape layout selection: the candidate-selection term of Sec. 4.4 evaluated over the
// handful of rewrites this library implements (Table 2), instead of over a solver's
// candidate list.  Host arithmetic only (the one call into the kernel side asks whether the
// stencil-unrolling GEMM stage takes the shape).
#include "../../include/conv2d_int8.h"
#include "desc_check.h"
#include "kernels.h"

#include <stdint.h>

namespace {

// Extents of the matrix intrinsic the dimensions are padded to (Sec. 4.2.4 rule b):
// 32 output pixels x 32 output channels per MFMA block, depth in 64-byte steps.
constexpr int64_t UNIT_PIXELS = 32, UNIT_CHANNELS = 32, UNIT_DEPTH = CONV_DEPTH_ALIGN;

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Cand {
    int layout, cb;
};

}  // namespace

extern "C" int layout_overheads(const conv_desc_t *d, int layout, int cb,
                                int64_t *o_mac, int64_t *o_data, int64_t *rewritten)
{
    const int rc0 = c2i8::check_conv_desc(d);
    if (rc0 != CONV_OK) return rc0;
    const int64_t P = ((int64_t)d->H + 2 * (int64_t)d->pad - d->R) / d->stride + 1;
    const int64_t Q = ((int64_t)d->W + 2 * (int64_t)d->pad - d->S) / d->stride + 1;
    const int64_t M = (int64_t)d->N * P * Q;
    const int64_t taps = (int64_t)d->R * d->S;
    const int64_t mac_min = M * d->K * d->C * taps;
    if (layout == CONV_LAYOUT_IMAGE_PACK) {
        // the packed stride-1 problem in its inner layout, against the MACs of the original definition
        conv_desc_t d2;
        int rc = image_pack_desc(d, &d2);
        if (rc != CONV_OK) return rc;
        if (cb != 0 && cb != 16 && cb != 32 && cb != 64) return CONV_ERR_INVALID_ARG;
        int64_t om, od, rw;
        rc = layout_overheads(&d2, cb == 0 ? CONV_LAYOUT_IMPLICIT : CONV_LAYOUT_PACKED, cb, &om, &od, &rw);
        if (rc != CONV_OK) return rc;
        const int64_t inner_min = M * d->K * d2.C * d2.R * d2.S;  // includes the zero taps of the split kernel
        const int64_t x2 = (int64_t)d2.N * d2.C * d2.H * d2.W, w2 = (int64_t)d2.K * d2.C * d2.R * d2.S;
        if (o_mac) *o_mac = om + inner_min - mac_min;
        if (o_data) *o_data = od + 2 * (x2 + w2);
        if (rewritten) *rewritten = rw + x2 + w2;
        return CONV_OK;
    }
    if (layout == CONV_LAYOUT_IMPLICIT) {
        // nothing rewritten, nothing moved twice; pixels padded per output row, kernel rows to dwords
        if (P > 2147483647LL || Q > 2147483647LL) return CONV_ERR_UNSUPPORTED;
        const c2i8::WindowProblem g{nullptr, nullptr, nullptr, d->N, d->C, d->H, d->W, d->K, (int)P, (int)Q,
                                    d->R, d->S, d->stride, d->pad, 0, c2i8::ActOut{}, 0, 0};
        const bool pointwise = c2i8::pointwise_shape(d->C, d->R, d->S);
        if (!(pointwise ? c2i8::pointwise_fits(g) : c2i8::window_fits(g))) return CONV_ERR_UNSUPPORTED;
        // 1x1 over whole 64-channel multiples: pixels padded per image, depth as it is
        const int64_t depth = pointwise ? d->C : round_up((int64_t)d->C * d->R * round_up(d->S, 4), UNIT_DEPTH);
        const int64_t pixels = pointwise ? (int64_t)d->N * round_up(P * Q, UNIT_PIXELS)
                                         : (int64_t)d->N * P * round_up(Q, UNIT_PIXELS);
        const int64_t mac_total = pixels * round_up(d->K, UNIT_CHANNELS) * depth;
        if (o_mac) *o_mac = mac_total - mac_min;
        if (o_data) *o_data = 0;
        if (rewritten) *rewritten = 0;
        return CONV_OK;
    }
    if (layout == CONV_LAYOUT_PAD_ONLY) cb = (int)round_up(d->C, 16);
    if (layout != CONV_LAYOUT_IM2COL && layout != CONV_LAYOUT_PACKED && layout != CONV_LAYOUT_PAD_ONLY)
        return CONV_ERR_INVALID_ARG;
    if (layout != CONV_LAYOUT_IM2COL && (cb <= 0 || cb % 16)) return CONV_ERR_INVALID_ARG;

    int64_t depth, x_elems;
    if (layout == CONV_LAYOUT_IM2COL) {
        depth = round_up(d->C * taps, UNIT_DEPTH);
        x_elems = M * depth;
    } else {
        const int64_t cpad = round_up(d->C, cb);
        depth = round_up(cpad * taps, UNIT_DEPTH);
        x_elems = (int64_t)d->N * cpad * ((int64_t)d->H + 2 * (int64_t)d->pad) * ((int64_t)d->W + 2 * (int64_t)d->pad);
    }
    const int64_t w_elems = (int64_t)d->K * depth;
    const int64_t mac_total = round_up(M, UNIT_PIXELS) * round_up(d->K, UNIT_CHANNELS) * depth;
    if (o_mac) *o_mac = mac_total - mac_min;
    // rewrite writes X' and W', the GEMM stage reads them again; in, wt, out are the minimum
    if (o_data) *o_data = 2 * x_elems + 2 * w_elems;
    if (rewritten) *rewritten = x_elems + w_elems;
    return CONV_OK;
}

extern "C" int select_layout_weighted(const conv_desc_t *d, double w_mac, double w_data,
                                      int *layout, int *cb, double *score)
{
    if (!d || !layout || !cb) return CONV_ERR_INVALID_ARG;
    const Cand cands[] = {{CONV_LAYOUT_PACKED, 64}, {CONV_LAYOUT_PACKED, 32}, {CONV_LAYOUT_PACKED, 16},
                          {CONV_LAYOUT_IM2COL, 0},  {CONV_LAYOUT_PAD_ONLY, 0},  {CONV_LAYOUT_IMPLICIT, 0},
                          {CONV_LAYOUT_IMAGE_PACK, 0}, {CONV_LAYOUT_IMAGE_PACK, 64}, {CONV_LAYOUT_IMAGE_PACK, 32},
                          {CONV_LAYOUT_IMAGE_PACK, 16}};
    bool have = false;
    double best_score = 0;
    int64_t best_ws = 0;
    Cand best{0, 0};
    for (const Cand &c0 : cands) {
        Cand c = c0;
        if (c.layout == CONV_LAYOUT_PAD_ONLY) c.cb = (int)round_up(d->C, 16);
        int64_t om, od, ws;
        int rc = layout_overheads(d, c.layout, c.cb, &om, &od, &ws);
        if (rc == CONV_ERR_UNSUPPORTED && (c.layout == CONV_LAYOUT_IMPLICIT || c.layout == CONV_LAYOUT_IMAGE_PACK))
            continue;  // outside its domain
        if (rc != CONV_OK) return rc;
        const double sc = w_mac * (double)om + w_data * (double)od;
        bool better = !have;
        if (have) {
            if (sc != best_score) better = sc < best_score;
            else if (ws != best_ws) better = ws < best_ws;
            else if (c.layout != best.layout) better = c.layout < best.layout;
            else better = c.cb > best.cb;
        }
        if (better) {
            have = true;
            best_score = sc;
            best_ws = ws;
            best = c;
        }
    }
    *layout = best.layout;
    *cb = best.cb;
    if (score) *score = best_score;
    return CONV_OK;
}

// MI355X weights -- the "used hardware" the paper leaves w to: seconds per issued MAC and per
// moved int8 element at the rates this library's own kernels sustain there (GEMM stage about
// 0.6e15 MAC/s, layout kernels about 4e12 B/s), not at the data-sheet peaks.
extern "C" int select_layout(const conv_desc_t *d, int *layout, int *cb, double *score)
{
    const double w_mac = 1.0 / 0.6e15, w_data = 1.0 / 4.0e12;
    return select_layout_weighted(d, w_mac, w_data, layout, cb, score);
}
