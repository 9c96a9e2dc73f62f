// The one validity check of a convolution descriptor, shared by every entry point that takes one
// (the conv calls, the size queries, the layout selector): 64-bit extents throughout.
#pragma once
#include "../../include/conv2d_int8.h"

namespace c2i8 {

inline int check_conv_desc(const conv_desc_t *d)
{
    constexpr long long INT_LIMIT = 2147483647LL;
    if (!d) return CONV_ERR_INVALID_ARG;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 ||
        d->stride <= 0 || d->pad < 0)
        return CONV_ERR_INVALID_ARG;
    const long long Hp = (long long)d->H + 2LL * d->pad, Wp = (long long)d->W + 2LL * d->pad;
    if (d->R > Hp || d->S > Wp) return CONV_ERR_INVALID_ARG;
    if ((long long)d->C * d->R * d->S > 131072LL) return CONV_ERR_OVERFLOW_RISK;  // an int32 accumulator could wrap
    const long long P = (Hp - d->R) / d->stride + 1, Q = (Wp - d->S) / d->stride + 1;
    if (Hp > INT_LIMIT || Wp > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    if (P * Q > INT_LIMIT || (long long)d->N * P * Q > INT_LIMIT) return CONV_ERR_UNSUPPORTED;
    return CONV_OK;
}

}  // namespace c2i8
