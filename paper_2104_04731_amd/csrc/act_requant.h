// The ALU step between two int8 layers (Sec. 5.1 names the accelerator's shift / min / max unit and gives
// no formula): rounding right shift, optional max(., 0), clip to int8.  The one definition every kernel
// that applies the activation includes.
#pragma once
#include <hip/hip_runtime.h>

namespace c2i8 {

__device__ __forceinline__ int act_requant(int x, int shift, int relu)
{
    // floor(x / 2^shift + 1/2) without leaving 32 bits: floor(x / 2^shift) + bit (shift-1) of x
    int v = shift > 0 ? (x >> shift) + ((x >> (shift - 1)) & 1) : x;
    if (relu) v = max(v, 0);
    return min(max(v, -128), 127);
}

}  // namespace c2i8
