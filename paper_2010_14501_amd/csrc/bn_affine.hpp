// BatchNorm's apply step as one multiply-add per element: y = a * x + b with a = gamma * invstd and
// b = beta - mean * a.
//
// Three kernels apply it: the stand-alone apply kernel, the fused BatchNorm (+ add) + ReLU pass, and the epilogue of a
// recomputed convolution whose BatchNorm statistics are already known.  All go through the two functions below, so
// a tensor has the same bits whichever of them wrote it (explicit fused multiply-adds, no re-association).
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace monet {

__device__ inline void bn_affine_coeffs(const float *__restrict__ gamma, const float *__restrict__ beta, const float *__restrict__ stats,
                                        int C, int c, float &a, float &b) {
#pragma clang fp contract(off)
    a = gamma[c] * stats[C + c];
    b = __builtin_fmaf(-stats[c], a, beta[c]);
}

__device__ inline float bn_affine(float x, float a, float b) { return __builtin_fmaf(x, a, b); }

// ReLU (mode 1) / ReLU6 (mode 2) as the stand-alone kernels compute it: strict comparisons, NaN and -0.0 give +0.0
__device__ inline float relu_clamp(float e, int mode) {
    float r = e > 0.0f ? e : 0.0f;
    if (mode == 2) r = r < 6.0f ? r : 6.0f;
    return r;
}

}  // namespace monet
