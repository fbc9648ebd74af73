// Pieces of the KL stability rule shared by the reduction that produces its cross term and the
// decision that consumes it (the per-token rule Section 2 describes: a small KL divergence
// between the distributions of consecutive steps marks a prediction that has stopped moving).
#pragma once
#include "jot_device.h"

// jot_merge() with the cross term A = sum_v 2^(l_v log2 e - M) (l_v - l'_v) riding along: it is
// scaled by the same exact powers of two as the exponent sum.
__device__ __forceinline__ void jot_merge_kl(float& m1, int32_t& idx, float& m2, float& M, float& s, float& a,
                                             float bm1, int32_t bidx, float bm2, float bM, float bs, float ba)
{
    const float newM = fmaxf(M, bM);
    const float fa = (M == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(M - newM);
    const float fb = (bM == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(bM - newM);
    a = a * fa + ba * fb;
    jot_merge(m1, idx, m2, M, s, bm1, bidx, bm2, bM, bs);
}
