// Running log-sum-exp pair shared by the kernels that turn logits into token losses.
#ifndef FQ_LSE_H
#define FQ_LSE_H

#include <hip/hip_runtime.h>

// (m, s) stands for s * exp(m) = sum of exp(l) over the logits seen so far, m their maximum.  Merging keeps
// the larger maximum; a pair that has seen nothing (or only -inf) is (-inf, 0).
__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2)
{
    const float mx = fmaxf(m, m2);
    if (mx == -INFINITY) {
        m = mx;
        s = 0.f;
        return;
    }
    s = s * __expf(m - mx) + s2 * __expf(m2 - mx);
    m = mx;
}

#endif
