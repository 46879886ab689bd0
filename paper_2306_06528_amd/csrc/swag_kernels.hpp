// Multi-SWAG running moments (paper Sec. 2: SWAG keeps the first and second moments of a network's
// parameter trajectory; multi-SWAG does so for every particle).  One more iterate X is absorbed
// into the running means of all n*D parameters after `count` earlier updates:
//     mean <- (count*mean + x)/(count+1),   sq <- (count*sq + x*x)/(count+1)
// evaluated in the incremental form m += (x - m)/(count+1), which does not lose accuracy as count
// grows; the first update (count = 0) copies x and x*x, whatever the arrays held before.  A pure
// streaming kernel: 12 bytes read and 8 written per parameter.
#pragma once
#include "common.hpp"

namespace svgd {

__global__ __launch_bounds__(256) void swag_moments_kernel(float *__restrict__ mean,
                                                           float *__restrict__ sq,
                                                           const float *__restrict__ X,
                                                           int64_t total, float inv, bool first)
{
    // all three arrays are only 4-byte aligned in general; 16-byte accesses need no more than that
    const int64_t ngroups = (total + 3) >> 2;
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    for (int64_t grp = (int64_t)blockIdx.x * 256 + threadIdx.x; grp < ngroups; grp += nthreads) {
        const int64_t e = grp << 2;
        const bool full = (e + 4 <= total);
        const f32x4 x = load4_stream(X, e, total, full);
        f32x4 m = load4(mean, e, total, full);
        f32x4 s = load4(sq, e, total, full);
        if (first) {
            m = x;
            s = x * x;
        } else {
            m += (x - m) * inv;
            s += (x * x - s) * inv;
        }
        store4(mean, e, total, full, m);
        store4(sq, e, total, full, s);
    }
}

} // namespace svgd
