// Measurement helpers: stand-in compute kernel and plain copy with the mover's inner loop.
// Included by rb.hip only, after rb_device.h.
#pragma once

#include "rb_device.h"

namespace {

// ---------------------------------------------------------------------------
// Measurement helpers
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) rb_standin_kernel(float* __restrict__ sink, int64_t iters)
{
    float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1.f, x2 = x0 + 2.f, x3 = x0 + 3.f;
    const float m = 0.999f, d = 1e-3f;
    for (int64_t i = 0; i < iters; ++i) {
        x0 = fmaf(x0, m, d); x1 = fmaf(x1, m, d); x2 = fmaf(x2, m, d); x3 = fmaf(x3, m, d);
        x0 = fmaf(x0, m, d); x1 = fmaf(x1, m, d); x2 = fmaf(x2, m, d); x3 = fmaf(x3, m, d);
    }
    sink[(int64_t)blockIdx.x * TPB + threadIdx.x] = x0 + x1 + x2 + x3;
}

template <int U, bool NT, int PACE>       // PACE: 1 - every store waited for; 64 - the stores of a tile in one burst
__global__ void __launch_bounds__(TPB) rb_copy_kernel(vec16* __restrict__ dst, const vec16* __restrict__ src, int64_t nvec)
{
    const int64_t lo = (int64_t)blockIdx.x * (TPB * U);
    const int64_t hi = lo + TPB * U < nvec ? lo + TPB * U : nvec;
    Tile<U, NT, TPB, PACE> t;
    t.load(src, lo, hi);
    t.store(dst, lo, hi);
}


}  // namespace
