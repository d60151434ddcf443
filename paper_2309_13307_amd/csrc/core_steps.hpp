// Small kernels around a round: the statistic and step of Algorithm 3, its comparison step, the
// squared norms of the projections, and the device-resident round counter.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_common.hpp"

namespace core {

// Algorithm 3 (non-convex CORE-GD), Option I: the norm statistic p = c * sqrt(mean_j pbar_j^2)
// (each combined projection is N(0, |grad f|^2), so the mean square estimates |grad f|^2) and the
// step h = min{first, second_over_sqrt_p / sqrt(p)} with
// first = m / (16 r1) and second_over_sqrt_p = H^(-1/2) d^(-3/4) m^(3/4) / 1600 from the host.
// One block; squares are summed in fp64 in a fixed order (thread-strided, then an LDS tree).
__global__ void __launch_bounds__(kThreads) nonconvex_step_kernel(const float* pbar, uint32_t m, float c,
                                                                  float first, float second_over_sqrt_p,
                                                                  float* p_out, float* h_out)
{
    __shared__ double part[kThreads];
    const uint32_t t = threadIdx.x;
    double s = 0.0;
    for (uint32_t j = t; j < m; j += kThreads) {
        const double v = (double)pbar[j];
        s += v * v;
    }
    part[t] = s;
    __syncthreads();
    for (uint32_t w = kThreads / 2; w > 0; w >>= 1) {
        if (t < w) part[t] += part[t + w];
        __syncthreads();
    }
    if (t == 0) {
        const float p = c * (float)sqrt(part[0] / (double)m);
        float h = first;
        if (p > 0.0f) h = fminf(first, second_over_sqrt_p / sqrtf(p));
        if (p_out) *p_out = p;
        *h_out = h;
    }
}

// Squared norms of the released projections (appendix on differential privacy, lemma on the law of
// C(a)): sq[c] = sum_j P[c][j]^2.  C(a) is N(0, |a|^2 I_m), so sq[c] / m estimates |g_c|^2 and sq[c]
// is all of P[c] that the privacy loss depends on.  One block per client; squares are summed in fp64
// in a fixed order (thread-strided, then an LDS tree), as in nonconvex_step_kernel.
__global__ void __launch_bounds__(kThreads) projection_sqnorms_kernel(const float* P, uint32_t m, double* sq)
{
    __shared__ double part[kThreads];
    const uint32_t t = threadIdx.x;
    const float* row = P + (uint64_t)blockIdx.x * m;
    double s = 0.0;
    for (uint32_t j = t; j < m; j += kThreads) {
        const double v = (double)row[j];
        s += v * v;
    }
    part[t] = s;
    __syncthreads();
    for (uint32_t w = kThreads / 2; w > 0; w >>= 1) {
        if (t < w) part[t] += part[t + w];
        __syncthreads();
    }
    if (t == 0) sq[blockIdx.x] = part[0];
}

// Comparison step of Algorithm 3, part 1: the decision (strict decrease; NaN rejects).
__global__ void accept_decide_kernel(float* f_cur, const float* f_trial, int32_t* accepted)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const float fc = *f_cur, ft = *f_trial;
        const int32_t take = ft < fc ? 1 : 0;
        if (take) *f_cur = ft;
        *accepted = take;
    }
}

// Part 2: x <- x_trial where the decision says so.  Every block reads the flag written by the
// previous kernel on the same stream; nothing is touched on a reject.
__global__ void __launch_bounds__(kThreads) accept_copy_kernel(const int32_t* accepted, float* x,
                                                               const float* x_trial, uint64_t d, int vec)
{
    if (*accepted == 0) return;
    const uint64_t t = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (vec) {
        const uint64_t i = 4 * t;
        if (i + 4 <= d) {
            *reinterpret_cast<float4*>(x + i) = *reinterpret_cast<const float4*>(x_trial + i);
        } else {
            for (uint64_t k = i; k < d; ++k) x[k] = x_trial[k];
        }
    } else {
        const uint64_t i = 4 * t;
        for (uint64_t k = i; k < i + 4 && k < d; ++k) x[k] = x_trial[k];
    }
}

// Device-resident round counter for replayed launch sequences (HIP graphs): one thread adds 1.
__global__ void advance_round_kernel(uint64_t* round_dev)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *round_dev += 1;
}

}  // namespace core
