// Cross-chunk sum of the projection's partial sums and the client mean (Eq. (tildefdef)).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_common.hpp"

namespace core {

// Cross-chunk sum (a4), stage A: psum[z][c][j] = sum over the chunks of slice z of part[k][c][j],
// fp64, fixed order.  grid = (ceil(m/32), n, Z); block = 32 vectors x 8 interleaved sub-slices.
// Chunk k belongs to slice k % Z and, inside it, to sub-slice (k / Z) % 8.
__global__ void __launch_bounds__(kThreads) reduce_chunks_kernel(const float* __restrict__ part,
                                                                 uint32_t m, uint32_t n, uint32_t nchunks,
                                                                 double* __restrict__ psum)
{
    __shared__ double sh[8][32];
    const uint32_t jl = threadIdx.x & 31u;
    const uint32_t sl = threadIdx.x >> 5;
    const uint32_t j = blockIdx.x * 32u + jl;
    const uint32_t c = blockIdx.y;
    const uint32_t z = blockIdx.z, Z = gridDim.z;
    const uint64_t E = (uint64_t)n * m;
    double s = 0.0;
    if (j < m) {
        const float* src = part + (uint64_t)c * m + j;
        const uint64_t step = 8ull * Z;
        uint64_t k = (uint64_t)sl * Z + z;
        // four independent loads in flight per thread; each sub-slice still adds in increasing k
        for (; k + 3 * step < nchunks; k += 4 * step) {
            const float v0 = src[k * E], v1 = src[(k + step) * E];
            const float v2 = src[(k + 2 * step) * E], v3 = src[(k + 3 * step) * E];
            s += (double)v0; s += (double)v1; s += (double)v2; s += (double)v3;
        }
        for (; k < nchunks; k += step) s += (double)src[k * E];
    }
    sh[sl][jl] = s;
    __syncthreads();
    if (sl == 0 && j < m) {
        double tot = sh[0][jl];
#pragma unroll
        for (int q = 1; q < 8; ++q) tot += sh[q][jl];
        psum[((uint64_t)z * n + c) * m + j] = tot;
    }
}

// Stage B: P[c][j] = sum_z psum[z][c][j]; the client mean of Eq. (tildefdef),
// (with at most 16 chunks stage A is skipped and this kernel sums the fp32 partials directly)
// pbar[j] = (1/n) sum_c P[c][j].  Block = 32 vectors x 8 client lanes (lane cl takes clients
// cl, cl+8, ...); fp64, fixed order.
template <typename T>   // double: slices from stage A; float: the partials themselves (few chunks)
__global__ void __launch_bounds__(kThreads) reduce_clients_kernel(const T* __restrict__ psum,
                                                                  uint32_t m, uint32_t n, uint32_t Z,
                                                                  float* __restrict__ P,
                                                                  float* __restrict__ pbar)
{
    __shared__ double sh[8][32];
    const uint32_t jl = threadIdx.x & 31u;
    const uint32_t cl = threadIdx.x >> 5;
    const uint32_t j = blockIdx.x * 32u + jl;
    const uint64_t E = (uint64_t)n * m;
    double tot = 0.0;
    if (j < m) {
        for (uint32_t c = cl; c < n; c += 8) {
            const T* src = psum + (uint64_t)c * m + j;
            double s = 0.0;
            for (uint32_t z = 0; z < Z; ++z) s += (double)src[(uint64_t)z * E];
            if (P) P[(uint64_t)c * m + j] = (float)s;
            tot += s;
        }
    }
    sh[cl][jl] = tot;
    __syncthreads();
    if (cl == 0 && j < m) {
        double t = sh[0][jl];
#pragma unroll
        for (int q = 1; q < 8; ++q) t += sh[q][jl];
        pbar[j] = (float)(t / (double)n);
    }
}

}  // namespace core
