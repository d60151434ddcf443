// Test-only generator dumps.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_common.hpp"
#include "core_rng.hpp"

namespace core {

// ---- test-only generator dumps ----------------------------------------------------------------

// out[(jj * nq + qq) * 4 + w] = word w of Philox block q0 + qq of vector j0 + jj, produced with the
// generator instantiation and the lane layout of one family of production kernels, so that the
// split between scalar-unit rounds and vector rounds (and the three-input xor) is the one they run:
//   LAYOUT 0  Generator<10,10>: every round key on the scalar path; one thread per block q
//   LAYOUT 1  Generator<3,4>, lanes over the vector index j, q the wave-uniform loop index
//             (project_kernel, project_mfma_kernel)
//   LAYOUT 2  Generator<2,3>, lanes over the block index q, j the wave-uniform loop index
//             (reconstruct_kernel, reconstruct_batched_kernel, project_q_kernel)
//   LAYOUT 3  Generator<4,4>, lanes over q, j a kernel argument (debug_xi_kernel)
struct DebugPhiloxArgs {
    uint32_t k0, k1, r0, r1;
    uint32_t j0, nj;
    uint64_t q0, nq;
    uint32_t* out;
};

template <int LAYOUT>
__global__ void __launch_bounds__(kThreads) debug_philox_kernel(DebugPhiloxArgs a)
{
    const uint64_t t = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    auto put = [&](uint64_t jj, uint64_t qq, const Words& w) {
        uint32_t* o = a.out + (jj * a.nq + qq) * 4;
        o[0] = w.x0; o[1] = w.x1; o[2] = w.x2; o[3] = w.x3;
    };
    if constexpr (LAYOUT == 1) {
        Generator<3, 4> gen;
        gen.init(a.k0, a.k1, a.r0, a.r1);
        const uint32_t j = a.j0 + (uint32_t)t;
        for (uint64_t qq = 0; qq < a.nq; ++qq) {
            const Words w = gen.words((uint32_t)(a.q0 + qq), j);
            if (t < a.nj) put(t, qq, w);
        }
    } else if constexpr (LAYOUT == 2) {
        Generator<2, 3> gen;
        gen.init(a.k0, a.k1, a.r0, a.r1);
        const uint32_t q = (uint32_t)(a.q0 + t);
        for (uint32_t jj = 0; jj < a.nj; ++jj) {
            const Words w = gen.words(q, a.j0 + jj);
            if (t < a.nq) put(jj, t, w);
        }
    } else if constexpr (LAYOUT == 4) {
        // lanes over vectors and Philox blocks at once (tiles of fewer than 64 vectors)
        Generator<1, 1> gen;
        gen.init(a.k0, a.k1, a.r0, a.r1);
        const uint64_t jj = t % a.nj, qq = t / a.nj;
        const Words w = gen.words((uint32_t)(a.q0 + qq), a.j0 + (uint32_t)jj);
        if (qq < a.nq) put(jj, qq, w);
    } else {
        Generator<(LAYOUT == 3 ? 4 : 10), (LAYOUT == 3 ? 4 : 10)> gen;
        gen.init(a.k0, a.k1, a.r0, a.r1);
        const uint32_t q = (uint32_t)(a.q0 + t);
        for (uint32_t jj = 0; jj < a.nj; ++jj) {
            const Words w = gen.words(q, a.j0 + jj);
            if (t < a.nq) put(jj, t, w);
        }
    }
}

__global__ void __launch_bounds__(kThreads) debug_xi_kernel(uint32_t k0, uint32_t k1, uint32_t r0,
                                                            uint32_t r1, uint32_t j, uint64_t i0,
                                                            uint64_t count, float* out)
{
    const uint64_t tt = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (tt >= count) return;
    const uint64_t i = i0 + tt;
    Generator<4, 4> gen;
    gen.init(k0, k1, r0, r1);
    float z0, z1, z2, z3;
    gen.block((uint32_t)(i >> 2), j, z0, z1, z2, z3);
    const uint32_t k = (uint32_t)(i & 3u);
    out[tt] = kXiScale * ((k == 0) ? z0 : (k == 1) ? z1 : (k == 2) ? z2 : z3);
}

}  // namespace core
