// Device-side common random generator of CORE (Algorithm 1, REQUIRE line, Section 3 of
// arXiv 2309.13307): Philox4x32-10 words -> 24-bit uniforms -> Box-Muller normals, all in
// registers.  xi_j[4q .. 4q+3] is a pure function of (seed, round, j, q), so the projection and
// the reconstruction kernels regenerate identical values and Xi never exists in memory.
//
// Written for gfx950.  Measured issue costs that shape this code (cycles per wave64
// instruction per SIMD): plain two-operand VALU ops with VGPR/literal operands ~2.4,
// the same ops with an SGPR operand ~4.4, v_mad_u64_u32 ~4.9 (v_mul_lo + v_mul_hi ~9),
// v_cvt ~4.3, transcendentals (v_log/v_sqrt/v_sin/v_cos) ~8.2.  Hence: one 64-bit
// multiply-add per Philox product, literals for the multipliers, hardware transcendentals
// (their absolute error against fp64 is ~1e-7 on this domain), and wave-uniform parts of
// the first Philox rounds left to the scalar unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace core {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

struct Words { uint32_t x0, x1, x2, x3; };

// Philox4x32-10 (Salmon et al., SC'11).  Counter (c0,c1,c2,c3), key (k0,k1).
// Values that are uniform across the wave stay on the scalar unit: the compiler's
// uniformity analysis sees that from the arguments.
__device__ __forceinline__ Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pa = (uint64_t)c0 * kPhiloxM0;
        const uint64_t pb = (uint64_t)c2 * kPhiloxM1;
        const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    return Words{c0, c1, c2, c3};
}

// Two words -> two standard normals.  The 24-bit uniforms are exact in fp32, so the only
// difference from an fp64 evaluation is the error of log2/sqrt/sin/cos themselves.
// v_sin_f32 / v_cos_f32 take their argument in revolutions, so u2 is used as is.
__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float& z_even, float& z_odd)
{
    const float u1 = (float)((xa >> 8) + 1u) * 0x1p-24f;   // (0, 1]
    const float u2 = (float)(xb >> 8) * 0x1p-24f;          // [0, 1)
    // -2 ln(u1) = (-2 ln 2) log2(u1)
    const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));
    z_even = r * __builtin_amdgcn_cosf(u2);
    z_odd  = r * __builtin_amdgcn_sinf(u2);
}

struct Normals { float z0, z1, z2, z3; };

// xi_j[4q .. 4q+3] for key (k0,k1) = seed halves and (r0,r1) = round halves.
__device__ __forceinline__ Normals xi_block(uint32_t q, uint32_t j, uint32_t r0, uint32_t r1,
                                            uint32_t k0, uint32_t k1)
{
    const Words w = philox4x32_10(q, j, r0, r1, k0, k1);
    Normals z;
    box_muller(w.x0, w.x1, z.z0, z.z1);
    box_muller(w.x2, w.x3, z.z2, z.z3);
    return z;
}

}  // namespace core
