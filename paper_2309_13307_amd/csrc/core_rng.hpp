// Device-side common random generator of CORE (Algorithm 1, REQUIRE line, Section 3 of
// arXiv 2309.13307): Philox4x32-10 words -> 24-bit uniforms -> Box-Muller normals, all in
// registers.  xi_j[4q .. 4q+3] is a pure function of (seed, round, j, q), so the projection and
// the reconstruction kernels regenerate identical values and Xi never exists in memory.
//
// Written for gfx950.  Measured issue costs that shape this code (cycles per wave64
// instruction per SIMD): plain two-operand VALU ops with VGPR/literal operands ~2.4 (also
// v_fma / v_bitop3 when src0 and src1 sit in different VGPR banks, as the Philox xors do),
// the same ops with an SGPR operand ~4.4, v_mad_u64_u32 ~4.9 (v_mul_lo + v_mul_hi ~9),
// v_cvt ~4.3, transcendentals (v_log/v_sqrt/v_sin/v_cos) ~8.2.  Hence: one 64-bit
// multiply-add per Philox product, literals for the multipliers, round keys and constants of
// the fully divergent rounds held in VGPRs, hardware transcendentals (their absolute error
// against fp64 is ~1e-7 on this domain), and the wave-uniform parts of the first Philox
// rounds left to the scalar unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace core {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

// The generator produces xi / kXiScale; callers multiply their sums by kXiScale once.
// r = sqrt(-2 ln u1) = sqrt(2 ln 2) * sqrt(-log2 u1): the constant factor leaves the hot loop.
constexpr float kXiScale = 1.17741002251547469f;   // sqrt(2 ln 2)

struct Words { uint32_t x0, x1, x2, x3; };

// A wave-uniform value copied into a vector register.  The compiler then treats it as divergent
// and uses it as a VGPR operand, which is the cheap operand kind on this chip.
__device__ __forceinline__ uint32_t to_vgpr(uint32_t s)
{
    uint32_t v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(v) : "s"(s));
    return v;
}

// Per-kernel generator state: key schedule on the scalar unit for the first rounds, where part
// of the counter is still wave-uniform and the key is folded into a scalar xor, and the same
// schedule in VGPRs from round kVecFrom0 (first key word) / kVecFrom1 (second key word) on,
// where both operands of the xor are divergent.
template <int kVecFrom0, int kVecFrom1>
struct Generator {
    uint32_t r0, r1;            // round counter halves (counter words 2, 3)
    uint32_t ks0, ks1;          // seed halves (key), scalar
    uint32_t kv[10][2];         // VGPR copies of the round keys, valid from kVecFrom0/1 on
    float two_m24;              // 2^-24 in a VGPR

    __device__ __forceinline__ void init(uint32_t k0, uint32_t k1, uint32_t rr0, uint32_t rr1)
    {
        r0 = rr0; r1 = rr1; ks0 = k0; ks1 = k1;
#pragma unroll
        for (int r = 0; r < 10; ++r) {
            kv[r][0] = (r >= kVecFrom0) ? to_vgpr(k0 + (uint32_t)r * kPhiloxW0) : 0u;
            kv[r][1] = (r >= kVecFrom1) ? to_vgpr(k1 + (uint32_t)r * kPhiloxW1) : 0u;
        }
        two_m24 = __uint_as_float(to_vgpr(0x33800000u));
    }

    // Philox4x32-10 (Salmon et al., SC'11) on counter (q, j, r0, r1).
    __device__ __forceinline__ Words words(uint32_t q, uint32_t j) const
    {
        uint32_t c0 = q, c1 = j, c2 = r0, c3 = r1;
#pragma unroll
        for (int r = 0; r < 10; ++r) {
            const uint32_t k0 = (r >= kVecFrom0) ? kv[r][0] : ks0 + (uint32_t)r * kPhiloxW0;
            const uint32_t k1 = (r >= kVecFrom1) ? kv[r][1] : ks1 + (uint32_t)r * kPhiloxW1;
            const uint64_t pa = (uint64_t)c0 * kPhiloxM0;
            const uint64_t pb = (uint64_t)c2 * kPhiloxM1;
            // three-way xor: one v_bitop3_b32 (truth table 0x96) once all three inputs are divergent
            const uint32_t n0 = (r >= kVecFrom0) ? __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), c1, k0, 0x96)
                                                 : (uint32_t)(pb >> 32) ^ c1 ^ k0;
            const uint32_t n2 = (r >= kVecFrom1) ? __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), c3, k1, 0x96)
                                                 : (uint32_t)(pa >> 32) ^ c3 ^ k1;
            c1 = (uint32_t)pb;
            c3 = (uint32_t)pa;
            c0 = n0;
            c2 = n2;
        }
        return Words{c0, c1, c2, c3};
    }

    // Two words -> two normals divided by kXiScale.  The 24-bit uniforms are exact in fp32, so
    // the only difference from an fp64 evaluation is the error of log2/sqrt/sin/cos themselves.
    // v_sin_f32 / v_cos_f32 take their argument in revolutions, so u2 is used as is.
    __device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float& z_even, float& z_odd) const
    {
        const float u1 = fmaf((float)(xa >> 8), two_m24, two_m24);   // ((xa>>8)+1) 2^-24 in (0, 1], exact
        const float u2 = (float)(xb >> 8) * 0x1p-24f;                // [0, 1), exact
        const float r = __builtin_amdgcn_sqrtf(-__builtin_amdgcn_logf(u1));
        z_even = r * __builtin_amdgcn_cosf(u2);
        z_odd  = r * __builtin_amdgcn_sinf(u2);
    }

    // Polar form of the same two normals: radius / kXiScale, cosine, sine.  A consumer that
    // multiplies every normal by one factor p can fold p into the radius (one multiply per pair
    // instead of two).
    __device__ __forceinline__ void polar(uint32_t xa, uint32_t xb, float& r, float& c, float& s) const
    {
        const float u1 = fmaf((float)(xa >> 8), two_m24, two_m24);
        const float u2 = (float)(xb >> 8) * 0x1p-24f;
        r = __builtin_amdgcn_sqrtf(-__builtin_amdgcn_logf(u1));
        c = __builtin_amdgcn_cosf(u2);
        s = __builtin_amdgcn_sinf(u2);
    }

    // xi_j[4q .. 4q+3] / kXiScale
    __device__ __forceinline__ void block(uint32_t q, uint32_t j, float& z0, float& z1, float& z2, float& z3) const
    {
        const Words w = words(q, j);
        box_muller(w.x0, w.x1, z0, z1);
        box_muller(w.x2, w.x3, z2, z3);
    }
};

}  // namespace core
