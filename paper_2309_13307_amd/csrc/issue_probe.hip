// Instruction-issue microbenchmark for gfx950 (MI355X): how many SIMD cycles one wave64 VALU
// instruction of each class costs when the SIMD is kept full (8 waves per SIMD).  The CORE kernels
// are bound by VALU issue, so their design (which instructions the generator is written with,
// where the scalar unit is used, why fp32 MFMA does not help at 8 clients) rests on this table.
//
// Standalone program, not part of libcore_hip.so:   ./issue_probe
// Each kernel runs kIters trips of a straight-line block of inline-asm instructions over 8
// independent register chains; cycles = launch time x 2.4 GHz / (instructions per wave x waves per
// SIMD).  The clock under load can sit below 2.4 GHz, so the figures are upper bounds by that ratio.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

namespace {

constexpr int kIters = 2048;
constexpr int kBlocks = 256 * 8;   // x 4 waves = 8 waves per SIMD on 256 CUs x 4 SIMDs
constexpr double kClockHz = 2.4e9;

// one instruction applied to each of the 8 chains a..h (operand %8 = y, a VGPR)
#define EACH8(ins)                                                                             \
    ins " %0, %0, %8\n" ins " %1, %1, %8\n" ins " %2, %2, %8\n" ins " %3, %3, %8\n" ins        \
        " %4, %4, %8\n" ins " %5, %5, %8\n" ins " %6, %6, %8\n" ins " %7, %7, %8\n"
#define EACH8_UNARY(ins)                                                                   \
    ins " %0, %0\n" ins " %1, %1\n" ins " %2, %2\n" ins " %3, %3\n" ins " %4, %4\n" ins    \
        " %5, %5\n" ins " %6, %6\n" ins " %7, %7\n"
#define EACH8_3OP(ins)                                                                               \
    ins " %0, %0, %8, %8\n" ins " %1, %1, %8, %8\n" ins " %2, %2, %8, %8\n" ins " %3, %3, %8, %8\n" \
    ins " %4, %4, %8, %8\n" ins " %5, %5, %8, %8\n" ins " %6, %6, %8, %8\n" ins " %7, %7, %8, %8\n"
#define REGS8 : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e), "+v"(f), "+v"(g), "+v"(h) : "v"(y)

enum Op {
    kXor, kAddU32, kLshr, kMulF32, kAddF32, kFmaSgpr, kAdd3, kMulLo, kMulHi, kMad64,
    kCvt, kLog, kSqrt, kSin, kCos, kMadThenXor, kMfma4x4
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int OP>
__global__ void __launch_bounds__(256) probe(uint32_t* out, uint32_t seed)
{
    uint32_t a = threadIdx.x * 2654435761u + seed, b = a ^ 0x1234567u, c = a + 77u, d = a * 3u + 1u;
    uint32_t e = a ^ 0xdeadbeefu, f = b + 0x9e3779b9u, g = c ^ 0x85ebca6bu, h = d + 0xc2b2ae35u;
    uint32_t y = 0x3f800001u ^ (seed & 1u);
    uint64_t w0 = a, w1 = b, w2 = c, w3 = d;
    f32x4 m0 = {0.f, 0.f, 0.f, 0.f}, m1 = m0, m2 = m0, m3 = m0;
#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (OP == kXor) asm volatile(EACH8("v_xor_b32") REGS8);
            else if constexpr (OP == kAddU32) asm volatile(EACH8("v_add_u32") REGS8);
            else if constexpr (OP == kLshr)
                asm volatile("v_lshrrev_b32 %0, 8, %0\n v_lshrrev_b32 %1, 8, %1\n v_lshrrev_b32 %2, 8, %2\n"
                             "v_lshrrev_b32 %3, 8, %3\n v_lshrrev_b32 %4, 8, %4\n v_lshrrev_b32 %5, 8, %5\n"
                             "v_lshrrev_b32 %6, 8, %6\n v_lshrrev_b32 %7, 8, %7\n" REGS8);
            else if constexpr (OP == kMulF32) asm volatile(EACH8("v_mul_f32") REGS8);
            else if constexpr (OP == kAddF32) asm volatile(EACH8("v_add_f32") REGS8);
            else if constexpr (OP == kFmaSgpr)
                asm volatile("v_fma_f32 %0, s4, %8, %0\n v_fma_f32 %1, s4, %8, %1\n v_fma_f32 %2, s4, %8, %2\n"
                             "v_fma_f32 %3, s4, %8, %3\n v_fma_f32 %4, s4, %8, %4\n v_fma_f32 %5, s4, %8, %5\n"
                             "v_fma_f32 %6, s4, %8, %6\n v_fma_f32 %7, s4, %8, %7\n" REGS8);
            else if constexpr (OP == kAdd3) asm volatile(EACH8_3OP("v_add3_u32") REGS8);
            else if constexpr (OP == kMulLo) asm volatile(EACH8("v_mul_lo_u32") REGS8);
            else if constexpr (OP == kMulHi) asm volatile(EACH8("v_mul_hi_u32") REGS8);
            else if constexpr (OP == kMad64 || OP == kMadThenXor) {
                asm volatile("v_mad_u64_u32 %0, vcc, %4, %8, 0\n v_mad_u64_u32 %1, vcc, %5, %8, 0\n"
                             "v_mad_u64_u32 %2, vcc, %6, %8, 0\n v_mad_u64_u32 %3, vcc, %7, %8, 0\n"
                             : "=&v"(w0), "=&v"(w1), "=&v"(w2), "=&v"(w3), "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(y)
                             :
                             : "vcc");
                if constexpr (OP == kMadThenXor) asm volatile(EACH8("v_xor_b32") REGS8);
                else
                    asm volatile("v_mad_u64_u32 %0, vcc, %4, %8, 0\n v_mad_u64_u32 %1, vcc, %5, %8, 0\n"
                                 "v_mad_u64_u32 %2, vcc, %6, %8, 0\n v_mad_u64_u32 %3, vcc, %7, %8, 0\n"
                                 : "=&v"(w0), "=&v"(w1), "=&v"(w2), "=&v"(w3), "+v"(e), "+v"(f), "+v"(g), "+v"(h), "+v"(y)
                                 :
                                 : "vcc");
            } else if constexpr (OP == kCvt) asm volatile(EACH8_UNARY("v_cvt_f32_u32") REGS8);
            else if constexpr (OP == kLog) asm volatile(EACH8_UNARY("v_log_f32") REGS8);
            else if constexpr (OP == kSqrt) asm volatile(EACH8_UNARY("v_sqrt_f32") REGS8);
            else if constexpr (OP == kSin) asm volatile(EACH8_UNARY("v_sin_f32") REGS8);
            else if constexpr (OP == kCos) asm volatile(EACH8_UNARY("v_cos_f32") REGS8);
            else if constexpr (OP == kMfma4x4) {
                const float fa = __uint_as_float(a), fb = __uint_as_float(b);
                m0 = __builtin_amdgcn_mfma_f32_4x4x1f32(fa, fb, m0, 0, 0, 0);
                m1 = __builtin_amdgcn_mfma_f32_4x4x1f32(fa, fb, m1, 0, 0, 0);
                m2 = __builtin_amdgcn_mfma_f32_4x4x1f32(fb, fa, m2, 0, 0, 0);
                m3 = __builtin_amdgcn_mfma_f32_4x4x1f32(fb, fa, m3, 0, 0, 0);
                m0 = __builtin_amdgcn_mfma_f32_4x4x1f32(fa, fa, m0, 0, 0, 0);
                m1 = __builtin_amdgcn_mfma_f32_4x4x1f32(fb, fb, m1, 0, 0, 0);
                m2 = __builtin_amdgcn_mfma_f32_4x4x1f32(fa, fb, m2, 0, 0, 0);
                m3 = __builtin_amdgcn_mfma_f32_4x4x1f32(fb, fa, m3, 0, 0, 0);
            }
        }
    }
    const f32x4 ms = m0 + m1 + m2 + m3;
    out[blockIdx.x * 256 + threadIdx.x] = a ^ b ^ c ^ d ^ e ^ f ^ g ^ h ^ (uint32_t)(w0 ^ w1 ^ w2 ^ w3) ^
                                          (uint32_t)((w0 ^ w1 ^ w2 ^ w3) >> 32) ^
                                          __float_as_uint(ms.x + ms.y + ms.z + ms.w);
}

// VGPR bank effects (bank = register number mod 4), with explicit registers: eight destination /
// accumulator registers v100, v104, ... (bank 0) and sources picked from chosen banks.
#define BANK_CLOBBERS "v100", "v104", "v108", "v112", "v116", "v120", "v124", "v128", "v101", "v102", "v132"
#define BANK8(ins, tail)                                                                      \
    ins " v100, " tail "\n" ins " v104, " tail "\n" ins " v108, " tail "\n" ins " v112, " tail "\n" \
    ins " v116, " tail "\n" ins " v120, " tail "\n" ins " v124, " tail "\n" ins " v128, " tail "\n"

enum BankCase { kFmacClean, kFmacSrc0InAccBank, kFmaClean, kFmaSrc0Src1SameBank, kBitop3Clean, kBitop3Src0Src1SameBank };

template <int CASE>
__global__ void __launch_bounds__(256) bank_probe(uint32_t* out, uint32_t seed)
{
    asm volatile(BANK8("v_mov_b32", "0") "v_mov_b32 v101, 1.0\n v_mov_b32 v102, 1.0\n v_mov_b32 v132, 1.0\n"
                 ::: BANK_CLOBBERS);
#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (CASE == kFmacClean) asm volatile(BANK8("v_fmac_f32", "v101, v102") ::: BANK_CLOBBERS);
            else if constexpr (CASE == kFmacSrc0InAccBank) asm volatile(BANK8("v_fmac_f32", "v132, v102") ::: BANK_CLOBBERS);
            else if constexpr (CASE == kFmaClean) asm volatile(BANK8("v_fma_f32", "v101, v102, v132") ::: BANK_CLOBBERS);
            else if constexpr (CASE == kFmaSrc0Src1SameBank) asm volatile(BANK8("v_fma_f32", "v132, v100, v102") ::: BANK_CLOBBERS);
            else if constexpr (CASE == kBitop3Clean)
                asm volatile(BANK8("v_bitop3_b32", "v101, v102, v132 bitop3:0x96") ::: BANK_CLOBBERS);
            else asm volatile(BANK8("v_bitop3_b32", "v132, v100, v102 bitop3:0x96") ::: BANK_CLOBBERS);
        }
    }
    uint32_t r;
    asm volatile("v_mov_b32 %0, v100" : "=v"(r)::BANK_CLOBBERS);
    out[blockIdx.x * 256 + threadIdx.x] = r ^ seed;
}

int time_kernel(void (*kern)(uint32_t*, uint32_t), const char* name, int instr_per_group, uint32_t* dout)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(kBlocks), dim3(256), 0, 0, dout, 1u);   // warm-up
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(kBlocks), dim3(256), 0, 0, dout, 3u);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double waves_per_simd = kBlocks * 4 / 1024.0;
    const double instr = (double)kIters * 4 * instr_per_group * waves_per_simd;   // per SIMD
    std::printf("%-44s %8.3f ms   %5.2f cycles per wave64 instruction\n", name, ms, ms * 1e-3 * kClockHz / instr);
    std::fflush(stdout);
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return 0;
}

template <int OP>
int run(const char* name, int instr_per_group, uint32_t* dout)
{
    return time_kernel(probe<OP>, name, instr_per_group, dout);
}

}   // namespace

int main()
{
    uint32_t* dout = nullptr;
    CK(hipMalloc(&dout, (size_t)kBlocks * 256 * sizeof(uint32_t)));
    int rc = 0;
    rc |= run<kXor>("v_xor_b32", 8, dout);
    rc |= run<kAddU32>("v_add_u32", 8, dout);
    rc |= run<kLshr>("v_lshrrev_b32", 8, dout);
    rc |= run<kMulF32>("v_mul_f32", 8, dout);
    rc |= run<kAddF32>("v_add_f32", 8, dout);
    rc |= run<kFmaSgpr>("v_fma_f32 (one SGPR operand)", 8, dout);
    rc |= run<kAdd3>("v_add3_u32", 8, dout);
    rc |= run<kMulLo>("v_mul_lo_u32", 8, dout);
    rc |= run<kMulHi>("v_mul_hi_u32", 8, dout);
    rc |= run<kMad64>("v_mad_u64_u32", 8, dout);
    rc |= run<kCvt>("v_cvt_f32_u32", 8, dout);
    rc |= run<kLog>("v_log_f32", 8, dout);
    rc |= run<kSqrt>("v_sqrt_f32", 8, dout);
    rc |= run<kSin>("v_sin_f32", 8, dout);
    rc |= run<kCos>("v_cos_f32", 8, dout);
    rc |= run<kMadThenXor>("4 v_mad_u64_u32 then 8 v_xor_b32 (average)", 12, dout);
    rc |= run<kMfma4x4>("v_mfma_f32_4x4x1_16B_f32", 8, dout);
    rc |= time_kernel(bank_probe<kFmacClean>, "v_fmac_f32, operands in three banks", 8, dout);
    rc |= time_kernel(bank_probe<kFmacSrc0InAccBank>, "v_fmac_f32, src0 in the accumulator's bank", 8, dout);
    rc |= time_kernel(bank_probe<kFmaClean>, "v_fma_f32, src0/src1 in different banks", 8, dout);
    rc |= time_kernel(bank_probe<kFmaSrc0Src1SameBank>, "v_fma_f32, src0/src1 in the same bank", 8, dout);
    rc |= time_kernel(bank_probe<kBitop3Clean>, "v_bitop3_b32, src0/src1 in different banks", 8, dout);
    rc |= time_kernel(bank_probe<kBitop3Src0Src1SameBank>, "v_bitop3_b32, src0/src1 in the same bank", 8, dout);
    CK(hipFree(dout));
    return rc;
}
