// HIP kernels of the CORE hot path for gfx950 (wave64, 256 CUs in 8 XCDs, 160 KB LDS per CU).
//
//   project_kernel      Algorithm 1 compression line / Algorithm 2 "machine i sends p_ij":
//                       per-chunk partial sums of P[c][j] = <G[c], xi_j>
//   reduce_*_kernel     sum of the partials over chunks (fp64, fixed order) and the client mean
//                       pbar[j] = (1/n) sum_c P[c][j]            (Eq. (tildefdef))
//   reconstruct_kernel  gtilde[i] = scale * sum_j pbar[j] xi_j[i]  (Eq. (reconstruction))
//
// Both heavy kernels are bound by VALU issue (the generator: ~40 integer/transcendental
// lane-ops per normal), not by HBM: G is read once per 256-vector tile and gtilde written once.
// The lane mappings are chosen to make the generator as cheap as possible:
//   - projection: lanes run over the vector index j, all lanes of a wave share the Philox
//     block q.  Then counter words 0, 2, 3 are wave-uniform, the scalar unit does 4 of the 20
//     Philox products, every lane owns its (j, client) sums (no cross-lane reduction), and the
//     wave-uniform G values arrive as LDS broadcast reads (VGPR operands; an SGPR operand
//     would nearly double the cost of each FMA on this chip).
//   - reconstruction: lanes run over q (coalesced 128-bit stores), j is the loop index and
//     wave-uniform: 2 of the 20 products are scalar, pbar[j] is an LDS broadcast read.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_rng.hpp"

namespace core {

constexpr int kThreads = 256;     // threads per block in every kernel
constexpr int kTile = 256;        // coordinates of G staged in LDS per step (64 Philox blocks)
constexpr int kPbarTile = 1024;   // pbar values staged in LDS per step

struct ProjectArgs {
    const void* G;        // [n][ld], element type by template
    uint64_t ld;
    uint64_t d;
    uint32_t m;
    uint32_t n;           // total clients (row count of the partial array)
    uint32_t c0;          // first client of this pass
    uint32_t nc;          // clients in this pass (<= NC)
    uint32_t k0, k1;      // seed halves
    uint32_t r0, r1;      // round halves
    const uint32_t* round_dev;   // when non-null, the round counter (lo, hi) is read from here instead
    uint32_t jtiles;      // vector tiles of this launch: tiles of 256, 64 or JW vectors, or groups of QJ vectors
    uint32_t j_begin;     // first vector of this launch (the small-tile launches follow the tiles of 256)
    uint32_t nchunks;     // chunks of d
    uint32_t tiles_per_chunk;
    float* part;          // [nchunks][n][m]
    float* xi_store;      // materialised variant only: [ceil(d/4)][m][4], else unused
    int vec_load;         // rows of G start on 16-byte (fp32) / 8-byte (bf16) boundaries, so a thread of the
                          // kernels that fetch 4 coordinates per lane may do it with one load
};

template <bool BF16>
__device__ __forceinline__ float load_g(const void* G, uint64_t idx)
{
    if constexpr (BF16) {
        return __uint_as_float((uint32_t)((const uint16_t*)G)[idx] << 16);
    } else {
        return ((const float*)G)[idx];
    }
}

// STORE_XI: the materialised-Xi comparison variant.  The kernel additionally writes every normal
// it generates to xi_store[q][j][0..3] = xi_j[4q..4q+3], so that reconstruct_xi_kernel can read
// them back instead of regenerating them.
template <int NC, bool BF16, bool STORE_XI = false>
__global__ void __launch_bounds__(kThreads) project_kernel(ProjectArgs a)
{
    __shared__ __attribute__((aligned(16))) float tile[NC][kTile];

    // Consecutive block ids are dealt round-robin to the 8 XCDs; keep all vector tiles
    // of one chunk of G on one XCD so the chunk is fetched into a single L2.
    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b & 7u;
    const uint32_t s = b >> 3;
    const uint32_t chunk = (s / a.jtiles) * 8u + xcd;
    const uint32_t jt = s % a.jtiles;
    if (chunk >= a.nchunks) return;

    const uint32_t t = threadIdx.x;
    const uint32_t j = jt * kThreads + t;
    const bool wave_active = (jt * kThreads + (t & ~63u)) < a.m;   // wave-uniform

    const uint64_t tiles_total = (a.d + kTile - 1) / kTile;
    const uint64_t tile_begin = (uint64_t)chunk * a.tiles_per_chunk;
    uint64_t tile_end = tile_begin + a.tiles_per_chunk;
    if (tile_end > tiles_total) tile_end = tiles_total;

    // lanes differ in j (counter word 1) only: the state is fully divergent after 3 rounds
    Generator<3, 4> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float acc_outer[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc_outer[c] = 0.0f;

    // register prefetch of the next tile: thread t holds coordinate i0 + t of every client
    float pre[NC];
    auto fetch = [&](uint64_t tl) {
        const uint64_t i = tl * kTile + t;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float v = 0.0f;
            if (i < a.d && (uint32_t)c < a.nc) v = load_g<BF16>(a.G, (uint64_t)(a.c0 + c) * a.ld + i);
            pre[c] = v;
        }
    };
    if (tile_begin < tile_end) fetch(tile_begin);

    for (uint64_t tl = tile_begin; tl < tile_end; ++tl) {
        __syncthreads();
#pragma unroll
        for (int c = 0; c < NC; ++c) tile[c][t] = pre[c];
        __syncthreads();
        if (tl + 1 < tile_end) fetch(tl + 1);

        float acc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] = 0.0f;
        const uint32_t q0 = (uint32_t)(tl * (kTile / 4));
        if (!wave_active) continue;   // this wave only helps staging G (m is not a multiple of 256)
#pragma unroll 2
        for (int qq = 0; qq < kTile / 4; ++qq) {
            float z0, z1, z2, z3;
            gen.block(q0 + (uint32_t)qq, j, z0, z1, z2, z3);
            if constexpr (STORE_XI) {
                const uint64_t q = (uint64_t)q0 + (uint32_t)qq;
                if (j < a.m && 4 * q < a.d)
                    *reinterpret_cast<float4*>(a.xi_store + (q * a.m + j) * 4) =
                        make_float4(kXiScale * z0, kXiScale * z1, kXiScale * z2, kXiScale * z3);
            }
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 g = *reinterpret_cast<const float4*>(&tile[c][4 * qq]);
                acc[c] = fmaf(z0, g.x, acc[c]);
                acc[c] = fmaf(z1, g.y, acc[c]);
                acc[c] = fmaf(z2, g.z, acc[c]);
                acc[c] = fmaf(z3, g.w, acc[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) acc_outer[c] += acc[c];
    }

    if (j < a.m) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if ((uint32_t)c < a.nc)
                a.part[((uint64_t)chunk * a.n + a.c0 + c) * a.m + j] = kXiScale * acc_outer[c];
        }
    }
}

// The lanes-over-vectors projection for 64 vectors per block instead of 256: serves the whole waves
// of a vector count that does not fill a tile of 256 (the rest m mod 256).  A wave of project_kernel is
// latency-bound on its own (the generator is one long dependency chain) and only about 8 busy waves per
// SIMD saturate the issue port, so a block of 256 with idle waves wastes wave slots.  Here all four
// waves of a block take the SAME 64 vectors, a.j_begin + 64 jt + lane, and share the chunk's
// coordinates instead: the chunk is walked in steps of 64 coordinates and wave w takes the steps
// w, w + 4, w + 8, ...; each wave stages its own step of G in its own part of LDS, and the four
// partial sums are added in wave order at the end, so the block writes one partial sum per (vector,
// client) exactly like a block of project_kernel.  a.jtiles counts tiles of 64 vectors here.
// Inside the loop the waves do not wait for each other: a wave's part of LDS is written and read by
// that wave alone, and the LDS operations of one wave are performed in program order.
constexpr int kNarrow = 64;

template <int NC, bool BF16>
__global__ void __launch_bounds__(kThreads) project_narrow_kernel(ProjectArgs a)
{
    __shared__ __attribute__((aligned(16))) float tile[kThreads / 64][NC][kNarrow];
    __shared__ float red[kThreads / 64][NC][kNarrow];

    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b & 7u;
    const uint32_t s = b >> 3;
    const uint32_t chunk = (s / a.jtiles) * 8u + xcd;
    const uint32_t jt = s % a.jtiles;
    if (chunk >= a.nchunks) return;

    const uint32_t t = threadIdx.x, lane = t & 63u;
    const uint32_t w = (uint32_t)__builtin_amdgcn_readfirstlane((int)(t >> 6));   // wave-uniform, so scalar
    const uint32_t j = a.j_begin + jt * kNarrow + lane;

    constexpr uint32_t kStepsPerTile = kTile / kNarrow;
    const uint64_t steps_total = (a.d + kNarrow - 1) / kNarrow;
    const uint64_t step_begin = (uint64_t)chunk * a.tiles_per_chunk * kStepsPerTile;
    uint64_t step_end = step_begin + (uint64_t)a.tiles_per_chunk * kStepsPerTile;
    if (step_end > steps_total) step_end = steps_total;

    Generator<3, 4> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float acc_outer[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc_outer[c] = 0.0f;

    // register prefetch of this wave's next step: lane l holds coordinate 64 step + l of every client
    float pre[NC];
    auto fetch = [&](uint64_t step) {
        const uint64_t i = step * kNarrow + lane;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float v = 0.0f;
            if (step < step_end && i < a.d && (uint32_t)c < a.nc) v = load_g<BF16>(a.G, (uint64_t)(a.c0 + c) * a.ld + i);
            pre[c] = v;
        }
    };
    fetch(step_begin + w);

    for (uint64_t step = step_begin + w; step < step_end; step += 4) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < NC; ++c) tile[w][c][lane] = pre[c];
        __builtin_amdgcn_wave_barrier();
        fetch(step + 4);

        float acc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] = 0.0f;
        const uint32_t q0 = (uint32_t)(step * (kNarrow / 4));
#pragma unroll 2
        for (int qq = 0; qq < kNarrow / 4; ++qq) {
            float z0, z1, z2, z3;
            gen.block(q0 + (uint32_t)qq, j, z0, z1, z2, z3);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 g = *reinterpret_cast<const float4*>(&tile[w][c][4 * qq]);
                acc[c] = fmaf(z0, g.x, acc[c]);
                acc[c] = fmaf(z1, g.y, acc[c]);
                acc[c] = fmaf(z2, g.z, acc[c]);
                acc[c] = fmaf(z3, g.w, acc[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) acc_outer[c] += acc[c];
    }

#pragma unroll
    for (int c = 0; c < NC; ++c) red[w][c][lane] = acc_outer[c];
    __syncthreads();
    if (w == 0 && j < a.m) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if ((uint32_t)c < a.nc) {
                const float tot = ((red[0][c][lane] + red[1][c][lane]) + red[2][c][lane]) + red[3][c][lane];
                a.part[((uint64_t)chunk * a.n + a.c0 + c) * a.m + j] = kXiScale * tot;
            }
        }
    }
}

// Matrix-pipe variant of the projection, used for passes of more than 8 clients (and selectable
// with the environment variable CORE_PROJECT_VARIANT=mfma|valu for A/B runs).  Same lane mapping and generator as
// project_kernel; the 4*NC v_fmac per call are replaced by NC v_mfma_f32_4x4x1_16B_f32: block
// b = lane/4 of the instruction computes the 4x4 outer product of (xi of vectors 4b..4b+3) and
// (G of clients 4g..4g+3) at one coordinate.  Lane l supplies A = its own normal and
// B = G[4g + l%4][coordinate]; it receives D[i] = sum for vector 4(l/4)+i and client 4g + l%4.
// fp32 MFMA has the same peak as the vector FMA on this chip and its issue does not overlap the
// generator's VALU work (a probe with 16x16x4 and 32x32x2 instructions next to the generator showed
// the two times adding up exactly, at 1 to 8 waves per SIMD), so what it buys is fewer LDS reads and
// registers per FMA.  Measured on a ResNet-50-sized gradient, m = 1024, projection alone: 8 clients
// 13.85 ms at best against 13.7 ms on the vector ALU; 9 clients 15.9 against 19.5 ms, 12 clients 16.0
// against 19.8 ms, 16 clients 16.8 against 20.5 ms.
typedef float mfma_f32x4 __attribute__((ext_vector_type(4)));

// Occupancy targets.  Left alone the compiler takes 112-180 registers for 3 to 8 client groups
// (4 to 2 waves per SIMD); asking for more waves makes it reuse registers and the kernel is faster at
// every width (measured at d = 2^23, m = 1024, bf16: 16 clients 6.31 -> 5.69 ms at 5 waves, 24 clients
// 7.73 -> 7.15 ms at 3 waves, 32 clients 10.26 -> 8.94 ms at 3 waves; only the 8-group kernel then spills,
// 23 registers of the tile prefetch).
template <int NG, bool BF16>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(NG >= 6 ? 3 : NG >= 3 ? 5 : 1)))
project_mfma_kernel(ProjectArgs a)
{
    constexpr int NC = 4 * NG;
    constexpr int kRow = kTile + 4;   // 16-byte skew: the 4 client rows a wave reads hit distinct banks
    __shared__ __attribute__((aligned(16))) float tile[NC][kRow];

    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b & 7u;
    const uint32_t s = b >> 3;
    const uint32_t chunk = (s / a.jtiles) * 8u + xcd;
    const uint32_t jt = s % a.jtiles;
    if (chunk >= a.nchunks) return;

    const uint32_t t = threadIdx.x;
    const uint32_t j = jt * kThreads + t;
    const uint32_t csub = t & 3u;
    const bool wave_active = (jt * kThreads + (t & ~63u)) < a.m;   // wave-uniform

    const uint64_t tiles_total = (a.d + kTile - 1) / kTile;
    const uint64_t tile_begin = (uint64_t)chunk * a.tiles_per_chunk;
    uint64_t tile_end = tile_begin + a.tiles_per_chunk;
    if (tile_end > tiles_total) tile_end = tiles_total;

    Generator<3, 4> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    mfma_f32x4 outer[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) outer[g] = mfma_f32x4{0.f, 0.f, 0.f, 0.f};

    float pre[NC];
    auto fetch = [&](uint64_t tl) {
        const uint64_t i = tl * kTile + t;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float v = 0.0f;
            if (i < a.d && (uint32_t)c < a.nc) v = load_g<BF16>(a.G, (uint64_t)(a.c0 + c) * a.ld + i);
            pre[c] = v;
        }
    };
    if (tile_begin < tile_end) fetch(tile_begin);

    for (uint64_t tl = tile_begin; tl < tile_end; ++tl) {
        __syncthreads();
#pragma unroll
        for (int c = 0; c < NC; ++c) tile[c][t] = pre[c];
        __syncthreads();
        if (tl + 1 < tile_end) fetch(tl + 1);

        // kSplit independent accumulator sets per client group: consecutive matrix instructions
        // never wait for each other's result
        constexpr int kSplit = (NG >= 4) ? 1 : (NG >= 2 ? 2 : 4);
        mfma_f32x4 acc[kSplit][NG];
#pragma unroll
        for (int sidx = 0; sidx < kSplit; ++sidx)
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[sidx][g] = mfma_f32x4{0.f, 0.f, 0.f, 0.f};
        const uint32_t q0 = (uint32_t)(tl * (kTile / 4));
        if (!wave_active) continue;   // this wave only helps staging G (m is not a multiple of 256)
#pragma unroll 2
        for (int qq = 0; qq < kTile / 4; ++qq) {
            float z0, z1, z2, z3;
            gen.block(q0 + (uint32_t)qq, j, z0, z1, z2, z3);
            float4 gv[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g) gv[g] = *reinterpret_cast<const float4*>(&tile[4 * g + csub][4 * qq]);
            // coordinate-major order: consecutive instructions update different accumulators
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[0][g] = __builtin_amdgcn_mfma_f32_4x4x1f32(z0, gv[g].x, acc[0][g], 0, 0, 0);
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[1 % kSplit][g] = __builtin_amdgcn_mfma_f32_4x4x1f32(z1, gv[g].y, acc[1 % kSplit][g], 0, 0, 0);
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[2 % kSplit][g] = __builtin_amdgcn_mfma_f32_4x4x1f32(z2, gv[g].z, acc[2 % kSplit][g], 0, 0, 0);
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[3 % kSplit][g] = __builtin_amdgcn_mfma_f32_4x4x1f32(z3, gv[g].w, acc[3 % kSplit][g], 0, 0, 0);
        }
#pragma unroll
        for (int sidx = 0; sidx < kSplit; ++sidx)
#pragma unroll
            for (int g = 0; g < NG; ++g) outer[g] += acc[sidx][g];
    }

    const uint32_t jrow = jt * kThreads + (t & ~3u);   // first of the 4 vectors this lane reports
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const uint32_t c = 4 * g + csub;
        if (c < a.nc) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (jrow + i < a.m)
                    a.part[((uint64_t)chunk * a.n + a.c0 + c) * a.m + jrow + i] = kXiScale * outer[g][i];
        }
    }
}

// Matrix-pipe projection for wide passes (33 to 64 clients at once), so that the normals are
// generated once for up to 64 machines (Eq. (tildefdef): the same xi_j serve all n machines).
// Same lane mapping, generator and matrix instruction as project_mfma_kernel; what differs is what
// lets 4*NG sums per lane fit: one level of accumulation (the launch plan caps a chunk at 4096
// coordinates for such calls, so an fp32 chain is never longer than that), tiles of 128
// coordinates staged straight from global memory (33.8 KB of LDS at 64 clients: three to four
// workgroups per CU), and the client groups taken four at a time so that only four LDS reads are
// live.  A lane reads its B operands with one 128-bit LDS read per client group and call, a quarter
// of the LDS traffic the vector-ALU form would need at this width.
constexpr int kWideTile = 128;

// Occupancy target of 4 waves per SIMD (128 registers): measured on a ResNet-50-sized gradient with
// m = 1024, 50 clients 34.4 ms against 35.4 ms at 3 waves and 35.7 ms at 2; 64 clients 39.9 / 40.0 / 49.3 ms.
template <int NG, bool BF16>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4)))
project_mfma_wide_kernel(ProjectArgs a)
{
    constexpr int NC = 4 * NG;
    constexpr int kRow = kWideTile + 4;   // 16-byte skew, as in project_mfma_kernel
    __shared__ __attribute__((aligned(16))) float tile[NC][kRow];

    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b & 7u;
    const uint32_t s = b >> 3;
    const uint32_t chunk = (s / a.jtiles) * 8u + xcd;
    const uint32_t jt = s % a.jtiles;
    if (chunk >= a.nchunks) return;

    const uint32_t t = threadIdx.x;
    const uint32_t j = jt * kThreads + t;
    const uint32_t csub = t & 3u;
    const bool wave_active = (jt * kThreads + (t & ~63u)) < a.m;   // wave-uniform

    const uint64_t chunk_len = (uint64_t)a.tiles_per_chunk * kTile;   // a multiple of kWideTile
    const uint64_t i_begin = (uint64_t)chunk * chunk_len;
    uint64_t i_end = i_begin + chunk_len;
    if (i_end > a.d) i_end = a.d;

    Generator<3, 4> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    mfma_f32x4 acc[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = mfma_f32x4{0.f, 0.f, 0.f, 0.f};

    const uint32_t col = t & (kWideTile - 1);   // coordinate of the tile this thread stages
    const uint32_t crow = t / kWideTile;        // ... for clients crow, crow + 2, crow + 4, ...
    for (uint64_t i0 = i_begin; i0 < i_end; i0 += kWideTile) {
        __syncthreads();
        const uint64_t i = i0 + col;
#pragma unroll
        for (int k = 0; k < NC / 2; ++k) {
            const uint32_t c = crow + 2 * k;
            float v = 0.0f;
            if (i < a.d && c < a.nc) v = load_g<BF16>(a.G, (uint64_t)(a.c0 + c) * a.ld + i);
            tile[c][col] = v;
        }
        __syncthreads();
        if (!wave_active) continue;   // this wave only helps staging G (m is not a multiple of 256)
        const uint32_t q0 = (uint32_t)(i0 / 4);
        for (int qq = 0; qq < kWideTile / 4; ++qq) {
            float z0, z1, z2, z3;
            gen.block(q0 + (uint32_t)qq, j, z0, z1, z2, z3);
#pragma unroll
            for (int g0 = 0; g0 < NG; g0 += 4) {
                constexpr int kBatchMax = 4;
                const int nb = (NG - g0 < kBatchMax) ? (NG - g0) : kBatchMax;   // compile-time after unrolling
                float4 gv[kBatchMax];
#pragma unroll
                for (int gg = 0; gg < kBatchMax; ++gg)
                    if (gg < nb) gv[gg] = *reinterpret_cast<const float4*>(&tile[4 * (g0 + gg) + csub][4 * qq]);
                // coordinate-major order: consecutive instructions update different accumulators
#pragma unroll
                for (int gg = 0; gg < kBatchMax; ++gg)
                    if (gg < nb) acc[g0 + gg] = __builtin_amdgcn_mfma_f32_4x4x1f32(z0, gv[gg].x, acc[g0 + gg], 0, 0, 0);
#pragma unroll
                for (int gg = 0; gg < kBatchMax; ++gg)
                    if (gg < nb) acc[g0 + gg] = __builtin_amdgcn_mfma_f32_4x4x1f32(z1, gv[gg].y, acc[g0 + gg], 0, 0, 0);
#pragma unroll
                for (int gg = 0; gg < kBatchMax; ++gg)
                    if (gg < nb) acc[g0 + gg] = __builtin_amdgcn_mfma_f32_4x4x1f32(z2, gv[gg].z, acc[g0 + gg], 0, 0, 0);
#pragma unroll
                for (int gg = 0; gg < kBatchMax; ++gg)
                    if (gg < nb) acc[g0 + gg] = __builtin_amdgcn_mfma_f32_4x4x1f32(z3, gv[gg].w, acc[g0 + gg], 0, 0, 0);
            }
        }
    }

    const uint32_t jrow = jt * kThreads + (t & ~3u);   // first of the 4 vectors this lane reports
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const uint32_t c = 4 * g + csub;
        if (c < a.nc) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (jrow + i < a.m)
                    a.part[((uint64_t)chunk * a.n + a.c0 + c) * a.m + jrow + i] = kXiScale * acc[g][i];
        }
    }
}

// Projection for very few vectors or for little work.  With lanes over the vectors a block of 256
// threads needs 256 vectors to keep its four waves busy (and the busy waves of partly filled blocks
// pile up on the same SIMDs); here lanes run over the Philox block q, as in the reconstruction, so
// every lane works whatever the number of vectors is.  A block owns QJ consecutive vectors and a
// chunk of 1024-coordinate tiles; each thread loads G for its 4 coordinates once per tile (one 64- or
// 128-bit load per client when the rows allow it) and keeps it in registers for all QJ vectors, so
// there is no LDS traffic in the loop; the QJ x NC sums are combined across the block once per chunk
// (wave butterfly, then LDS in wave order; fixed order).
template <bool BF16>
__device__ __forceinline__ void load_g4(const void* G, uint64_t base, uint64_t i, uint64_t d, bool vec, float (&g)[4])
{
    if (vec && i + 4 <= d) {
        if constexpr (BF16) {
            const uint2 v = *reinterpret_cast<const uint2*>((const uint16_t*)G + base);
            g[0] = __uint_as_float(v.x << 16); g[1] = __uint_as_float(v.x & 0xffff0000u);
            g[2] = __uint_as_float(v.y << 16); g[3] = __uint_as_float(v.y & 0xffff0000u);
        } else {
            const float4 v = *reinterpret_cast<const float4*>((const float*)G + base);
            g[0] = v.x; g[1] = v.y; g[2] = v.z; g[3] = v.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) g[k] = (i + k < d) ? load_g<BF16>(G, base + k) : 0.0f;
    }
}

// The 4 coordinates of one client as they come from memory, kept in that form while the loads are
// in flight (prefetch of the next tile) and widened to fp32 only when the tile is used.
template <bool BF16> struct RawG4;

template <> struct RawG4<false> {
    float v[4];
    __device__ __forceinline__ void load(const void* G, uint64_t base, uint64_t i, uint64_t d, bool vec)
    {
        if (vec && i + 4 <= d) {
            const float4 x = *reinterpret_cast<const float4*>((const float*)G + base);
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = (i + k < d) ? ((const float*)G)[base + k] : 0.0f;
        }
    }
    __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.0f; }
    __device__ __forceinline__ void widen(float (&g)[4]) const { g[0] = v[0]; g[1] = v[1]; g[2] = v[2]; g[3] = v[3]; }
};

template <> struct RawG4<true> {
    uint32_t lo, hi;   // bf16 pairs: coordinates (0, 1) and (2, 3)
    __device__ __forceinline__ void load(const void* G, uint64_t base, uint64_t i, uint64_t d, bool vec)
    {
        const uint16_t* p = (const uint16_t*)G + base;
        if (vec && i + 4 <= d) {
            const uint2 x = *reinterpret_cast<const uint2*>(p);
            lo = x.x; hi = x.y;
        } else {
            uint32_t e[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) e[k] = (i + k < d) ? (uint32_t)p[k] : 0u;
            lo = e[0] | (e[1] << 16); hi = e[2] | (e[3] << 16);
        }
    }
    __device__ __forceinline__ void zero() { lo = hi = 0u; }
    __device__ __forceinline__ void widen(float (&g)[4]) const
    {
        g[0] = __uint_as_float(lo << 16); g[1] = __uint_as_float(lo & 0xffff0000u);
        g[2] = __uint_as_float(hi << 16); g[3] = __uint_as_float(hi & 0xffff0000u);
    }
};

// The lanes-over-vectors projection for tiles of JW = 8, 16 or 32 vectors: what is left of m mod 256
// after its whole waves, and few vectors on a long gradient.  As in project_narrow_kernel the four
// waves of a block take the same JW vectors and share the chunk's coordinates, wave w taking the
// 256-coordinate tiles w, w + 4, ... of the chunk and staging each in its own part of LDS; but the
// lanes of a wave split further: lane l works on vector a.j_begin + JW jt + (l mod JW) and, of the 64
// Philox blocks of a tile, on those congruent to l / JW modulo 64 / JW, so every lane is busy whatever
// the vector count.  The 64 / JW partial sums of a vector are added across the lanes once per chunk
// (butterfly over the upper lane bits), then the four waves' sums in wave order, and the block writes
// one partial sum per (vector, client) like a block of project_kernel.  a.jtiles counts tiles of JW
// vectors.  With so few generator calls per coordinate the loads of G must be wide and early: a lane
// fetches 4 consecutive coordinates per client with one 64- or 128-bit load where the rows allow it,
// a whole tile ahead, and keeps them in their stored form until the tile is used (with 64-coordinate
// steps and element loads the kernel took 0.37 ms at the ResNet-50 size whatever JW was, waiting for
// memory).  No block barrier in the loop: a wave's part of LDS is written and read by that wave
// alone, and the LDS operations of one wave are performed in program order.
template <int NC, bool BF16, int JW>
__global__ void __launch_bounds__(kThreads) project_sub_kernel(ProjectArgs a)
{
    static_assert(JW == 32 || JW == 16 || JW == 8, "vectors per tile");
    static_assert(NC <= 8, "LDS: four waves x NC x 256 floats");
    constexpr int QW = 64 / JW;             // lane groups of a wave, each with its own Philox blocks
    constexpr int kCalls = (kTile / 4) / QW;   // generator calls per lane per tile
    __shared__ __attribute__((aligned(16))) float tile[kThreads / 64][NC][kTile];
    __shared__ float red[kThreads / 64][NC][JW];

    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b & 7u;
    const uint32_t s = b >> 3;
    const uint32_t chunk = (s / a.jtiles) * 8u + xcd;
    const uint32_t jt = s % a.jtiles;
    if (chunk >= a.nchunks) return;

    const uint32_t t = threadIdx.x, lane = t & 63u;
    const uint32_t w = (uint32_t)__builtin_amdgcn_readfirstlane((int)(t >> 6));   // wave-uniform, so scalar
    const uint32_t jl = lane % JW, qs = lane / JW;
    const uint32_t j = a.j_begin + jt * JW + jl;

    const uint64_t tiles_total = (a.d + kTile - 1) / kTile;
    const uint64_t tile_begin = (uint64_t)chunk * a.tiles_per_chunk;
    uint64_t tile_end = tile_begin + a.tiles_per_chunk;
    if (tile_end > tiles_total) tile_end = tiles_total;

    // lanes differ in q and in j: every round after the first is fully divergent
    Generator<1, 1> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float acc_outer[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc_outer[c] = 0.0f;

    // register prefetch of this wave's next tile: lane l holds coordinates 256 tile + 4 l .. + 3 of every client
    RawG4<BF16> pre[NC];
    const bool vec = a.vec_load != 0;
    auto fetch = [&](uint64_t tl) {
        const uint64_t i = tl * kTile + 4 * lane;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (tl < tile_end && (uint32_t)c < a.nc) pre[c].load(a.G, (uint64_t)(a.c0 + c) * a.ld + i, i, a.d, vec);
            else pre[c].zero();
        }
    };
    fetch(tile_begin + w);

    for (uint64_t tl = tile_begin + w; tl < tile_end; tl += 4) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float g[4];
            pre[c].widen(g);
            *reinterpret_cast<float4*>(&tile[w][c][4 * lane]) = make_float4(g[0], g[1], g[2], g[3]);
        }
        __builtin_amdgcn_wave_barrier();
        fetch(tl + 4);

        float acc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] = 0.0f;
        const uint32_t q0 = (uint32_t)(tl * (kTile / 4));
#pragma unroll 2
        for (int k = 0; k < kCalls; ++k) {
            const uint32_t qq = qs + (uint32_t)(QW * k);
            float z0, z1, z2, z3;
            gen.block(q0 + qq, j, z0, z1, z2, z3);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const float4 g = *reinterpret_cast<const float4*>(&tile[w][c][4 * qq]);
                acc[c] = fmaf(z0, g.x, acc[c]);
                acc[c] = fmaf(z1, g.y, acc[c]);
                acc[c] = fmaf(z2, g.z, acc[c]);
                acc[c] = fmaf(z3, g.w, acc[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) acc_outer[c] += acc[c];
    }

    // the lane groups of a vector: butterfly over the lane bits above log2(JW)
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int off = JW; off < 64; off <<= 1) acc_outer[c] += __shfl_xor(acc_outer[c], off, 64);
    }
    if (qs == 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c) red[w][c][jl] = acc_outer[c];
    }
    __syncthreads();
    if (w == 0 && qs == 0 && j < a.m) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if ((uint32_t)c < a.nc) {
                const float tot = ((red[0][c][jl] + red[1][c][jl]) + red[2][c][jl]) + red[3][c][jl];
                a.part[((uint64_t)chunk * a.n + a.c0 + c) * a.m + j] = kXiScale * tot;
            }
        }
    }
}

template <int NC, bool BF16, int QJ>
__global__ void __launch_bounds__(kThreads) project_q_kernel(ProjectArgs a)
{
    __shared__ float red[kThreads / 64][QJ * NC];
    const uint32_t t = threadIdx.x;
    // As in project_kernel: consecutive block ids go round-robin over the 8 XCDs, so all vector groups
    // of one chunk of G are given ids congruent mod 8 and the chunk is fetched into a single L2
    // (each group re-reads the chunk: m / QJ times in all).
    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b & 7u;
    const uint32_t s = b >> 3;
    const uint32_t chunk = (s / a.jtiles) * 8u + xcd;   // a.jtiles = groups of QJ vectors here
    const uint32_t jg = s % a.jtiles;
    if (chunk >= a.nchunks) return;
    const uint32_t j0 = a.j_begin + jg * QJ;

    const uint64_t qtile = (uint64_t)kThreads * 4;      // coordinates per tile
    const uint64_t tiles_total = (a.d + qtile - 1) / qtile;
    const uint64_t tile_begin = (uint64_t)chunk * a.tiles_per_chunk;
    uint64_t tile_end = tile_begin + a.tiles_per_chunk;
    if (tile_end > tiles_total) tile_end = tiles_total;

    Generator<2, 3> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float acc[QJ][NC];
#pragma unroll
    for (int jj = 0; jj < QJ; ++jj)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[jj][c] = 0.0f;

    // A group with all QJ vectors present (every group but possibly the last) runs a loop body
    // without branches, so that the QJ independent generator calls can be interleaved.  The next
    // tile of G is fetched into registers before the current one is used: the workgroups of a CU
    // start together and stay in phase, so without it they would all wait for memory at once.
    auto walk = [&](auto full_group) {
        constexpr bool kFull = decltype(full_group)::value;
        RawG4<BF16> raw[NC];
        auto fetch = [&](uint64_t tl) {
            const uint64_t i = 4 * (tl * kThreads + t);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                if ((uint32_t)c < a.nc) raw[c].load(a.G, (uint64_t)(a.c0 + c) * a.ld + i, i, a.d, a.vec_load != 0);
                else                    raw[c].zero();
            }
        };
        if (tile_begin < tile_end) fetch(tile_begin);
        for (uint64_t tl = tile_begin; tl < tile_end; ++tl) {
            const uint64_t q = tl * kThreads + t;
            float g[NC][4];
#pragma unroll
            for (int c = 0; c < NC; ++c) raw[c].widen(g[c]);
            if (tl + 1 < tile_end) fetch(tl + 1);
#pragma unroll
            for (int jj = 0; jj < QJ; ++jj) {
                if constexpr (!kFull) {
                    if (j0 + jj >= a.m) break;           // block-uniform
                }
                float z0, z1, z2, z3;
                gen.block((uint32_t)q, j0 + jj, z0, z1, z2, z3);
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    acc[jj][c] = fmaf(z0, g[c][0], acc[jj][c]);
                    acc[jj][c] = fmaf(z1, g[c][1], acc[jj][c]);
                    acc[jj][c] = fmaf(z2, g[c][2], acc[jj][c]);
                    acc[jj][c] = fmaf(z3, g[c][3], acc[jj][c]);
                }
            }
        }
    };
    if (j0 + QJ <= a.m) walk(std::true_type{});
    else                walk(std::false_type{});

    // fixed-order combination: butterfly inside each wave, then waves 0..3 in order
#pragma unroll
    for (int jj = 0; jj < QJ; ++jj)
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float v = acc[jj][c];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
            if ((t & 63u) == 0) red[t >> 6][jj * NC + c] = v;
        }
    __syncthreads();
    if (t < (uint32_t)(QJ * NC)) {
        const uint32_t jj = t / NC, c = t % NC;
        if (j0 + jj < a.m && c < a.nc) {
            float tot = red[0][t];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) tot += red[w][t];
            a.part[((uint64_t)chunk * a.n + a.c0 + c) * a.m + j0 + jj] = kXiScale * tot;
        }
    }
}

// Projection, cross-chunk sum and client mean in one launch, for problems so small that launches
// are what a round costs (a few thousand coordinates, at most 8 clients): Algorithm 2's "machine i
// sends p_ij" and "central machine sends the combined p_j back" back to back.  One workgroup per
// vector j walks the whole of d, lanes over the Philox block q, each thread keeping its share of the
// NC sums; the workgroup then holds every term of P[c][j], adds them in a fixed order (butterfly
// inside each wave, then the waves in order) and writes P[c][j] (optional) and
// pbar[j] = (1/n) sum_c P[c][j] itself.  No partial sums leave the workgroup, so the workspace is
// not touched.  blockDim.x is a multiple of 64, at most 1024.
struct ProjectSmallArgs {
    const void* G;        // [n][ld]
    uint64_t ld;
    uint64_t d;
    uint32_t m;
    uint32_t n;           // clients, n <= NC
    uint32_t k0, k1, r0, r1;
    const uint32_t* round_dev;
    int vec_load;         // rows start on 16-byte (fp32) / 8-byte (bf16) boundaries: 4 coordinates per load
    float* P;             // [n][m] or null
    float* pbar;          // [m]
};

template <int NC, bool BF16>
__global__ void __launch_bounds__(1024) project_small_kernel(ProjectSmallArgs a)
{
    __shared__ float red[16][NC];
    const uint32_t t = threadIdx.x, nthreads = blockDim.x;
    const uint32_t j = blockIdx.x;
    const uint64_t nblk = (a.d + 3) / 4;

    Generator<2, 3> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float acc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc[c] = 0.0f;

    for (uint64_t q = t; q < nblk; q += nthreads) {
        const uint64_t i = 4 * q;
        float g[NC][4];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if ((uint32_t)c < a.n) {
                load_g4<BF16>(a.G, (uint64_t)c * a.ld + i, i, a.d, a.vec_load != 0, g[c]);
            } else {
                g[c][0] = g[c][1] = g[c][2] = g[c][3] = 0.0f;
            }
        }
        float z0, z1, z2, z3;
        gen.block((uint32_t)q, j, z0, z1, z2, z3);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            acc[c] = fmaf(z0, g[c][0], acc[c]);
            acc[c] = fmaf(z1, g[c][1], acc[c]);
            acc[c] = fmaf(z2, g[c][2], acc[c]);
            acc[c] = fmaf(z3, g[c][3], acc[c]);
        }
    }

#pragma unroll
    for (int c = 0; c < NC; ++c) {
        float v = acc[c];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if ((t & 63u) == 0) red[t >> 6][c] = v;
    }
    __syncthreads();
    // lane c of the first wave adds client c's per-wave sums in wave order; lane 0 then adds the
    // clients in order (values fetched from the other lanes) for the mean
    if (t < 64) {
        const uint32_t waves = nthreads >> 6;
        float tot = 0.0f;
        if (t < a.n) {
            tot = red[0][t];
            for (uint32_t w = 1; w < waves; ++w) tot += red[w][t];
            tot *= kXiScale;
            if (a.P) a.P[(uint64_t)t * a.m + j] = tot;
        }
        double mean = 0.0;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const float v = __shfl(tot, c);
            if ((uint32_t)c < a.n) mean += (double)v;
        }
        if (t == 0) a.pbar[j] = (float)(mean / (double)a.n);
    }
}

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

struct ReconArgs {
    const float* pbar;    // [m]
    float* gtilde;        // [d]
    uint64_t d;
    uint32_t m;
    float scale;
    uint32_t k0, k1, r0, r1;
    const uint32_t* round_dev;   // when non-null, the round counter (lo, hi) is read from here instead
    int vec_store;        // every output (and y, x_cur) is 16-byte aligned
    // fused optimiser step (UPDATE variant only)
    const float* y;       // [d] point the gradients were taken at
    float* x_new;         // [d] y - h * gtilde
    const float* x_cur;   // [d] current iterate, for the heavy-ball extrapolation (or null)
    float* y_next;        // [d] x_new + omb * (x_new - x_cur) (or null)
    float h;
    float omb;            // 1 - beta
    const float* h_dev;   // when non-null, the step is read from device memory instead of h
};

// Epilogue shared by the reconstruction kernels: the four sums of Philox block q become
// gtilde[4q..4q+3] = scale * sum (Eq. (reconstruction)) and, with UPDATE, feed the optimiser step
// instead of (or as well as) being written: x_new = y - h * gtilde (last line of the loop of
// Algorithm 2; with y = y^k it is the update of CORE-AGD), and optionally the next heavy-ball
// point y_next = x_new + (1 - beta)(x_new - x_cur) (first line of the loop of CORE-AGD).
template <bool UPDATE>
__device__ __forceinline__ void finish_block(const ReconArgs& a, uint64_t q, const float (&sum)[4])
{
    const uint64_t nblk = (a.d + 3) / 4;   // Philox blocks in the vector
    if (q >= nblk) return;
    const uint64_t i = 4 * q;
    const float sc = a.scale * kXiScale;
    float v[4] = {sc * sum[0], sc * sum[1], sc * sum[2], sc * sum[3]};
    const bool full = a.vec_store && i + 4 <= a.d;
    if (a.gtilde) {
        if (full) {
            *reinterpret_cast<float4*>(a.gtilde + i) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) if (i + k < a.d) a.gtilde[i + k] = v[k];
        }
    }
    if constexpr (UPDATE) {
        float yv[4] = {0.f, 0.f, 0.f, 0.f}, xc[4] = {0.f, 0.f, 0.f, 0.f};
        if (full) {
            const float4 t4 = *reinterpret_cast<const float4*>(a.y + i);
            yv[0] = t4.x; yv[1] = t4.y; yv[2] = t4.z; yv[3] = t4.w;
            if (a.y_next) {
                const float4 c4 = *reinterpret_cast<const float4*>(a.x_cur + i);
                xc[0] = c4.x; xc[1] = c4.y; xc[2] = c4.z; xc[3] = c4.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) if (i + k < a.d) {
                yv[k] = a.y[i + k];
                if (a.y_next) xc[k] = a.x_cur[i + k];
            }
        }
        const float h = a.h_dev ? *a.h_dev : a.h;
        float xn[4], yn[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            xn[k] = fmaf(-h, v[k], yv[k]);
            yn[k] = fmaf(a.omb, xn[k] - xc[k], xn[k]);
        }
        if (full) {
            *reinterpret_cast<float4*>(a.x_new + i) = make_float4(xn[0], xn[1], xn[2], xn[3]);
            if (a.y_next) *reinterpret_cast<float4*>(a.y_next + i) = make_float4(yn[0], yn[1], yn[2], yn[3]);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) if (i + k < a.d) {
                a.x_new[i + k] = xn[k];
                if (a.y_next) a.y_next[i + k] = yn[k];
            }
        }
    }
}

template <bool UPDATE, int kReconBlocks>
__global__ void __launch_bounds__(kThreads) reconstruct_kernel(ReconArgs a)
{
    __shared__ float pb[kPbarTile];
    const uint32_t t = threadIdx.x;
    const uint64_t qbase = (uint64_t)blockIdx.x * (kThreads * kReconBlocks) + t;

    // lanes differ in q (counter word 0) only: the state is fully divergent after 2-3 rounds
    Generator<2, 3> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float outer[kReconBlocks][4];
#pragma unroll
    for (int r = 0; r < kReconBlocks; ++r)
#pragma unroll
        for (int k = 0; k < 4; ++k) outer[r][k] = 0.0f;

    for (uint32_t j0 = 0; j0 < a.m; j0 += kPbarTile) {
        const uint32_t jn = (a.m - j0 < (uint32_t)kPbarTile) ? (a.m - j0) : (uint32_t)kPbarTile;
        __syncthreads();
        for (uint32_t x = t; x < jn; x += kThreads) pb[x] = a.pbar[j0 + x];
        __syncthreads();
        // inner sums of 64 vectors, then added to the running sum: keeps fp32 chains short
        for (uint32_t jb = 0; jb < jn; jb += 64) {
            const uint32_t je = (jn - jb < 64u) ? (jn - jb) : 64u;
            float acc[kReconBlocks][4];
#pragma unroll
            for (int r = 0; r < kReconBlocks; ++r)
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[r][k] = 0.0f;
            for (uint32_t jj = 0; jj < je; ++jj) {
                const float p = pb[jb + jj];
                const uint32_t j = j0 + jb + jj;
#pragma unroll
                for (int r = 0; r < kReconBlocks; ++r) {
                    const uint32_t q = (uint32_t)(qbase + (uint64_t)r * kThreads);
                    const Words w = gen.words(q, j);
                    float ra, ca, sa, rb, cb, sb;
                    gen.polar(w.x0, w.x1, ra, ca, sa);
                    gen.polar(w.x2, w.x3, rb, cb, sb);
                    const float pa = p * ra, pb2 = p * rb;   // pbar[j] folded into the radius
                    acc[r][0] = fmaf(pa, ca, acc[r][0]);
                    acc[r][1] = fmaf(pa, sa, acc[r][1]);
                    acc[r][2] = fmaf(pb2, cb, acc[r][2]);
                    acc[r][3] = fmaf(pb2, sb, acc[r][3]);
                }
            }
#pragma unroll
            for (int r = 0; r < kReconBlocks; ++r)
#pragma unroll
                for (int k = 0; k < 4; ++k) outer[r][k] += acc[r][k];
        }
    }

#pragma unroll
    for (int r = 0; r < kReconBlocks; ++r) finish_block<UPDATE>(a, qbase + (uint64_t)r * kThreads, outer[r]);
}

// Reconstruction for short vectors (too few Philox blocks to fill the chip with one thread per
// block).  A workgroup owns 64 consecutive Philox blocks and has JS = blockDim.x / 64 waves; wave w
// sums the vectors j = w, w + JS, w + 2 JS, ... for those blocks, the JS partial sums are added in
// wave order through LDS, and wave 0 finishes the block.  Every wave regenerates only its own share
// of the normals, so nothing is generated twice; the order of every sum is fixed by (d, m).
constexpr int kSplitMaxWaves = 16;

template <bool UPDATE>
__global__ void __launch_bounds__(64 * kSplitMaxWaves) reconstruct_split_kernel(ReconArgs a)
{
    __shared__ float pb[kPbarTile];
    extern __shared__ float red[];   // [JS][4][64], sized by the launch
    const uint32_t t = threadIdx.x;
    const uint32_t lane = t & 63u, w = t >> 6, JS = blockDim.x >> 6;
    const uint64_t q64 = (uint64_t)blockIdx.x * 64 + lane;
    const uint32_t q = (uint32_t)q64;

    Generator<2, 3> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float outer[4] = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t j0 = 0; j0 < a.m; j0 += kPbarTile) {
        const uint32_t jn = (a.m - j0 < (uint32_t)kPbarTile) ? (a.m - j0) : (uint32_t)kPbarTile;
        __syncthreads();
        for (uint32_t x = t; x < jn; x += blockDim.x) pb[x] = a.pbar[j0 + x];
        __syncthreads();
        float acc[4] = {0.f, 0.f, 0.f, 0.f};   // at most kPbarTile / JS <= 512 terms
        for (uint32_t jj = w; jj < jn; jj += JS) {
            const float p = pb[jj];
            const Words wd = gen.words(q, j0 + jj);
            float ra, ca, sa, rb, cb, sb;
            gen.polar(wd.x0, wd.x1, ra, ca, sa);
            gen.polar(wd.x2, wd.x3, rb, cb, sb);
            const float pa = p * ra, pb2 = p * rb;
            acc[0] = fmaf(pa, ca, acc[0]);
            acc[1] = fmaf(pa, sa, acc[1]);
            acc[2] = fmaf(pb2, cb, acc[2]);
            acc[3] = fmaf(pb2, sb, acc[3]);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) outer[k] += acc[k];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) red[(w * 4 + k) * 64 + lane] = outer[k];
    __syncthreads();
    if (w != 0) return;
    float sum[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float s = red[k * 64 + lane];
        for (uint32_t ww = 1; ww < JS; ++ww) s += red[(ww * 4 + k) * 64 + lane];
        sum[k] = s;
    }
    finish_block<UPDATE>(a, q64, sum);
}

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

// Reconstruction for several machines at once (decentralized CORE-GD with the machines batched on one
// device: after gossip every machine holds its own averaged vector p_v and reconstructs from it with
// the same xi_j).  The normals are generated once per (coordinate block, j) and feed NB accumulators,
// the mirror image of the projection: X[v][i] -= h * scale * sum_j P[v][j] xi_j[i], or the sums
// themselves into Gt.  Lanes over q, j the wave-uniform loop; P is staged in LDS as [j][NB] so that a
// lane reads the NB factors of one j with NB/4 broadcast reads.
struct ReconBatchArgs {
    const float* P;       // [nb][ldp]
    uint64_t ldp;
    float* X;             // [nb][ldx] updated in place, or null
    float* Gt;            // [nb][ldx] scale * sum, or null
    uint64_t ldx;
    uint64_t d;
    uint32_t m;
    uint32_t v0, nv;      // first machine of this pass, machines in this pass (<= NB)
    float scale, h;
    uint32_t k0, k1, r0, r1;
};

constexpr int kBatchPTile = 256;   // vectors j staged per step

template <int NB>
__global__ void __launch_bounds__(kThreads) reconstruct_batched_kernel(ReconBatchArgs a)
{
    __shared__ __attribute__((aligned(16))) float pb[kBatchPTile][NB];
    const uint32_t t = threadIdx.x;
    const uint64_t nblk = (a.d + 3) / 4;
    const uint64_t q64 = (uint64_t)blockIdx.x * kThreads + t;
    const uint32_t q = (uint32_t)q64;

    Generator<2, 3> gen;
    gen.init(a.k0, a.k1, a.r0, a.r1);

    float outer[NB][4];
#pragma unroll
    for (int v = 0; v < NB; ++v)
#pragma unroll
        for (int k = 0; k < 4; ++k) outer[v][k] = 0.0f;

    for (uint32_t j0 = 0; j0 < a.m; j0 += kBatchPTile) {
        const uint32_t jn = (a.m - j0 < (uint32_t)kBatchPTile) ? (a.m - j0) : (uint32_t)kBatchPTile;
        __syncthreads();
        for (uint32_t x = t; x < jn * NB; x += kThreads) {
            const uint32_t jj = x / NB, v = x % NB;
            pb[jj][v] = (v < a.nv) ? a.P[(uint64_t)(a.v0 + v) * a.ldp + j0 + jj] : 0.0f;
        }
        __syncthreads();
        // inner sums of 64 vectors, then added to the running sum: keeps fp32 chains short
        for (uint32_t jb = 0; jb < jn; jb += 64) {
            const uint32_t je = (jn - jb < 64u) ? (jn - jb) : 64u;
            float acc[NB][4];
#pragma unroll
            for (int v = 0; v < NB; ++v)
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[v][k] = 0.0f;
            for (uint32_t jj = 0; jj < je; ++jj) {
                float z0, z1, z2, z3;
                gen.block(q, j0 + jb + jj, z0, z1, z2, z3);
#pragma unroll
                for (int v = 0; v < NB; ++v) {
                    const float p = pb[jb + jj][v];
                    acc[v][0] = fmaf(p, z0, acc[v][0]);
                    acc[v][1] = fmaf(p, z1, acc[v][1]);
                    acc[v][2] = fmaf(p, z2, acc[v][2]);
                    acc[v][3] = fmaf(p, z3, acc[v][3]);
                }
            }
#pragma unroll
            for (int v = 0; v < NB; ++v)
#pragma unroll
                for (int k = 0; k < 4; ++k) outer[v][k] += acc[v][k];
        }
    }

    if (q64 >= nblk) return;
    const uint64_t i = 4 * q64;
    const float sc = a.scale * kXiScale;
#pragma unroll
    for (int v = 0; v < NB; ++v) {
        if ((uint32_t)v >= a.nv) break;
        const uint64_t row = (uint64_t)(a.v0 + v) * a.ldx;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i + k < a.d) {
                const float g = sc * outer[v][k];
                if (a.Gt) a.Gt[row + i + k] = g;
                if (a.X) a.X[row + i + k] = fmaf(-a.h, g, a.X[row + i + k]);
            }
        }
    }
}

// Device-resident round counter for replayed launch sequences (HIP graphs): one thread adds 1.
__global__ void advance_round_kernel(uint64_t* round_dev)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *round_dev += 1;
}

// Materialised-Xi comparison variant of the reconstruction: gtilde[4q+k] = scale * sum_j pbar[j] *
// xi[q][j][k] with the normals read back from memory (Xi = [xi_1 ... xi_m]^T of the privacy
// appendix, stored in 4-coordinate blocks).  One wave per Philox block q, lanes over j
// (coalesced 1 KB reads), then a wave butterfly; HBM-bound by construction (16 bytes per 4 pairs).
struct ReconXiArgs {
    const float* pbar;
    const float* xi;      // [ceil(d/4)][m][4]
    float* gtilde;
    uint64_t d;
    uint32_t m;
    float scale;
};

__global__ void __launch_bounds__(kThreads) reconstruct_xi_kernel(ReconXiArgs a)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t q = (uint64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    const uint64_t nblk = (a.d + 3) / 4;
    if (q >= nblk) return;   // whole wave leaves together
    const float4* row = reinterpret_cast<const float4*>(a.xi) + q * a.m;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    for (uint32_t j = lane; j < a.m; j += 64) {
        const float4 v = row[j];
        const float p = a.pbar[j];
        s0 = fmaf(p, v.x, s0); s1 = fmaf(p, v.y, s1); s2 = fmaf(p, v.z, s2); s3 = fmaf(p, v.w, s3);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        s0 += __shfl_xor(s0, off); s1 += __shfl_xor(s1, off);
        s2 += __shfl_xor(s2, off); s3 += __shfl_xor(s3, off);
    }
    if (lane == 0) {
        const uint64_t i = 4 * q;
        if (i + 0 < a.d) a.gtilde[i + 0] = a.scale * s0;
        if (i + 1 < a.d) a.gtilde[i + 1] = a.scale * s1;
        if (i + 2 < a.d) a.gtilde[i + 2] = a.scale * s2;
        if (i + 3 < a.d) a.gtilde[i + 3] = a.scale * s3;
    }
}

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
