// Projection (Algorithm 1 compression line / Algorithm 2 "machine i sends p_ij") with lanes over the
// vector index j, for whole tiles of 256 vectors: the VALU kernel and the two matrix-pipe kernels.
// These are the kernels the headline workloads run.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_common.hpp"
#include "core_rng.hpp"

namespace core {

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

}  // namespace core
