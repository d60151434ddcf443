// Projection kernels for vector counts that do not fill tiles of 256, for few vectors, and for tiny
// problems: tiles of 64 vectors, tiles of 8 / 16 / 32 vectors, lanes over coordinates, and the
// one-launch kernel that also finishes the sums.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_common.hpp"
#include "core_rng.hpp"
#include "core_project.hpp"

namespace core {

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

// The same for 2 consecutive coordinates (one 32- or 64-bit load).
template <bool BF16> struct RawG2;

template <> struct RawG2<false> {
    float v[2];
    __device__ __forceinline__ void load(const void* G, uint64_t base, uint64_t i, uint64_t d, bool vec)
    {
        if (vec && i + 2 <= d) {
            const float2 x = *reinterpret_cast<const float2*>((const float*)G + base);
            v[0] = x.x; v[1] = x.y;
        } else {
#pragma unroll
            for (int k = 0; k < 2; ++k) v[k] = (i + k < d) ? ((const float*)G)[base + k] : 0.0f;
        }
    }
    __device__ __forceinline__ void zero() { v[0] = v[1] = 0.0f; }
    __device__ __forceinline__ void widen(float (&g)[2]) const { g[0] = v[0]; g[1] = v[1]; }
};

template <> struct RawG2<true> {
    uint32_t lo;   // a bf16 pair
    __device__ __forceinline__ void load(const void* G, uint64_t base, uint64_t i, uint64_t d, bool vec)
    {
        const uint16_t* p = (const uint16_t*)G + base;
        if (vec && i + 2 <= d) {
            lo = *reinterpret_cast<const uint32_t*>(p);
        } else {
            const uint32_t e0 = (i < d) ? (uint32_t)p[0] : 0u, e1 = (i + 1 < d) ? (uint32_t)p[1] : 0u;
            lo = e0 | (e1 << 16);
        }
    }
    __device__ __forceinline__ void zero() { lo = 0u; }
    __device__ __forceinline__ void widen(float (&g)[2]) const
    {
        g[0] = __uint_as_float(lo << 16); g[1] = __uint_as_float(lo & 0xffff0000u);
    }
};

// The lanes-over-vectors projection for tiles of JW = 8, 16 or 32 vectors: what is left of m mod 256
// after its whole waves, and few vectors on a long gradient.  As in project_narrow_kernel the four
// waves of a block take the same JW vectors and share the chunk's coordinates, wave w taking the
// 128-coordinate trips w, w + 4, ... of the chunk and staging each in its own part of LDS; but the
// lanes of a wave split further: lane l works on vector a.j_begin + JW jt + (l mod JW) and, of the 32
// Philox blocks of a trip, on those congruent to l / JW modulo 64 / JW, so every lane is busy whatever
// the vector count.  The 64 / JW partial sums of a vector are added across the lanes once per chunk
// (butterfly over the upper lane bits), then the four waves' sums in wave order, and the block writes
// one partial sum per (vector, client) like a block of project_kernel.  a.jtiles counts tiles of JW
// vectors.  With so few generator calls per coordinate the loads of G must be wide and early: a lane
// fetches 2 consecutive coordinates per client with one 32- or 64-bit load where the rows allow it,
// a whole trip ahead, and keeps them in their stored form until the trip is used (with 64-coordinate
// steps and element loads the kernel took 0.37 ms at the ResNet-50 size whatever JW was, waiting for
// memory).  Trips of 128 rather than 256 coordinates keep a block at 16 KB of LDS for 8 clients, so
// that registers and not LDS bound the waves per SIMD: 3 to 10 % faster.  No block barrier in the
// loop: a wave's part of LDS is written and read by that wave alone, and the LDS operations of one
// wave are performed in program order.
constexpr int kSubTrip = 128;   // coordinates a wave stages at a time (32 Philox blocks)

template <int NC, bool BF16, int JW>
__global__ void __launch_bounds__(kThreads) project_sub_kernel(ProjectArgs a)
{
    static_assert(JW == 32 || JW == 16 || JW == 8, "vectors per tile");
    static_assert(NC <= 8, "LDS: four waves x NC x 128 floats");
    constexpr int TRIP = kSubTrip;
    constexpr int QW = 64 / JW;             // lane groups of a wave, each with its own Philox blocks
    constexpr int kCalls = (TRIP / 4) / QW;   // generator calls per lane per trip
    __shared__ __attribute__((aligned(16))) float tile[kThreads / 64][NC][TRIP];
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

    // trips of TRIP coordinates; a.tiles_per_chunk counts tiles of 256
    const uint64_t tiles_total = (a.d + TRIP - 1) / TRIP;
    const uint64_t tile_begin = (uint64_t)chunk * a.tiles_per_chunk * (kTile / TRIP);
    uint64_t tile_end = tile_begin + (uint64_t)a.tiles_per_chunk * (kTile / TRIP);
    if (tile_end > tiles_total) tile_end = tiles_total;

    // lanes differ in q and in j: every round after the first is fully divergent
    Generator<1, 1> gen;
    gen.init(a.k0, a.k1, a.round_dev ? a.round_dev[0] : a.r0, a.round_dev ? a.round_dev[1] : a.r1);

    float acc_outer[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc_outer[c] = 0.0f;

    // register prefetch of this wave's next trip: lane l holds coordinates 128 trip + 2 l, + 1 of every client
    RawG2<BF16> pre[NC];
    const bool vec = a.vec_load != 0;
    auto fetch = [&](uint64_t tl) {
        const uint64_t i = tl * TRIP + 2 * lane;
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
            float g[2];
            pre[c].widen(g);
            *reinterpret_cast<float2*>(&tile[w][c][2 * lane]) = make_float2(g[0], g[1]);
        }
        __builtin_amdgcn_wave_barrier();
        fetch(tl + 4);

        float acc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] = 0.0f;
        const uint32_t q0 = (uint32_t)(tl * (TRIP / 4));
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

}  // namespace core
