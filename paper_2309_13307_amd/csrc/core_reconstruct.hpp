// Reconstruction (Eq. (reconstruction)) with the normals regenerated in registers, its fused
// optimiser step, the form for short vectors, the form for several machines at once, and the
// comparison variant that reads a materialised Xi.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "core_common.hpp"
#include "core_rng.hpp"

namespace core {

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

}  // namespace core
