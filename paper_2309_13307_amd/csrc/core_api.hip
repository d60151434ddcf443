// Host side of the C ABI declared in include/core.h: argument validation, launch planning
// and kernel launches.  Nothing here touches device memory from the host or synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <atomic>
#include <cmath>
#include <mutex>

#include "../../include/core.h"
#include "core_kernels.hpp"

namespace {

using namespace core;

thread_local int g_last_hip_error = 0;

// Identifies the sources this binary was built from (set by the build step; the marker prefix lets
// a loader find the id in the file without loading it).
#ifndef CORE_BUILD_ID
#define CORE_BUILD_ID "unknown"
#endif
const char kBuildId[] = "CORE_BUILD_ID=" CORE_BUILD_ID;

constexpr uint64_t kMaxD = 1ull << 34;
// The kernels walk the vectors with 32-bit counters in steps of up to 1024; the cap keeps
// `j0 += step` from wrapping before `j0 < m` turns false.
constexpr uint32_t kMaxM = 0xFFFFFFFFu - 1023u;   // 2^32 - 1024
constexpr uint32_t kMaxN = 65535u;
constexpr uint32_t kMaxClientsPerPass = 16;       // VALU projection: accumulators held in registers per lane
constexpr uint32_t kMaxClientsPerPassMfma = 32;   // matrix-pipe projection (8 groups of 4 clients)
constexpr uint32_t kMaxClientsPerPassWide = 64;   // wide matrix-pipe projection (16 groups), one level of sums
// The wide kernel adds every term of a chunk into one fp32 sum per (vector, client): chunks are kept
// to 16 tiles = 4096 coordinates for calls that use it (rounding error of such a chain ~1e-6 of the
// chunk's norm; the two-level kernels allow 1024 tiles).
constexpr uint32_t kTilesPerChunkWide = 16;
constexpr uint32_t kTargetBlocks = 8192;      // projection blocks wanted: 4 per resident slot

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr uint32_t kBlockSlots = 2048;   // resident 256-thread blocks: 256 CUs x 8
constexpr uint64_t kWaveSlots = 8192;    // resident waves at 8 per SIMD: 256 CUs x 4 SIMDs x 8

// How the projection is laid out on the chip.
enum PlanMode : int {
    kPlanVectors = 0,   // lanes over the vectors j, blocks of 256 vectors x a chunk of 256-coordinate tiles
    kPlanCoords = 1,    // lanes over the coordinates, blocks of 4 or 8 vectors x a chunk of 1024-coordinate tiles
    kPlanSmall = 2      // one workgroup per vector over the whole of d, sums finished inside it (one launch)
};

struct Plan {
    int mode;
    uint32_t jtiles;       // tiles of 256 vectors given to the lanes-over-vectors kernels (0 in kPlanCoords;
                           // m in kPlanSmall)
    uint32_t narrow_tiles; // tiles of 64 vectors after those, given to project_narrow_kernel (whole waves of
                           // vectors that would not fill a block of 256)
    uint32_t sub_tiles;    // tiles of sub_jw vectors after those, same kernel with the lanes of a wave split
    uint32_t sub_jw;       // between vectors and Philox blocks (8, 16 or 32; 0 when there are none)
    uint32_t tail_groups;  // kPlanCoords: groups of qj vectors of the lanes-over-coordinates kernel; else 0
    uint32_t qj;           // vectors per block of that kernel (4 or 8)
    uint32_t nchunks;
    uint32_t tiles_per_chunk;   // in 256-coordinate tiles; a multiple of 4 in kPlanCoords, whose kernel walks
                                // 1024-coordinate tiles
    uint32_t Z;            // slices of the cross-chunk sum
    uint32_t small_threads;   // kPlanSmall: threads per workgroup
    bool wide;             // more than 32 clients: passes of up to 64 on the matrix pipe
    size_t part_off, psum_off, total;
};

// How the vectors that do not fill a tile of 256 are served (m mod 256 = rest).  A wave of the
// lanes-over-vectors kernels is latency-bound on its own and only about 8 busy waves per SIMD saturate
// the issue port, so a block of 256 with idle waves wastes wave slots: measured on a ResNet-50-sized
// gradient (8 clients, projection alone), 64 vectors as a quarter-filled block 1.71 ms, 320 vectors as
// one full and one quarter-filled tile 6.34 ms against 3.35 ms for 256.  So: a rest above 192 fills all
// four waves of one more block of 256; otherwise its whole waves go to blocks of 64 vectors whose four
// waves share the chunk's coordinates (project_narrow_kernel), and what is left after those to blocks
// of 8, 16 or 32 vectors of the same kernel (lanes split between vectors and Philox blocks), in the
// size that pads the count least (the larger one on a tie); more than 48 left-over vectors take a full
// block of 64 instead.  Measured there with 8 clients, projection + sums: 8 / 16 / 32 / 48 vectors
// 0.17 / 0.28 / 0.52 / 0.75 ms, and at 2^23 coordinates 0.070 / 0.10 / 0.17 / 0.25 ms (the
// lanes-over-coordinates kernel: 0.18 / 0.30 / 0.58 / 0.83 and 0.12 / 0.14 / 0.21 / 0.31 ms).
constexpr uint32_t kRestFullTile = 192;
constexpr uint32_t kSubTilesMaxVectors = 48;
// Fewer vectors than this on a gradient that is not tiny: the lanes-over-coordinates kernel.
constexpr uint32_t kVectorsPlanMin = 5;

constexpr uint64_t kSmallMaxD = 65536;      // kPlanSmall: a thread's fp32 chain stays <= 256 terms
constexpr uint32_t kSmallMaxClients = 8;

constexpr uint32_t kQTilesPerChunkMax = 64;   // bounds the fp32 chains of the lanes-over-q kernel
// A block adds one fp32 tile sum (256 terms) per tile to its fp32 chunk sum; the chunk sums are then
// combined in fp64.  Capping the tiles per chunk keeps that fp32 chain at the length the accuracy
// bar was verified for (GPT-2-sized d: 950), whatever d is.
constexpr uint32_t kTilesPerChunkMax = 1024;
constexpr uint64_t kMaxGridBlocks = 0x7fffffffull;   // HIP's limit on gridDim.x

// Which projection kernel to use: the library's own choice, or one forced for A/B runs and for
// the tests that drive every kernel over every shape.  Set with core_debug_set_projection (a
// test-only export); the environment variable CORE_PROJECT_VARIANT=valu|mfma|q gives the initial
// value and is read once per process.
enum Variant : int { kVariantAuto = 0, kVariantValu = 1, kVariantMfma = 2, kVariantQ = 3, kVariantSmall = 4 };

int variant_from_env()
{
    const char* v = getenv("CORE_PROJECT_VARIANT");
    if (!v) return kVariantAuto;
    if (strcmp(v, "valu") == 0) return kVariantValu;
    if (strcmp(v, "mfma") == 0) return kVariantMfma;
    if (strcmp(v, "q") == 0) return kVariantQ;
    if (strcmp(v, "small") == 0) return kVariantSmall;
    return kVariantAuto;
}

std::atomic<int>& variant_cell()
{
    static std::atomic<int> cell{variant_from_env()};
    return cell;
}

inline int forced_variant() { return variant_cell().load(std::memory_order_relaxed); }

// Split d into chunks of whole tiles so that (chunks x vector tiles) is about 8192 equal blocks:
// four per resident block slot (256 CUs x 8 blocks of 4 waves), which evens out speed differences
// between CUs.  With fewer than 64 vectors, or too little work to fill the chip that way, a
// lanes-over-coordinates plan is made instead (in one launch, sums included, when the problem is tiny).
// The plan depends only on (d, m, n) and on the forced kernel, if any.
bool make_plan(uint64_t d, uint32_t m, uint32_t n, bool allow_qmode, int forced, Plan& p)
{
    if (d == 0 || d > kMaxD || m == 0 || m > kMaxM || n == 0 || n > kMaxN) return false;
    const uint64_t tiles_total = ceil_div(d, kTile);
    const bool small_ok = allow_qmode && n <= kSmallMaxClients && d <= kSmallMaxD && m <= 0x7fffffffu;
    const bool little_work = ceil_div(m, 64) * tiles_total <= 1024;   // fewer than 1024 wave-tiles in all
    const bool force_vectors = forced == kVariantValu || forced == kVariantMfma || !allow_qmode;
    const uint32_t full_tiles = m / kThreads, rem = m % kThreads;
    p.small_threads = 0;
    p.qj = 0;
    p.wide = false;
    p.tail_groups = 0;
    p.narrow_tiles = 0;
    p.sub_tiles = 0;
    p.sub_jw = 0;
    if (!force_vectors && small_ok && (forced == kVariantSmall || (forced == kVariantAuto && little_work))) {
        // one Philox block per thread where d allows it: the serial chain of a thread is what a
        // launch-bound round waits for
        p.mode = kPlanSmall;
        uint64_t threads = ceil_div(ceil_div(d, 4), 64) * 64;
        if (threads > 1024) threads = 1024;
        p.small_threads = (uint32_t)threads;
        p.jtiles = m;
        p.nchunks = 1;
        p.tiles_per_chunk = (uint32_t)ceil_div(ceil_div(d, 4), threads);
    } else {
        // which vectors go to which kernel
        bool coords_all = false;
        uint32_t main_tiles = (uint32_t)ceil_div(m, kThreads), narrow = 0, sub_tiles = 0, sub_jw = 0;
        if (!force_vectors) {
            if (forced == kVariantQ || forced == kVariantSmall) coords_all = true;
            else coords_all = little_work || m < kVectorsPlanMin;
            if (!coords_all && rem > 0 && rem <= kRestFullTile) {
                main_tiles = full_tiles;
                narrow = rem / 64;
                const uint32_t left = rem % 64;
                if (left > 0) {
                    // more than 48 vectors: a full tile of 64 is faster than 7 or 8 small ones
                    uint32_t best_jw = 64, best_pad = 64;
                    for (uint32_t jw = 32; jw >= 8 && left <= kSubTilesMaxVectors; jw /= 2) {
                        const uint32_t padded = (uint32_t)ceil_div(left, jw) * jw;
                        if (padded < best_pad) { best_pad = padded; best_jw = jw; }
                    }
                    if (best_jw == 64) narrow += 1;
                    else { sub_jw = best_jw; sub_tiles = best_pad / best_jw; }
                }
            }
        }
        const uint64_t qtiles = ceil_div(d, (uint64_t)kThreads * 4);
        p.narrow_tiles = narrow;
        p.sub_tiles = sub_tiles;
        p.sub_jw = sub_jw;
        if (coords_all) {
            p.mode = kPlanCoords;
            p.jtiles = 0;
            // 8 vectors per block share every load of G when there is enough work to fill the chip
            // with such blocks; 4 otherwise (more, shorter blocks)
            p.qj = (m > 4 && ceil_div(m, 8) * qtiles >= 2 * kBlockSlots) ? 8 : 4;
            p.tail_groups = (uint32_t)ceil_div(m, p.qj);
            uint64_t want = ceil_div(kTargetBlocks / 2, p.tail_groups);
            if (want < 1) want = 1;
            if (want > qtiles) want = qtiles;
            uint64_t tpcq = ceil_div(qtiles, want);
            if (tpcq > kQTilesPerChunkMax) tpcq = kQTilesPerChunkMax;
            p.tiles_per_chunk = (uint32_t)(4 * tpcq);
            p.nchunks = (uint32_t)ceil_div(qtiles, tpcq);
        } else {
            p.mode = kPlanVectors;
            p.jtiles = main_tiles;
            // chunk length for about 8192 blocks in the launch of the 256-vector tiles, or in a
            // launch of smaller tiles when there is no other
            // (the one with the fewest tiles: the others then launch more blocks, which does no harm)
            const uint32_t side = narrow > sub_tiles ? narrow : sub_tiles;
            const uint32_t fewest = (narrow && sub_tiles) ? (narrow < sub_tiles ? narrow : sub_tiles) : side;
            uint64_t want = ceil_div(kTargetBlocks, main_tiles ? main_tiles : (fewest ? fewest : 1u));
            if (want < 1) want = 1;
            if (want > tiles_total) want = tiles_total;
            uint64_t tpc = ceil_div(tiles_total, want);
            if (tpc > kTilesPerChunkMax) tpc = kTilesPerChunkMax;
            // more than 32 clients: wide passes for the 256-vector tiles, with chunks of at most 16 tiles,
            // if those shorter chunks still give a launchable grid
            if (main_tiles > 0 && n > kMaxClientsPerPassMfma && forced != kVariantValu) {
                const uint64_t tpc_wide = tpc < kTilesPerChunkWide ? tpc : kTilesPerChunkWide;
                const uint64_t chunks_wide = ceil_div(tiles_total, tpc_wide);
                if (ceil_div(chunks_wide, 8) * 8 * main_tiles <= kMaxGridBlocks) {
                    p.wide = true;
                    tpc = tpc_wide;
                }
            }
            // a wave of the smaller tiles adds one fp32 sum per step of 64 coordinates into its chunk sum
            // and takes every fourth step, i.e. one sum per 256-coordinate tile: chunks of at most 256
            // tiles there, the chain length those kernels were checked with
            if (side > 0 && tpc > kTilesPerChunkMax / 4) tpc = kTilesPerChunkMax / 4;
            // the waves of a block of 8, 16 or 32 vectors take whole tiles in turn: chunks of a multiple
            // of 4 tiles keep them level
            if (sub_tiles > 0) tpc = ceil_div(tpc, 4) * 4;
            p.tiles_per_chunk = (uint32_t)tpc;
            p.nchunks = (uint32_t)ceil_div(tiles_total, tpc);
        }
    }
    // one block per (chunk, vector tile or group): both grids must stay valid launches
    const uint64_t chunk_slots = ceil_div(p.nchunks, 8) * 8;
    uint64_t widest = p.jtiles > p.tail_groups ? p.jtiles : p.tail_groups;
    if (p.narrow_tiles > widest) widest = p.narrow_tiles;
    if (p.sub_tiles > widest) widest = p.sub_tiles;
    const uint64_t grid = p.mode == kPlanSmall ? (uint64_t)p.jtiles : chunk_slots * widest;
    if (grid > kMaxGridBlocks) return false;
    uint32_t Z = p.nchunks / 128u;
    if (Z < 1) Z = 1;
    if (Z > 16) Z = 16;
    p.Z = Z;
    const uint64_t E = (uint64_t)n * m;
    size_t off = 0;
    p.part_off = p.psum_off = 0;
    if (p.mode != kPlanSmall) {   // the one-launch plan keeps every partial sum inside its workgroups
        p.part_off = off;  off = align_up(off + (size_t)p.nchunks * E * sizeof(float), 256);
        p.psum_off = off;  off = align_up(off + (size_t)Z * E * sizeof(double), 256);
    }
    p.total = off;
    return true;
}

bool make_plan(uint64_t d, uint32_t m, uint32_t n, bool allow_qmode, Plan& p)
{
    return make_plan(d, m, n, allow_qmode, forced_variant(), p);
}

// Workspace that serves every entry point for these sizes whichever projection kernel is chosen
// or forced: a buffer sized once stays valid when the kernel choice is switched afterwards.
// 0 if the sizes are out of range.
size_t workspace_bytes(uint64_t d, uint32_t m, uint32_t n)
{
    const int current = forced_variant();
    size_t need = 0;
    for (int forced = kVariantAuto; forced <= kVariantSmall; ++forced)
        for (int allow = 0; allow < 2; ++allow) {
            Plan p;
            if (!make_plan(d, m, n, allow != 0, forced, p)) {
                if (forced == current) return 0;   // the plan a call would use now must exist
                continue;                          // a forced kernel may not cover extreme sizes
            }
            if (p.total > need) need = p.total;
        }
    return need;
}

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return CORE_ERR_HIP;
}

// Whether the process has a usable GPU: asked of the runtime once, then remembered.
int check_device()
{
    static const int rc = [] {
        int count = 0;
        if (hipGetDeviceCount(&count) != hipSuccess || count <= 0) {
            (void)hipGetLastError();
            return (int)CORE_ERR_NO_DEVICE;
        }
        return (int)CORE_OK;
    }();
    return rc;
}

// One kernel launch whose status is the return value of the launch call itself, so an error
// left behind by some earlier HIP call on this thread is never mistaken for a failure here.
template <typename T> struct same_type { using type = T; };

template <typename... Params>
hipError_t launch_lds(void (*kernel)(Params...), dim3 grid, dim3 block, size_t dynamic_lds, hipStream_t st,
                      typename same_type<Params>::type... args)
{
    void* ptrs[] = {(void*)&args...};
    return hipLaunchKernel((const void*)kernel, grid, block, ptrs, dynamic_lds, st);
}

template <typename... Params>
hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t st,
                  typename same_type<Params>::type... args)
{
    return launch_lds(kernel, grid, block, 0, st, args...);
}

bool aligned_to(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

template <int NC>
hipError_t launch_project_narrow(const ProjectArgs& a, bool bf16, uint32_t blocks, hipStream_t st)
{
    const dim3 g(blocks), b(kThreads);
    return bf16 ? launch(project_narrow_kernel<NC, true>, g, b, st, a)
                : launch(project_narrow_kernel<NC, false>, g, b, st, a);
}

template <int NC, int JW>
hipError_t launch_project_sub_jw(const ProjectArgs& a, bool bf16, uint32_t blocks, hipStream_t st)
{
    const dim3 g(blocks), b(kThreads);
    return bf16 ? launch(project_sub_kernel<NC, true, JW>, g, b, st, a)
                : launch(project_sub_kernel<NC, false, JW>, g, b, st, a);
}

template <int NC>
hipError_t launch_project_sub(const ProjectArgs& a, bool bf16, uint32_t jw, uint32_t blocks, hipStream_t st)
{
    switch (jw) {
        case 8:  return launch_project_sub_jw<NC, 8>(a, bf16, blocks, st);
        case 16: return launch_project_sub_jw<NC, 16>(a, bf16, blocks, st);
        default: return launch_project_sub_jw<NC, 32>(a, bf16, blocks, st);
    }
}

template <int NC>
hipError_t launch_project(const ProjectArgs& a, bool bf16, bool store_xi, uint32_t blocks, hipStream_t st)
{
    const dim3 g(blocks), b(kThreads);
    if (store_xi) return bf16 ? launch(project_kernel<NC, true, true>, g, b, st, a)
                              : launch(project_kernel<NC, false, true>, g, b, st, a);
    return bf16 ? launch(project_kernel<NC, true, false>, g, b, st, a)
                : launch(project_kernel<NC, false, false>, g, b, st, a);
}

template <int NG>
hipError_t launch_project_mfma(const ProjectArgs& a, bool bf16, uint32_t blocks, hipStream_t st)
{
    const dim3 g(blocks), b(kThreads);
    return bf16 ? launch(project_mfma_kernel<NG, true>, g, b, st, a)
                : launch(project_mfma_kernel<NG, false>, g, b, st, a);
}

template <int NG>
hipError_t launch_project_mfma_wide(const ProjectArgs& a, bool bf16, uint32_t blocks, hipStream_t st)
{
    const dim3 g(blocks), b(kThreads);
    return bf16 ? launch(project_mfma_wide_kernel<NG, true>, g, b, st, a)
                : launch(project_mfma_wide_kernel<NG, false>, g, b, st, a);
}

template <int NC>
hipError_t launch_project_q(const ProjectArgs& a, bool bf16, uint32_t qj, uint32_t blocks, hipStream_t st)
{
    const dim3 g(blocks), b(kThreads);
    if (qj == 8) return bf16 ? launch(project_q_kernel<NC, true, 8>, g, b, st, a)
                             : launch(project_q_kernel<NC, false, 8>, g, b, st, a);
    return bf16 ? launch(project_q_kernel<NC, true, 4>, g, b, st, a)
                : launch(project_q_kernel<NC, false, 4>, g, b, st, a);
}

// Which projection kernel serves a pass of nc clients.  Measured on MI355X (ResNet-50-sized
// gradient, m = 1024, every n from 9 to 16): the matrix-pipe kernel is 18-22 % faster than the VALU
// kernel (which pads 9..15 clients to 16), and 1 % slower at 8, so it is the default above 8 clients.
bool use_mfma_projection(uint32_t nc)
{
    const int forced = forced_variant();
    if (forced == kVariantMfma) return true;
    if (forced == kVariantValu) return false;
    return nc > 8;
}

int validate_compress(uint64_t d, uint32_t m, uint32_t n, const void* G, core_dtype dt, uint64_t ld,
                      const float* P, const float* pbar, const void* ws, size_t ws_bytes, Plan& plan,
                      bool allow_qmode = true)
{
    if (!G || !pbar || !ws) return CORE_ERR_INVALID_ARGUMENT;
    if (dt != CORE_DTYPE_F32 && dt != CORE_DTYPE_BF16) return CORE_ERR_INVALID_ARGUMENT;
    if (ld < d) return CORE_ERR_INVALID_ARGUMENT;
    if (!make_plan(d, m, n, allow_qmode, plan)) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(G, dt == CORE_DTYPE_F32 ? 4 : 2)) return CORE_ERR_MISALIGNED;
    if (!aligned_to(pbar, 4) || (P && !aligned_to(P, 4)) || !aligned_to(ws, 16)) return CORE_ERR_MISALIGNED;
    if (ws_bytes < workspace_bytes(d, m, n)) return CORE_ERR_WORKSPACE_TOO_SMALL;
    return CORE_OK;
}

int validate_reconstruct(uint64_t d, uint32_t m, const float* pbar, const float* gtilde)
{
    if (!pbar || !gtilde) return CORE_ERR_INVALID_ARGUMENT;
    if (d == 0 || d > kMaxD || m == 0 || m > kMaxM) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(pbar, 4) || !aligned_to(gtilde, 4)) return CORE_ERR_MISALIGNED;
    return CORE_OK;
}

// Tiles of jw vectors starting at vector j_begin: jw = 64 in passes of at most 16 clients
// (project_narrow_kernel), jw = 8, 16 or 32 in passes of at most 8 (project_sub_kernel).
int enqueue_narrow(const ProjectArgs& a, bool bf16, uint32_t n, uint32_t jw, uint32_t tiles, uint32_t j_begin,
                   uint32_t chunk_slots, hipStream_t st)
{
    ProjectArgs w = a;
    w.jtiles = tiles;
    w.j_begin = j_begin;
    const uint32_t blocks = chunk_slots * tiles;
    const uint32_t cap = jw == 64 ? kMaxClientsPerPass : 8u;
    for (uint32_t c0 = 0; c0 < n; c0 += cap) {
        const uint32_t nc = (n - c0 < cap) ? (n - c0) : cap;
        w.c0 = c0; w.nc = nc;
        hipError_t e;
        if (jw == 64) {
            if (nc <= 1)      e = launch_project_narrow<1>(w, bf16, blocks, st);
            else if (nc <= 2) e = launch_project_narrow<2>(w, bf16, blocks, st);
            else if (nc <= 4) e = launch_project_narrow<4>(w, bf16, blocks, st);
            else if (nc <= 8) e = launch_project_narrow<8>(w, bf16, blocks, st);
            else              e = launch_project_narrow<16>(w, bf16, blocks, st);
        } else {
            if (nc <= 1)      e = launch_project_sub<1>(w, bf16, jw, blocks, st);
            else if (nc <= 2) e = launch_project_sub<2>(w, bf16, jw, blocks, st);
            else if (nc <= 4) e = launch_project_sub<4>(w, bf16, jw, blocks, st);
            else              e = launch_project_sub<8>(w, bf16, jw, blocks, st);
        }
        if (e != hipSuccess) return hip_fail(e);
    }
    return CORE_OK;
}

int enqueue_compress(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                     const void* G, core_dtype dt, uint64_t ld, float* P, float* pbar,
                     void* ws, const Plan& plan, hipStream_t st, float* xi_store = nullptr,
                     const uint64_t* round_dev = nullptr)
{
    char* base = (char*)ws;
    float* part = (float*)(base + plan.part_off);
    double* psum = (double*)(base + plan.psum_off);

    ProjectArgs a;
    a.G = G; a.ld = ld; a.d = d; a.m = m; a.n = n;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32);
    a.r0 = (uint32_t)round; a.r1 = (uint32_t)(round >> 32);
    a.round_dev = reinterpret_cast<const uint32_t*>(round_dev);   // little-endian: lo word first
    a.jtiles = plan.jtiles; a.nchunks = plan.nchunks; a.tiles_per_chunk = plan.tiles_per_chunk;
    a.j_begin = 0;
    a.part = part;
    a.xi_store = xi_store;
    const bool bf16 = (dt == CORE_DTYPE_BF16);
    a.vec_load = (aligned_to(G, bf16 ? 8 : 16) && ld % 4 == 0) ? 1 : 0;

    if (plan.mode == kPlanSmall) {
        ProjectSmallArgs sa;
        sa.G = G; sa.ld = ld; sa.d = d; sa.m = m; sa.n = n;
        sa.k0 = a.k0; sa.k1 = a.k1; sa.r0 = a.r0; sa.r1 = a.r1; sa.round_dev = a.round_dev;
        sa.vec_load = a.vec_load;
        sa.P = P; sa.pbar = pbar;
        const dim3 g(m), b(plan.small_threads);
        hipError_t e;
        if (n <= 1)      e = bf16 ? launch(project_small_kernel<1, true>, g, b, st, sa) : launch(project_small_kernel<1, false>, g, b, st, sa);
        else if (n <= 2) e = bf16 ? launch(project_small_kernel<2, true>, g, b, st, sa) : launch(project_small_kernel<2, false>, g, b, st, sa);
        else if (n <= 4) e = bf16 ? launch(project_small_kernel<4, true>, g, b, st, sa) : launch(project_small_kernel<4, false>, g, b, st, sa);
        else             e = bf16 ? launch(project_small_kernel<8, true>, g, b, st, sa) : launch(project_small_kernel<8, false>, g, b, st, sa);
        return e == hipSuccess ? CORE_OK : hip_fail(e);
    }

    const uint32_t chunk_slots = (uint32_t)(ceil_div(plan.nchunks, 8) * 8);
    if (plan.jtiles > 0) {   // lanes-over-vectors kernels: the tiles of 256 vectors
        const uint32_t blocks = chunk_slots * plan.jtiles;
        for (uint32_t c0 = 0; c0 < n;) {
            const uint32_t left = n - c0;
            const bool store = (xi_store != nullptr) && c0 == 0;   // later passes regenerate, store once
            // Every pass regenerates the normals, so a pass takes as many clients as its kernel can
            // hold: 64 on the wide matrix-pipe kernel when more than 32 are left (ResNet-50-sized
            // gradient, m = 1024, projection alone: n = 50 in one pass 32.6 ms against 48.2 ms in passes
            // of 32 + 18, n = 64 39.5 against 52.9 ms, n = 36 25.4 against 37.4 ms), 32 on the two-level
            // matrix-pipe kernel, 16 on the VALU.
            const bool mfma = !store && use_mfma_projection(left);
            const bool wide = mfma && plan.wide && left > kMaxClientsPerPassMfma;
            const uint32_t cap = wide ? kMaxClientsPerPassWide : mfma ? kMaxClientsPerPassMfma : kMaxClientsPerPass;
            const uint32_t nc = left < cap ? left : cap;
            a.c0 = c0; a.nc = nc;
            c0 += nc;
            hipError_t e;
            if (wide) {
                switch ((nc + 3) / 4) {   // client groups of 4: 9 to 16
                    case 9:  e = launch_project_mfma_wide<9>(a, bf16, blocks, st); break;
                    case 10: e = launch_project_mfma_wide<10>(a, bf16, blocks, st); break;
                    case 11: e = launch_project_mfma_wide<11>(a, bf16, blocks, st); break;
                    case 12: e = launch_project_mfma_wide<12>(a, bf16, blocks, st); break;
                    case 13: e = launch_project_mfma_wide<13>(a, bf16, blocks, st); break;
                    case 14: e = launch_project_mfma_wide<14>(a, bf16, blocks, st); break;
                    case 15: e = launch_project_mfma_wide<15>(a, bf16, blocks, st); break;
                    default: e = launch_project_mfma_wide<16>(a, bf16, blocks, st); break;
                }
            } else
            if (mfma) {
                if (nc <= 4)       e = launch_project_mfma<1>(a, bf16, blocks, st);
                else if (nc <= 8)  e = launch_project_mfma<2>(a, bf16, blocks, st);
                else if (nc <= 12) e = launch_project_mfma<3>(a, bf16, blocks, st);
                else if (nc <= 16) e = launch_project_mfma<4>(a, bf16, blocks, st);
                else if (nc <= 24) e = launch_project_mfma<6>(a, bf16, blocks, st);
                else               e = launch_project_mfma<8>(a, bf16, blocks, st);
            } else
            if (nc <= 1)      e = launch_project<1>(a, bf16, store, blocks, st);
            else if (nc <= 2) e = launch_project<2>(a, bf16, store, blocks, st);
            else if (nc <= 4) e = launch_project<4>(a, bf16, store, blocks, st);
            else if (nc <= 8) e = launch_project<8>(a, bf16, store, blocks, st);
            else              e = launch_project<16>(a, bf16, store, blocks, st);
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    uint32_t j_next = plan.jtiles * (uint32_t)kThreads;
    if (plan.narrow_tiles > 0) {   // whole waves of the rest: blocks of 64 vectors
        const int rc = enqueue_narrow(a, bf16, n, 64, plan.narrow_tiles, j_next, chunk_slots, st);
        if (rc != CORE_OK) return rc;
        j_next += plan.narrow_tiles * 64u;
    }
    if (plan.sub_tiles > 0) {      // what is left: blocks of 8, 16 or 32 vectors
        const int rc = enqueue_narrow(a, bf16, n, plan.sub_jw, plan.sub_tiles, j_next, chunk_slots, st);
        if (rc != CORE_OK) return rc;
    }
    if (plan.tail_groups > 0) {   // lanes-over-coordinates kernel (kPlanCoords): all vectors
        ProjectArgs q = a;
        q.jtiles = plan.tail_groups;
        q.j_begin = 0;
        q.tiles_per_chunk = plan.tiles_per_chunk / 4;   // its tiles are 1024 coordinates
        const uint32_t blocks = chunk_slots * plan.tail_groups;
        for (uint32_t c0 = 0; c0 < n; c0 += 8) {
            const uint32_t nc = (n - c0 < 8u) ? (n - c0) : 8u;
            q.c0 = c0; q.nc = nc;
            hipError_t e;
            if (nc <= 1)      e = launch_project_q<1>(q, bf16, plan.qj, blocks, st);
            else if (nc <= 2) e = launch_project_q<2>(q, bf16, plan.qj, blocks, st);
            else if (nc <= 4) e = launch_project_q<4>(q, bf16, plan.qj, blocks, st);
            else              e = launch_project_q<8>(q, bf16, plan.qj, blocks, st);
            if (e != hipSuccess) return hip_fail(e);
        }
    }

    const uint64_t E = (uint64_t)n * m;
    hipError_t e;
    if (plan.nchunks <= 16) {
        // few chunks: one kernel sums them and the clients
        e = launch(reduce_clients_kernel<float>, dim3((uint32_t)ceil_div(m, 32)), dim3(kThreads), st,
                   (const float*)part, m, n, plan.nchunks, P, pbar);
        return e == hipSuccess ? CORE_OK : hip_fail(e);
    }
    e = launch(reduce_chunks_kernel, dim3((uint32_t)ceil_div(m, 32), n, plan.Z), dim3(kThreads), st,
               (const float*)part, m, n, plan.nchunks, psum);
    if (e != hipSuccess) return hip_fail(e);
    e = launch(reduce_clients_kernel<double>, dim3((uint32_t)ceil_div(m, 32)), dim3(kThreads), st,
               (const double*)psum, m, n, plan.Z, P, pbar);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

struct UpdateArgs {
    const float* y = nullptr;
    float* x_new = nullptr;
    const float* x_cur = nullptr;
    float* y_next = nullptr;
    float h = 0.0f, omb = 0.0f;
    const float* h_dev = nullptr;
    const uint64_t* round_dev = nullptr;
};

int enqueue_reconstruct(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, const float* pbar,
                        float scale, float* gtilde, hipStream_t st, const UpdateArgs* up = nullptr)
{
    ReconArgs a;
    a.pbar = pbar; a.gtilde = gtilde; a.d = d; a.m = m; a.scale = scale;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32);
    a.r0 = (uint32_t)round; a.r1 = (uint32_t)(round >> 32);
    bool vec = !gtilde || aligned_to(gtilde, 16);
    a.y = nullptr; a.x_new = nullptr; a.x_cur = nullptr; a.y_next = nullptr; a.h = 0.0f; a.omb = 0.0f;
    a.h_dev = nullptr;
    a.round_dev = up ? reinterpret_cast<const uint32_t*>(up->round_dev) : nullptr;
    if (up) {
        a.y = up->y; a.x_new = up->x_new; a.x_cur = up->x_cur; a.y_next = up->y_next;
        a.h = up->h; a.omb = up->omb; a.h_dev = up->h_dev;
        vec = vec && aligned_to(up->y, 16) && aligned_to(up->x_new, 16) &&
              (!up->y_next || (aligned_to(up->y_next, 16) && aligned_to(up->x_cur, 16)));
    }
    a.vec_store = vec ? 1 : 0;
    const uint64_t nblk = ceil_div(d, 4);
    // two Philox blocks per thread share the scalar work of a vector; one per thread when that
    // would leave block slots empty (small d)
    const bool two = ceil_div(nblk, (uint64_t)kThreads * 2) >= 2 * kBlockSlots;
    hipError_t e;
    // short vectors: fewer 64-block columns than 4 waves per SIMD.  Split the vectors j of a
    // column over several waves of one workgroup until there are that many (measured at 2^20
    // coordinates, 4096 columns: one wave per column 122 us, two 129 us, four 127 us; at 4096
    // coordinates, 16 columns: 17 us unsplit, 9 us with 16 waves per column).
    const uint64_t columns = ceil_div(nblk, 64);
    uint32_t split = 1;
    while (split < (uint32_t)kSplitMaxWaves && columns * split < kWaveSlots / 2 && 2 * split <= m) split *= 2;
    if (!two && split >= 2) {
        const dim3 g((uint32_t)columns), b(64 * split);
        const size_t lds = (size_t)split * 4 * 64 * sizeof(float);
        e = up ? launch_lds(reconstruct_split_kernel<true>, g, b, lds, st, a)
               : launch_lds(reconstruct_split_kernel<false>, g, b, lds, st, a);
        return e == hipSuccess ? CORE_OK : hip_fail(e);
    }
    const uint32_t blocks = (uint32_t)ceil_div(nblk, (uint64_t)kThreads * (two ? 2 : 1));
    const dim3 g(blocks), b(kThreads);
    if (up) e = two ? launch(reconstruct_kernel<true, 2>, g, b, st, a) : launch(reconstruct_kernel<true, 1>, g, b, st, a);
    else    e = two ? launch(reconstruct_kernel<false, 2>, g, b, st, a) : launch(reconstruct_kernel<false, 1>, g, b, st, a);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

// [a, a + na floats) and [b, b + nb floats) share at least one element (null never does)
bool intersects(const float* a, uint64_t na, const float* b, uint64_t nb)
{
    if (!a || !b) return false;
    const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + (uintptr_t)nb * sizeof(float) && pb < pa + (uintptr_t)na * sizeof(float);
}
bool intersects(const float* a, const float* b, uint64_t count) { return intersects(a, count, b, count); }

// the two ranges intersect without being the same range (an in-place alias is element-wise safe,
// a shifted one is not)
bool overlaps_shifted(const float* a, const float* b, uint64_t count) { return a != b && intersects(a, b, count); }

int validate_update(uint64_t d, const float* y, const float* x_new, const float* x_cur, const float* y_next,
                    const float* gtilde)
{
    if (!y || !x_new) return CORE_ERR_INVALID_ARGUMENT;
    if ((x_cur == nullptr) != (y_next == nullptr)) return CORE_ERR_INVALID_ARGUMENT;
    if (intersects(y_next, x_new, d) || intersects(y_next, gtilde, d)) return CORE_ERR_INVALID_ARGUMENT;
    if (intersects(gtilde, x_new, d) || intersects(gtilde, y, d) || intersects(gtilde, x_cur, d))
        return CORE_ERR_INVALID_ARGUMENT;
    if (overlaps_shifted(y, x_new, d) || overlaps_shifted(x_cur, x_new, d) || overlaps_shifted(y_next, x_cur, d) ||
        overlaps_shifted(y_next, y, d))
        return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(y, 4) || !aligned_to(x_new, 4) || !aligned_to(x_cur, 4) || !aligned_to(y_next, 4) ||
        !aligned_to(gtilde, 4))
        return CORE_ERR_MISALIGNED;
    return CORE_OK;
}

int validate_nonconvex_step(uint64_t d, uint32_t m, const float* pbar, float c, double r1, double H,
                            const float* p_out, const float* h_out)
{
    if (!pbar || !h_out || d == 0 || d > kMaxD || m == 0 || m > kMaxM) return CORE_ERR_INVALID_ARGUMENT;
    if (!(c > 0.0f) || !(r1 > 0.0) || !(H > 0.0)) return CORE_ERR_INVALID_ARGUMENT;
    if (h_out == p_out || h_out == pbar || p_out == pbar) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(pbar, 4) || !aligned_to(p_out, 4) || !aligned_to(h_out, 4)) return CORE_ERR_MISALIGNED;
    return CORE_OK;
}

int enqueue_nonconvex_step(uint64_t d, uint32_t m, const float* pbar, float c, double r1, double H,
                           float* p_out, float* h_out, hipStream_t st)
{
    const double first = (double)m / (16.0 * r1);
    const double second = std::pow(H, -0.5) * std::pow((double)d, -0.75) * std::pow((double)m, 0.75) / 1600.0;
    const hipError_t e = launch(nonconvex_step_kernel, dim3(1), dim3(kThreads), st, pbar, m, c, (float)first,
                                (float)second, p_out, h_out);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

int validate_trial(uint64_t d, const float* h, const float* x, const float* x_trial, const float* gtilde)
{
    if (!h || !x || !x_trial || intersects(x, x_trial, d)) return CORE_ERR_INVALID_ARGUMENT;
    if (intersects(gtilde, x, d) || intersects(gtilde, x_trial, d)) return CORE_ERR_INVALID_ARGUMENT;
    if (intersects(h, 1, x_trial, d) || intersects(h, 1, gtilde, d)) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(h, 4) || !aligned_to(x, 4) || !aligned_to(x_trial, 4) || !aligned_to(gtilde, 4))
        return CORE_ERR_MISALIGNED;
    return CORE_OK;
}

int enqueue_reconstruct_xi(uint64_t d, uint32_t m, const float* pbar, float scale, const float* xi,
                           float* gtilde, hipStream_t st)
{
    ReconXiArgs a;
    a.pbar = pbar; a.xi = xi; a.gtilde = gtilde; a.d = d; a.m = m; a.scale = scale;
    const uint64_t nblk = ceil_div(d, 4);
    const hipError_t e = launch(reconstruct_xi_kernel, dim3((uint32_t)ceil_div(nblk, kThreads / 64)), dim3(kThreads), st, a);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

// bytes of the materialised Xi for (d, m); 0 if it cannot be addressed
size_t xi_bytes(uint64_t d, uint32_t m)
{
    if (d == 0 || d > kMaxD || m == 0 || m > kMaxM) return 0;
    const uint64_t nblk = ceil_div(d, 4);
    if (nblk > (~(uint64_t)0) / 16 / m) return 0;
    if (ceil_div(nblk, kThreads / 64) > 0x7fffffffull) return 0;
    return (size_t)(nblk * m * 16);
}

// ---- fixed scratch for callers that cannot allocate ---------------------------------------------
// core_round_static runs core_round with its workspace in this array instead of caller memory.
// Every GPU the library runs on holds its own copy until the process ends.  In host code the
// array's name is only a handle for the runtime's symbol lookup: the device address is asked for
// once per device and that address is what the kernels get.
static __device__ __align__(256) unsigned char scratch[CORE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return CORE_ERR_INVALID_ARGUMENT;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // address of this device's copy
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CORE_OK;
}

}  // namespace

extern "C" {

const char* core_build_id(void) { return kBuildId + 14; }

const char* core_strerror(int code)
{
    switch (code) {
        case CORE_OK: return "success";
        case CORE_ERR_INVALID_ARGUMENT: return "invalid argument (null pointer, zero or out-of-range size, ld < d, or unknown dtype)";
        case CORE_ERR_MISALIGNED: return "pointer not aligned to its element size (workspace: 16 bytes)";
        case CORE_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than core_workspace_bytes(d, m, n)";
        case CORE_ERR_HIP: return "HIP runtime error on launch (see core_last_hip_error)";
        case CORE_ERR_NO_DEVICE: return "no usable GPU device";
        case CORE_ERR_STATIC_SCRATCH_TOO_SMALL:
            return "sizes need more scratch than the library's fixed CORE_STATIC_SCRATCH_BYTES; use core_round with a caller workspace";
        default: return "unknown error code";
    }
}

int core_last_hip_error(void) { return g_last_hip_error; }

size_t core_workspace_bytes(uint64_t d, uint32_t m, uint32_t n) { return workspace_bytes(d, m, n); }

int core_compress_batched(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                          const void* G, core_dtype dt, uint64_t ld, float* P, float* pbar,
                          void* ws, size_t ws_bytes, core_stream stream)
{
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, P, pbar, ws, ws_bytes, plan);
    if (rc != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    return enqueue_compress(seed, round, d, m, n, G, dt, ld, P, pbar, ws, plan, (hipStream_t)stream);
}

int core_compress(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, const void* g, core_dtype dt,
                  float* p, void* ws, size_t ws_bytes, core_stream stream)
{
    // one client: the mean over clients is the projection itself
    return core_compress_batched(seed, round, d, m, 1, g, dt, d, nullptr, p, ws, ws_bytes, stream);
}

int core_reconstruct(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, const float* pbar,
                     float scale, float* gtilde, core_stream stream)
{
    int rc = validate_reconstruct(d, m, pbar, gtilde);
    if (rc != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    return enqueue_reconstruct(seed, round, d, m, pbar, scale, gtilde, (hipStream_t)stream);
}

int core_round(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n, const void* G,
               core_dtype dt, uint64_t ld, float* pbar, float* gtilde, void* ws, size_t ws_bytes,
               core_stream stream)
{
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, nullptr, pbar, ws, ws_bytes, plan);
    if (rc != CORE_OK) return rc;
    if ((rc = validate_reconstruct(d, m, pbar, gtilde)) != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    rc = enqueue_compress(seed, round, d, m, n, G, dt, ld, nullptr, pbar, ws, plan, (hipStream_t)stream);
    if (rc != CORE_OK) return rc;
    return enqueue_reconstruct(seed, round, d, m, pbar, 1.0f / (float)m, gtilde, (hipStream_t)stream);
}

int core_round_static(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n, const void* G,
                      core_dtype dt, uint64_t ld, float* pbar, float* gtilde, core_stream stream)
{
    const size_t need = workspace_bytes(d, m, n);
    if (need == 0) return CORE_ERR_INVALID_ARGUMENT;
    if (need > (size_t)CORE_STATIC_SCRATCH_BYTES) return CORE_ERR_STATIC_SCRATCH_TOO_SMALL;
    // validation needs a non-null, aligned workspace pointer; the real one is looked up only
    // after every argument has passed
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, nullptr, pbar, (const void*)(uintptr_t)256, need, plan);
    if (rc != CORE_OK) return rc;
    if ((rc = validate_reconstruct(d, m, pbar, gtilde)) != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != CORE_OK) return rc;
    rc = enqueue_compress(seed, round, d, m, n, G, dt, ld, nullptr, pbar, ws, plan, (hipStream_t)stream);
    if (rc != CORE_OK) return rc;
    return enqueue_reconstruct(seed, round, d, m, pbar, 1.0f / (float)m, gtilde, (hipStream_t)stream);
}

int core_reconstruct_update(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, const float* pbar,
                            float scale, float h, const float* y, float* x_new, const float* x_cur,
                            float one_minus_beta, float* y_next, float* gtilde, core_stream stream)
{
    if (!pbar || d == 0 || d > kMaxD || m == 0 || m > kMaxM) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(pbar, 4)) return CORE_ERR_MISALIGNED;
    int rc = validate_update(d, y, x_new, x_cur, y_next, gtilde);
    if (rc != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    UpdateArgs up;
    up.y = y; up.x_new = x_new; up.x_cur = x_cur; up.y_next = y_next; up.h = h; up.omb = one_minus_beta;
    return enqueue_reconstruct(seed, round, d, m, pbar, scale, gtilde, (hipStream_t)stream, &up);
}

int core_round_update(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n, const void* G,
                      core_dtype dt, uint64_t ld, float* pbar, float h, const float* y, float* x_new,
                      const float* x_cur, float one_minus_beta, float* y_next, float* gtilde,
                      void* ws, size_t ws_bytes, core_stream stream)
{
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, nullptr, pbar, ws, ws_bytes, plan);
    if (rc != CORE_OK) return rc;
    if ((rc = validate_update(d, y, x_new, x_cur, y_next, gtilde)) != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    rc = enqueue_compress(seed, round, d, m, n, G, dt, ld, nullptr, pbar, ws, plan, (hipStream_t)stream);
    if (rc != CORE_OK) return rc;
    UpdateArgs up;
    up.y = y; up.x_new = x_new; up.x_cur = x_cur; up.y_next = y_next; up.h = h; up.omb = one_minus_beta;
    return enqueue_reconstruct(seed, round, d, m, pbar, 1.0f / (float)m, gtilde, (hipStream_t)stream, &up);
}

int core_round_update_r(uint64_t seed, const uint64_t* round_dev, uint64_t d, uint32_t m, uint32_t n,
                        const void* G, core_dtype dt, uint64_t ld, float* pbar, float h, const float* y,
                        float* x_new, const float* x_cur, float one_minus_beta, float* y_next, float* gtilde,
                        void* ws, size_t ws_bytes, core_stream stream)
{
    if (!round_dev) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(round_dev, 8)) return CORE_ERR_MISALIGNED;
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, nullptr, pbar, ws, ws_bytes, plan);
    if (rc != CORE_OK) return rc;
    if ((rc = validate_update(d, y, x_new, x_cur, y_next, gtilde)) != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    rc = enqueue_compress(seed, 0, d, m, n, G, dt, ld, nullptr, pbar, ws, plan, (hipStream_t)stream, nullptr,
                          round_dev);
    if (rc != CORE_OK) return rc;
    UpdateArgs up;
    up.y = y; up.x_new = x_new; up.x_cur = x_cur; up.y_next = y_next; up.h = h; up.omb = one_minus_beta;
    up.round_dev = round_dev;
    return enqueue_reconstruct(seed, 0, d, m, pbar, 1.0f / (float)m, gtilde, (hipStream_t)stream, &up);
}

int core_advance_round(uint64_t* round_dev, core_stream stream)
{
    if (!round_dev) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(round_dev, 8)) return CORE_ERR_MISALIGNED;
    int rc = check_device();
    if (rc != CORE_OK) return rc;
    const hipError_t e = launch(advance_round_kernel, dim3(1), dim3(64), (hipStream_t)stream, round_dev);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

int core_reconstruct_update_batched(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t nb,
                                    const float* P, uint64_t ldp, float scale, float h, float* X, float* Gt,
                                    uint64_t ldx, core_stream stream)
{
    if (!P || (!X && !Gt) || d == 0 || d > kMaxD || m == 0 || m > kMaxM || nb == 0 || nb > kMaxN) return CORE_ERR_INVALID_ARGUMENT;
    if (ldp < m || ldx < d) return CORE_ERR_INVALID_ARGUMENT;
    if (X && Gt && intersects(X, (uint64_t)nb * ldx, Gt, (uint64_t)nb * ldx)) return CORE_ERR_INVALID_ARGUMENT;
    if (intersects(P, (uint64_t)nb * ldp, X, (uint64_t)nb * ldx) || intersects(P, (uint64_t)nb * ldp, Gt, (uint64_t)nb * ldx))
        return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(P, 4) || !aligned_to(X, 4) || !aligned_to(Gt, 4)) return CORE_ERR_MISALIGNED;
    int rc = check_device();
    if (rc != CORE_OK) return rc;
    ReconBatchArgs a;
    a.P = P; a.ldp = ldp; a.X = X; a.Gt = Gt; a.ldx = ldx; a.d = d; a.m = m; a.scale = scale; a.h = h;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32);
    a.r0 = (uint32_t)round; a.r1 = (uint32_t)(round >> 32);
    const uint32_t blocks = (uint32_t)ceil_div(ceil_div(d, 4), (uint64_t)kThreads);
    for (uint32_t v0 = 0; v0 < nb; v0 += 8) {
        const uint32_t nv = (nb - v0 < 8u) ? (nb - v0) : 8u;
        a.v0 = v0; a.nv = nv;
        const hipError_t e = nv <= 4 ? launch(reconstruct_batched_kernel<4>, dim3(blocks), dim3(kThreads), (hipStream_t)stream, a)
                                     : launch(reconstruct_batched_kernel<8>, dim3(blocks), dim3(kThreads), (hipStream_t)stream, a);
        if (e != hipSuccess) return hip_fail(e);
    }
    return CORE_OK;
}

int core_nonconvex_step(uint64_t d, uint32_t m, const float* pbar, float c, double r1, double H,
                        float* p_out, float* h_out, core_stream stream)
{
    int rc = validate_nonconvex_step(d, m, pbar, c, r1, H, p_out, h_out);
    if (rc != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    return enqueue_nonconvex_step(d, m, pbar, c, r1, H, p_out, h_out, (hipStream_t)stream);
}

int core_step_size_option2(uint64_t d, uint32_t m, double r1, double H, double L, double Delta, double* h)
{
    if (!h || d == 0 || d > kMaxD || m == 0 || m > kMaxM) return CORE_ERR_INVALID_ARGUMENT;
    if (!(r1 > 0.0) || !(H > 0.0) || !(L > 0.0) || !(Delta > 0.0)) return CORE_ERR_INVALID_ARGUMENT;
    const double first = (double)m / (16.0 * r1);
    const double second = std::pow(H, -0.5) * std::pow(L * Delta, -0.25) * std::pow((double)d, -0.75) *
                          std::pow((double)m, 0.75) / 1600.0;
    *h = first < second ? first : second;
    return CORE_OK;
}

int core_projection_sqnorms(uint32_t m, uint32_t n, const float* P, double* sq, core_stream stream)
{
    if (!P || !sq || m == 0 || m > kMaxM || n == 0 || n > kMaxN) return CORE_ERR_INVALID_ARGUMENT;
    if (intersects((const float*)sq, 2 * (uint64_t)n, P, (uint64_t)n * m)) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(P, 4) || !aligned_to(sq, 8)) return CORE_ERR_MISALIGNED;
    const int rc = check_device();
    if (rc != CORE_OK) return rc;
    const hipError_t e = launch(projection_sqnorms_kernel, dim3(n), dim3(kThreads), (hipStream_t)stream, P, m, sq);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

int core_privacy_loss(double sqnorm, uint32_t m, double sigma1, double sigma2, double* loss)
{
    if (!loss || m == 0 || m > kMaxM) return CORE_ERR_INVALID_ARGUMENT;
    if (!(sqnorm >= 0.0) || !(sigma1 > 0.0) || !(sigma2 > 0.0)) return CORE_ERR_INVALID_ARGUMENT;
    if (std::isinf(sqnorm) || std::isinf(sigma1) || std::isinf(sigma2)) return CORE_ERR_INVALID_ARGUMENT;
    *loss = 0.5 * sqnorm * (1.0 / (sigma2 * sigma2) - 1.0 / (sigma1 * sigma1)) + (double)m * std::log(sigma2 / sigma1);
    return CORE_OK;
}

int core_reconstruct_trial(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, const float* pbar,
                           float scale, const float* h, const float* x, float* x_trial, float* gtilde,
                           core_stream stream)
{
    if (!pbar || d == 0 || d > kMaxD || m == 0 || m > kMaxM) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(pbar, 4)) return CORE_ERR_MISALIGNED;
    int rc = validate_trial(d, h, x, x_trial, gtilde);
    if (rc != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    UpdateArgs up;
    up.y = x; up.x_new = x_trial; up.h_dev = h;
    return enqueue_reconstruct(seed, round, d, m, pbar, scale, gtilde, (hipStream_t)stream, &up);
}

static int round_trial_impl(uint64_t seed, uint64_t round, const uint64_t* round_dev, uint64_t d, uint32_t m,
                            uint32_t n, const void* G, core_dtype dt, uint64_t ld, float* pbar, float c, double r1,
                            double H, float* p_out, float* h_out, const float* x, float* x_trial, float* gtilde,
                            void* ws, size_t ws_bytes, core_stream stream)
{
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, nullptr, pbar, ws, ws_bytes, plan);
    if (rc != CORE_OK) return rc;
    if ((rc = validate_nonconvex_step(d, m, pbar, c, r1, H, p_out, h_out)) != CORE_OK) return rc;
    if ((rc = validate_trial(d, h_out, x, x_trial, gtilde)) != CORE_OK) return rc;
    if ((rc = check_device()) != CORE_OK) return rc;
    rc = enqueue_compress(seed, round, d, m, n, G, dt, ld, nullptr, pbar, ws, plan, (hipStream_t)stream, nullptr,
                          round_dev);
    if (rc != CORE_OK) return rc;
    if ((rc = enqueue_nonconvex_step(d, m, pbar, c, r1, H, p_out, h_out, (hipStream_t)stream)) != CORE_OK)
        return rc;
    UpdateArgs up;
    up.y = x; up.x_new = x_trial; up.h_dev = h_out; up.round_dev = round_dev;
    return enqueue_reconstruct(seed, round, d, m, pbar, 1.0f / (float)m, gtilde, (hipStream_t)stream, &up);
}

int core_round_trial(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n, const void* G,
                     core_dtype dt, uint64_t ld, float* pbar, float c, double r1, double H, float* p_out,
                     float* h_out, const float* x, float* x_trial, float* gtilde, void* ws, size_t ws_bytes,
                     core_stream stream)
{
    return round_trial_impl(seed, round, nullptr, d, m, n, G, dt, ld, pbar, c, r1, H, p_out, h_out, x, x_trial,
                            gtilde, ws, ws_bytes, stream);
}

int core_round_trial_r(uint64_t seed, const uint64_t* round_dev, uint64_t d, uint32_t m, uint32_t n, const void* G,
                       core_dtype dt, uint64_t ld, float* pbar, float c, double r1, double H, float* p_out,
                       float* h_out, const float* x, float* x_trial, float* gtilde, void* ws, size_t ws_bytes,
                       core_stream stream)
{
    if (!round_dev) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(round_dev, 8)) return CORE_ERR_MISALIGNED;
    return round_trial_impl(seed, 0, round_dev, d, m, n, G, dt, ld, pbar, c, r1, H, p_out, h_out, x, x_trial,
                            gtilde, ws, ws_bytes, stream);
}

int core_accept_trial(uint64_t d, float* f_cur, const float* f_trial, float* x, const float* x_trial,
                      int32_t* accepted, core_stream stream)
{
    if (!f_cur || !f_trial || !x || !x_trial || !accepted || d == 0 || d > kMaxD)
        return CORE_ERR_INVALID_ARGUMENT;
    if (intersects(x, x_trial, d) || f_cur == f_trial) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(f_cur, 4) || !aligned_to(f_trial, 4) || !aligned_to(x, 4) || !aligned_to(x_trial, 4) ||
        !aligned_to(accepted, 4))
        return CORE_ERR_MISALIGNED;
    int rc = check_device();
    if (rc != CORE_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = launch(accept_decide_kernel, dim3(1), dim3(64), st, f_cur, f_trial, accepted);
    if (e != hipSuccess) return hip_fail(e);
    const int vec = (aligned_to(x, 16) && aligned_to(x_trial, 16)) ? 1 : 0;
    const uint32_t blocks = (uint32_t)ceil_div(ceil_div(d, 4), (uint64_t)kThreads);
    e = launch(accept_copy_kernel, dim3(blocks), dim3(kThreads), st, (const int32_t*)accepted, x, x_trial, d, vec);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

size_t core_xi_bytes(uint64_t d, uint32_t m) { return xi_bytes(d, m); }

int core_compress_batched_store_xi(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                                   const void* G, core_dtype dt, uint64_t ld, float* P, float* pbar,
                                   float* xi, size_t xi_buf_bytes, void* ws, size_t ws_bytes,
                                   core_stream stream)
{
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, P, pbar, ws, ws_bytes, plan, false);
    if (rc != CORE_OK) return rc;
    if (!xi) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(xi, 16)) return CORE_ERR_MISALIGNED;
    const size_t need = xi_bytes(d, m);
    if (need == 0) return CORE_ERR_INVALID_ARGUMENT;
    if (xi_buf_bytes < need) return CORE_ERR_WORKSPACE_TOO_SMALL;
    if ((rc = check_device()) != CORE_OK) return rc;
    return enqueue_compress(seed, round, d, m, n, G, dt, ld, P, pbar, ws, plan, (hipStream_t)stream, xi);
}

int core_reconstruct_from_xi(uint64_t d, uint32_t m, const float* pbar, float scale, const float* xi,
                             size_t xi_buf_bytes, float* gtilde, core_stream stream)
{
    int rc = validate_reconstruct(d, m, pbar, gtilde);
    if (rc != CORE_OK) return rc;
    if (!xi) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(xi, 16)) return CORE_ERR_MISALIGNED;
    const size_t need = xi_bytes(d, m);
    if (need == 0) return CORE_ERR_INVALID_ARGUMENT;
    if (xi_buf_bytes < need) return CORE_ERR_WORKSPACE_TOO_SMALL;
    if ((rc = check_device()) != CORE_OK) return rc;
    return enqueue_reconstruct_xi(d, m, pbar, scale, xi, gtilde, (hipStream_t)stream);
}

int core_round_materialized(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                            const void* G, core_dtype dt, uint64_t ld, float* pbar, float* gtilde,
                            float* xi, size_t xi_buf_bytes, void* ws, size_t ws_bytes, core_stream stream)
{
    Plan plan;
    int rc = validate_compress(d, m, n, G, dt, ld, nullptr, pbar, ws, ws_bytes, plan, false);
    if (rc != CORE_OK) return rc;
    if ((rc = validate_reconstruct(d, m, pbar, gtilde)) != CORE_OK) return rc;
    if (!xi) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(xi, 16)) return CORE_ERR_MISALIGNED;
    const size_t need = xi_bytes(d, m);
    if (need == 0) return CORE_ERR_INVALID_ARGUMENT;
    if (xi_buf_bytes < need) return CORE_ERR_WORKSPACE_TOO_SMALL;
    if ((rc = check_device()) != CORE_OK) return rc;
    rc = enqueue_compress(seed, round, d, m, n, G, dt, ld, nullptr, pbar, ws, plan, (hipStream_t)stream, xi);
    if (rc != CORE_OK) return rc;
    return enqueue_reconstruct_xi(d, m, pbar, 1.0f / (float)m, xi, gtilde, (hipStream_t)stream);
}

int core_debug_plan(uint64_t d, uint32_t m, uint32_t n, uint64_t plan[10])
{
    Plan p;
    if (!plan || !make_plan(d, m, n, true, p)) return CORE_ERR_INVALID_ARGUMENT;
    const uint64_t chunk_slots = ceil_div(p.nchunks, 8) * 8;
    plan[0] = (uint64_t)p.mode;
    plan[1] = p.mode == kPlanCoords ? p.tail_groups : p.jtiles;
    plan[2] = p.nchunks;
    plan[3] = p.mode == kPlanCoords ? p.tiles_per_chunk / 4 : p.tiles_per_chunk;
    plan[4] = p.Z;
    plan[5] = p.mode == kPlanSmall ? (uint64_t)p.jtiles : chunk_slots * plan[1];
    plan[6] = p.sub_tiles;
    plan[7] = p.qj;
    plan[8] = p.narrow_tiles;
    plan[9] = p.sub_jw;
    return CORE_OK;
}

int core_debug_philox_layout(int layout, uint64_t seed, uint64_t round, uint32_t j0, uint32_t nj, uint64_t q0,
                             uint64_t nq, uint32_t* out, core_stream stream)
{
    if (!out || layout < 0 || layout > 4 || nj == 0 || nq == 0) return CORE_ERR_INVALID_ARGUMENT;
    if ((uint64_t)j0 + nj > (1ull << 32) || nq > (1ull << 32) || q0 + nq > (1ull << 32) ||
        (uint64_t)nj * nq > (1ull << 28))
        return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(out, 4)) return CORE_ERR_MISALIGNED;
    int rc = check_device();
    if (rc != CORE_OK) return rc;
    DebugPhiloxArgs a;
    a.k0 = (uint32_t)seed; a.k1 = (uint32_t)(seed >> 32);
    a.r0 = (uint32_t)round; a.r1 = (uint32_t)(round >> 32);
    a.j0 = j0; a.nj = nj; a.q0 = q0; a.nq = nq; a.out = out;
    const uint64_t threads = layout == 1 ? nj : layout == 4 ? (uint64_t)nj * nq : nq;
    const dim3 g((uint32_t)ceil_div(threads, kThreads)), b(kThreads);
    hipError_t e;
    switch (layout) {
        case 1: e = launch(debug_philox_kernel<1>, g, b, (hipStream_t)stream, a); break;
        case 2: e = launch(debug_philox_kernel<2>, g, b, (hipStream_t)stream, a); break;
        case 3: e = launch(debug_philox_kernel<3>, g, b, (hipStream_t)stream, a); break;
        case 4: e = launch(debug_philox_kernel<4>, g, b, (hipStream_t)stream, a); break;
        default: e = launch(debug_philox_kernel<0>, g, b, (hipStream_t)stream, a); break;
    }
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

int core_debug_philox(uint64_t seed, uint64_t round, uint32_t j, uint64_t q0, uint64_t nblocks,
                      uint32_t* out, core_stream stream)
{
    if (nblocks > (1ull << 28)) return CORE_ERR_INVALID_ARGUMENT;
    return core_debug_philox_layout(0, seed, round, j, 1, q0, nblocks, out, stream);
}

int core_debug_set_projection(int variant)
{
    if (variant < kVariantAuto || variant > kVariantSmall) return CORE_ERR_INVALID_ARGUMENT;
    variant_cell().store(variant, std::memory_order_relaxed);
    return CORE_OK;
}

int core_debug_xi(uint64_t seed, uint64_t round, uint32_t j, uint64_t i0, uint64_t count, float* out,
                  core_stream stream)
{
    if (!out || count == 0 || count > (1ull << 32) || i0 + count > kMaxD) return CORE_ERR_INVALID_ARGUMENT;
    if (!aligned_to(out, 4)) return CORE_ERR_MISALIGNED;
    int rc = check_device();
    if (rc != CORE_OK) return rc;
    const hipError_t e = launch(debug_xi_kernel, dim3((uint32_t)ceil_div(count, kThreads)), dim3(kThreads),
                                (hipStream_t)stream, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)round,
                                (uint32_t)(round >> 32), j, i0, count, out);
    return e == hipSuccess ? CORE_OK : hip_fail(e);
}

}  // extern "C"
