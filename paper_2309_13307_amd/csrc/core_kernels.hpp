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
//
// The kernels live in one header per family:
//   core_project.hpp       projection for whole tiles of 256 vectors (VALU and matrix pipe)
//   core_project_few.hpp   projection for other vector counts and for tiny problems
//   core_reduce.hpp        cross-chunk sum and client mean
//   core_reconstruct.hpp   reconstruction and its variants
//   core_steps.hpp         Algorithm 3's scalar steps, diagnostics, round counter
//   core_debug.hpp         test-only generator dumps
#pragma once
#include "core_common.hpp"
#include "core_rng.hpp"
#include "core_project.hpp"
#include "core_project_few.hpp"
#include "core_reduce.hpp"
#include "core_reconstruct.hpp"
#include "core_steps.hpp"
#include "core_debug.hpp"
