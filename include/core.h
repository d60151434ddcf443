/*
 * core.h -- C ABI of the CORE (Common Random Reconstruction) hot path for AMD MI355X (gfx950).
 *
 * The method is that of "CORE: Common Random Reconstruction for Distributed
 * Optimization with Provable Low Communication Complexity" (arXiv 2309.13307):
 *
 *   compression     p_j = <a, xi_j>,  j = 1..m              (Algorithm 1, Section 3)
 *   reconstruction  a~  = (1/m) sum_j p_j xi_j              (Eq. (reconstruction), Section 3)
 *   n machines      g~  = (1/(n m)) sum_i sum_j <g_i, xi_j> xi_j
 *                                                           (Eq. (tildefdef), Section 4;
 *                                                            Algorithm 2, the three
 *                                                            communication lines)
 *
 * xi_1..xi_m ~ N(0, I_d) come from a generator every machine shares (Algorithm 1,
 * REQUIRE line).  They are never stored: each kernel regenerates the values it
 * needs in registers from (seed, round, j, i):
 *
 *   Philox4x32-10 with key (seed lo32, seed hi32) and counter
 *   (q = floor(i/4), j, round lo32, round hi32) yields four words x0..x3;
 *   u1 = ((xa>>8)+1) 2^-24, u2 = (xb>>8) 2^-24, r = sqrt(-2 ln u1),
 *   (x0,x1) -> xi_j[4q] = r cos(2 pi u2), xi_j[4q+1] = r sin(2 pi u2); (x2,x3) -> xi_j[4q+2], xi_j[4q+3].
 *   j and i are 0-based.  A new `round` gives fresh vectors (Algorithm 1 / Algorithm 2,
 *   "generate fresh i.i.d. Gaussian vectors"); all n clients of a call share them.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     allocates nothing, frees nothing and keeps no pointer after it returns.
 *   - Work is enqueued on `stream` (a hipStream_t; NULL = the default stream) and
 *     the call returns without synchronising.  Outputs are overwritten, never
 *     accumulated into.  Results are a pure function of the arguments and
 *     bit-identical from run to run on the same device and build (all sums run
 *     in a fixed order; no floating-point atomics).
 *   - Return value: CORE_OK (0) or a negative CORE_ERR_* code.  Arguments are
 *     validated on the host before anything is launched, so a call that fails
 *     validation enqueues nothing and writes nothing.  CORE_ERR_HIP is the one
 *     exception: it reports that the runtime refused a launch, and an entry point
 *     that issues several launches may already have enqueued the earlier ones
 *     (its outputs are then undefined).  Launch status is taken from the launch
 *     call itself, never from the thread's sticky last-error state.
 *   - Limits: 1 <= d <= 2^34, 1 <= m <= 2^32-1024, 1 <= n <= 65535, ld >= d, and
 *     ceil(d / 2^18) * ceil(m / 256) < 2^31 (one projection block per 2^18 coordinates x 256
 *     vectors at the largest sizes; d * m below ~1.4e17 always qualifies).  Sizes outside
 *     the limits are refused with CORE_ERR_INVALID_ARGUMENT by every entry point.
 *     fp32 pointers must be 4-byte aligned, bf16 pointers 2-byte aligned; rows of G
 *     may start at any element.  gtilde is written with 128-bit stores when it is
 *     16-byte aligned and with scalar stores otherwise.
 *   - Arithmetic: fp32 throughout on the device; per-(client, vector) sums are
 *     blocked (256-coordinate inner sums, then per-chunk sums, then an fp64 sum
 *     over chunks) so that rounding error stays near fp32 epsilon at any d.
 *     Subnormal inputs, products and sums are kept (no flush to zero); a projection is
 *     finite as long as |<g, xi_j>| fits fp32; non-finite inputs give non-finite outputs.
 */
#ifndef CORE_H_
#define CORE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CORE_DTYPE_F32 = 0,  /* IEEE binary32 */
    CORE_DTYPE_BF16 = 1  /* upper 16 bits of a binary32, widened exactly on load */
} core_dtype;

typedef void *core_stream; /* hipStream_t */

enum {
    CORE_OK = 0,
    CORE_ERR_INVALID_ARGUMENT = -1,   /* NULL required pointer, zero or out-of-range size, ld < d, unknown dtype */
    CORE_ERR_MISALIGNED = -2,         /* pointer not aligned to its element size */
    CORE_ERR_WORKSPACE_TOO_SMALL = -3,/* ws_bytes < core_workspace_bytes(d, m, n) */
    CORE_ERR_HIP = -4,                /* the HIP runtime refused a launch (see core_last_hip_error) */
    CORE_ERR_NO_DEVICE = -5,          /* no usable GPU in this process */
    CORE_ERR_STATIC_SCRATCH_TOO_SMALL = -6 /* core_round_static: sizes need more than CORE_STATIC_SCRATCH_BYTES */
};

/* Static, human-readable text for a return code. */
const char *core_strerror(int code);

/* hipError_t of the most recent CORE_ERR_HIP on the calling thread (0 if none). */
int core_last_hip_error(void);

/* Identifier of the sources the library was built from (a hash set by the build step, or
 * "unknown").  Static string.  A loader can compare it with the sources it has at hand and
 * refuse, or rebuild, a stale binary. */
const char *core_build_id(void);

/* Bytes of device scratch the compress/round entry points need for these sizes
 * (per-chunk partial projections and the staged cross-chunk sums).  Returns 0 if
 * the sizes are out of range.  The scratch needs 16-byte alignment and carries
 * no state between calls. */
size_t core_workspace_bytes(uint64_t d, uint32_t m, uint32_t n);

/* Algorithm 1, compression line, for one vector:  p[j] = <g, xi_j>, j < m.
 *   g  [d] device, dtype dt;  p [m] device fp32 (out);  ws device scratch. */
int core_compress(uint64_t seed, uint64_t round, uint64_t d, uint32_t m,
                  const void *g, core_dtype dt,
                  float *p,
                  void *ws, size_t ws_bytes, core_stream stream);

/* Algorithm 2, "machine i sends p_ij" for n machines batched on one device, and the
 * combination of Eq. (tildefdef):
 *   P[c][j]  = <G[c], xi_j>                     c < n, j < m
 *   pbar[j]  = (1/n) sum_c P[c][j]
 *   G    [n][ld] device, row-major, dtype dt, ld >= d (elements)
 *   P    [n][m]  device fp32 (out), may be NULL when only the mean is wanted
 *   pbar [m]     device fp32 (out) */
int core_compress_batched(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                          const void *G, core_dtype dt, uint64_t ld,
                          float *P, float *pbar,
                          void *ws, size_t ws_bytes, core_stream stream);

/* Eq. (reconstruction):  gtilde[i] = scale * sum_{j<m} pbar[j] * xi_j[i],  i < d.
 * scale = 1/m is the paper's estimator of the mean gradient; scale = n/m applied to
 * the client mean gives the sum-over-machines form written in Algorithm 2.
 *   pbar [m] device fp32;  gtilde [d] device fp32 (out). */
int core_reconstruct(uint64_t seed, uint64_t round, uint64_t d, uint32_t m,
                     const float *pbar, float scale,
                     float *gtilde, core_stream stream);

/* One communication round of Algorithm 2 without the x update:
 * core_compress_batched(P = NULL) followed by core_reconstruct(scale = 1/m),
 * i.e. Eq. (tildefdef).  pbar [m] and gtilde [d] are both outputs. */
int core_round(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
               const void *G, core_dtype dt, uint64_t ld,
               float *pbar, float *gtilde,
               void *ws, size_t ws_bytes, core_stream stream);

/* core_round for callers that cannot allocate device memory or supply a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results as core_round, but the scratch (per-chunk partial projections
 * and the staged cross-chunk sums) lives in a fixed array inside the library, of
 * CORE_STATIC_SCRATCH_BYTES per GPU, which each GPU the library runs on holds until the process
 * ends.  The call allocates and frees nothing; the first call on a device looks up that device's
 * copy of the array (the device current on the calling thread must be the stream's device).
 *   - Sizes with core_workspace_bytes(d, m, n) > CORE_STATIC_SCRATCH_BYTES are refused with
 *     CORE_ERR_STATIC_SCRATCH_TOO_SMALL before anything is launched (the ResNet-50-sized case,
 *     d = 25,557,032, m = 1024, n = 8, needs 68 MB and fits).
 *   - All calls on one GPU share the one array: calls that may overlap in time on the same GPU
 *     (different streams, or different host threads) race on it and must be serialised by the
 *     caller; use core_round with separate workspaces for concurrent rounds.
 *   - The array keeps the previous call's contents.  Nothing needs clearing: every partial sum is
 *     written by the call's own projection kernels before its reduction kernels read it. */
#define CORE_STATIC_SCRATCH_BYTES (80u << 20)
int core_round_static(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                      const void *G, core_dtype dt, uint64_t ld,
                      float *pbar, float *gtilde, core_stream stream);

/* ---- reconstruction fused with the optimiser step -------------------------------------------
 * Algorithm 2 ends each round with x^{k+1} = x^k - h_k * gtilde; CORE-AGD (appendix, heavy-ball
 * form) takes the gradients at y^k = x^k + (1-beta)(x^k - x^{k-1}) and sets
 * x^{k+1} = y^k - h * gtilde.  These entry points do that step in the epilogue of the
 * reconstruction kernel, so gtilde need not be written and re-read:
 *   x_new[i]  = y[i] - h * scale * sum_j pbar[j] xi_j[i]
 *   y_next[i] = x_new[i] + one_minus_beta * (x_new[i] - x_cur[i])     (only if y_next != NULL)
 *   y      [d] device fp32: the point the gradients were taken at (x^k for CORE-GD)
 *   x_new  [d] device fp32 out; may be the same buffer as y (in-place step)
 *   x_cur, y_next: both NULL (plain gradient step) or both non-NULL; x_cur is the iterate
 *           x^k; y_next may be the same buffer as x_cur or y, but not x_new
 *   gtilde [d] device fp32 out, or NULL when the estimate itself is not wanted; must not alias
 *           the other buffers.
 * Every element is read before the same thread writes it, which is what makes the stated
 * aliasing safe.  "The same buffer" means the same address: ranges that overlap at different
 * addresses are rejected with CORE_ERR_INVALID_ARGUMENT, here and in the Algorithm 3 entry points. */
int core_reconstruct_update(uint64_t seed, uint64_t round, uint64_t d, uint32_t m,
                            const float *pbar, float scale, float h,
                            const float *y, float *x_new,
                            const float *x_cur, float one_minus_beta, float *y_next,
                            float *gtilde, core_stream stream);

/* core_compress_batched(P = NULL) followed by core_reconstruct_update(scale = 1/m): one whole
 * iteration of Algorithm 2 (or of CORE-AGD) apart from the evaluation of the client gradients. */
int core_round_update(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                      const void *G, core_dtype dt, uint64_t ld,
                      float *pbar, float h,
                      const float *y, float *x_new,
                      const float *x_cur, float one_minus_beta, float *y_next,
                      float *gtilde,
                      void *ws, size_t ws_bytes, core_stream stream);

/* Reconstruction for nb machines at once, each from its own vector of (averaged) projections, as in
 * decentralized CORE-GD (appendix) when the machines are batched on one device: the common vectors
 * are generated once and feed all nb sums,
 *   g_v[i]   = scale * sum_j P[v][j] xi_j[i]           v < nb, i < d
 *   Gt[v][i] = g_v[i]                                   (if Gt != NULL)
 *   X[v][i] -= h * g_v[i]                               (if X != NULL; in place)
 *   P  [nb][ldp] device fp32, ldp >= m;  X, Gt [nb][ldx] device fp32, ldx >= d; at least one of X, Gt;
 *   the three arrays must not overlap.  (The decentralized algorithm uses scale = n/m on the
 *   averaged vector.)
 * The library's share of the decentralized algorithm is the projection (core_compress_batched with
 * P requested) and this reconstruction.  The exchange between the two -- every machine averaging
 * its neighbours' projection vectors with the gossip matrix -- is the caller's: on real hardware
 * it is the network step, and with the machines batched on one device it is one small product
 * W * P that the caller forms before this call. */
int core_reconstruct_update_batched(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t nb,
                                    const float *P, uint64_t ldp, float scale, float h,
                                    float *X, float *Gt, uint64_t ldx, core_stream stream);

/* ---- round counter in device memory (for replayed launch sequences) --------------------------
 * Algorithms 1 and 2 draw fresh Gaussian vectors every round, so the round counter must change
 * from one round to the next.  A caller that records one iteration into a HIP graph and replays it
 * cannot change a by-value argument between replays; core_round_update_r is core_round_update
 * with the counter read from device memory when the kernels run:
 *   round = *round_dev      (device uint64, 8-byte aligned; every kernel of the call reads it, so it
 *                            must not change while the call's kernels are in flight)
 * core_advance_round enqueues *round_dev += 1 on `stream`; put it after the round in the recorded
 * sequence.  Neither call uses a memset node, so both may be captured. */
int core_round_update_r(uint64_t seed, const uint64_t *round_dev, uint64_t d, uint32_t m, uint32_t n,
                        const void *G, core_dtype dt, uint64_t ld,
                        float *pbar, float h,
                        const float *y, float *x_new,
                        const float *x_cur, float one_minus_beta, float *y_next,
                        float *gtilde,
                        void *ws, size_t ws_bytes, core_stream stream);

int core_advance_round(uint64_t *round_dev, core_stream stream);

/* core_round_trial (Algorithm 3, below) with the counter read from device memory, for the same use. */
int core_round_trial_r(uint64_t seed, const uint64_t *round_dev, uint64_t d, uint32_t m, uint32_t n,
                       const void *G, core_dtype dt, uint64_t ld,
                       float *pbar, float c, double r1, double H, float *p_out, float *h_out,
                       const float *x, float *x_trial, float *gtilde,
                       void *ws, size_t ws_bytes, core_stream stream);

/* ---- CORE-GD for non-convex objectives (Algorithm 3, Section 5) -----------------------------
 * An iteration of Algorithm 3 is a round of Algorithm 2 plus three things: a scalar p formed from
 * the combined projections, a step size h_k chosen from p (Option I) or from constants
 * (Option II), and a comparison step that keeps x^k unless the trial point
 * xt = x^k - h_k * gtilde has a strictly smaller objective value.  None of them needs the host
 * to read device memory: p, h_k, the two objective values and the accept flag all stay on the
 * device, so the iterations can be queued back to back.
 *
 * The statistic.  The printed definition of p (a plain average of the summed projections, with
 * the machine and vector indices exchanged) cannot give the event p >= 2 |grad f(x^k)| that the
 * proof of Theorem 5.1 uses; since each combined projection is N(0, |grad f|^2) (lemma on the
 * law of C(a)), the library forms the norm estimate
 *   p = c * sqrt((1/m) sum_j pbar[j]^2),        c >= 2 chosen by the caller,
 * for which m (p/c)^2 / |grad f|^2 is chi-square with m degrees of freedom.
 *
 * core_nonconvex_step: Option I of Algorithm 3,
 *   h = min{ m/(16 r1), (1/1600) H^(-1/2) p^(-1/2) d^(-3/4) m^(3/4) }     (first term if p = 0)
 *   pbar [m] device fp32 (in);  p_out, h_out: device fp32 scalars (out; p_out may be NULL)
 *   r1 > 0 (bound on the trace of the Hessian), H > 0 (Lipschitz constant of the Hessian), c > 0;
 *   the two constant factors are evaluated on the host in fp64 and rounded to fp32 once. */
int core_nonconvex_step(uint64_t d, uint32_t m, const float *pbar, float c, double r1, double H,
                        float *p_out, float *h_out, core_stream stream);

/* Option II of Algorithm 3: h = min{ m/(16 r1), (1/1600) H^(-1/2) (L Delta)^(-1/4) d^(-3/4) m^(3/4) }.
 * Pure host arithmetic (fp64); h is a host pointer.  Use the result with
 * core_reconstruct_update / core_round_update, which take h by value. */
int core_step_size_option2(uint64_t d, uint32_t m, double r1, double H, double L, double Delta,
                           double *h);

/* Trial point of Algorithm 3 with the step read from device memory:
 *   x_trial[i] = x[i] - (*h) * scale * sum_j pbar[j] xi_j[i]
 *   h device fp32 scalar (e.g. h_out of core_nonconvex_step, written earlier on the same stream)
 *   x [d] device fp32 (in);  x_trial [d] device fp32 (out), a different buffer from x
 *   gtilde [d] device fp32 out or NULL; must not alias x or x_trial. */
int core_reconstruct_trial(uint64_t seed, uint64_t round, uint64_t d, uint32_t m,
                           const float *pbar, float scale, const float *h,
                           const float *x, float *x_trial,
                           float *gtilde, core_stream stream);

/* core_compress_batched(P = NULL), core_nonconvex_step and core_reconstruct_trial(scale = 1/m):
 * everything of one iteration of Algorithm 3 (Option I) between the evaluation of the client
 * gradients and the evaluation of f at the trial point.  Outputs: pbar [m], p_out (may be NULL),
 * h_out, x_trial [d], gtilde [d] (may be NULL). */
int core_round_trial(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                     const void *G, core_dtype dt, uint64_t ld,
                     float *pbar, float c, double r1, double H, float *p_out, float *h_out,
                     const float *x, float *x_trial, float *gtilde,
                     void *ws, size_t ws_bytes, core_stream stream);

/* Comparison step of Algorithm 3: x^{k+1} = argmin over {x^k, xt} of f.  With the two objective
 * values supplied by the caller as device scalars,
 *   if (*f_trial < *f_cur) { x[0..d) = x_trial[0..d); *f_cur = *f_trial; *accepted = 1; }
 *   else                   { *accepted = 0; }            (ties and NaN keep x)
 *   f_cur device fp32 scalar (in/out), f_trial device fp32 scalar (in)
 *   x [d] device fp32 (in/out), x_trial [d] device fp32 (in), a different buffer from x
 *   accepted: device int32 scalar (out, required: it carries the decision between the two
 *   kernels of this call). */
int core_accept_trial(uint64_t d, float *f_cur, const float *f_trial,
                      float *x, const float *x_trial, int32_t *accepted, core_stream stream);

/* ---- diagnostics from the privacy appendix ---------------------------------------------------
 * The appendix on differential privacy writes one machine's message as p = C(a) = Xi a and shows
 * (lemma on the law of C(a)) that p is N(0, |a|^2 I_m): an observer of the projections learns the
 * norm of the gradient and nothing about its direction.  Two consequences are exported.
 *
 * core_projection_sqnorms: sq[c] = sum_j P[c][j]^2 for every machine c (fp64, fixed summation
 *   order).  sq[c] / m is an unbiased estimate of |g_c|^2 with relative standard deviation
 *   sqrt(2/m), and m * (sq[c]/m) / |g_c|^2 is chi-square with m degrees of freedom.
 *   P [n][m] device fp32, row-major without padding, as core_compress_batched writes it (in);
 *   sq [n] device fp64 (out), 8-byte aligned, must not overlap P.
 *
 * core_privacy_loss: the privacy loss of the proof of the privacy theorem for one released
 *   message with squared norm sqnorm = |p|^2, when the two adjacent gradients have norms sigma1
 *   and sigma2:  L = (sqnorm / 2) (1/sigma2^2 - 1/sigma1^2) + m ln(sigma2 / sigma1),
 *   i.e. the log-ratio of the N(0, sigma1^2 I_m) and N(0, sigma2^2 I_m) densities at p.
 *   Pure host arithmetic (fp64); loss is a host pointer.  sqnorm >= 0, sigma1, sigma2 > 0, all
 *   finite, else CORE_ERR_INVALID_ARGUMENT. */
int core_projection_sqnorms(uint32_t m, uint32_t n, const float *P, double *sq, core_stream stream);
int core_privacy_loss(double sqnorm, uint32_t m, double sigma1, double sigma2, double *loss);

/* ---- materialised-Xi comparison variant ---------------------------------------------------
 * The matrix Xi = [xi_1 ... xi_m]^T of the paper's privacy appendix (p = Xi a) is normally never
 * stored.  These entry points store it once, while projecting, and read it back to reconstruct,
 * so that "generate twice" can be measured against "generate once + 8 bytes of HBM traffic per
 * normal".  Layout of xi: [ceil(d/4)][m][4] fp32, xi[q][j][k] = xi_j[4q+k]; entries with
 * 4q+k >= d are written but never used.  xi must be 16-byte aligned and hold
 * core_xi_bytes(d, m) bytes (0 = sizes out of range); it is caller-owned device memory. */
size_t core_xi_bytes(uint64_t d, uint32_t m);

/* core_compress_batched that also writes xi (outputs: P (may be NULL), pbar, xi). */
int core_compress_batched_store_xi(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                                   const void *G, core_dtype dt, uint64_t ld,
                                   float *P, float *pbar,
                                   float *xi, size_t xi_buf_bytes,
                                   void *ws, size_t ws_bytes, core_stream stream);

/* Eq. (reconstruction) from a stored xi: gtilde[i] = scale * sum_j pbar[j] xi_j[i]. */
int core_reconstruct_from_xi(uint64_t d, uint32_t m, const float *pbar, float scale,
                             const float *xi, size_t xi_buf_bytes,
                             float *gtilde, core_stream stream);

/* core_round through the stored xi (same outputs as core_round; xi is scratch). */
int core_round_materialized(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                            const void *G, core_dtype dt, uint64_t ld,
                            float *pbar, float *gtilde,
                            float *xi, size_t xi_buf_bytes,
                            void *ws, size_t ws_bytes, core_stream stream);

/* ---- test-only exports: raw generator output -------------------------------- */

/* The launch plan core_compress_batched / core_round would use for these sizes (host arithmetic,
 * nothing is launched; `plan` is a HOST pointer to 10 values):
 *   plan[0] 0 = lanes-over-vectors projection, 1 = lanes-over-coordinates projection (fewer than 5
 *           vectors, or little work), 2 = one workgroup per vector with the sums finished inside it (tiny
 *           problems with at most 8 clients and d <= 65536: projection, cross-chunk sum and client
 *           mean are then a single launch and the workspace is not used)
 *   plan[1] vector tiles (256 vectors each; groups of plan[7] vectors in mode 1; m in mode 2)
 *   plan[2] chunks of d            plan[3] tiles per chunk (256 coordinates each; 1024 in mode 1;
 *                                          Philox blocks per thread in mode 2)
 *   plan[4] slices of the cross-chunk sum
 *   plan[5] projection blocks launched per pass of clients (mode 0: by the 256-vector kernel)
 *   Mode 0 serves the rest m mod 256, when it is at most 192, without half-empty blocks of 256:
 *   plan[8] tiles of 64 vectors that follow the tiles of 256 (a second launch: blocks whose four waves
 *           share the chunk's coordinates), and
 *   plan[6] tiles of plan[9] = 8, 16 or 32 vectors that follow those (a third launch of the same kernel
 *           with the lanes of a wave split between vectors and Philox blocks; both 0 if there are none);
 *   plan[7] vectors per block of the lanes-over-coordinates kernel (4 or 8; 0 if it is not used)
 * Returns CORE_ERR_INVALID_ARGUMENT for sizes out of range. */
int core_debug_plan(uint64_t d, uint32_t m, uint32_t n, uint64_t plan[10]);

/* out[b][0..3] = Philox words of block q0 + b of vector j,  b < nblocks <= 2^28.  out device uint32.
 * (Layout 0 of core_debug_philox_layout with one vector.) */
int core_debug_philox(uint64_t seed, uint64_t round, uint32_t j, uint64_t q0, uint64_t nblocks,
                      uint32_t *out, core_stream stream);

/* The same words for nj vectors x nq blocks, out[jj][qq][0..3] = words of block q0 + qq of vector
 * j0 + jj (Algorithm 1, REQUIRE line: every machine must draw the same stream, so the words must
 * equal the reference generator's bit for bit), produced with the generator instantiation and
 * lane layout of one family of production kernels:
 *   layout 0  every round key on the scalar path, one thread per block
 *   layout 1  the projection kernels: lanes over vectors, the block index wave-uniform
 *   layout 2  the reconstruction kernels and the small-problem projection: lanes over blocks, the
 *             vector index wave-uniform
 *   layout 3  the generator of core_debug_xi
 *   layout 4  the projection of tiles of fewer than 64 vectors: lanes over vectors and blocks at once
 * j0 + nj <= 2^32, q0 + nq <= 2^32, nj * nq <= 2^28.  out device uint32 [nj][nq][4]. */
int core_debug_philox_layout(int layout, uint64_t seed, uint64_t round, uint32_t j0, uint32_t nj,
                             uint64_t q0, uint64_t nq, uint32_t *out, core_stream stream);

/* Force the projection kernel for every later call in this process (A/B measurements and tests
 * that drive each kernel over each shape): 0 = the library's own choice, 1 = vector-ALU kernel
 * with lanes over vectors, 2 = matrix-pipe kernel, 3 = lanes-over-coordinates kernel, 4 = the
 * one-launch kernel for tiny problems where its limits allow (else as 3).  The environment
 * variable CORE_PROJECT_VARIANT = valu | mfma | q | small sets the initial value; it is read
 * once.  Not synchronised with calls in flight on other host threads. */
int core_debug_set_projection(int variant);

/* out[t] = xi_j[i0 + t] as the kernels compute it (fp32), t < count.  out device fp32. */
int core_debug_xi(uint64_t seed, uint64_t round, uint32_t j, uint64_t i0, uint64_t count,
                  float *out, core_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CORE_H_ */
