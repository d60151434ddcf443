/*
 * CORE (Common Random Reconstruction) -- CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, fp64
 * definition of what the GPU library computes.  Nothing in the product path
 * may link, load or call it; it shares no code, header, table or constant
 * generator with the HIP kernels.
 *
 * What is computed (citations are to the paper, arXiv 2309.13307):
 *   - Algorithm 1 (Section 3): compression p_j = <a, xi_j>, j = 1..m, and the
 *     reconstruction of Eq. (reconstruction), a~ = (1/m) sum_j p_j xi_j.
 *   - Eq. (tildefdef) (Section 4): with n machines every machine projects onto
 *     the SAME xi_j; the estimator is (1/(n m)) sum_i sum_j <grad f_i, xi_j> xi_j.
 *     Appendix "decentralized CORE-GD" writes the client mean explicitly,
 *     p_j = (1/n) sum_i p_ij.
 *   - Algorithm 2 (Section 4), the three communication lines: machine i sends
 *     p_ij, the centre combines them over i, machines reconstruct.
 *
 * The paper only asks for "a common random number generator" producing fresh
 * i.i.d. N(0, I_d) vectors (Section 3, Algorithm 1 REQUIRE line).  The
 * generator convention used here is fixed by this build:
 *   - Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), counter-based.
 *   - key     = (seed mod 2^32, seed div 2^32)
 *   - counter = (q, j, round mod 2^32, round div 2^32),  q = floor(i / 4)
 *     one call yields xi_j[4q .. 4q+3]; j is 0-based; i is 0-based.
 *   - each 32-bit word x gives a 24-bit uniform: u1 = ((x>>8)+1) 2^-24 in (0,1],
 *     u2 = (x>>8) 2^-24 in [0,1);  Box-Muller on word pairs (x0,x1), (x2,x3):
 *     r = sqrt(-2 ln u1), z_even = r cos(2 pi u2), z_odd = r sin(2 pi u2).
 *
 * Every floating-point quantity is fp64; inputs are taken exactly as stored
 * (fp64, fp32, or bf16 widened exactly).  Sums run in index order.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/* ---- Philox4x32-10 -------------------------------------------------------- */

/* One Philox4x32 round: two 32x32->64 products, a fixed word shuffle, and the
 * round key folded into the two high halves. */
void core_oracle_philox_round(uint32_t c[4], const uint32_t k[2])
{
    const uint64_t prod_a = (uint64_t)0xD2511F53u * (uint64_t)c[0];
    const uint64_t prod_b = (uint64_t)0xCD9E8D57u * (uint64_t)c[2];
    const uint32_t hi_a = (uint32_t)(prod_a >> 32), lo_a = (uint32_t)prod_a;
    const uint32_t hi_b = (uint32_t)(prod_b >> 32), lo_b = (uint32_t)prod_b;
    const uint32_t n0 = hi_b ^ c[1] ^ k[0];
    const uint32_t n2 = hi_a ^ c[3] ^ k[1];
    c[0] = n0;
    c[1] = lo_b;
    c[2] = n2;
    c[3] = lo_a;
}

/* Ten rounds; the key is advanced by the Weyl constants between rounds. */
void core_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                               uint32_t out[4])
{
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    uint32_t k[2] = { key[0], key[1] };
    for (int r = 0; r < 10; ++r) {
        core_oracle_philox_round(c, k);
        k[0] += 0x9E3779B9u;
        k[1] += 0xBB67AE85u;
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* ---- uniform map and Box-Muller ------------------------------------------- */

/* Two words -> two independent standard normals. */
void core_oracle_box_muller(uint32_t xa, uint32_t xb, double *z_even, double *z_odd)
{
    const double two_pi = 6.283185307179586476925286766559;
    const double u1 = ((double)(xa >> 8) + 1.0) / 16777216.0; /* (0, 1] */
    const double u2 = (double)(xb >> 8) / 16777216.0;         /* [0, 1) */
    const double r = sqrt(-2.0 * log(u1));
    *z_even = r * cos(two_pi * u2);
    *z_odd  = r * sin(two_pi * u2);
}

/* The generator's words for block q of vector j in a given (seed, round). */
void core_oracle_words(uint64_t seed, uint64_t round, uint32_t j, uint64_t q,
                       uint32_t w[4])
{
    const uint32_t ctr[4] = { (uint32_t)q, j, (uint32_t)round, (uint32_t)(round >> 32) };
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    core_oracle_philox4x32_10(ctr, key, w);
}

/* xi_j[4q .. 4q+3] */
void core_oracle_xi_block(uint64_t seed, uint64_t round, uint32_t j, uint64_t q,
                          double z[4])
{
    uint32_t w[4];
    core_oracle_words(seed, round, j, q, w);
    core_oracle_box_muller(w[0], w[1], &z[0], &z[1]);
    core_oracle_box_muller(w[2], w[3], &z[2], &z[3]);
}

/* xi_j[i] */
double core_oracle_xi(uint64_t seed, uint64_t round, uint32_t j, uint64_t i)
{
    double z[4];
    core_oracle_xi_block(seed, round, j, i >> 2, z);
    return z[i & 3];
}

/* out[t] = xi_j[i0 + t], t < count */
void core_oracle_xi_fill(uint64_t seed, uint64_t round, uint32_t j, uint64_t i0,
                         uint64_t count, double *out)
{
    for (uint64_t t = 0; t < count; ++t) out[t] = core_oracle_xi(seed, round, j, i0 + t);
}

/* ---- inputs as stored ------------------------------------------------------ */

enum { ORACLE_F64 = 0, ORACLE_F32 = 1, ORACLE_BF16 = 2 };

static double load_elem(const void *base, int dtype, uint64_t idx)
{
    if (dtype == ORACLE_F64) return ((const double *)base)[idx];
    if (dtype == ORACLE_F32) return (double)((const float *)base)[idx];
    /* bf16: the upper 16 bits of an fp32 */
    union { uint32_t u; float f; } cvt;
    cvt.u = (uint32_t)((const uint16_t *)base)[idx] << 16;
    return (double)cvt.f;
}

/* ---- Algorithm 1, compression line; Algorithm 2, "machine i sends p_ij" ---- */

/* P[c][t] = sum_{i<d} G[c][i] * xi_{jidx[t]}[i]   for c < n, t < nj.
 * G is [n][ld] row-major of the given dtype.  xi_j[i] is evaluated once per
 * (j, i) and used for every client, which is the method's point: all machines
 * share the vector.  Returns 0, or -1 on a bad argument. */
int core_oracle_compress(uint64_t seed, uint64_t round, uint64_t d, uint32_t n,
                         const void *G, int dtype, uint64_t ld,
                         const uint32_t *jidx, uint64_t nj, double *P)
{
    if (!G || !jidx || !P || d == 0 || n == 0 || ld < d) return -1;
    if (dtype < ORACLE_F64 || dtype > ORACLE_BF16) return -1;
    for (uint64_t t = 0; t < nj; ++t) {
        const uint32_t j = jidx[t];
        for (uint32_t c = 0; c < n; ++c) P[(uint64_t)c * nj + t] = 0.0;
        for (uint64_t q = 0; 4 * q < d; ++q) {
            double z[4];
            core_oracle_xi_block(seed, round, j, q, z);
            for (int k = 0; k < 4; ++k) {
                const uint64_t i = 4 * q + (uint64_t)k;
                if (i >= d) break; /* normals past the end of the vector are dropped */
                for (uint32_t c = 0; c < n; ++c)
                    P[(uint64_t)c * nj + t] += load_elem(G, dtype, (uint64_t)c * ld + i) * z[k];
            }
        }
    }
    return 0;
}

/* ---- client mean, p_j = (1/n) sum_i p_ij ----------------------------------- */

int core_oracle_client_mean(const double *P, uint32_t n, uint64_t nj, double *pbar)
{
    if (!P || !pbar || n == 0) return -1;
    for (uint64_t t = 0; t < nj; ++t) {
        double s = 0.0;
        for (uint32_t c = 0; c < n; ++c) s += P[(uint64_t)c * nj + t];
        pbar[t] = s / (double)n;
    }
    return 0;
}

/* ---- Eq. (reconstruction) -------------------------------------------------- */

/* out[t] = scale * sum_{j<m} pbar[j] * xi_j[i0 + t]   for t < count.
 * scale = 1/m gives Eq. (reconstruction) / Eq. (tildefdef) on a client mean. */
int core_oracle_reconstruct(uint64_t seed, uint64_t round, uint32_t m,
                            const double *pbar, double scale,
                            uint64_t i0, uint64_t count, double *out)
{
    if (!pbar || !out || m == 0) return -1;
    if (count == 0) return 0;
    /* The generator hands out four coordinates per call, so walk the range one
     * generator block at a time; each coordinate's sum still runs over j in order. */
    const uint64_t i_end = i0 + count;
    for (uint64_t q = i0 >> 2; 4 * q < i_end; ++q) {
        double s[4] = { 0.0, 0.0, 0.0, 0.0 };
        for (uint32_t j = 0; j < m; ++j) {
            double z[4];
            core_oracle_xi_block(seed, round, j, q, z);
            for (int k = 0; k < 4; ++k) s[k] += pbar[j] * z[k];
        }
        for (int k = 0; k < 4; ++k) {
            const uint64_t i = 4 * q + (uint64_t)k;
            if (i >= i0 && i < i_end) out[i - i0] = scale * s[k];
        }
    }
    return 0;
}

/* ---- one communication round of Algorithm 2 (without the x update) --------- */

/* P[c][j] = <G[c], xi_j>,  pbar[j] = (1/n) sum_c P[c][j],
 * gtilde = (1/m) sum_j pbar[j] xi_j.   P is [n][m], pbar [m], gtilde [d]. */
int core_oracle_round(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n,
                      const void *G, int dtype, uint64_t ld,
                      const uint32_t *all_j /* 0..m-1 */,
                      double *P, double *pbar, double *gtilde)
{
    if (!all_j || !P || !pbar || !gtilde || m == 0) return -1;
    if (core_oracle_compress(seed, round, d, n, G, dtype, ld, all_j, m, P)) return -1;
    if (core_oracle_client_mean(P, n, m, pbar)) return -1;
    return core_oracle_reconstruct(seed, round, m, pbar, 1.0 / (double)m, 0, d, gtilde);
}
