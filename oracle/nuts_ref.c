/*
 * Reference ("oracle") implementation of multi-chain NUTS on the CPU.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists to define, in the plainest
 * possible way, what the GPU library must compute.  It is recursive, slow and
 * unoptimised on purpose, it shares no code, header, table or helper with the
 * HIP path, and only the test-suite, the smoke check and the CPU-baseline leg
 * of the benchmark may load it.  Nothing in the product path may call it.
 *
 * What it follows.  The paper (Radul et al., "Automatically batching
 * control-intensive programs for modern accelerators", Sections 3-4) batches
 * the No-U-Turn Sampler, which is usually presented as a recursive function
 * (Section 4).  The paper does not restate NUTS, so the recursion
 * below is the published tree-doubling scheme in its multinomial form:
 *   - one leapfrog step per tree leaf (nuts_ref_sample_k: a fixed number k of them),
 *   - uniform progressive (multinomial) selection inside a subtree,
 *     biased progressive selection min(1, w'/w) at the top level,
 *   - the end-point U-turn criterion on every merged subtree and on the whole
 *     trajectory, continuing while both dot products are >= 0,
 *   - a leaf whose energy error exceeds 1000 (or is not finite) is divergent:
 *     it has weight zero and stops the trajectory,
 *   - identity mass matrix, fixed step size, no adaptation.
 * Every random number is a pure function of (seed, chain, iteration, purpose,
 * position) through the Philox4x32-10 counter generator (Salmon et al., SC'11),
 * so the outcome does not depend on the order in which chains are advanced
 * (the per-member independence argument of Section 2 of the paper).
 *
 * Precision.  `NUTS_REF_F64`: everything in binary64.  `NUTS_REF_F32`: state
 * vectors and target data are binary32 and element-wise updates round to
 * binary32; every reduction (dot products, log-density sums, matrix-vector
 * products) accumulates in binary64 in ascending index order, and all decision
 * scalars (energies, log-weights, U-turn dot products) are binary64.
 * Compile with -ffp-contract=off so a*b+c is two roundings.
 *
 * Pins.  Every exported function is pinned by tests/test_oracle_*.py against
 * closed forms, invariants, brute force or independent re-derivations; see the
 * docstrings there.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { NUTS_REF_F32 = 0, NUTS_REF_F64 = 1 };
enum {
    NUTS_REF_STD_NORMAL = 0,  /* log p = -1/2 |x|^2                              */
    NUTS_REF_GAUSS_DENSE = 1, /* log p = -1/2 x' P x, P given                     */
    NUTS_REF_GAUSS_DIAG = 2,  /* log p = -1/2 sum x_i^2 / sigma_i^2               */
    NUTS_REF_LOGREG = 3       /* Bernoulli-logit likelihood, N(0, s^2 I) prior    */
};
/* purposes of a random draw; they go into counter word 1 */
enum { TAG_INIT = 0, TAG_MOMENTUM = 1, TAG_DIRECTION = 2, TAG_SUBTREE = 3, TAG_TOP = 4, TAG_SLICE = 5 };
/* how candidates are weighted: by exp(-H) (multinomial), or equally under a slice (the published form) */
enum { NUTS_REF_MULTINOMIAL = 0, NUTS_REF_SLICE = 1 };

#define DELTA_MAX 1000.0

/* ---------------------------------------------------------------- Philox -- */

/* One Philox4x32 block with 10 rounds: the bijection of Salmon et al. (SC'11),
 * Section 3.3: two 32x32->64 multiplications per round, the high halves are
 * xored with the neighbouring counter word and a round key, the key is bumped
 * by the Weyl constants between rounds. */
void nuts_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The draw for (seed; index, purpose, level, iteration, chain). */
void nuts_ref_draw(uint64_t seed, uint32_t index, uint32_t tag, uint32_t level,
                   uint32_t iteration, uint32_t chain, uint32_t out[4])
{
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { index, tag | (level << 8), iteration, chain };
    nuts_ref_philox4x32_10(ctr, key, out);
}

/* 52 random bits -> the midpoint of one of 2^52 equal cells of (0,1); the value
 * is exact in binary64 and never 0 or 1. */
double nuts_ref_uniform(uint32_t a, uint32_t b)
{
    uint64_t m = ((uint64_t)(a >> 6) << 26) | (uint64_t)(b >> 6);
    return (double)(2 * m + 1) * 0x1p-53;
}

/* Box-Muller: two independent standard normals from one Philox block. */
void nuts_ref_normal_pair(const uint32_t w[4], double z[2])
{
    double u1 = nuts_ref_uniform(w[0], w[1]);
    double u2 = nuts_ref_uniform(w[2], w[3]);
    double rho = sqrt(-2.0 * log(u1));
    double phi = 6.283185307179586476925286766559 * u2;
    z[0] = rho * cos(phi);
    z[1] = rho * sin(phi);
}

/* log(exp(a) + exp(b)), with -inf as the log of zero weight. */
double nuts_ref_logaddexp(double a, double b)
{
    double m = a > b ? a : b;
    if (m == -INFINITY) return -INFINITY;
    return m + log1p(exp(-fabs(a - b)));
}

/* ------------------------------------------------- typed implementations -- */

#define REAL double
#define FN(name) name##_f64
#include "nuts_ref_typed.inc"
#undef REAL
#undef FN

#define REAL float
#define FN(name) name##_f32
#include "nuts_ref_typed.inc"
#undef REAL
#undef FN

/* ------------------------------------------------------------ public API -- */

/* log-density and gradient of a target at one point.
 * Data pointers are host arrays of the target's dtype:
 *   precision  [dim*dim] row-major  (GAUSS_DENSE)
 *   scales     [dim] sigma_i        (GAUSS_DIAG)
 *   X [n_data*dim] row-major, y [n_data] in {0,1}, prior_scale   (LOGREG)
 * Returns 0, or -1 on a bad argument. */
int nuts_ref_logp_grad(int dtype, int kind, int64_t dim, const void* precision, const void* scales,
                       const void* X, const void* y, int64_t n_data, double prior_scale,
                       const void* theta, void* grad_out, double* logp_out)
{
    if (dtype == NUTS_REF_F64)
        return logp_grad_api_f64(kind, dim, precision, scales, X, y, n_data, prior_scale, theta, grad_out, logp_out);
    if (dtype == NUTS_REF_F32)
        return logp_grad_api_f32(kind, dim, precision, scales, X, y, n_data, prior_scale, theta, grad_out, logp_out);
    return -1;
}

/* n_steps leapfrog steps of signed size h from (theta, r), in place.
 * logp_out receives the log-density at the end point. */
int nuts_ref_leapfrog(int dtype, int kind, int64_t dim, const void* precision, const void* scales,
                      const void* X, const void* y, int64_t n_data, double prior_scale,
                      void* theta, void* r, double h, int64_t n_steps, double* logp_out)
{
    if (dtype == NUTS_REF_F64)
        return leapfrog_api_f64(kind, dim, precision, scales, X, y, n_data, prior_scale, theta, r, h, n_steps, logp_out);
    if (dtype == NUTS_REF_F32)
        return leapfrog_api_f32(kind, dim, precision, scales, X, y, n_data, prior_scale, theta, r, h, n_steps, logp_out);
    return -1;
}

/* 1 if the trajectory with ends (theta_minus, r_minus), (theta_plus, r_plus)
 * has not turned back on itself. */
int nuts_ref_uturn_ok(int dtype, int64_t dim, const void* theta_minus, const void* r_minus,
                      const void* theta_plus, const void* r_plus)
{
    double margin = INFINITY;
    if (dtype == NUTS_REF_F64) return uturn_ok_f64(dim, theta_minus, r_minus, theta_plus, r_plus, &margin);
    if (dtype == NUTS_REF_F32) return uturn_ok_f32(dim, theta_minus, r_minus, theta_plus, r_plus, &margin);
    return -1;
}

/* Run NUTS for a set of chains.
 *   chain_ids   NULL: chains 0..n_chains-1; else the global ids to run (a chain's
 *               result depends on its id only, never on its companions)
 *   init_states NULL: x0 ~ N(0, I) from the INIT draws; else [n_chains][dim]
 *   out_states  [n_iters][n_chains][dim] of the target's dtype
 *   out_tree_depths, out_n_leapfrog  [n_iters][n_chains] int32
 *   out_margin  optional [n_iters][n_chains]: the smallest distance of any
 *               decision taken in that iteration from its threshold (diagnostic)
 *   n_threads   worker threads (chains are split evenly); <= 0 means 1
 *   sampler     NUTS_REF_MULTINOMIAL (the form described at the top of this file) or NUTS_REF_SLICE
 *               (Algorithm 3 of Hoffman & Gelman, JMLR 2014: see build_slice in nuts_ref_typed.inc)
 *   leaf_steps  leapfrog steps per tree leaf: 1 is the published algorithm; the paper's own runs
 *               used 4 (Section 4.1).  out_n_leapfrog counts leapfrog steps, i.e. leaf_steps per leaf.
 * Any output pointer may be NULL.  Returns 0, or -1 on a bad argument. */
int nuts_ref_sample_k(int dtype, int kind, int64_t dim, const void* precision, const void* scales,
                      const void* X, const void* y, int64_t n_data, double prior_scale,
                      int64_t n_chains, const int64_t* chain_ids, const void* init_states,
                      int64_t n_iters, double step_size, int32_t max_tree_depth, int32_t leaf_steps, int32_t sampler,
                      uint64_t seed, void* out_states, int32_t* out_tree_depths, int32_t* out_n_leapfrog,
                      double* out_margin, int32_t n_threads)
{
    if (n_chains < 1 || n_iters < 1 || dim < 1) return -1;
    if (leaf_steps < 1 || leaf_steps > 64) return -1;
    if (sampler != NUTS_REF_MULTINOMIAL && sampler != NUTS_REF_SLICE) return -1;
    if (!(step_size > 0.0) || !isfinite(step_size)) return -1;
    if (max_tree_depth < 1 || max_tree_depth > 20) return -1;
    if (dtype == NUTS_REF_F64)
        return sample_api_f64(kind, dim, precision, scales, X, y, n_data, prior_scale, n_chains, chain_ids,
                              init_states, n_iters, step_size, max_tree_depth, leaf_steps, sampler, seed, out_states,
                              out_tree_depths, out_n_leapfrog, out_margin, n_threads);
    if (dtype == NUTS_REF_F32)
        return sample_api_f32(kind, dim, precision, scales, X, y, n_data, prior_scale, n_chains, chain_ids,
                              init_states, n_iters, step_size, max_tree_depth, leaf_steps, sampler, seed, out_states,
                              out_tree_depths, out_n_leapfrog, out_margin, n_threads);
    return -1;
}

/* Multinomial sampler, one leapfrog step per leaf. */
int nuts_ref_sample(int dtype, int kind, int64_t dim, const void* precision, const void* scales,
                    const void* X, const void* y, int64_t n_data, double prior_scale,
                    int64_t n_chains, const int64_t* chain_ids, const void* init_states,
                    int64_t n_iters, double step_size, int32_t max_tree_depth, uint64_t seed,
                    void* out_states, int32_t* out_tree_depths, int32_t* out_n_leapfrog,
                    double* out_margin, int32_t n_threads)
{
    return nuts_ref_sample_k(dtype, kind, dim, precision, scales, X, y, n_data, prior_scale, n_chains, chain_ids,
                             init_states, n_iters, step_size, max_tree_depth, 1, NUTS_REF_MULTINOMIAL, seed, out_states, out_tree_depths,
                             out_n_leapfrog, out_margin, n_threads);
}
