// Binary64 logistic functions for the batched gradient, written for throughput:
// on this chip binary64 MFMA and binary64 vector instructions do not overlap, so
// every vector instruction spent here is paid in full.
//
// For a logit z the gradient step needs softplus(-z) = log(1 + e^{-z}) and
// sigma(-z) = 1/(1 + e^{z}).  Both come from one even function,
//     F(a) = log(2 cosh(a/2)) = a/2 + log(1 + e^{-a}),  a = |z|:
//     softplus(-z) = F(|z|) - z/2,     sigma(-z) = 1/2 - sign(z) F'(|z|),
// with F'(a) = tanh(a/2)/2 = sigma(a) - 1/2.  F' is evaluated as a degree-6
// polynomial around the nearest multiple of 1/16 (y = 16 a - round(16 a) in
// [-1/2, 1/2]) from a table in LDS: 6 FMAs.  The gradient loop never evaluates F
// itself: sum_i log(1 + e^{-a_i}) = -log prod_i sigma(a_i), so it multiplies the
// sigma(a_i) = F'(a_i) + 1/2 together and takes one logarithm per lane and round.
// Where F of a single argument is wanted (the weight merges of the chain program),
// it is the table's F at the node plus the integral of the same polynomial.
// Beyond a = 37, F'(a) = 1/2 and F(a) = a/2 to rounding, which the last table
// entry encodes, so no clamping of z is needed; a NaN or infinite z propagates.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <vector>

namespace nuts {

constexpr int kFtabIntervals = 37 * 16;           // nodes k / 16, k = 0 .. 37 * 16 - 1
constexpr int kFtabEntries = kFtabIntervals + 1;  // + the linear tail
constexpr int kFtabStride = 10;                   // doubles per entry: 7 coefficients of F' and F at the node, padded
                                                  // to an 80-byte stride so that neighbouring entries fall in different banks
constexpr int kFtabDoubles = kFtabEntries * kFtabStride;
constexpr double kFtabScale = 16.0;               // intervals per unit of a

// Host: fit the table in extended precision (interpolation at Chebyshev nodes of each interval).
inline void build_softplus_table(std::vector<double>* out)
{
    out->assign((size_t)kFtabDoubles, 0.0);
    const long double pi = 3.14159265358979323846264338327950288L;
    constexpr int kC = 7;  // coefficients of F'
    for (int k = 0; k < kFtabIntervals; ++k) {
        long double V[kC][kC + 1];
        for (int i = 0; i < kC; ++i) {
            const long double y = -0.5L * cosl(pi * (2 * i + 1) / (2.0L * kC));  // Chebyshev nodes of [-1/2, 1/2]
            const long double a = ((long double)k + y) / (long double)kFtabScale;  // (node 0 reaches into a < 0)
            long double pw = 1.0L;
            for (int j = 0; j < kC; ++j) {
                V[i][j] = pw;
                pw *= y;
            }
            V[i][kC] = 0.5L * tanhl(0.5L * a);
        }
        for (int col = 0; col < kC; ++col) {  // Gaussian elimination with partial pivoting
            int piv = col;
            for (int r = col + 1; r < kC; ++r)
                if (fabsl(V[r][col]) > fabsl(V[piv][col])) piv = r;
            for (int j = 0; j <= kC; ++j) {
                const long double tmp = V[col][j];
                V[col][j] = V[piv][j];
                V[piv][j] = tmp;
            }
            for (int r = 0; r < kC; ++r) {
                if (r == col) continue;
                const long double f = V[r][col] / V[col][col];
                for (int j = col; j <= kC; ++j) V[r][j] -= f * V[col][j];
            }
        }
        for (int j = 0; j < kC; ++j) (*out)[(size_t)k * kFtabStride + j] = (double)(V[j][kC] / V[j][j]);
        const long double node = (long double)k / (long double)kFtabScale;
        (*out)[(size_t)k * kFtabStride + kC] = (double)(0.5L * node + log1pl(expl(-node)));
    }
    // tail: F'(a) = 1/2, F(a) = a/2 with a = (kFtabIntervals + y) / 16
    (*out)[(size_t)kFtabIntervals * kFtabStride + 0] = 0.5;
    (*out)[(size_t)kFtabIntervals * kFtabStride + kC] = (double)kFtabIntervals / (2.0 * kFtabScale);
}

// ---- logarithm of a product of sigmas ----------------------------------------
// log x for 0 < x <= 1 (x = m 2^e, m in [1/2, 1)): a table over the top 7 bits of the mantissa
// holds inv ~ 1/c (c the middle of the cell) and -log(inv), so that r = m inv - 1 is exact in one
// FMA and |r| < 2^-8; then log x = e ln 2 - log(inv) + log1p(r) with a degree-7 series.
// About 20 instructions instead of the 90 of the library routine; error below 2 ulp.
constexpr int kLogTabEntries = 128;
constexpr int kLogTabDoubles = 2 * kLogTabEntries;

inline void build_log_table(std::vector<double>* out)
{
    out->assign((size_t)kLogTabDoubles, 0.0);
    for (int i = 0; i < kLogTabEntries; ++i) {
        const long double c = 0.5L + ((long double)i + 0.5L) / 256.0L;
        const double inv = (double)(1.0L / c);
        (*out)[2 * i] = inv;
        (*out)[2 * i + 1] = (double)(-logl((long double)inv));
    }
}

__device__ __forceinline__ double log_unit(double x, const double* __restrict__ logtab)
{
    const int e = __builtin_amdgcn_frexp_exp(x);     // x = m 2^e
    const double m = __builtin_amdgcn_frexp_mant(x);  // [1/2, 1)
    const unsigned cell = ((unsigned)__double2hiint(m) >> 13) & (kLogTabEntries - 1);  // top 7 mantissa bits
    const double2 t = reinterpret_cast<const double2*>(logtab)[cell];
    const double r = fma(m, t.x, -1.0);
    double p = fma(r, 1.0 / 7.0, -1.0 / 6.0);
    p = fma(p, r, 0.2);
    p = fma(p, r, -0.25);
    p = fma(p, r, 1.0 / 3.0);
    p = fma(p, r, -0.5);
    p = fma(p * r, r, r);
    return fma((double)e, 0.69314718055994530942, t.y + p);
}

// ---- a point of the unit circle ------------------------------------------------
// sin(phi) or cos(phi) for an angle in [0, 2 pi], the angle of a Box-Muller draw.  The library routine
// carries the reduction of arbitrarily large arguments along (a wave executes both of its paths); here
// the quarter turn q = round(phi / (pi/2)) is at most 4, phi - q pi/2 is exact in one FMA against the
// leading 53 bits of pi/2 (both terms are multiples of 2^-52 below 8) and the next 53 bits correct it.
// On |r| <= pi/4 the Taylor polynomials to r^15 and r^16 leave less than 7e-17 of the value.
__device__ __forceinline__ double circle_point(double phi, bool sine)
{
    const double q = rint(phi * 0.63661977236758134308);
    double r = fma(q, -1.57079632679489655800, phi);
    r = fma(q, -6.12323399573676603587e-17, r);
    const double r2 = r * r;
    double ps = fma(r2, -1.0 / 1307674368000.0, 1.0 / 6227020800.0);
    double pc = fma(r2, 1.0 / 20922789888000.0, -1.0 / 87178291200.0);
    ps = fma(ps, r2, -1.0 / 39916800.0);
    pc = fma(pc, r2, 1.0 / 479001600.0);
    ps = fma(ps, r2, 1.0 / 362880.0);
    pc = fma(pc, r2, -1.0 / 3628800.0);
    ps = fma(ps, r2, -1.0 / 5040.0);
    pc = fma(pc, r2, 1.0 / 40320.0);
    ps = fma(ps, r2, 1.0 / 120.0);
    pc = fma(pc, r2, -1.0 / 720.0);
    ps = fma(ps, r2, -1.0 / 6.0);
    pc = fma(pc, r2, 1.0 / 24.0);
    const double sn = fma(r * r2, ps, r);                // sin r
    const double cs = fma(r2, fma(pc, r2, -0.5), 1.0);  // cos r
    // sin(phi) = sin(r + q pi/2); cos(phi) = sin(phi + pi/2)
    const int n = (int)q + (sine ? 0 : 1);
    const double v = (n & 1) ? cs : sn;
    return (n & 2) ? -v : v;
}

// ---- the weight of a trajectory point -------------------------------------------
// e^x for x <= 700 (the tile kernel keeps a trajectory's weights as numbers, not logarithms, in a unit that
// it moves when the energy falls far): 0 below -745 and for -infinity (a divergent leaf).  x = k ln 2 + r with
// |r| <= ln(2)/2; k ln2_hi is exact (ln2_hi has 33 bits); on that range the Taylor polynomial to r^13 leaves
// less than 1e-17 of the value.
__device__ __forceinline__ double exp_bounded(double x)
{
    const double xc = fmax(x, -800.0);
    const double kf = rint(xc * 1.4426950408889634);
    double r = fma(kf, -0x1.62e42fef00000p-1, xc);
    r = fma(kf, -0x1.473de6af278edp-34, r);
    // (Horner's form on purpose: the phases of the chain program are bound by how many instructions they issue,
    // and the shallower Estrin form, three instructions longer, measured slower)
    double p = fma(r, 1.0 / 6227020800.0, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)kf);
}

// Table entry and position inside its interval for |z|.
__device__ __forceinline__ const double2* ftab_entry(double z, const double* __restrict__ tab, double& y)
{
    // 16|z| + (2^52 + 2^32) rounds to an integer whose low word is the node index round(16|z|)
    constexpr double kMagic = 0x1p52 + 0x1p32;
    const double m = fmin(fma(fabs(z), kFtabScale, kMagic), kMagic + (double)kFtabIntervals);
    const double kf = m - kMagic;
    y = fma(fabs(z), kFtabScale, -kf);  // exact product, one rounding
    const int byte_off = (int)__umul24((unsigned)__double2loint(m), (unsigned)(kFtabStride * sizeof(double)));
    return reinterpret_cast<const double2*>(reinterpret_cast<const char*>(tab) + byte_off);
}

// slope = F'(|z|) = sigma(|z|) - 1/2, in [0, 1/2].
__device__ __forceinline__ double logistic_slope(double z, const double* __restrict__ tab)
{
    double y;
    const double2* c = ftab_entry(z, tab, y);
    const double2 c01 = c[0], c23 = c[1], c45 = c[2];
    const double c6 = reinterpret_cast<const double*>(c)[6];
    double d = fma(c6, y, c45.y);
    d = fma(d, y, c45.x);
    d = fma(d, y, c23.y);
    d = fma(d, y, c23.x);
    d = fma(d, y, c01.y);
    d = fma(d, y, c01.x);
    return d;
}

// F' of kN logits at once, step by step across all of them: the gradient loop shares a SIMD with
// another wave's MFMAs, each of which holds the issue port for 64 ticks, so what counts there is how
// many dependent steps the section has, not only how many instructions.
template <int kN>
__device__ __forceinline__ void logistic_slopes(const double (&z)[kN], const double* __restrict__ tab, double (&slope)[kN])
{
    double y[kN], c6[kN];
    double2 c01[kN], c23[kN], c45[kN];
#pragma unroll
    for (int i = 0; i < kN; ++i) {
        const double2* c = ftab_entry(z[i], tab, y[i]);
        c45[i] = c[2];
        c6[i] = reinterpret_cast<const double*>(c)[6];
        c23[i] = c[1];
        c01[i] = c[0];
    }
#pragma unroll
    for (int i = 0; i < kN; ++i) slope[i] = fma(c6[i], y[i], c45[i].y);
#pragma unroll
    for (int i = 0; i < kN; ++i) slope[i] = fma(slope[i], y[i], c45[i].x);
#pragma unroll
    for (int i = 0; i < kN; ++i) slope[i] = fma(slope[i], y[i], c23[i].y);
#pragma unroll
    for (int i = 0; i < kN; ++i) slope[i] = fma(slope[i], y[i], c23[i].x);
#pragma unroll
    for (int i = 0; i < kN; ++i) slope[i] = fma(slope[i], y[i], c01[i].y);
#pragma unroll
    for (int i = 0; i < kN; ++i) slope[i] = fma(slope[i], y[i], c01[i].x);
}

// value = F(|z|);  slope = F'(|z|).
__device__ __forceinline__ void softplus_sym(double z, const double* __restrict__ tab, double& value, double& slope)
{
    double y;
    const double2* c = ftab_entry(z, tab, y);
    const double2 c01 = c[0], c23 = c[1], c45 = c[2], c67 = c[3];  // c67.y is F at the node
    double d = fma(c67.x, y, c45.y);
    d = fma(d, y, c45.x);
    d = fma(d, y, c23.y);
    d = fma(d, y, c23.x);
    d = fma(d, y, c01.y);
    d = fma(d, y, c01.x);
    slope = d;
    // F(node + y/16) = F(node) + (y/16) (c0 + c1 y/2 + ... + c6 y^6/7)
    double q = c67.x * (1.0 / 7.0);
    q = fma(q, y, c45.y * (1.0 / 6.0));
    q = fma(q, y, c45.x * 0.2);
    q = fma(q, y, c23.y * 0.25);
    q = fma(q, y, c23.x * (1.0 / 3.0));
    q = fma(q, y, c01.y * 0.5);
    q = fma(q, y, c01.x);
    value = fma(q, y * (1.0 / kFtabScale), c67.y);
}

// For two finite log-weights: log(e^a + e^b), and the probability e^b / (e^a + e^b).
__device__ __forceinline__ void merge_logweights(double a, double b, const double* tab, double& lse, double& p_b)
{
    const double diff = b - a;
    double val, slope;
    softplus_sym(diff, tab, val, slope);
    lse = 0.5 * (a + b) + val;  // max + log(1 + e^-|diff|)
    p_b = 0.5 + __builtin_copysign(slope, diff);
}

}  // namespace nuts
