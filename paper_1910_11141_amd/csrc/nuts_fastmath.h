// Binary64 logistic functions for the batched gradient, written for throughput:
// on this chip binary64 MFMA and binary64 vector instructions do not overlap, so
// every vector instruction spent here is paid in full.
//
// For a logit z the gradient step needs softplus(-z) = log(1 + e^{-z}) and
// sigma(-z) = 1/(1 + e^{z}).  Both come from one even function,
//     F(a) = log(2 cosh(a/2)) = a/2 + log(1 + e^{-a}),  a = |z|:
//     softplus(-z) = F(|z|) - z/2,     sigma(-z) = 1/2 - sign(z) F'(|z|),
// and F is evaluated as a degree-7 polynomial around the nearest multiple of
// 1/16 (y = 16 a - round(16 a) in [-1/2, 1/2]) from a table in LDS, value and
// derivative sharing one Horner sweep (13 FMAs).  Beyond a = 37, F(a) = a/2 to
// rounding, which the last table entry encodes as a straight line, so no
// clamping of z is needed; a NaN or infinite z propagates into the value.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <vector>

namespace nuts {

constexpr int kFtabIntervals = 37 * 16;           // nodes k / 16, k = 0 .. 37 * 16 - 1
constexpr int kFtabEntries = kFtabIntervals + 1;  // + the linear tail
constexpr int kFtabStride = 10;                   // doubles per entry: 8 coefficients, padded to an 80-byte
                                                  // stride so that neighbouring entries fall in different banks
constexpr int kFtabDoubles = kFtabEntries * kFtabStride;
constexpr double kFtabScale = 16.0;               // intervals per unit of a

// Host: fit the table in extended precision (interpolation at Chebyshev nodes of each interval).
inline void build_softplus_table(std::vector<double>* out)
{
    out->assign((size_t)kFtabDoubles, 0.0);
    const long double pi = 3.14159265358979323846264338327950288L;
    for (int k = 0; k < kFtabIntervals; ++k) {
        long double V[8][9];
        for (int i = 0; i < 8; ++i) {
            const long double y = -0.5L * cosl(pi * (2 * i + 1) / 16.0L);  // Chebyshev nodes of [-1/2, 1/2]
            const long double a = ((long double)k + y) / (long double)kFtabScale;
            long double pw = 1.0L;
            for (int j = 0; j < 8; ++j) {
                V[i][j] = pw;
                pw *= y;
            }
            // F(a) = a/2 + log(1 + e^{-a}) holds for every real a (node 0 reaches into a < 0): fit the
            // decaying part, the linear part is added exactly below
            V[i][8] = log1pl(expl(-a));
        }
        for (int col = 0; col < 8; ++col) {  // Gaussian elimination with partial pivoting
            int piv = col;
            for (int r = col + 1; r < 8; ++r)
                if (fabsl(V[r][col]) > fabsl(V[piv][col])) piv = r;
            for (int j = 0; j < 9; ++j) {
                const long double tmp = V[col][j];
                V[col][j] = V[piv][j];
                V[piv][j] = tmp;
            }
            for (int r = 0; r < 8; ++r) {
                if (r == col) continue;
                const long double f = V[r][col] / V[col][col];
                for (int j = col; j < 9; ++j) V[r][j] -= f * V[col][j];
            }
        }
        long double coef[8];
        for (int j = 0; j < 8; ++j) coef[j] = V[j][8] / V[j][j];
        coef[0] += (long double)k / (2.0L * kFtabScale);  // a/2 with a = (k + y)/16
        coef[1] += 1.0L / (2.0L * kFtabScale);
        for (int j = 0; j < 8; ++j) (*out)[(size_t)k * kFtabStride + j] = (double)coef[j];
    }
    // tail: F(a) = a/2 with a = (kFtabIntervals + y) / 16
    (*out)[(size_t)kFtabIntervals * kFtabStride + 0] = (double)kFtabIntervals / (2.0 * kFtabScale);
    (*out)[(size_t)kFtabIntervals * kFtabStride + 1] = 1.0 / (2.0 * kFtabScale);
}

// value = F(|z|);  dslope = dF/dy = F'(|z|) / 16  (y is the position inside the interval).
__device__ __forceinline__ void softplus_sym(double z, const double* __restrict__ tab, double& value, double& dslope)
{
    // 16|z| + (2^52 + 2^32) rounds to an integer whose low word is the node index round(16|z|)
    constexpr double kMagic = 0x1p52 + 0x1p32;
    const double a16 = fabs(z) * kFtabScale;  // exact (a power of two), so the sums below round as the fused forms would
    const double m = fmin(a16 + kMagic, kMagic + (double)kFtabIntervals);
    const double kf = m - kMagic;
    const double y = a16 - kf;
    const int byte_off = (int)__umul24((unsigned)__double2loint(m), (unsigned)(kFtabStride * sizeof(double)));
    const double2* c = reinterpret_cast<const double2*>(reinterpret_cast<const char*>(tab) + byte_off);
    const double2 c01 = c[0], c23 = c[1], c45 = c[2], c67 = c[3];
    double p = fma(c67.y, y, c67.x);
    double d = fma(c67.y, y, p);
    p = fma(p, y, c45.y);
    d = fma(d, y, p);
    p = fma(p, y, c45.x);
    d = fma(d, y, p);
    p = fma(p, y, c23.y);
    d = fma(d, y, p);
    p = fma(p, y, c23.x);
    d = fma(d, y, p);
    p = fma(p, y, c01.y);
    d = fma(d, y, p);
    p = fma(p, y, c01.x);
    value = p;
    dslope = d;
}

// For two finite log-weights: log(e^a + e^b), and the probability e^b / (e^a + e^b).
__device__ __forceinline__ void merge_logweights(double a, double b, const double* tab, double& lse, double& p_b)
{
    const double diff = b - a;
    double val, dy;
    softplus_sym(diff, tab, val, dy);
    lse = 0.5 * (a + b) + val;  // max + log(1 + e^-|diff|)
    p_b = 0.5 + __builtin_copysign(dy * kFtabScale, diff);
}

}  // namespace nuts
