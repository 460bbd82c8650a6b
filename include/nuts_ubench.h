/*
 * nuts_ubench.h - C ABI of the instruction-issue microbenchmark (libnuts_ubench.so).
 *
 * Not part of the sampler: a measurement tool that backs the roofline discussion of the
 * logistic-regression kernels.  The unit the paper counts is one gradient evaluation (Section 4.1);
 * how many of them a compute unit can do per second is bounded by how its SIMDs issue matrix and
 * vector instructions, which is what this library times.
 */
#ifndef NUTS_UBENCH_H_
#define NUTS_UBENCH_H_

#ifdef __cplusplus
extern "C" {
#endif

/* One workgroup of 8 waves on one compute unit: waves 0..3 run instruction mix `mix_a`, waves 4..7
 * `mix_b` (wave w and w + 4 share a SIMD), each for `iters` loop iterations (1 .. 2^20).
 *   out  HOST, 8 rows (one per wave) of 6 doubles: loop duration in shader-clock ticks, the same in
 *        ticks of the constant 100 MHz clock, SIMD id read from the hardware, mix, instructions (or
 *        instruction groups) the wave issued, 0.
 * Mix numbers: see the enum in csrc/ubench/issue_ubench.hip (0 = idle).  Synchronous.
 * Returns 0, -1 (bad argument) or -3 (device error); reason in nuts_ubench_last_error(). */
int nuts_ubench_pair(int mix_a, int mix_b, int iters, double* out);

/* `blocks` workgroups of 4 waves issue nothing but v_mfma_f64_16x16x4_f64 (16 * iters each);
 * *out_tflops is the rate over the launch's duration by HIP events (best of `reps`), *out_ms that
 * duration.  Both HOST pointers.  Synchronous.  Same return codes. */
int nuts_ubench_mfma_peak(int blocks, int iters, int reps, double* out_tflops, double* out_ms);

/* The same with any instruction mix (*out_tflops counts binary64 matrix flop only). */
int nuts_ubench_fill(int mix, int blocks, int iters, int reps, double* out_tflops, double* out_ms);

/* The sampler kernels' table-driven logistic function, on its own, for n logits (the gradient of the
 * logistic-regression target, Section 4, needs log(1 + e^{-z}) and 1/(1 + e^{z}); both come from it).
 *   z, out_value, out_slope  DEVICE binary64 arrays of n values;
 *   out_value[i] = log(2 cosh(z[i]/2)) = |z|/2 + log(1 + exp(-|z|)),
 *   out_slope[i] = (1/2) tanh(|z[i]|/2) = 1/(1 + exp(-|z|)) - 1/2.
 * Synchronous, null stream.  Same return codes. */
int nuts_ubench_logistic(const double* z, long long n, double* out_value, double* out_slope);

/* The gradient loop's logarithm (it sums log(1 + e^{-z}) over the data as minus the logarithm of a
 * product of sigmas in (0, 1], one logarithm per lane and round), on its own:
 *   x, out  DEVICE binary64 arrays of n values, 0 < x[i] <= 1 (normal numbers); out[i] = log(x[i]).
 * Synchronous, null stream.  Same return codes. */
int nuts_ubench_log_unit(const double* x, long long n, double* out);

/* The sine and cosine of the tile kernel's Box-Muller draws (Section 4.1's sampler draws a Gaussian
 * momentum per iteration), on their own:
 *   phi, out_sin, out_cos  DEVICE binary64 arrays of n values, 0 <= phi[i] <= 2 pi.
 * Synchronous, null stream.  Same return codes. */
int nuts_ubench_circle_point(const double* phi, long long n, double* out_sin, double* out_cos);

/* The exponential that turns a leaf's energy error into its weight in the tile kernel (the multinomial
 * weights exp(H0 - H) of the sampler Section 4.1 batches), on its own:
 *   x, out  DEVICE binary64 arrays of n values, x[i] <= 700 (-infinity allowed); out[i] = exp(x[i]).
 * Synchronous, null stream.  Same return codes. */
int nuts_ubench_exp_bounded(const double* x, long long n, double* out);

const char* nuts_ubench_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* NUTS_UBENCH_H_ */
