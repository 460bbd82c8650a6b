// Instruction-issue microbenchmark for one MI355X compute unit: how fast a SIMD
// issues binary64 matrix (MFMA) instructions, plain vector instructions, and
// whether the two overlap when they come from different waves of one SIMD or
// from one wave's own instruction stream.
//
// One workgroup of 8 waves runs on one compute unit; the hardware places the
// waves round-robin on the 4 SIMDs, so waves w and w + 4 share a SIMD (each
// wave reports the SIMD id it reads from the hardware-id register, so the
// placement is checked, not assumed).  Waves 0..3 run instruction mix A,
// waves 4..7 mix B; every wave times its own loop with the shader clock and
// with the constant 100 MHz clock.  Comparing
//     time(A beside idle), time(B beside idle), time(A beside B)
// tells whether a SIMD runs the two streams at the same time (max) or one
// after the other (sum).
//
// A second entry point fills the whole chip with the binary64 MFMA loop and
// reports the rate it reaches, i.e. the practical matrix peak at the clock the
// chip holds under that load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../nuts_fastmath.h"

namespace {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef double v2d __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

enum Mix : int {
    kIdle = 0,
    kMfmaF64 = 1,        // v_mfma_f64_16x16x4_f64, 4 independent accumulators
    kMfmaF64Dep = 2,     // the same, one accumulator (each instruction waits for the one before)
    kFmaF64 = 3,         // v_fma_f64, 8 independent registers
    kFmaF32 = 4,         // v_fma_f32
    kXorB32 = 5,         // v_xor_b32 (plain 32-bit integer)
    kMulHiU32 = 6,       // v_mul_hi_u32 (the multiplier of the Philox rounds)
    kLdsRead = 7,        // ds_read_b128, conflict-free
    kMfmaPlusFmaF64 = 8, // one wave: 1 MFMA then 4 independent v_fma_f64, repeated
    kMfmaPlusFmaF32 = 9, // one wave: 1 MFMA then 4 independent v_fma_f32
    kMfmaPlusXor = 10,   // one wave: 1 MFMA then 4 independent v_xor_b32
    kMfmaF64Small = 11,  // v_mfma_f64_4x4x4_4b_f64 (four 4x4x4 blocks)
    kMfmaF32 = 12,       // v_mfma_f32_32x32x2_f32, 2 independent accumulators
    kMfmaF32PlusFma = 13,// one wave: 1 binary32 MFMA then 4 independent v_fma_f32
    kExpF32 = 14,        // v_exp_f32 (transcendental unit)
    kMfmaPlusLds = 15,   // one wave: 1 MFMA then 1 ds_read_b128
    kMfmaF64SmallDep = 16,  // v_mfma_f64_4x4x4_4b_f64, one accumulator
    kMfmaF32Small = 17,     // v_mfma_f32_4x4x1_16b_f32 (sixteen 4x4x1 blocks), 4 independent accumulators
    kMfmaF32SmallDep = 18,  // the same, one accumulator
    kMixCount = 19
};

// Instructions per loop iteration of each mix (what the rate is divided by).
__host__ __device__ inline int per_iter(int mix)
{
    switch (mix) {
    case kIdle: return 0;
    case kMfmaF64: case kMfmaF64Dep: case kMfmaF64Small: case kMfmaF64SmallDep: return 16;
    case kMfmaF32: case kMfmaF32Small: case kMfmaF32SmallDep: return 16;
    case kFmaF64: case kFmaF32: case kXorB32: case kMulHiU32: case kExpF32: return 64;
    case kLdsRead: return 16;
    case kMfmaPlusFmaF64: case kMfmaPlusFmaF32: case kMfmaPlusXor: case kMfmaF32PlusFma: return 16;  // groups of 1 + 4
    case kMfmaPlusLds: return 16;  // groups of 1 + 1
    default: return 0;
    }
}

#define VALU8(op, x, a, b)                                             \
    asm volatile(op " %0, %8, %9, %0\n\t" op " %1, %8, %9, %1\n\t"     \
                 op " %2, %8, %9, %2\n\t" op " %3, %8, %9, %3\n\t"     \
                 op " %4, %8, %9, %4\n\t" op " %5, %8, %9, %5\n\t"     \
                 op " %6, %8, %9, %6\n\t" op " %7, %8, %9, %7"         \
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]) \
                 : "v"(a), "v"(b))
#define VALU4(op, x, o, a, b)                                          \
    asm volatile(op " %0, %4, %5, %0\n\t" op " %1, %4, %5, %1\n\t"     \
                 op " %2, %4, %5, %2\n\t" op " %3, %4, %5, %3"         \
                 : "+v"(x[o]), "+v"(x[o + 1]), "+v"(x[o + 2]), "+v"(x[o + 3]) \
                 : "v"(a), "v"(b))
#define INT8(op, x, a)                                                 \
    asm volatile(op " %0, %8, %0\n\t" op " %1, %8, %1\n\t"             \
                 op " %2, %8, %2\n\t" op " %3, %8, %3\n\t"             \
                 op " %4, %8, %4\n\t" op " %5, %8, %5\n\t"             \
                 op " %6, %8, %6\n\t" op " %7, %8, %7"                 \
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]) \
                 : "v"(a))
#define INT4(op, x, o, a)                                              \
    asm volatile(op " %0, %4, %0\n\t" op " %1, %4, %1\n\t"             \
                 op " %2, %4, %2\n\t" op " %3, %4, %3"                 \
                 : "+v"(x[o]), "+v"(x[o + 1]), "+v"(x[o + 2]), "+v"(x[o + 3]) \
                 : "v"(a))
#define UNARY8(op, x)                                                  \
    asm volatile(op " %0, %0\n\t" op " %1, %1\n\t" op " %2, %2\n\t" op " %3, %3\n\t" \
                 op " %4, %4\n\t" op " %5, %5\n\t" op " %6, %6\n\t" op " %7, %7"     \
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]))

struct WaveReport {
    unsigned long long shader_ticks;  // loop duration, shader clock
    unsigned long long wall_ticks;    // loop duration, 100 MHz clock
    unsigned int simd;                // SIMD id read from the hardware-id register
    unsigned int mix;
    double sink;                      // keeps the arithmetic alive
    unsigned long long pad;
};

__device__ __forceinline__ double run_mix(int mix, int iters, double seed, double* lds)
{
    double xd[8];
    float xf[8];
    unsigned xi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        xd[i] = seed + i;
        xf[i] = (float)(seed + i);
        xi[i] = (unsigned)(seed * 977.0) + i;
    }
    const double ad = 0.999999, bd = 1e-9;
    const float af = 0.9999f, bf = 1e-6f;
    const unsigned ai = 0x9E3779B9u;
    v4d acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = v4d{seed, 0.0, 0.0, 0.0};
    v16f accf[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) accf[i][q] = (float)seed;
    v4f accs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) accs[i] = v4f{(float)seed, 0.0f, 0.0f, 0.0f};
    double one = seed;
    double ldsum = 0.0;
    const double* my = lds + 2 * (threadIdx.x & 63);  // 16 bytes per lane, consecutive: conflict-free

    switch (mix) {
    case kMfmaF64:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, acc[i], 0, 0, 0);
        }
        break;
    case kMfmaF64Dep:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, acc[0], 0, 0, 0);
        }
        break;
    case kMfmaF64Small:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const double t = __builtin_amdgcn_mfma_f64_4x4x4f64(ad, bd, (r & 1) ? xd[1] : xd[0], 0, 0, 0);
                if (r & 1) xd[1] = t; else xd[0] = t;
            }
        }
        break;
    case kMfmaF64SmallDep:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) xd[0] = __builtin_amdgcn_mfma_f64_4x4x4f64(ad, bd, xd[0], 0, 0, 0);
        }
        break;
    case kMfmaF32:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r)
#pragma unroll
                for (int i = 0; i < 2; ++i) accf[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, accf[i], 0, 0, 0);
        }
        break;
    case kMfmaF32Small:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) accs[r & 3] = __builtin_amdgcn_mfma_f32_4x4x1f32(af, bf, accs[r & 3], 0, 0, 0);
        }
        break;
    case kMfmaF32SmallDep:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) accs[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(af, bf, accs[0], 0, 0, 0);
        }
        break;
    case kFmaF64:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) VALU8("v_fma_f64", xd, ad, bd);
        }
        break;
    case kFmaF32:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) VALU8("v_fma_f32", xf, af, bf);
        }
        break;
    case kXorB32:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) INT8("v_xor_b32", xi, ai);
        }
        break;
    case kMulHiU32:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) INT8("v_mul_hi_u32", xi, ai);
        }
        break;
    case kExpF32:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) UNARY8("v_exp_f32", xf);
        }
        break;
    case kLdsRead:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const v2d v = *reinterpret_cast<const volatile v2d*>(my + 128 * r);
                ldsum += v.x;
            }
        }
        break;
    case kMfmaPlusFmaF64:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[r & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, acc[r & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                VALU4("v_fma_f64", xd, (r & 1) * 4, ad, bd);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        break;
    case kMfmaPlusFmaF32:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[r & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, acc[r & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                VALU4("v_fma_f32", xf, (r & 1) * 4, af, bf);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        break;
    case kMfmaPlusXor:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[r & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, acc[r & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                INT4("v_xor_b32", xi, (r & 1) * 4, ai);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        break;
    case kMfmaF32PlusFma:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                accf[r & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, accf[r & 1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                VALU4("v_fma_f32", xf, (r & 1) * 4, af, bf);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        break;
    case kMfmaPlusLds:
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[r & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(ad, bd, acc[r & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                const v2d v = *reinterpret_cast<const volatile v2d*>(my + 128 * r);
                ldsum += v.x;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        break;
    default:
        break;
    }
    for (int i = 0; i < 8; ++i) one += xd[i] + (double)xf[i] + (double)xi[i];
    for (int i = 0; i < 4; ++i) one += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    for (int i = 0; i < 2; ++i) one += (double)accf[i][0] + (double)accf[i][7];
    for (int i = 0; i < 4; ++i) one += (double)accs[i][0] + (double)accs[i][3];
    return one + ldsum;
}

__global__ __launch_bounds__(512) void issue_pair_kernel(int mix_a, int mix_b, int iters, WaveReport* out)
{
    __shared__ __align__(16) double lds[128 * 16 + 128];
    for (int i = threadIdx.x; i < 128 * 16 + 128; i += blockDim.x) lds[i] = 1.0 / (1 + i);
    const int wave = threadIdx.x >> 6;
    const int mix = wave < 4 ? mix_a : mix_b;
    __syncthreads();
    const unsigned long long w0 = wall_clock64();
    const unsigned long long t0 = clock64();
    const double r = run_mix(mix, iters, 1.0 + wave, lds);
    const unsigned long long t1 = clock64();
    const unsigned long long w1 = wall_clock64();
    if ((threadIdx.x & 63) == 0) {
        WaveReport& o = out[blockIdx.x * 8 + wave];
        o.shader_ticks = t1 - t0;
        o.wall_ticks = w1 - w0;
        // hardware-id register: bits 4..5 hold the SIMD the wave runs on
        o.simd = (__builtin_amdgcn_s_getreg((2 - 1) << 11 | 4 << 6 | 4)) & 3u;
        o.mix = (unsigned)mix;
        o.sink = r;
        o.pad = 0;
    }
}

__global__ __launch_bounds__(256) void mfma_fill_kernel(int mix, int iters, double* sink)
{
    __shared__ __align__(16) double lds[128 * 16 + 128];
    for (int i = threadIdx.x; i < 128 * 16 + 128; i += blockDim.x) lds[i] = 1.0 / (1 + i);
    __syncthreads();
    const double r = run_mix(mix, iters, 1.0 + (threadIdx.x >> 6), lds);
    if (r == 12345.678) sink[0] = r;  // never true: keeps the loop alive
}

__global__ void logistic_kernel(const double* z, long n, const double* ftab, double* out_value, double* out_slope)
{
    extern __shared__ __align__(16) double tab[];
    for (int i = threadIdx.x; i < nuts::kFtabDoubles; i += blockDim.x) tab[i] = ftab[i];
    __syncthreads();
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
        double v, slope;
        nuts::softplus_sym(z[i], tab, v, slope);
        out_value[i] = v;
        out_slope[i] = nuts::logistic_slope(z[i], tab);
        if (out_slope[i] != slope) out_slope[i] = NAN;  // the two evaluations of F' are the same arithmetic
    }
}

__global__ void log_unit_kernel(const double* x, long n, const double* logtab, double* out)
{
    __shared__ __align__(16) double tab[nuts::kLogTabDoubles];
    for (int i = threadIdx.x; i < nuts::kLogTabDoubles; i += blockDim.x) tab[i] = logtab[i];
    __syncthreads();
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x)
        out[i] = nuts::log_unit(x[i], tab);
}

__global__ void circle_point_kernel(const double* phi, long n, double* out_sin, double* out_cos)
{
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
        out_sin[i] = nuts::circle_point(phi[i], true);
        out_cos[i] = nuts::circle_point(phi[i], false);
    }
}

__global__ void exp_bounded_kernel(const double* x, long n, double* out)
{
    for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x)
        out[i] = nuts::exp_bounded(x[i]);
}

thread_local char g_err[256] = "";

}  // namespace

extern "C" {

// Runs mixes (mix_a on waves 0..3, mix_b on waves 4..7) of one 8-wave workgroup for `iters` loop
// iterations.  out (HOST, 8 rows of 6 doubles): shader ticks, 100 MHz ticks, SIMD id, mix,
// instructions issued by the wave (for the "1 MFMA + k others" mixes: groups), 0.
int nuts_ubench_pair(int mix_a, int mix_b, int iters, double* out)
{
    if (mix_a < 0 || mix_a >= kMixCount || mix_b < 0 || mix_b >= kMixCount || iters < 1 || iters > (1 << 20) || !out) {
        snprintf(g_err, sizeof(g_err), "bad argument");
        return -1;
    }
    WaveReport* dev = nullptr;
    hipError_t e = hipMalloc((void**)&dev, 8 * sizeof(WaveReport));
    if (e != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "hipMalloc: %s", hipGetErrorString(e));
        return -3;
    }
    // once untimed (instruction cache, clocks), then the run that is reported
    for (int rep = 0; rep < 2; ++rep) hipLaunchKernelGGL(issue_pair_kernel, dim3(1), dim3(512), 0, 0, mix_a, mix_b, iters, dev);
    WaveReport host[8];
    e = hipMemcpy(host, dev, sizeof(host), hipMemcpyDeviceToHost);
    (void)hipFree(dev);
    if (e != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "kernel or copy failed: %s", hipGetErrorString(e));
        return -3;
    }
    for (int w = 0; w < 8; ++w) {
        out[6 * w + 0] = (double)host[w].shader_ticks;
        out[6 * w + 1] = (double)host[w].wall_ticks;
        out[6 * w + 2] = (double)host[w].simd;
        out[6 * w + 3] = (double)host[w].mix;
        out[6 * w + 4] = (double)per_iter((int)host[w].mix) * iters;
        out[6 * w + 5] = 0.0;
    }
    return 0;
}

// Fills the chip (blocks x 4 waves) with one instruction mix (1: the binary64 16x16x4 MFMA loop);
// *out_tflops = matrix flop (2 * 1024 per 16x16x4, 2 * 256 per 4x4x4_4b instruction; 0 for mixes without
// a binary64 MFMA) over the launch's duration by HIP events (best of `reps`), *out_ms that duration.
int nuts_ubench_fill(int mix, int blocks, int iters, int reps, double* out_tflops, double* out_ms)
{
    if (mix < 1 || mix >= kMixCount || blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 22) || reps < 1 ||
        reps > 100 || !out_tflops || !out_ms) {
        snprintf(g_err, sizeof(g_err), "bad argument");
        return -1;
    }
    double* sink = nullptr;
    hipEvent_t a, b;
    if (hipMalloc((void**)&sink, 64) != hipSuccess || hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "set-up failed");
        return -3;
    }
    float best = 1e30f;
    for (int r = 0; r <= reps; ++r) {
        (void)hipEventRecord(a, 0);
        hipLaunchKernelGGL(mfma_fill_kernel, dim3(blocks), dim3(256), 0, 0, mix, iters, sink);
        (void)hipEventRecord(b, 0);
        if (hipEventSynchronize(b) != hipSuccess) {
            snprintf(g_err, sizeof(g_err), "kernel failed");
            return -3;
        }
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, a, b);
        if (r > 0 && ms < best) best = ms;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    (void)hipFree(sink);
    double per_instr = 0.0;  // matrix flop per instruction (or group) of the mix
    switch (mix) {
    case kMfmaF64: case kMfmaF64Dep: case kMfmaPlusFmaF64: case kMfmaPlusFmaF32: case kMfmaPlusXor: case kMfmaPlusLds:
        per_instr = 2.0 * 16 * 16 * 4; break;
    case kMfmaF64Small: case kMfmaF64SmallDep: per_instr = 2.0 * 4 * 4 * 4 * 4; break;
    default: break;
    }
    const double flop = per_instr * per_iter(mix) * iters * 4.0 * blocks;
    *out_ms = best;
    *out_tflops = flop / (best * 1e-3) / 1e12;
    return 0;
}

int nuts_ubench_mfma_peak(int blocks, int iters, int reps, double* out_tflops, double* out_ms)
{
    return nuts_ubench_fill(kMfmaF64, blocks, iters, reps, out_tflops, out_ms);
}

// The sampler kernels' table-driven logistic function on n logits (all DEVICE binary64 arrays):
// out_value = log(2 cosh(z/2)), out_slope = (1/2) tanh(|z|/2).  Synchronous, null stream.
int nuts_ubench_logistic(const double* z, long long n, double* out_value, double* out_slope)
{
    if (!z || !out_value || !out_slope || n < 1) {
        snprintf(g_err, sizeof(g_err), "null pointer or n < 1");
        return -1;
    }
    std::vector<double> ftab;
    nuts::build_softplus_table(&ftab);
    double* dev = nullptr;
    if (hipMalloc((void**)&dev, ftab.size() * sizeof(double)) != hipSuccess ||
        hipMemcpy(dev, ftab.data(), ftab.size() * sizeof(double), hipMemcpyHostToDevice) != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "table upload failed");
        return -3;
    }
    hipLaunchKernelGGL(logistic_kernel, dim3(256), dim3(256), nuts::kFtabDoubles * sizeof(double), 0, z, (long)n, dev,
                       out_value, out_slope);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipDeviceSynchronize();
    (void)hipFree(dev);
    if (e != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "diagnostic kernel failed: %s", hipGetErrorString(e));
        return -3;
    }
    return 0;
}

int nuts_ubench_log_unit(const double* x, long long n, double* out)
{
    if (!x || !out || n < 1) {
        snprintf(g_err, sizeof(g_err), "null pointer or n < 1");
        return -1;
    }
    std::vector<double> tab;
    nuts::build_log_table(&tab);
    double* dev = nullptr;
    if (hipMalloc((void**)&dev, tab.size() * sizeof(double)) != hipSuccess ||
        hipMemcpy(dev, tab.data(), tab.size() * sizeof(double), hipMemcpyHostToDevice) != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "table upload failed");
        return -3;
    }
    hipLaunchKernelGGL(log_unit_kernel, dim3(256), dim3(256), 0, 0, x, (long)n, dev, out);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipDeviceSynchronize();
    (void)hipFree(dev);
    if (e != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "diagnostic kernel failed: %s", hipGetErrorString(e));
        return -3;
    }
    return 0;
}

int nuts_ubench_circle_point(const double* phi, long long n, double* out_sin, double* out_cos)
{
    if (!phi || !out_sin || !out_cos || n < 1) {
        snprintf(g_err, sizeof(g_err), "null pointer or n < 1");
        return -1;
    }
    hipLaunchKernelGGL(circle_point_kernel, dim3(256), dim3(256), 0, 0, phi, (long)n, out_sin, out_cos);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "diagnostic kernel failed: %s", hipGetErrorString(e));
        return -3;
    }
    return 0;
}

int nuts_ubench_exp_bounded(const double* x, long long n, double* out)
{
    if (!x || !out || n < 1) {
        snprintf(g_err, sizeof(g_err), "null pointer or n < 1");
        return -1;
    }
    hipLaunchKernelGGL(exp_bounded_kernel, dim3(256), dim3(256), 0, 0, x, (long)n, out);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        snprintf(g_err, sizeof(g_err), "diagnostic kernel failed: %s", hipGetErrorString(e));
        return -3;
    }
    return 0;
}

const char* nuts_ubench_last_error(void) { return g_err; }

}  // extern "C"
