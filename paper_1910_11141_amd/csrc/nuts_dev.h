// Device-side definitions shared by the sampler kernels: kernel argument
// blocks, the program-counter vocabulary of the hand-lowered NUTS recursion,
// and wavefront-level reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nuts {

constexpr int kWave = 64;
constexpr double kDeltaMax = 1000.0;  // a leaf whose energy error exceeds this is divergent

enum TargetKind : int { kStdNormal = 0, kGaussDense = 1, kGaussDiag = 2, kLogReg = 3 };

// Target data on the device, in the layouts the kernels read.
template <typename T>
struct DevTarget {
    int kind;
    int d;            // dimension
    int dstride;      // padded length of one state vector in the workspace (elements)
    int kl;           // logistic regression, wave kernel: lanes along the feature axis (power of two <= 64)
    int lds_matrix;   // dense Gaussian, wave kernel: the precision matrix is copied to LDS at kernel start
    long n;           // data rows
    const T* PT;      // dense Gaussian: transpose of the precision, [k][i]
    const T* inv_var; // diagonal Gaussian: 1/sigma_i^2
    const T* X;       // logistic regression: [n][d]
    const T* XT;      // logistic regression: [d][n]
    const T* y;       // logistic regression: [n]
    double prior_prec;
};

// Per-call arguments.
struct DevSample {
    long n_chains;
    long first_chain;   // global id of local chain 0
    int n_iters;
    int iter_begin;     // this launch runs iterations [iter_begin, iter_end) of the n_iters
    int iter_end;
    int max_depth;
    int leaf_steps;     // leapfrog steps per tree leaf (>= 1)
    int sampler;        // kSamplerMultinomial or kSamplerSlice
    double eps;
    uint32_t key0, key1;
    void* out_states;
    int* out_depths;
    int* out_nleap;
    const void* init_states;
    char* workspace;
    size_t slot_bytes;  // workspace bytes per resident chain slot
    unsigned long long* counters;
};

// How the leaves of a trajectory are weighted.  Multinomial: leaf weight exp(H0 - H), subtrees carry
// the log of their summed weights.  Slice (Algorithm 3 of Hoffman & Gelman, the published form): a
// height is drawn below exp(-H0) once per iteration, leaves at or above it count 1, the others 0,
// and subtrees carry their count.  The count travels in the same variables as the log-weight
// (an integer below 2^21 is exact in binary64).
enum : int { kSamplerMultinomial = 0, kSamplerSlice = 1 };

// counters[] slots
enum : int {
    kCtrQueue = 0, kCtrIssued = 1, kCtrUseful = 2, kCtrExtra = 3, kCtrRounds = 4,
    kCtrCycControl = 5, kCtrCycGrad = 6, kCtrCycPost = 7,  // shader-clock ticks, summed over workgroups
    kCtrSlotMax = 8,  // wave and element-wise kernels: most gradient evaluations done by one slot in this launch
    kCtrCount = 9
};

// Program points of one chain.  This is the NUTS recursion written in the
// vocabulary of program-counter batching (Figure 4 / Algorithm 2 of the paper):
// BUILD is the body of the recursive tree builder, AFTER_LEFT / AFTER_RIGHT are
// the return points of its two recursive calls, DOUBLE_END is the return point
// of the top-level call.  LEAF and INIT_EVAL are the points where a chain needs
// the target's gradient: the scheduler runs every chain up to such a point and
// then evaluates all waiting gradients together.  Blocks are numbered in
// program order, which is also the order the scheduler picks them in
// ("earliest block first", Section 2).
enum Pc : int {
    kPcFetch = 0,       // take the next chain from the queue, make x0
    kPcIterBegin = 1,   // draw the momentum, H0, reset the trajectory
    kPcDoubleBegin = 2, // draw the direction, call BUILD(level = j)
    kPcBuild = 3,       // level == 0 ? LEAF : call BUILD(level-1), return to AFTER_LEFT
    kPcAfterLeft = 4,   // left half done: stop early, or save its summary and call BUILD for the right half
    kPcAfterRight = 5,  // right half done: merge weights, select the proposal, U-turn test over the span
    kPcDoubleEnd = 6,   // top level: accept the new half, whole-trajectory U-turn test, loop or finish
    kPcIterEnd = 7,     // emit the iteration's outputs
    kPcInitEval = 8,    // waiting for (logp, grad) at x0
    kPcLeaf = 9,        // waiting for a leapfrog step
    kPcHalt = 10
};

// Return addresses live in a 2-bit-per-entry stack packed into 64 bits
// (depth <= max_tree_depth + 1 <= 21 entries).
enum RetCode : unsigned { kRetAfterLeft = 0, kRetAfterRight = 1, kRetDoubleEnd = 2 };

__device__ __forceinline__ int ret_to_pc(unsigned code)
{
    return code == kRetAfterLeft ? kPcAfterLeft : (code == kRetAfterRight ? kPcAfterRight : kPcDoubleEnd);
}

// Butterfly sums: every lane ends with the same bits (a+b == b+a exactly).
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
    return x;
}

__device__ __forceinline__ void wave_sum2(double& a, double& b)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        a += __shfl_xor(a, o, kWave);
        b += __shfl_xor(b, o, kWave);
    }
}

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

}  // namespace nuts
