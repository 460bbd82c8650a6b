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
    const T* band;    // dense Gaussian whose precision is banded (|i - k| <= kBandHalf): [row][k - i + kBandHalf],
                      // kBandRows rows, zero outside the matrix; NULL otherwise
    const T* inv_var; // diagonal Gaussian: 1/sigma_i^2
    const T* X;       // logistic regression: [n][d]
    const T* XT;      // logistic regression: [d][n]
    const T* y;       // logistic regression: [n]
    double prior_prec;
};

// A precision matrix with at most this many off-diagonals on each side is treated as banded.
constexpr int kBandHalf = 4;
constexpr int kBandRows = 128;

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
// their summed weights (tile, dense and quad kernels: as numbers in a unit that moves when the energy falls
// far; the other kernels: as logarithms).  Slice (Algorithm 3 of Hoffman & Gelman, the published form):
// a height is drawn below exp(-H0) once per iteration, leaves at or above it count 1, the others 0,
// and subtrees carry their count.  The count travels in the same variables as the weight
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

// For caches keyed by a leapfrog count: a count that no leaf has, and none a few leaves further on.
constexpr int kNoLeaf = -(1 << 30);

__device__ __forceinline__ int ret_to_pc(unsigned code)
{
    return code == kRetAfterLeft ? kPcAfterLeft : (code == kRetAfterRight ? kPcAfterRight : kPcDoubleEnd);
}

// A binary64 value moved between lanes by a DPP control word (two 32-bit moves).
template <int kCtrl>
__device__ __forceinline__ double dpp_rotate(double x)
{
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), kCtrl, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), kCtrl, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double read_lane(double x, int src_lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), src_lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src_lane);
    return __hiloint2double(hi, lo);
}

// Sums over the 64 lanes of a wave (all lanes active).  Inside each row of 16 lanes: rotations by
// 8, 4, 2, 1 (DPP, no LDS traffic; at each step the two partners add the same pair of values, so a
// row's lanes end with the same bits).  The four row totals are then read as scalars and added in
// one fixed order, so every lane of the wave holds the same bits.
__device__ __forceinline__ double wave_sum(double x)
{
    x += dpp_rotate<0x128>(x);  // row_ror:8
    x += dpp_rotate<0x124>(x);  // row_ror:4
    x += dpp_rotate<0x122>(x);  // row_ror:2
    x += dpp_rotate<0x121>(x);  // row_ror:1
    return (read_lane(x, 0) + read_lane(x, 16)) + (read_lane(x, 32) + read_lane(x, 48));
}

__device__ __forceinline__ void wave_sum2(double& a, double& b)
{
    a += dpp_rotate<0x128>(a);
    b += dpp_rotate<0x128>(b);
    a += dpp_rotate<0x124>(a);
    b += dpp_rotate<0x124>(b);
    a += dpp_rotate<0x122>(a);
    b += dpp_rotate<0x122>(b);
    a += dpp_rotate<0x121>(a);
    b += dpp_rotate<0x121>(b);
    a = (read_lane(a, 0) + read_lane(a, 16)) + (read_lane(a, 32) + read_lane(a, 48));
    b = (read_lane(b, 0) + read_lane(b, 16)) + (read_lane(b, 32) + read_lane(b, 48));
}

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

}  // namespace nuts
