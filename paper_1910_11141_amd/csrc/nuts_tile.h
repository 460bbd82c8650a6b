// Tile kernel: 16 chains per workgroup advance in lock step and their
// logistic-regression gradients are evaluated together on the matrix cores.
//
// This is program-counter batching (Algorithm 2 of the paper) at workgroup
// scale.  A workgroup of 8 wavefronts owns 16 chain slots.  Each chain has its
// own program counter, return-address stack and tree state, held in the
// registers of a 32-lane group (lane k owns component k of every state vector;
// the per-level frame scalars sit one level per lane).  A round is:
//   1. control: every wave sweeps the blocks of the chain program in program
//      order and runs each block for exactly those of its chains that wait at
//      it (masked), until all of them stand at a point that needs the target's
//      gradient;
//   2. the 16 positions are gathered into an LDS tile, and all 8 waves evaluate
//      the 16 gradients as two chained GEMMs on binary64 MFMA tiles
//        Z = X~ Theta           (rows of data  x chains, contraction over features)
//        G = X~' sigma(-Z)      (features      x chains, contraction over rows)
//      with the logistic functions applied to Z in the accumulator registers,
//      so Z never leaves the register file.  X~ is X with the rows of y = 0
//      negated, which turns  y z - log(1+e^z)  into  -log(1+e^{-z~})  and
//      X'(y - sigma(z))  into  X~' sigma(-z~)  exactly (sign flips are exact);
//   3. each chain sums the 8 per-wave partial gradients in a fixed order and
//      finishes its leapfrog step.
// A chain that ends its last iteration takes the next chain from the queue, so
// slots stay occupied until the queue is empty.
//
// A constant column (an intercept) whose removal saves a k-step of the first
// GEMM (d = 1 mod 4: the paper's logistic regression has 24 features and an
// intercept) does not go through that GEMM: its share c theta_c of every logit
// is the accumulators' initial value.  Since the functions of the logit used here
// are even or odd, both GEMMs then multiply by X itself (|z~| = |z| and
// X~' (sign(z~) F') = X' (sign(z) F'), bit for bit), so that the column is the same
// constant in every row; the labels enter through the column sums of X~ alone.
//
// The tree storage that is indexed by level (proposal pool of the open frames,
// first-leaf slots) lives in LDS for the shallow levels and in global memory
// beyond; each element is only ever read by the lane that wrote it.  Everything
// else is in registers.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "nuts_dev.h"
#include "nuts_fastmath.h"
#include "nuts_rng.h"

namespace nuts {

constexpr int kTileMaxDim = 32;
constexpr int kTileMaxDepth = 12;
constexpr int kTileChains = 16;    // chains per workgroup = MFMA N
constexpr int kTileLanes = 32;     // lanes per chain in the control phase
constexpr int kTileWaves = 8;
constexpr int kTileThreads = kTileWaves * kWave;
constexpr int kTileRows = 16;      // data rows per MFMA tile = MFMA M of the first GEMM
constexpr int kTileLdsPool = 5;    // proposal-pool buffers 0..4 of every chain live in LDS
constexpr int kTileLdsFirst = 4;   // first-leaf slots 1..4 of every chain live in LDS (with the tables 158 KB of the 160)

struct TileData {
    double* base = nullptr;  // device: operands of every row tile, in MFMA lane order
    double* ftab = nullptr;  // device: softplus table (kFtabDoubles) followed by the logarithm table (kLogTabDoubles)
    double* colsum = nullptr;  // device: column sums of X~ (kTileMaxDim values, zero padded)
    int d = 0;
    int ks1 = 0;             // k-steps of the first GEMM  = ceil(d / 4)
    int mt = 0;              // M-tiles of the second GEMM = ceil(d / 16)
    int n_tiles = 0;         // row tiles that are run
    int n_alloc_tiles = 0;   // row tiles in the operand stream
    long n_rows = 0, n_pad = 0;
    int z0_col = -1;         // the constant column that stays out of the first GEMM, or -1
    double z0_val = 0.0;     // its value
};

struct TileLaunch {
    int blocks = 0;
    size_t block_bytes = 0, workspace_bytes = 0;
};

struct TileArgs {
    const double* ops;
    const double* ftab;
    const double* colsum;
    int d, n_tiles;
    double prior_prec;
    double n_pad;  // zero rows appended to fill the last tiles
    unsigned ops_bytes;  // size of the operand stream
    int rem_rows;        // kZ0 kernels: real rows of the last tile if that tile is not full, else 0
    int z0_col;          // the constant column that is the accumulators' initial value (kZ0 kernels), and its value
    double z0_val;
};

// (the operand stream is read through a buffer descriptor with 32-bit offsets: 512 bytes per data row at most, so
// four million rows stay below 2 GiB)
inline bool tile_supports_shape(int64_t d, int64_t n) { return d >= 1 && d <= kTileMaxDim && n >= 1 && n <= 4000000; }

// Operand stream: for every row tile t (16 rows), KS1 operands of 64 doubles for
// the first GEMM (padded to an even count) then 4*MT for the second; operand
// element l is what lane l feeds to the MFMA.  Operands are stored in pairs,
// element by element (pair p holds [2p][l], [2p+1][l] for l = 0..63), so that one
// 16-byte load per lane brings two of them.  Rows beyond n are zero, features
// beyond d are zero.
__host__ __device__ constexpr int tile_pairs_per_tile(int ks1, int mt) { return (ks1 + 1) / 2 + 2 * mt; }
inline void tile_pack_operands(const double* X, const double* y, int64_t n, int64_t d, TileData* td,
                               std::vector<double>* out, std::vector<double>* colsum)
{
    colsum->assign(kTileMaxDim, 0.0);
    for (int64_t f = 0; f < d; ++f) {
        double acc = 0.0;
        for (int64_t r = 0; r < n; ++r) acc += y[r] != 0.0 ? X[r * d + f] : -X[r * d + f];
        (*colsum)[(size_t)f] = acc;
    }
    td->d = (int)d;
    td->ks1 = (int)((d + 3) / 4);
    td->mt = (int)((d + 15) / 16);
    td->z0_col = -1;
    td->z0_val = 0.0;
    if (d % 4 == 1 && d > 1) {  // one feature less is one k-step less
        for (int64_t f = 0; f < d && td->z0_col < 0; ++f) {
            bool same = X[f] != 0.0 && std::isfinite(X[f]);
            for (int64_t r = 1; r < n && same; ++r) same = X[r * d + f] == X[f];
            if (same) {
                td->z0_col = (int)f;
                td->z0_val = X[f];
                td->ks1 = (int)((d - 1) / 4);
            }
        }
    }
    const bool z0 = td->z0_col >= 0;
    const int64_t tiles = (n + kTileRows - 1) / kTileRows;
    // (the stream always holds a multiple of kTileWaves tiles: every wave asks for its first tile unconditionally)
    td->n_alloc_tiles = (int)((tiles + kTileWaves - 1) / kTileWaves * kTileWaves);
    // Rows of zeros have logit 0, which is harmless (a known constant in the log-likelihood, nothing in the gradient),
    // unless the accumulators start from the constant column's share: then only real tiles are run, and the rows that
    // fill the last one start from zero.
    td->n_tiles = z0 ? (int)tiles : td->n_alloc_tiles;
    td->n_rows = (long)n;
    td->n_pad = (long)td->n_tiles * kTileRows - (long)n;
    const int pairs1 = (td->ks1 + 1) / 2;
    const int per_tile = 2 * tile_pairs_per_tile(td->ks1, td->mt);
    out->assign((size_t)td->n_alloc_tiles * per_tile * 64, 0.0);
    auto xs = [&](int64_t row, int64_t feat) -> double {
        if (row >= n || feat >= d) return 0.0;
        const double v = X[row * d + feat];
        return (z0 || y[row] != 0.0) ? v : -v;
    };
    // slot of the first GEMM's contraction -> feature: with a constant column c the last feature takes its slot
    // (the chains' lanes c and d - 1 write their positions to each other's place to match)
    auto feat1 = [&](int64_t slot) -> int64_t {
        if (!z0) return slot;
        if (slot >= d - 1) return d;  // (no feature: zero)
        return slot == td->z0_col ? d - 1 : slot;
    };
    for (int t = 0; t < td->n_alloc_tiles; ++t) {
        double* o = out->data() + (size_t)t * per_tile * 64;
        auto at = [&](int operand, int l) -> double& { return o[((operand >> 1) * 64 + l) * 2 + (operand & 1)]; };
        for (int s = 0; s < td->ks1; ++s)          // A[i][k] = X~[16t + i][4s + k], lane = i + 16k
            for (int l = 0; l < 64; ++l) at(s, l) = xs((int64_t)t * 16 + (l & 15), feat1(4 * s + (l >> 4)));
        for (int u = 0; u < td->mt; ++u)           // A[i][k] = X~[16t + 4s + k][16u + i]
            for (int s = 0; s < 4; ++s)
                for (int l = 0; l < 64; ++l)
                    at(2 * pairs1 + u * 4 + s, l) = xs((int64_t)t * 16 + 4 * s + (l >> 4), 16 * u + (l & 15));
    }
}

// Global-memory vectors of one chain slot, 32 doubles each:
//   proposal pool  2*b + c            b <= D,  c in {theta, grad}
//   first-leaf     2*(D+1) + 2*s + c  s <= D,  c in {theta, r}
__host__ __device__ inline int tile_num_vectors(int max_depth) { return 4 * (max_depth + 1); }

inline void tile_plan(const TileData&, long n_chains, int max_depth, TileLaunch* tl)
{
    long blocks = (n_chains + kTileChains - 1) / kTileChains;
    const long cap = 256L * 2;  // two resident workgroups per compute unit is the most that fits
    if (blocks > cap) blocks = cap;
    tl->blocks = (int)blocks;
    tl->block_bytes = (size_t)kTileChains * tile_num_vectors(max_depth) * kTileLanes * sizeof(double);
    tl->workspace_bytes = tl->block_bytes * (size_t)blocks;
}

typedef double v4d __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// ---- reductions over the 32 lanes of one chain ------------------------------
// Rotations inside each row of 16 lanes (DPP), then one exchange between the
// two rows (swizzle).  Every lane ends with the same bits: at each step the two
// partners add the same pair of values.
__device__ __forceinline__ double swap_rows(double x)  // lane ^ 16
{
    const int lo = __builtin_amdgcn_ds_swizzle(__double2loint(x), 0x401F);
    const int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(x), 0x401F);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double add_other_row(double x)  // x[lane] + x[lane ^ 16]
{
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}
__device__ __forceinline__ double add_other_half(double x)  // x[lane] + x[lane ^ 32]
{
    const unsigned lo = (unsigned)__double2loint(x), hi = (unsigned)__double2hiint(x);
    const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
}
__device__ __forceinline__ double group_sum(double x)
{
    x += dpp_rotate<0x128>(x);  // row_ror:8
    x += dpp_rotate<0x124>(x);  // row_ror:4
    x += dpp_rotate<0x122>(x);  // row_ror:2
    x += dpp_rotate<0x121>(x);  // row_ror:1
    x += swap_rows(x);
    return x;
}
__device__ __forceinline__ void group_sum2(double& a, double& b)
{
    a += dpp_rotate<0x128>(a);
    b += dpp_rotate<0x128>(b);
    a += dpp_rotate<0x124>(a);
    b += dpp_rotate<0x124>(b);
    a += dpp_rotate<0x122>(a);
    b += dpp_rotate<0x122>(b);
    a += dpp_rotate<0x121>(a);
    b += dpp_rotate<0x121>(b);
    a += swap_rows(a);
    b += swap_rows(b);
}

// Two sums over the 32 lanes of one chain in one sweep, for where only their signs are wanted: the rows change halves
// first (row 0 takes a, row 1 takes b), then one set of rotations sums both.  Lanes 0..15 end with sum(a), lanes 16..31
// with sum(b).
__device__ __forceinline__ double group_sum_split(double a, double b, bool upper_row)
{
    const double keep = upper_row ? b : a, give = upper_row ? a : b;
    double x = keep + swap_rows(give);
    x += dpp_rotate<0x128>(x);
    x += dpp_rotate<0x124>(x);
    x += dpp_rotate<0x122>(x);
    x += dpp_rotate<0x121>(x);
    return x;
}
// ... and whether both are >= 0, the same answer in all 32 lanes (all of them must be running).
__device__ __forceinline__ bool group_both_nonnegative(double a, double b, int lane)
{
    const double x = group_sum_split(a, b, (lane & 16) != 0);
    const unsigned long long votes = __ballot(x >= 0.0);
    return (uint32_t)(votes >> (lane & 32)) == 0xffffffffu;
}

// Workgroup barrier that orders LDS traffic only.  The chains of a workgroup talk to each other through
// LDS alone (positions in, partial gradients out); what a lane has in flight to global memory - operands
// asked for ahead of the barrier, output samples, its own deep tree levels - nobody else in the workgroup
// reads, so the barrier need not wait for it as __syncthreads() would.
__device__ __forceinline__ void tile_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// State of one chain, replicated over (and partly distributed across) its 32 lanes.
struct TileChain {
    int pc, level, j, v, m, nleap, iter, cur_s, cur_idx, frame_idx;
    int sub;  // leapfrog steps already taken inside the current leaf
    uint64_t ret;
    long chain;
    uint32_t gchain, free_mask;
    // Weights of trajectory points are kept as numbers, not logarithms: a leaf weighs exp(H0 - H) / unit, a subtree the sum of
    // its leaves (slice sampler: 1 or 0 per leaf, the count per subtree), so a merge is an add and a selection one product
    // and a comparison.  `log_unit` is the logarithm of the unit, 0 until a leaf's energy falls more than 600 below what the
    // unit can represent; then that leaf becomes the unit and what the iteration holds is rescaled.
    double H0, w_tree, cur_w, log_unit_w, edge_logp, top_logp;
    // Lane-distributed scalars (lane k of the chain's 32 lanes):
    double frame_w;    // k = 1..12: weight of the open frame of level k; k = 16 + j: the next iteration's TOP uniform of doubling j
    double pool_logp;  // k = 0..12: log-density of pool buffer k;            k = 16 + j: this iteration's TOP uniform of doubling j
                       // (slice sampler: k = 31 of both carries log(slice height / exp(-H0)), the log of a uniform)
    double u_sub;      // k = 0..12: SUBTREE uniform of level k for the leaf that ends with leapfrog count `u_sub_leaf`;
                       // k = 16 + l: that of level l for the next leaf that can complete a merge (two leaves on)
    // component k of the two ends of the trajectory: the one the current doubling extends (direction v) and the other;
    // they change places when a doubling turns round, so that a leapfrog step and the tests on it select nothing
    double tha, ra, ga, tho, ro, go;
    double tt, tg;                    // component k of the trajectory's current proposal and its gradient
    double rn;                        // component k of the momentum drawn ahead for iteration `ahead_iter`
    double kin_n;                     // |rn|^2
    int ahead_iter, u_sub_leaf;
    uint32_t dirbits, dirbits_n;      // bit j: direction of doubling j (this / the drawn-ahead iteration)
};

template <int KS1, int MT, bool kSlice, bool kZ0>
__global__ __launch_bounds__(kTileThreads) void nuts_tile_kernel(TileArgs ta, DevSample sa)
{
    __shared__ double sTheta[kTileChains][kTileLanes + 1];
    // odd row stride: an accumulator store (lanes = 16 chains x 4 feature offsets) would otherwise pile onto 4 banks
    __shared__ double sG[kTileWaves][kTileChains][kTileLanes + 1];
    __shared__ double sLL[kTileWaves][kTileChains];
    __shared__ int sHalted;  // chains of this workgroup that have halted (a chain that has not waits for a gradient after every sweep)
    __shared__ __align__(16) double sFtab[kFtabDoubles + kLogTabDoubles];
    __shared__ double sPool[kTileChains][kTileLdsPool][2][kTileLanes];
    __shared__ double sFirst[kTileChains][kTileLdsFirst][2][kTileLanes];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = uni(tid >> 6);  // the wave index as a scalar: loops over it are uniform
    const int grp = tid / kTileLanes;      // chain slot in the workgroup
    const int k = tid & (kTileLanes - 1);  // component owned by this lane
    const int d = ta.d, D = sa.max_depth;
    const bool kin_range = k < d;
    const DrawKey key{sa.key0, sa.key1};
    constexpr bool slice = kSlice;  // the sampler is a compile-time choice: each form keeps its own register budget
    const uint32_t all_bufs = (1u << (D + 1)) - 1u;

    double* const wsc = reinterpret_cast<double*>(sa.workspace + (size_t)blockIdx.x * sa.slot_bytes) +
                        (size_t)grp * tile_num_vectors(D) * kTileLanes + k;
    // The shallow part of the level-indexed tree storage is in LDS (trees are mostly shallow, and the
    // pool hands out its lowest free buffer first); deeper levels fall back to global memory.
    // (a load reads LDS always - a clamped slot when the level is deep - and global memory on top of that when
    // it has to: the LDS read then needs no branch and no wait of its own, so it travels together with the
    // other LDS traffic of its block.  The pointer is typed as LDS and volatile on purpose: left to itself the
    // compiler folds the two reads into one flat load from a selected address, which takes the long way
    // round even when it ends in LDS.)
    typedef volatile __attribute__((address_space(3))) double LdsDouble;
    auto pool_load = [&](int b, int c) __attribute__((always_inline)) -> double {
        double v = *(LdsDouble*)(&sPool[grp][min(b, kTileLdsPool - 1)][c][k]);
        if (b >= kTileLdsPool) v = wsc[(size_t)(2 * b + c) * kTileLanes];
        return v;
    };
    auto pool_store = [&](int b, int c, double v) __attribute__((always_inline)) {
        if (b < kTileLdsPool) sPool[grp][b][c][k] = v;
        else wsc[(size_t)(2 * b + c) * kTileLanes] = v;
    };
    auto first_load = [&](int s, int c) __attribute__((always_inline)) -> double {
        double v = *(LdsDouble*)(&sFirst[grp][min(s, kTileLdsFirst) - 1][c][k]);
        if (s > kTileLdsFirst) v = wsc[(size_t)(2 * (D + 1) + 2 * s + c) * kTileLanes];
        return v;
    };
    auto first_store = [&](int s, int c, double v) __attribute__((always_inline)) {
        if (s <= kTileLdsFirst) sFirst[grp][s - 1][c][k] = v;
        else wsc[(size_t)(2 * (D + 1) + 2 * s + c) * kTileLanes] = v;
    };

    for (int i = threadIdx.x; i < kFtabDoubles + kLogTabDoubles; i += kTileThreads) sFtab[i] = ta.ftab[i];
    if (tid == 0) sHalted = 0;
    __syncthreads();

    const double half_colsum = 0.5 * ta.colsum[k];
    // where lane k puts its position for the first GEMM (see feat1 in tile_pack_operands)
    const int k_slot = !kZ0 ? k : (k == ta.z0_col ? ta.d - 1 : (k == ta.d - 1 ? ta.z0_col : k));
    const __amdgpu_buffer_rsrc_t ops_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(ta.ops), 0, (int)ta.ops_bytes, 0x00020000);

    TileChain c{};
    c.pc = kPcFetch;
    c.cur_idx = -1;
    unsigned long long n_leaf = 0, n_extra = 0, n_rounds = 0;
    long long cyc_control = 0, cyc_grad = 0, cyc_post = 0;  // wave 0's view of where a round's time goes

    // Box-Muller as in normal_of(), with the logarithm of the gradient loop (its table is in LDS here)
    auto normal_from = [&](const Words4& w, bool second) __attribute__((always_inline)) -> double {
        const double u1 = uniform52(w.w0, w.w1);
        const double u2 = uniform52(w.w2, w.w3);
        const double rho = sqrt(-2.0 * log_unit(u1, sFtab + kFtabDoubles));
        const double phi = 6.283185307179586476925286766559 * u2;
        return rho * circle_point(phi, second);
    };
    auto push_ret = [&](unsigned code) __attribute__((always_inline)) { c.ret = (c.ret << 2) | code; };
    auto do_return = [&]() __attribute__((always_inline)) {
        c.pc = ret_to_pc((unsigned)(c.ret & 3u));
        c.ret >>= 2;
        c.level += 1;
    };
    // BUILD(level) calls BUILD(level - 1) down to a leaf: one return address per level
    auto descend_to_leaf = [&]() __attribute__((always_inline)) {
        static_assert(kRetAfterLeft == 0, "pushing it `level` times is a shift");
        c.ret <<= 2 * c.level;
        c.level = 0;
        c.pc = kPcLeaf;
    };
    // Make sure the current proposal owns a pool buffer (a fresh leaf lives in the edge registers).
    auto materialise_cur = [&]() __attribute__((always_inline)) {
        if (c.cur_idx >= 0) return;
        const int b = __ffs(c.free_mask) - 1;
        c.free_mask &= ~(1u << b);
        pool_store(b, 0, c.tha);
        pool_store(b, 1, c.ga);
        if (k == b) c.pool_logp = c.edge_logp;
        c.cur_idx = b;
    };

    // ---- blocks of the chain program; each runs for the lanes whose chain waits at it ----
    auto block_after_right = [&]() __attribute__((always_inline)) {
        if (c.cur_s) {
            // the first leaf of this subtree was saved when it was computed; ask for it early
            const int f = c.m - (1 << c.level) + 1;  // 1-based
            const int s = (f == 1) ? c.j : min(__ffs(f - 1) - 1, c.j);
            const double tf = first_load(s, 0), rf = first_load(s, 1);
            const double l_w = __shfl(c.frame_w, c.level, kTileLanes);
            const int l_idx = __shfl(c.frame_idx, c.level, kTileLanes);
            const double u = __shfl(c.u_sub, c.level + (c.u_sub_leaf != c.nleap ? 16 : 0), kTileLanes);
            // right with probability w_R / (w_L + w_R) (never when both are zero)
            const double w_new = l_w + c.cur_w;
            if (u * w_new < c.cur_w) {  // keep the right half's proposal
                c.free_mask |= (1u << l_idx);
            } else {
                if (c.cur_idx >= 0) c.free_mask |= (1u << c.cur_idx);
                c.cur_idx = l_idx;
            }
            c.cur_w = w_new;
            // (theta+ - theta-) . r at both ends of the subtree; going backwards the span is the negative of
            // last leaf - first leaf, and so, exactly, are the sums: their signs are turned by the direction
            const double span = c.v > 0 ? c.tha - tf : tf - c.tha;
            c.cur_s = group_both_nonnegative(span * rf, span * c.ra, lane);
        }
        do_return();
    };
    auto block_after_left = [&]() __attribute__((always_inline)) {
        if (!c.cur_s) {  // the right half is never built
            do_return();
            return;
        }
        materialise_cur();
        if (k == c.level) {
            c.frame_w = c.cur_w;
            c.frame_idx = c.cur_idx;
        }
        c.level -= 1;
        push_ret(kRetAfterRight);
        descend_to_leaf();
    };
    auto block_double_end = [&]() __attribute__((always_inline)) {
        bool go_on = false;
        if (c.cur_s) {
            const double u = __shfl(c.pool_logp, 16 + c.j, kTileLanes);
            if (u * c.w_tree < c.cur_w) {  // accept the new half with probability min(1, w_new / w_tree)
                if (c.cur_idx < 0) {
                    c.tt = c.tha;
                    c.tg = c.ga;
                    c.top_logp = c.edge_logp;
                } else {
                    c.tt = pool_load(c.cur_idx, 0);
                    c.tg = pool_load(c.cur_idx, 1);
                    c.top_logp = __shfl(c.pool_logp, c.cur_idx, kTileLanes);
                }
            }
            c.w_tree += c.cur_w;
            const double span = c.v > 0 ? c.tha - c.tho : c.tho - c.tha;  // forward end - backward end
            go_on = group_both_nonnegative(span * c.ro, span * c.ra, lane);
        }
        c.j += 1;
        c.free_mask = all_bufs;  // nothing of the finished doubling stays in the pool
        c.pc = (go_on && c.j < D) ? kPcDoubleBegin : kPcIterEnd;
    };
    auto block_iter_end = [&]() __attribute__((always_inline)) {
        const size_t row = (size_t)c.iter * (size_t)sa.n_chains + (size_t)c.chain;
        if (sa.out_states && kin_range) static_cast<double*>(sa.out_states)[row * d + k] = c.tt;
        if (k == 0) {
            if (sa.out_depths) sa.out_depths[row] = c.j;
            if (sa.out_nleap) sa.out_nleap[row] = c.nleap;
        }
        c.iter += 1;
        c.pc = (c.iter < sa.iter_end) ? kPcIterBegin : kPcFetch;
    };
    auto block_fetch = [&]() __attribute__((always_inline)) {
        unsigned long long q = 0;
        if (k == 0) q = atomicAdd(&sa.counters[kCtrQueue], 1ull);
        q = __shfl(q, 0, kTileLanes);
        c.tt = 0.0;
        if ((long)q >= sa.n_chains) {
            c.pc = kPcHalt;
            if (k == 0) atomicAdd(&sHalted, 1);
            return;
        }
        c.chain = (long)q;
        c.gchain = (uint32_t)(sa.first_chain + c.chain);
        c.iter = sa.iter_begin;
        c.ahead_iter = -1;
        c.u_sub_leaf = kNoLeaf;
        c.free_mask = all_bufs;
        if (kin_range) {
            if (sa.init_states) {
                c.tt = static_cast<const double*>(sa.init_states)[(size_t)c.chain * d + k];
            } else {
                const Words4 w = draw(key, (uint32_t)(k >> 1), kDrawInit, 0, 0, c.gchain);
                c.tt = normal_from(w, k & 1);
            }
        }
        c.pc = kPcInitEval;
    };
    // Every random number of an iteration that does not depend on where the trajectory goes: the
    // momentum, the direction of each doubling, the top-level acceptance uniforms.  The draws are
    // keyed by (chain, iteration, purpose, position), so they can be made at any time; a chain
    // makes them one iteration ahead in a round in which it has little else to do.
    auto draw_iteration = [&](int it) __attribute__((always_inline)) {
        double r = 0.0;
        if (kin_range) {
            const Words4 w = draw(key, (uint32_t)(k >> 1), kDrawMomentum, 0, (uint32_t)it, c.gchain);
            r = normal_from(w, k & 1);
        }
        c.rn = r;
        c.kin_n = group_sum(r * r);
        // lanes 0..15: direction of doubling k; lanes 16..31: acceptance uniform of doubling k - 16
        const bool slice_lane = slice && k == kTileLanes - 1;
        const Words4 w = draw(key, slice_lane ? 0u : (uint32_t)(k & 15),
                              k < 16 ? kDrawDirection : (slice_lane ? kDrawSlice : kDrawTop), 0, (uint32_t)it, c.gchain);
        const unsigned long long votes = __ballot((k < 16) && (w.w0 >> 31));
        c.dirbits_n = (uint32_t)(votes >> (lane & 32)) & 0xffffu;
        if (k >= 16) c.frame_w = uniform52(w.w0, w.w1);
        if (slice_lane) c.frame_w = log(c.frame_w);
        c.ahead_iter = it;
    };
    auto block_iter_begin = [&]() __attribute__((always_inline)) {
        if (c.ahead_iter != c.iter) draw_iteration(c.iter);
        const double r = c.rn;
        c.dirbits = c.dirbits_n;
        if (k >= 16) c.pool_logp = c.frame_w;
        c.tha = c.tho = c.tt;
        c.ga = c.go = c.tg;
        c.ra = c.ro = r;
        c.H0 = -c.top_logp + 0.5 * c.kin_n;
        c.w_tree = 1.0;  // the starting point: weight exp(0), or the first candidate
        c.log_unit_w = 0.0;
        c.j = 0;
        c.nleap = 0;
        c.u_sub_leaf = kNoLeaf;  // leaf counts restart: the cached SUBTREE uniforms belong to the old iteration
        c.pc = kPcDoubleBegin;
    };
    auto block_double_begin = [&]() __attribute__((always_inline)) {
        const int v = ((c.dirbits >> c.j) & 1u) ? 1 : -1;
        if (v != c.v) {  // the doubling turns round (in the first doubling the two ends are the same point)
            double t;
            t = c.tha, c.tha = c.tho, c.tho = t;
            t = c.ra, c.ra = c.ro, c.ro = t;
            t = c.ga, c.ga = c.go, c.go = t;
        }
        c.v = v;
        c.m = 0;
        c.level = c.j;
        push_ret(kRetDoubleEnd);
        c.pc = kPcBuild;
        descend_to_leaf();  // BUILD has no work of its own: fall straight through to the leaf
    };

    for (;;) {
        const long long t0 = clock64();
        // ---- 1. control: one sweep over the chain program in program order (a static
        // choice of the "which block next" freedom of Section 2; no block can starve).
        // Returns cascade: a finished subtree may complete its parent, and so on.
        // Every merge that a leaf can complete draws at the same position (the leapfrog count), one level
        // per lane; only leaves that close a right half complete merges, and those are two leaves apart,
        // so one pass of the generator serves two of them: lanes 0..15 this leaf, lanes 16..31 the next.
        // (before the loop and under a condition of its own: inside, the compiler would hoist the generator
        // out of the loop and run it in every round)
        if (c.pc == kPcAfterRight && c.cur_s && c.u_sub_leaf != c.nleap && c.u_sub_leaf + 2 * sa.leaf_steps != c.nleap) {
            const Words4 w = draw(key, (uint32_t)(c.nleap + (k >= 16 ? 2 * sa.leaf_steps : 0)), kDrawSubtree, (uint32_t)(k & 15),
                                  (uint32_t)c.iter, c.gchain);
            c.u_sub = uniform52(w.w0, w.w1);
            c.u_sub_leaf = c.nleap;
        }
        for (;;) {
            const int pa = __builtin_amdgcn_readlane(c.pc, 0), pb = __builtin_amdgcn_readlane(c.pc, kTileLanes);
            const bool any_right = pa == kPcAfterRight || pb == kPcAfterRight;
            const bool any_left = pa == kPcAfterLeft || pb == kPcAfterLeft;
            if (!any_right && !any_left) break;
            if (any_right && c.pc == kPcAfterRight) block_after_right();
            if (c.pc == kPcAfterLeft) block_after_left();
        }
        const bool wave_busy = __any(c.pc == kPcDoubleEnd);  // a doubling ends in this wave: it may be the round's slowest
        if (c.pc == kPcDoubleEnd) block_double_end();
        if (c.pc == kPcIterEnd) block_iter_end();
        if (c.pc == kPcFetch) block_fetch();
        if (c.pc == kPcIterBegin) block_iter_begin();
        if (c.pc == kPcDoubleBegin) block_double_begin();
        if (!wave_busy && c.pc == kPcLeaf && c.ahead_iter != c.iter + 1 && c.nleap >= 1 && c.iter + 1 < sa.iter_end)
            draw_iteration(c.iter + 1);

        // ---- 2. batched gradient of every waiting chain ----
        const bool at_leaf = c.pc == kPcLeaf, at_init = c.pc == kPcInitEval;
        const double half = 0.5 * (c.v * sa.eps), full = c.v * sa.eps;
        double theta_in = 0.0, r_half = 0.0;
        if (at_leaf) {
            r_half = c.ra + half * c.ga;
            theta_in = c.tha + full * r_half;
        } else if (at_init) {
            theta_in = c.tt;
        }
        // The operands of this wave's first row tile do not depend on the chains: ask for them
        // before the barrier so that their latency overlaps the wait.
        constexpr int kP1 = (KS1 + 1) / 2, kP2 = 2 * MT;   // operand pairs of the two GEMMs
        constexpr int kPerTile = (kP1 + kP2) * 64;         // double2 elements per tile
        double2 a1[kP1], a2[kP2];
        // (buffer loads: the tile's place in the stream is a scalar offset and the lane's a constant, so fetching
        // operands costs no vector instruction for addresses)
        auto load_pair = [&](int tile, int pair) __attribute__((always_inline)) -> double2 {
            const v4u raw = __builtin_amdgcn_raw_buffer_load_b128(ops_rsrc, lane * 16, (tile * kPerTile + pair * 64) * 16, 0);
            return __builtin_bit_cast(double2, raw);
        };
#pragma unroll
        for (int i = 0; i < kP1; ++i) a1[i] = load_pair(wave, i);
#pragma unroll
        for (int i = 0; i < kP2; ++i) a2[i] = load_pair(wave, kP1 + i);
        sTheta[grp][k_slot] = theta_in;
        tile_lds_barrier();
        // (counted up before this barrier, read after it, counted up again only after the round's second barrier)
        if (*const_cast<volatile int*>(&sHalted) == kTileChains) break;  // every chain of the workgroup has halted
        n_rounds += 1;
        const long long t1 = clock64();

        {
            v4d G[MT];
#pragma unroll
            for (int u = 0; u < MT; ++u) G[u] = v4d{0.0, 0.0, 0.0, 0.0};
            // log-likelihood: sum_i log(1 + e^{-z~_i}) = sum max(-z~, 0) - log prod sigma(|z~|), and
            // sum max(-z~, 0) = (1/2) sum |z~| - (1/2) sum z~ (the last sum is colsum . theta, added per chain below)
            double sum_abs = 0.0, prod = 1.0, log_prod = 0.0;
            // One row tile: Z = X~ Theta, the logistic functions on the accumulator, G += X~' s.
            // Each operand register is refilled for the next tile as soon as its MFMA has consumed
            // it, so every load has most of a tile's duration to arrive.
            // (the product is folded into a logarithm every 64 tiles of a wave - 256 factors in [1/2, 1], far
            // from underflow - in an outer loop, so that the hot loop has no branch in its body)
            double b1[KS1];
#pragma unroll
            for (int s = 0; s < KS1; ++s) b1[s] = sTheta[lane & 15][4 * s + (lane >> 4)];
            // The share of the constant column in every logit of a real row: the first GEMM starts from it.
            v4d z_init = v4d{0.0, 0.0, 0.0, 0.0};
            if (kZ0) {
                const double z0 = ta.z0_val * sTheta[lane & 15][ta.d - 1];
                z_init = v4d{z0, z0, z0, z0};
            }
            auto row_tile = [&](const int t, const v4d z_start, const bool more) __attribute__((always_inline)) {
                v4d z = z_start;
#pragma unroll
                for (int s = 0; s < KS1; ++s)
                    z = __builtin_amdgcn_mfma_f64_16x16x4f64((s & 1) ? a1[s >> 1].y : a1[s >> 1].x, b1[s], z, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (more) {
#pragma unroll
                    for (int i = 0; i < kP1; ++i) a1[i] = load_pair(t + kTileWaves, i);
                }
                double sg[4];
                {
                    const double zq[4] = {z[0], z[1], z[2], z[3]};
                    double slope[4];
                    logistic_slopes<4>(zq, sFtab, slope);  // a NaN or infinite logit makes its slope NaN
#pragma unroll
                    for (int q = 0; q < 4; ++q) sg[q] = __builtin_copysign(slope[q], zq[q]);
                    // (absolute values are operand modifiers: they cost no instruction)
#pragma unroll
                    for (int q = 0; q < 4; ++q)  // (written out: the compiler would clear the sign bit with an instruction of its own)
                        asm("v_add_f64 %0, %0, |%1|" : "+v"(sum_abs) : "v"(zq[q]));
                    prod *= ((fabs(sg[0]) + 0.5) * (fabs(sg[1]) + 0.5)) * ((fabs(sg[2]) + 0.5) * (fabs(sg[3]) + 0.5));
                }
#pragma unroll
                for (int u = 0; u < MT; ++u)
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        G[u] = __builtin_amdgcn_mfma_f64_16x16x4f64((s & 1) ? a2[u * 2 + (s >> 1)].y : a2[u * 2 + (s >> 1)].x, sg[s],
                                                                    G[u], 0, 0, 0);
                if (more) {
#pragma unroll
                    for (int i = 0; i < kP2; ++i) a2[i] = load_pair(t + kTileWaves, kP1 + i);
                }
            };
            // (a last tile that is not full is run after the loop, by the wave whose turn it is)
            const int n_loop = (kZ0 && ta.rem_rows != 0) ? ta.n_tiles - 1 : ta.n_tiles;
            for (int t_chunk = wave; t_chunk < n_loop; t_chunk += 64 * kTileWaves) {
                const int t_stop = min(n_loop, t_chunk + 64 * kTileWaves);
                for (int t = t_chunk; t < t_stop; t += kTileWaves) row_tile(t, z_init, t + kTileWaves < ta.n_tiles);
                if (t_chunk + 64 * kTileWaves < n_loop) {  // more follow
                    log_prod += log_unit(prod, sFtab + kFtabDoubles);
                    prod = 1.0;
                }
            }
            if (kZ0 && ta.rem_rows != 0 && wave == ((ta.n_tiles - 1) & (kTileWaves - 1))) {
                v4d z_part;  // accumulator element (register q, lane) belongs to row 4q + lane/16 of the tile
#pragma unroll
                for (int q = 0; q < 4; ++q) z_part[q] = (4 * q + (lane >> 4) < ta.rem_rows) ? z_init[q] : 0.0;
                row_tile(ta.n_tiles - 1, z_part, false);
            }
            log_prod += log_unit(prod, sFtab + kFtabDoubles);
            double ll = log_prod - 0.5 * sum_abs;
            // accumulator element (register q, lane) = G[feature 16u + 4q + lane/16][chain lane%16]
#pragma unroll
            for (int u = 0; u < MT; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) sG[wave][lane & 15][16 * u + 4 * q + (lane >> 4)] = G[u][q];
            ll = add_other_row(ll);
            ll = add_other_half(ll);
            if (lane < 16) sLL[wave][lane] = ll;
        }
        tile_lds_barrier();
        const long long t2 = clock64();

        // ---- 3. every chain collects its gradient and finishes its step ----
        if (at_leaf || at_init) {
            double gk = 0.0;
            // (the eight partial log-likelihoods ride on lanes 0..7 of the sum over the chain's lanes below)
            const double ll_part = (k < kTileWaves) ? sLL[k & (kTileWaves - 1)][grp] : 0.0;
            if (k < 16 * MT) {
#pragma unroll
                for (int w = 0; w < kTileWaves; ++w) gk += sG[w][grp][k];
            }
            // G = X~' sigma(-z~) = colsum/2 - X~' s,  s = sign(z~) F'(|z~|)
            gk = kin_range ? (half_colsum - gk) - theta_in * ta.prior_prec : 0.0;
            if (at_leaf) {
                const double r_new = r_half + half * gk;
                c.tha = theta_in;
                c.ra = r_new;
                c.ga = gk;
                c.nleap += 1;
                n_leaf += 1;
                c.sub += 1;
                if (c.sub >= sa.leaf_steps) {  // otherwise the leaf is not finished: the chain stays at LEAF
                    c.sub = 0;
                    // |theta|^2 for the prior, (1/2) colsum . theta = (1/2) sum z~ for the likelihood
                    double sq = fma(theta_in, theta_in * (-0.5 * ta.prior_prec), half_colsum * theta_in) + ll_part, kin = r_new * r_new;
                    group_sum2(sq, kin);
                    const double logp = ta.n_pad * 0.6931471805599453 + sq;
                    c.edge_logp = logp;
                    c.m += 1;
                    double delta = (-logp + 0.5 * kin) - c.H0;
                    if (!(fabs(delta) < INFINITY)) delta = INFINITY;
                    if (slice) {
                        const double log_slice = __shfl(c.pool_logp, kTileLanes - 1, kTileLanes);
                        c.cur_w = (log_slice <= -delta) ? 1.0 : 0.0;
                        c.cur_s = (log_slice < kDeltaMax - delta);
                    } else {
                        double e = c.log_unit_w - delta;  // logarithm of the leaf's weight in the current unit
                        if (e > 600.0) {  // the energy has fallen far: this leaf becomes the unit
                            const double shrink = exp_bounded(-e);
                            c.w_tree *= shrink;
                            if (k < 16) c.frame_w *= shrink;
                            c.log_unit_w = delta;
                            e = 0.0;
                        }
                        c.cur_w = exp_bounded(e);
                        c.cur_s = (delta <= kDeltaMax);
                    }
                    c.cur_idx = -1;  // the proposal of a one-leaf subtree is the edge itself
                    if ((c.m & 1) && c.j >= 1) {
                        // first leaf of every open subtree it starts; one copy serves them all
                        const int s = (c.m == 1) ? c.j : min(__ffs(c.m - 1) - 1, c.j);
                        first_store(s, 0, theta_in);
                        first_store(s, 1, r_new);
                    }
                    do_return();
                }
            } else {
                const double sq = group_sum(fma(theta_in, theta_in * (-0.5 * ta.prior_prec), half_colsum * theta_in) + ll_part);
                c.tg = gk;
                c.top_logp = ta.n_pad * 0.6931471805599453 + sq;
                n_extra += 1;
                c.pc = kPcIterBegin;
            }
        }
        cyc_control += t1 - t0;
        cyc_grad += t2 - t1;
        cyc_post += clock64() - t2;
    }

    if (k == 0) {
        atomicAdd(&sa.counters[kCtrUseful], n_leaf);
        atomicAdd(&sa.counters[kCtrExtra], n_extra);
    }
    if (tid == 0) {
        atomicAdd(&sa.counters[kCtrIssued], n_rounds * kTileChains);
        atomicAdd(&sa.counters[kCtrRounds], n_rounds);
        atomicAdd(&sa.counters[kCtrCycControl], (unsigned long long)cyc_control);
        atomicAdd(&sa.counters[kCtrCycGrad], (unsigned long long)cyc_grad);
        atomicAdd(&sa.counters[kCtrCycPost], (unsigned long long)cyc_post);
    }
}

template <int KS1, int MT, bool kZ0>
inline void tile_launch_inst(const TileArgs& ta, const DevSample& sa, int blocks, hipStream_t stream)
{
    if (sa.sampler == kSamplerSlice)
        hipLaunchKernelGGL((nuts_tile_kernel<KS1, MT, true, kZ0>), dim3((unsigned)blocks), dim3(kTileThreads), 0, stream, ta, sa);
    else
        hipLaunchKernelGGL((nuts_tile_kernel<KS1, MT, false, kZ0>), dim3((unsigned)blocks), dim3(kTileThreads), 0, stream, ta, sa);
}

inline void tile_launch(const TileData& td, const DevSample& sa, double prior_prec, const TileLaunch& tl,
                        hipStream_t stream)
{
    const bool z0 = td.z0_col >= 0;
    TileArgs ta{td.base, td.ftab, td.colsum, td.d, td.n_tiles, prior_prec, (double)td.n_pad,
                (unsigned)((size_t)td.n_alloc_tiles * 2 * tile_pairs_per_tile(td.ks1, td.mt) * 64 * sizeof(double)),
                z0 ? (int)(td.n_rows % kTileRows) : 0, td.z0_col, td.z0_val};
    if (z0) {  // d = 4 ks1 + 1
        switch (td.ks1) {
        case 1: tile_launch_inst<1, 1, true>(ta, sa, tl.blocks, stream); break;
        case 2: tile_launch_inst<2, 1, true>(ta, sa, tl.blocks, stream); break;
        case 3: tile_launch_inst<3, 1, true>(ta, sa, tl.blocks, stream); break;
        case 4: tile_launch_inst<4, 2, true>(ta, sa, tl.blocks, stream); break;
        case 5: tile_launch_inst<5, 2, true>(ta, sa, tl.blocks, stream); break;
        case 6: tile_launch_inst<6, 2, true>(ta, sa, tl.blocks, stream); break;
        default: tile_launch_inst<7, 2, true>(ta, sa, tl.blocks, stream); break;
        }
        return;
    }
    switch (td.ks1) {
    case 1: tile_launch_inst<1, 1, false>(ta, sa, tl.blocks, stream); break;
    case 2: tile_launch_inst<2, 1, false>(ta, sa, tl.blocks, stream); break;
    case 3: tile_launch_inst<3, 1, false>(ta, sa, tl.blocks, stream); break;
    case 4: tile_launch_inst<4, 1, false>(ta, sa, tl.blocks, stream); break;
    case 5: tile_launch_inst<5, 2, false>(ta, sa, tl.blocks, stream); break;
    case 6: tile_launch_inst<6, 2, false>(ta, sa, tl.blocks, stream); break;
    case 7: tile_launch_inst<7, 2, false>(ta, sa, tl.blocks, stream); break;
    default: tile_launch_inst<8, 2, false>(ta, sa, tl.blocks, stream); break;
    }
}

}  // namespace nuts
