// Quad kernel: dense Gaussian targets (d <= 128, binary64) with the precision-matrix product of
// four chains at a time on the matrix cores.
//
// Program-counter batching (Algorithm 2 of the paper) at wavefront scale.  A wavefront owns four
// chain slots; each chain has its own program counter, return-address stack and tree state in the
// registers of a 16-lane group (lane l of the group owns components 8l .. 8l+7 of every state
// vector; the per-level frame scalars sit one level per lane).  A round of a wave is:
//   1. control: the wave sweeps the blocks of the chain program in program order and runs each
//      block for exactly those of its chains that wait at it (masked), until all of them stand at
//      a point that needs the target's gradient;
//   2. the four positions go to LDS and G = P Theta (d x d times d x 4) is evaluated with
//      v_mfma_f64_4x4x4_4b_f64: four independent 4x4x4 blocks per instruction, here four groups of
//      4 rows of P against the same 4 columns of Theta.  The matrix sits in LDS in operand order
//      (one copy per workgroup, 128 KB at d = 128), every entry is read once per round and used
//      for four chains;
//   3. each chain takes its gradient back from LDS and finishes its leapfrog step.
// The four waves of a workgroup share nothing but the matrix: there is no barrier after start-up.
// A chain that ends its last iteration takes the next chain from the queue.
//
// Both ends of the trajectory, the current proposal and the momentum drawn ahead are in registers
// (one wave per SIMD, so a wave may use the whole register file); the level-indexed tree storage
// (proposal pool, first-leaf slots) is in global memory, 1 KB per vector, read and written as
// coalesced 64-byte pieces by the lane that owns them.
//
// Against one chain per wavefront with the matrix-vector product on the vector ALUs (the dense
// kernel) this pays once a compute unit has more than a handful of chains: the matrix product of
// four chains costs about what one chain's costs there, but a wave's control work is that of four
// chains.
#pragma once
#include <hip/hip_runtime.h>

#include <vector>

#include "nuts_dev.h"
#include "nuts_fastmath.h"
#include "nuts_rng.h"

namespace nuts {

constexpr int kQuadMaxDim = 128;
constexpr int kQuadMaxDepth = 12;
constexpr int kQuadChains = 4;     // chains per wavefront = the N of one MFMA block
constexpr int kQuadLanes = 16;     // lanes per chain
constexpr int kQuadV = 8;          // components per lane
constexpr int kQuadWaves = 4;      // wavefronts per workgroup, one per SIMD
constexpr int kQuadThreads = kQuadWaves * kWave;
constexpr int kQuadPitch = 144;    // doubles per chain in the LDS staging area (128 + 16: rows of different chains on different banks)
constexpr int kQuadVecLen = 128;   // doubles per workspace vector
constexpr long kQuadAutoChains = 2560;  // automatic choice: from this many chains on (10 per compute unit; measured
                                        // at d = 100: level with the one-chain-per-wavefront kernel at 2048 chains,
                                        // twice its rate from 4096 on)

struct QuadData {
    double* ops = nullptr;  // device: P in MFMA operand order, see quad_pack_operands
    int d = 0, n_r = 0, n_kb = 0;
};

struct QuadArgs {
    const double* ops;
    int d, n_r, n_kb;
};

// Operand stream of P (symmetric, d x d): for column block kb (columns 4kb .. 4kb+3) and row group R
// (rows 16R .. 16R+15), 64 doubles; element l = 16k + 4b + i is A[i][k] of block b, i.e.
// P[16R + 4b + i][4kb + k] (zero beyond d).  Order: kb outermost, then R.  The number of column blocks is
// rounded up to an even number (the kernel takes them two at a time); the extra one is zero.
inline void quad_pack_operands(const double* P, int64_t d, QuadData* qd, std::vector<double>* out)
{
    qd->d = (int)d;
    qd->n_r = (int)((d + 15) / 16);
    qd->n_kb = (int)((d + 3) / 4);
    qd->n_kb += qd->n_kb & 1;
    out->assign((size_t)qd->n_r * qd->n_kb * 64, 0.0);
    for (int kb = 0; kb < qd->n_kb; ++kb)
        for (int R = 0; R < qd->n_r; ++R)
            for (int l = 0; l < 64; ++l) {
                const int64_t row = 16 * R + 4 * ((l >> 2) & 3) + (l & 3), col = 4 * kb + (l >> 4);
                if (row < d && col < d) (*out)[((size_t)kb * qd->n_r + R) * 64 + l] = P[row * d + col];
            }
}

inline size_t quad_matrix_bytes(const QuadData& qd) { return (size_t)qd.n_r * qd.n_kb * 64 * sizeof(double); }
inline size_t quad_stage_bytes() { return (size_t)kQuadWaves * kQuadChains * kQuadPitch * sizeof(double); }

// Global-memory vectors of one chain slot, kQuadVecLen doubles each:
//   proposal pool  2*b + c            b <= D,  c in {theta, grad}
//   first-leaf     2*(D+1) + 2*s + c  s <= D,  c in {theta, r}
__host__ __device__ inline int quad_num_vectors(int max_depth) { return 4 * (max_depth + 1); }

// Sum over the 16 lanes of one chain (one DPP row): every lane ends with the same bits.
__device__ __forceinline__ double quad_sum(double x)
{
    x += dpp_rotate<0x128>(x);  // row_ror:8
    x += dpp_rotate<0x124>(x);  // row_ror:4
    x += dpp_rotate<0x122>(x);  // row_ror:2
    x += dpp_rotate<0x121>(x);  // row_ror:1
    return x;
}
__device__ __forceinline__ void quad_sum2(double& a, double& b)
{
    a += dpp_rotate<0x128>(a);
    b += dpp_rotate<0x128>(b);
    a += dpp_rotate<0x124>(a);
    b += dpp_rotate<0x124>(b);
    a += dpp_rotate<0x122>(a);
    b += dpp_rotate<0x122>(b);
    a += dpp_rotate<0x121>(a);
    b += dpp_rotate<0x121>(b);
}

// State of one chain, replicated over (and partly distributed across) its 16 lanes.
struct QuadChain {
    int pc, level, j, v, m, nleap, iter, cur_s, cur_idx, frame_idx;
    int sub;  // leapfrog steps already taken inside the current leaf
    uint64_t ret;
    long chain;
    uint32_t gchain, free_mask;
    // (weights of trajectory points are numbers exp(H0 - H) in a unit that moves when the energy falls far, as in the
    // tile kernel: a merge is an add, a selection a product and a comparison; log_unit_w is the logarithm of the unit)
    double H0, w_tree, cur_w, log_unit_w, edge_logp, top_logp, log_slice;
    // Lane-distributed scalars (lane l of the chain's 16 lanes):
    double frame_w;    // l = 1..12: weight of the open frame of level l
    double pool_logp;  // l = 0..12: log-density of pool buffer l
    double u_sub;      // l = 1..12: SUBTREE uniform of level l for the leaf counted in `u_sub_leaf`
    double u_top, u_top_n;  // l = doubling: TOP uniform of this / the drawn-ahead iteration
    // the end of the trajectory that the current doubling extends (direction v) and the other end; the two swap
    // places when the direction changes, so that a leapfrog step always reads and writes the same registers
    double tha[kQuadV], ra[kQuadV], ga[kQuadV], tho[kQuadV], ro[kQuadV], go[kQuadV];
    int act_v;  // direction of the end held in tha/ra/ga (0: both ends are the same point)
    double tt[kQuadV], tg[kQuadV];  // the trajectory's current proposal and its gradient
    double rn[kQuadV];              // the momentum drawn ahead for iteration `ahead_iter`
    double kin_n;                   // |rn|^2
    int ahead_iter, u_sub_leaf;
    uint32_t dirbits, dirbits_n;    // bit j: direction of doubling j (this / the drawn-ahead iteration)
};

// NR: row groups of 16 (ceil(d / 16)); the accumulators of one round are NR registers.
template <int NR, bool kSlice>
__global__ __launch_bounds__(kQuadThreads) void nuts_quad_kernel(QuadArgs qa, DevSample sa)
{
    extern __shared__ __align__(16) unsigned char quad_smem[];
    double* const sP = reinterpret_cast<double*>(quad_smem);
    const size_t mat_doubles = (size_t)qa.n_r * qa.n_kb * 64;
    double* const sStageAll = sP + mat_doubles;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = uni(tid >> 6);
    const int grp = lane >> 4;             // chain slot in the wave
    const int l16 = lane & (kQuadLanes - 1);
    const int c0 = kQuadV * l16;           // first component owned by this lane
    const int d = qa.d, D = sa.max_depth;
    const DrawKey key{sa.key0, sa.key1};
    constexpr bool slice = kSlice;
    const uint32_t all_bufs = (1u << (D + 1)) - 1u;
    double* const sStage = sStageAll + (size_t)wave * kQuadChains * kQuadPitch;  // this wave's positions / gradients
    // this lane's place in the operands of the matrix instruction: column (B, D) `ln`, block `lblk`;
    // `lq` is the contraction index of an A or B operand and the row of a D result
    const int ln = lane & 3, lblk = (lane >> 2) & 3, lq = lane >> 4;

    for (size_t i = tid; i < mat_doubles; i += kQuadThreads) sP[i] = qa.ops[i];
    for (int i = tid; i < kQuadWaves * kQuadChains * kQuadPitch; i += kQuadThreads) sStageAll[i] = 0.0;
    __syncthreads();

    const size_t slot = ((size_t)blockIdx.x * kQuadWaves + wave) * kQuadChains + grp;
    double* const wsc = reinterpret_cast<double*>(sa.workspace + slot * sa.slot_bytes) + c0;
    auto pool = [&](int b, int c) __attribute__((always_inline)) -> double* { return wsc + (size_t)(2 * b + c) * kQuadVecLen; };
    auto first = [&](int s, int c) __attribute__((always_inline)) -> double* {
        return wsc + (size_t)(2 * (D + 1) + 2 * s + c) * kQuadVecLen;
    };
    auto vload = [&](const double* src, double (&dst)[kQuadV]) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < kQuadV; e += 2) {
            const double2 x = *reinterpret_cast<const double2*>(src + e);
            dst[e] = x.x;
            dst[e + 1] = x.y;
        }
    };
    auto vstore = [&](double* dst, const double (&src)[kQuadV]) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < kQuadV; e += 2) *reinterpret_cast<double2*>(dst + e) = double2{src[e], src[e + 1]};
    };

    QuadChain c{};
    c.pc = kPcFetch;
    c.cur_idx = -1;
    unsigned long long n_leaf = 0, n_extra = 0, n_rounds = 0;
    long long cyc_control = 0, cyc_grad = 0, cyc_post = 0;  // where a round's time goes (shader-clock ticks)

    auto push_ret = [&](unsigned code) __attribute__((always_inline)) { c.ret = (c.ret << 2) | code; };
    auto do_return = [&]() __attribute__((always_inline)) {
        c.pc = ret_to_pc((unsigned)(c.ret & 3u));
        c.ret >>= 2;
        c.level += 1;
    };
    auto descend_to_leaf = [&]() __attribute__((always_inline)) {
        while (c.level > 0) {
            c.level -= 1;
            push_ret(kRetAfterLeft);
        }
        c.pc = kPcLeaf;
    };
    // Make sure the current proposal owns a pool buffer (a fresh leaf lives in the edge registers).
    auto materialise_cur = [&]() __attribute__((always_inline)) {
        if (c.cur_idx >= 0) return;
        const int b = __ffs(c.free_mask) - 1;
        c.free_mask &= ~(1u << b);
        vstore(pool(b, 0), c.tha);
        vstore(pool(b, 1), c.ga);
        if (l16 == b) c.pool_logp = c.edge_logp;
        c.cur_idx = b;
    };
    // ---- blocks of the chain program; each runs for the lanes whose chain waits at it ----
    auto block_after_right = [&]() __attribute__((always_inline)) {
        if (c.cur_s) {
            const int f = c.m - (1 << c.level) + 1;  // first leaf of this subtree, 1-based
            const int s = (f == 1) ? c.j : min(__ffs(f - 1) - 1, c.j);
            double tf[kQuadV], rf[kQuadV];
            vload(first(s, 0), tf);
            vload(first(s, 1), rf);
            const double l_w = __shfl(c.frame_w, c.level, kQuadLanes);
            const int l_idx = __shfl(c.frame_idx, c.level, kQuadLanes);
            const double u = __shfl(c.u_sub, c.level, kQuadLanes);
            // right with probability w_R / (w_L + w_R) (never when both are zero)
            const double w_new = l_w + c.cur_w;
            if (u * w_new < c.cur_w) {
                c.free_mask |= (1u << l_idx);
            } else {
                if (c.cur_idx >= 0) c.free_mask |= (1u << c.cur_idx);
                c.cur_idx = l_idx;
            }
            c.cur_w = w_new;
            // (theta+ - theta-) . r at both ends of the span; the difference is taken edge minus first leaf and
            // the direction's sign applied to the sums (negation is exact, so the values are the oracle's)
            double da = 0.0, db = 0.0;
#pragma unroll
            for (int e = 0; e < kQuadV; ++e) {
                const double delta = c.tha[e] - tf[e];
                da = fma(delta, rf[e], da);
                db = fma(delta, c.ra[e], db);
            }
            quad_sum2(da, db);
            c.cur_s = (c.v * da >= 0.0) && (c.v * db >= 0.0);
        }
        do_return();
    };
    auto block_after_left = [&]() __attribute__((always_inline)) {
        if (!c.cur_s) {  // the right half is never built
            do_return();
            return;
        }
        materialise_cur();
        if (l16 == c.level) {
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
            const double u = __shfl(c.u_top, c.j, kQuadLanes);
            if (u * c.w_tree < c.cur_w) {  // accept the new half with probability min(1, w_new / w_tree)
                if (c.cur_idx < 0) {
#pragma unroll
                    for (int e = 0; e < kQuadV; ++e) {
                        c.tt[e] = c.tha[e];
                        c.tg[e] = c.ga[e];
                    }
                    c.top_logp = c.edge_logp;
                } else {
                    vload(pool(c.cur_idx, 0), c.tt);
                    vload(pool(c.cur_idx, 1), c.tg);
                    c.top_logp = __shfl(c.pool_logp, c.cur_idx, kQuadLanes);
                }
            }
            c.w_tree += c.cur_w;
            double da = 0.0, db = 0.0;
#pragma unroll
            for (int e = 0; e < kQuadV; ++e) {
                const double delta = c.tha[e] - c.tho[e];
                da = fma(delta, c.ro[e], da);
                db = fma(delta, c.ra[e], db);
            }
            quad_sum2(da, db);
            go_on = (c.v * da >= 0.0) && (c.v * db >= 0.0);
        }
        c.j += 1;
        c.free_mask = all_bufs;  // nothing of the finished doubling stays in the pool
        c.pc = (go_on && c.j < D) ? kPcDoubleBegin : kPcIterEnd;
    };
    auto block_iter_end = [&]() __attribute__((always_inline)) {
        const size_t row = (size_t)c.iter * (size_t)sa.n_chains + (size_t)c.chain;
        if (sa.out_states) {
            double* dst = static_cast<double*>(sa.out_states) + row * d;
#pragma unroll
            for (int e = 0; e < kQuadV; ++e)
                if (c0 + e < d) dst[c0 + e] = c.tt[e];
        }
        if (l16 == 0) {
            if (sa.out_depths) sa.out_depths[row] = c.j;
            if (sa.out_nleap) sa.out_nleap[row] = c.nleap;
        }
        c.iter += 1;
        c.pc = (c.iter < sa.iter_end) ? kPcIterBegin : kPcFetch;
    };
    // normals for this lane's eight components from four draws (components 2k, 2k+1 share draw k)
    auto draw_normals = [&](uint32_t tag, uint32_t it, double (&out)[kQuadV]) __attribute__((always_inline)) {
        for (int p = 0; p < kQuadV / 2; ++p) {  // rolled: once per iteration, must not cost registers
            double z0 = 0.0, z1 = 0.0;
            const int comp = c0 + 2 * p;
            if (comp < d) {
                const Words4 w = draw(key, (uint32_t)(comp >> 1), tag, 0, it, c.gchain);
                normal_pair(w, z0, z1);
                if (comp + 1 >= d) z1 = 0.0;
            }
            // (static register indexes: the loop is rolled, so the pair is written through a switch)
            switch (p) {
            case 0: out[0] = z0; out[1] = z1; break;
            case 1: out[2] = z0; out[3] = z1; break;
            case 2: out[4] = z0; out[5] = z1; break;
            default: out[6] = z0; out[7] = z1; break;
            }
        }
    };
    auto block_fetch = [&]() __attribute__((always_inline)) {
        unsigned long long q = 0;
        if (l16 == 0) q = atomicAdd(&sa.counters[kCtrQueue], 1ull);
        q = __shfl(q, 0, kQuadLanes);
#pragma unroll
        for (int e = 0; e < kQuadV; ++e) c.tt[e] = 0.0;
        if ((long)q >= sa.n_chains) {
            c.pc = kPcHalt;
            return;
        }
        c.chain = (long)q;
        c.gchain = (uint32_t)(sa.first_chain + c.chain);
        c.iter = sa.iter_begin;
        c.ahead_iter = -1;
        c.u_sub_leaf = -1;
        c.free_mask = all_bufs;
        if (sa.init_states) {
            const double* src = static_cast<const double*>(sa.init_states) + (size_t)c.chain * d;
#pragma unroll
            for (int e = 0; e < kQuadV; ++e) c.tt[e] = c0 + e < d ? src[c0 + e] : 0.0;
        } else {
            draw_normals(kDrawInit, 0, c.tt);
        }
        c.pc = kPcInitEval;
    };
    // Every random number of an iteration that does not depend on where the trajectory goes: the
    // momentum, the direction of each doubling, the top-level acceptance uniforms (and the slice
    // height).  Keyed by (chain, iteration, purpose, position), so they can be made at any time.
    auto draw_iteration = [&](int it) __attribute__((always_inline)) {
        draw_normals(kDrawMomentum, (uint32_t)it, c.rn);
        double kin = 0.0;
#pragma unroll
        for (int e = 0; e < kQuadV; ++e) kin = fma(c.rn[e], c.rn[e], kin);
        c.kin_n = quad_sum(kin);
        const Words4 wd = draw(key, (uint32_t)l16, kDrawDirection, 0, (uint32_t)it, c.gchain);
        const unsigned long long votes = __ballot(wd.w0 >> 31);
        c.dirbits_n = (uint32_t)(votes >> (lane & 48)) & 0xffffu;
        const Words4 wt = draw(key, (uint32_t)l16, kDrawTop, 0, (uint32_t)it, c.gchain);
        c.u_top_n = uniform52(wt.w0, wt.w1);
        c.ahead_iter = it;
    };
    auto block_iter_begin = [&]() __attribute__((always_inline)) {
        if (c.ahead_iter != c.iter) draw_iteration(c.iter);
        c.dirbits = c.dirbits_n;
        c.u_top = c.u_top_n;
#pragma unroll
        for (int e = 0; e < kQuadV; ++e) {
            c.tha[e] = c.tho[e] = c.tt[e];
            c.ga[e] = c.go[e] = c.tg[e];
            c.ra[e] = c.ro[e] = c.rn[e];
        }
        c.act_v = 0;
        c.H0 = -c.top_logp + 0.5 * c.kin_n;
        c.w_tree = 1.0;  // the starting point: weight exp(0), or the first candidate
        c.log_unit_w = 0.0;
        if (slice) {
            const Words4 ws = draw(key, 0, kDrawSlice, 0, (uint32_t)c.iter, c.gchain);
            c.log_slice = log(uniform52(ws.w0, ws.w1));
        }
        c.j = 0;
        c.nleap = 0;
        c.u_sub_leaf = -1;
        c.pc = kPcDoubleBegin;
    };
    auto block_double_begin = [&]() __attribute__((always_inline)) {
        c.v = ((c.dirbits >> c.j) & 1u) ? 1 : -1;
        if (c.act_v == -c.v) {  // bring the end that is to be extended into the registers of the active end
#pragma unroll
            for (int e = 0; e < kQuadV; ++e) {
                double x;
                x = c.tha[e]; c.tha[e] = c.tho[e]; c.tho[e] = x;
                x = c.ra[e]; c.ra[e] = c.ro[e]; c.ro[e] = x;
                x = c.ga[e]; c.ga[e] = c.go[e]; c.go[e] = x;
            }
        }
        c.act_v = c.v;
        c.m = 0;
        c.level = c.j;
        push_ret(kRetDoubleEnd);
        c.pc = kPcBuild;
        descend_to_leaf();
    };

    for (;;) {
        const long long t0 = clock64();
        // ---- 1. control: one sweep over the chain program in program order; returns cascade ----
        // every merge that a leaf can complete draws at the same position (the leapfrog count): lane l draws for level
        // l, once per leaf (ahead of the loop and under a condition of its own: inside, the compiler hoists the generator
        // out of the loop and runs it in every round)
        if (c.pc == kPcAfterRight && c.cur_s && c.u_sub_leaf != c.nleap) {
            const Words4 w = draw(key, (uint32_t)c.nleap, kDrawSubtree, (uint32_t)l16, (uint32_t)c.iter, c.gchain);
            c.u_sub = uniform52(w.w0, w.w1);
            c.u_sub_leaf = c.nleap;
        }
        for (;;) {
            const bool any_right = __any(c.pc == kPcAfterRight), any_left = __any(c.pc == kPcAfterLeft);
            if (!any_right && !any_left) break;
            if (any_right && c.pc == kPcAfterRight) block_after_right();
            if (c.pc == kPcAfterLeft) block_after_left();
        }
        const bool wave_busy = __any(c.pc == kPcDoubleEnd);
        if (c.pc == kPcDoubleEnd) block_double_end();
        if (c.pc == kPcIterEnd) block_iter_end();
        if (c.pc == kPcFetch) block_fetch();
        if (c.pc == kPcIterBegin) block_iter_begin();
        if (c.pc == kPcDoubleBegin) block_double_begin();
        if (!wave_busy && c.pc == kPcLeaf && c.ahead_iter != c.iter + 1 && c.nleap >= 1 && c.iter + 1 < sa.iter_end)
            draw_iteration(c.iter + 1);

        // ---- 2. gradients of the wave's four chains ----
        const bool at_leaf = c.pc == kPcLeaf, at_init = c.pc == kPcInitEval;
        if (!__any(at_leaf || at_init)) break;  // every chain of the wave has halted
        n_rounds += 1;
        const double half = 0.5 * (c.v * sa.eps), full = c.v * sa.eps;
        double theta_in[kQuadV], r_half[kQuadV];
#pragma unroll
        for (int e = 0; e < kQuadV; ++e) {
            theta_in[e] = 0.0;
            r_half[e] = 0.0;
            if (at_leaf) {
                r_half[e] = c.ra[e] + half * c.ga[e];
                theta_in[e] = c.tha[e] + full * r_half[e];
            } else if (at_init) {
                theta_in[e] = c.tt[e];
            }
        }
        vstore(sStage + grp * kQuadPitch + c0, theta_in);
        __builtin_amdgcn_wave_barrier();
        const long long t1 = clock64();
        {
            double acc[NR];
#pragma unroll
            for (int R = 0; R < NR; ++R) acc[R] = 0.0;
            const double* a = sP + lane;
            const double* b = sStage + ln * kQuadPitch + lq;
            // Columns 4kb .. 4kb+3 of P against the same four components of the four positions, two column
            // blocks per trip with their operands in two sets of registers: while the instructions of one set
            // run, the other set's LDS reads are on their way (what is still outstanding where the loop closes was
            // requested a whole set of instructions earlier).
            double a0[NR], a1[NR], b0, b1;
#pragma unroll
            for (int R = 0; R < NR; ++R) a0[R] = a[R * 64];
            b0 = b[0];
#pragma unroll
            for (int R = 0; R < NR; ++R) a1[R] = a[(NR + R) * 64];
            b1 = b[4];
            // one pair of column blocks: each set's registers are refilled (two blocks ahead) as soon as its
            // instructions have been issued; past the end the first blocks are asked for again, nobody uses them
            auto pair_step = [&](int kb) __attribute__((always_inline)) {
                const bool more = kb + 2 < qa.n_kb;
                const double* an = more ? a + 2 * NR * 64 : sP + lane;
                const int bn = more ? 4 * kb + 8 : 0;
#pragma unroll
                for (int R = 0; R < NR; ++R) acc[R] = __builtin_amdgcn_mfma_f64_4x4x4f64(a0[R], b0, acc[R], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int R = 0; R < NR; ++R) a0[R] = an[R * 64];
                b0 = b[bn];
#pragma unroll
                for (int R = 0; R < NR; ++R) acc[R] = __builtin_amdgcn_mfma_f64_4x4x4f64(a1[R], b1, acc[R], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int R = 0; R < NR; ++R) a1[R] = an[(NR + R) * 64];
                b1 = b[bn + 4];
                a += 2 * NR * 64;
            };
            int kb = 0;
            for (; kb + 4 <= qa.n_kb; kb += 4) {  // two pairs per trip: the wait where the loop closes comes half as often
                pair_step(kb);
                pair_step(kb + 2);
            }
            for (; kb < qa.n_kb; kb += 2) pair_step(kb);
            __builtin_amdgcn_wave_barrier();
            // accumulator R, lane 16i + 4b + n: (P theta_n)[16R + 4b + i]
#pragma unroll
            for (int R = 0; R < NR; ++R) sStage[ln * kQuadPitch + 16 * R + 4 * lblk + lq] = acc[R];
            __builtin_amdgcn_wave_barrier();
        }

        const long long t2 = clock64();
        // ---- 3. every chain collects its gradient and finishes its step ----
        if (at_leaf || at_init) {
            double gk[kQuadV];
            vload(sStage + grp * kQuadPitch + c0, gk);
            double dot = 0.0;
#pragma unroll
            for (int e = 0; e < kQuadV; ++e) {
                gk[e] = c0 + e < d ? -gk[e] : 0.0;
                dot = fma(theta_in[e], gk[e], dot);
            }
            if (at_leaf) {
                double kin = 0.0;
#pragma unroll
                for (int e = 0; e < kQuadV; ++e) {
                    const double r_new = r_half[e] + half * gk[e];
                    kin = fma(r_new, r_new, kin);
                    c.tha[e] = theta_in[e];
                    c.ra[e] = r_new;
                    c.ga[e] = gk[e];
                }
                c.nleap += 1;
                n_leaf += 1;
                c.sub += 1;
                if (c.sub >= sa.leaf_steps) {  // otherwise the leaf is not finished: the chain stays at LEAF
                    c.sub = 0;
                    quad_sum2(dot, kin);
                    const double logp = 0.5 * dot;
                    c.edge_logp = logp;
                    c.m += 1;
                    double delta = (-logp + 0.5 * kin) - c.H0;
                    if (!(fabs(delta) < INFINITY)) delta = INFINITY;
                    if (slice) {
                        c.cur_w = (c.log_slice <= -delta) ? 1.0 : 0.0;
                        c.cur_s = (c.log_slice < kDeltaMax - delta);
                    } else {
                        double e = c.log_unit_w - delta;  // logarithm of the leaf's weight in the current unit
                        if (e > 600.0) {  // the energy has fallen far: this leaf becomes the unit
                            const double shrink = exp_bounded(-e);
                            c.w_tree *= shrink;
                            c.frame_w *= shrink;
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
                        vstore(first(s, 0), c.tha);
                        vstore(first(s, 1), c.ra);
                    }
                    do_return();
                }
            } else {
#pragma unroll
                for (int e = 0; e < kQuadV; ++e) c.tg[e] = gk[e];
                c.top_logp = 0.5 * quad_sum(dot);
                n_extra += 1;
                c.pc = kPcIterBegin;
            }
        }
        __builtin_amdgcn_wave_barrier();  // the staging area is written again at the top of the next round
        cyc_control += t1 - t0;
        cyc_grad += t2 - t1;
        cyc_post += clock64() - t2;
    }

    if (l16 == 0) {
        atomicAdd(&sa.counters[kCtrUseful], n_leaf);
        atomicAdd(&sa.counters[kCtrExtra], n_extra);
    }
    if (lane == 0) {
        atomicAdd(&sa.counters[kCtrIssued], n_rounds * kQuadChains);
        atomicAdd(&sa.counters[kCtrRounds], n_rounds);
        atomicAdd(&sa.counters[kCtrCycControl], (unsigned long long)cyc_control);
        atomicAdd(&sa.counters[kCtrCycGrad], (unsigned long long)cyc_grad);
        atomicAdd(&sa.counters[kCtrCycPost], (unsigned long long)cyc_post);
    }
}

template <int NR>
inline hipError_t quad_launch_inst(const QuadArgs& qa, const DevSample& sa, int blocks, size_t lds_bytes, hipStream_t stream)
{
    const void* fn = sa.sampler == kSamplerSlice ? reinterpret_cast<const void*>(nuts_quad_kernel<NR, true>)
                                                  : reinterpret_cast<const void*>(nuts_quad_kernel<NR, false>);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    if (sa.sampler == kSamplerSlice)
        hipLaunchKernelGGL((nuts_quad_kernel<NR, true>), dim3((unsigned)blocks), dim3(kQuadThreads), lds_bytes, stream, qa, sa);
    else
        hipLaunchKernelGGL((nuts_quad_kernel<NR, false>), dim3((unsigned)blocks), dim3(kQuadThreads), lds_bytes, stream, qa, sa);
    return hipGetLastError();
}

inline hipError_t quad_launch(const QuadArgs& qa, const DevSample& sa, int blocks, size_t lds_bytes, hipStream_t stream)
{
    switch (qa.n_r) {
    case 1: return quad_launch_inst<1>(qa, sa, blocks, lds_bytes, stream);
    case 2: return quad_launch_inst<2>(qa, sa, blocks, lds_bytes, stream);
    case 3: return quad_launch_inst<3>(qa, sa, blocks, lds_bytes, stream);
    case 4: return quad_launch_inst<4>(qa, sa, blocks, lds_bytes, stream);
    case 5: return quad_launch_inst<5>(qa, sa, blocks, lds_bytes, stream);
    case 6: return quad_launch_inst<6>(qa, sa, blocks, lds_bytes, stream);
    case 7: return quad_launch_inst<7>(qa, sa, blocks, lds_bytes, stream);
    default: return quad_launch_inst<8>(qa, sa, blocks, lds_bytes, stream);
    }
}

}  // namespace nuts
