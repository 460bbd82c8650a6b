// Register-resident kernel for element-wise targets (standard normal, diagonal
// Gaussian): the HBM-bound corner of the problem.
//
// One wavefront per chain slot, as in the general wave kernel, but the end of
// the trajectory that is being extended - position and momentum - stays in
// registers (kVpl values per lane), and the gradient -theta_i / sigma_i^2 is
// recomputed from the position instead of being stored.  A leapfrog step then
// moves no memory at all; what is left is the tree's own traffic:
//   * an odd leaf is written once as "first leaf" if it opens a subtree of more than two leaves,
//   * the proposal of a subtree of two or more leaves is written once to the pool if that subtree is
//     a left half,
//   * every merge above the lowest level reads one first-leaf state for its U-turn test,
//   * a change of direction swaps the register end with the one kept in memory.
// The lowest level of the tree never touches memory: an odd leaf is also kept in a second pair of
// register vectors until the next leaf has been merged with it (first leaf and left proposal of that
// two-leaf subtree), which takes away half of the merges' reads and of the first-leaf writes.
// All workspace vectors are padded to whole 16-byte lane accesses and the padding
// is kept at zero, so loads and stores are unguarded, fully coalesced dwordx4.
#pragma once
#include "nuts_dev.h"
#include "nuts_fastmath.h"
#include "nuts_rng.h"

namespace nuts {

// Workspace vectors of one slot, D = max_tree_depth:
//   0, 1                      the trajectory end that is not in registers (theta, r)
//   2                         (unused)
//   3 + b                     proposal pool, b < D + 2 (theta)
//   3 + (D+2) + 2*s + c       first-leaf slots, s <= D, c in {theta, r}
constexpr int kElemMaxBytes = 4096;  // largest state vector: 1024 binary32 or 512 binary64 components
__host__ __device__ inline int elem_num_vectors(int max_depth) { return 3 + (max_depth + 2) + 2 * (max_depth + 1); }

template <typename T>
struct ElemVec;
template <>
struct ElemVec<float> {
    static constexpr int kWidth = 4;
    typedef float4 type;
};
template <>
struct ElemVec<double> {
    static constexpr int kWidth = 2;
    typedef double2 type;
};

template <typename T, int kVpl>
struct ElemChain {
    static constexpr int kW = ElemVec<T>::kWidth;
    static constexpr int kChunks = kVpl / kW;
    typedef typename ElemVec<T>::type Vec;

    const DevTarget<T>& tg;
    const DevSample& sa;
    const int lane, d, D, dstride;
    T* const ws;
    const double* const ftab;  // LDS: table of the logistic function for weight merges
    const T* const wv;         // LDS: 1/sigma^2, zero padded to whole lane accesses (one copy per workgroup)
    double* const usub;        // LDS, 64 doubles of this wave: SUBTREE uniform of level l for the leaf counted in u_sub_leaf
    int u_sub_leaf = -1;       // (the same for the whole wave: a scalar register)

    T th[kVpl], r[kVpl];    // the register end of the trajectory
    T pth[kVpl], pr[kVpl];  // the last odd leaf, until the leaf after it has been merged with it
    double prev_logp = 0;   // its log-density
    static constexpr int kInEdge = -1, kInPrev = -2;  // cur_idx / frame_idx: the proposal is th, or pth

    int pc = kPcFetch, level = 0, j = 0, v = 1, m = 0, nleap = 0, iter = 0, act = 1;
    uint64_t ret = 0;
    long chain = 0;
    uint32_t gchain = 0, free_mask = 0;
    double H0 = 0, lw_tree = 0, cur_lw = 0, edge_logp = 0, log_slice = 0;
    int cur_s = 0, cur_idx = -1, top_idx = 0;
    double frame_lw = 0, pool_logp = 0;  // lane k: level k / pool buffer k
    int frame_idx = 0;
    unsigned long long n_leaf = 0, n_extra = 0;

    __device__ ElemChain(const DevTarget<T>& tg_, const DevSample& sa_, int lane_, T* ws_, const double* ftab_, const T* wv_,
                         double* usub_)
        : tg(tg_), sa(sa_), lane(lane_), d(tg_.d), D(sa_.max_depth), dstride(tg_.dstride), ws(ws_), ftab(ftab_), wv(wv_),
          usub(usub_) {}

    __device__ int elem(int q, int e) const { return (q * kWave + lane) * kW + e; }  // component of register q*kW+e
    __device__ T* other(int c) const { return ws + (size_t)c * dstride; }
    __device__ const T* wvec() const { return wv; }
    __device__ T* pool(int b) const { return ws + (size_t)(3 + b) * dstride; }
    __device__ T* first(int s, int c) const { return ws + (size_t)(3 + (D + 2) + 2 * s + c) * dstride; }
    __device__ DrawKey key() const { return DrawKey{sa.key0, sa.key1}; }

    __device__ void load(const T* src, T (&dst)[kVpl]) const
    {
#pragma unroll
        for (int q = 0; q < kChunks; ++q) {
            if (elem(q, 0) < dstride) {
                const Vec x = *reinterpret_cast<const Vec*>(src + elem(q, 0));
                const T* xs = reinterpret_cast<const T*>(&x);
#pragma unroll
                for (int e = 0; e < kW; ++e) dst[q * kW + e] = xs[e];
            } else {
#pragma unroll
                for (int e = 0; e < kW; ++e) dst[q * kW + e] = T(0);
            }
        }
    }
    __device__ void store(T* dst, const T (&src)[kVpl]) const
    {
#pragma unroll
        for (int q = 0; q < kChunks; ++q) {
            if (elem(q, 0) < dstride) {
                Vec x;
                T* xs = reinterpret_cast<T*>(&x);
#pragma unroll
                for (int e = 0; e < kW; ++e) xs[e] = src[q * kW + e];
                *reinterpret_cast<Vec*>(dst + elem(q, 0)) = x;
            }
        }
    }
    // Standard normals for every component (zero beyond d), written to a workspace vector.  A rolled
    // loop over memory: this runs once per iteration and must not cost registers.
    __device__ void draw_normals_to(uint32_t tag, uint32_t iteration, T* dst) const
    {
        for (int i = 2 * lane; i < dstride; i += 2 * kWave) {  // components i, i+1 share a Philox block
            T z0 = T(0), z1 = T(0);
            if (i < d) {
                const Words4 wd = draw(key(), (uint32_t)(i >> 1), tag, 0, iteration, gchain);
                z0 = (T)normal_of(wd, false);
                if (i + 1 < d) z1 = (T)normal_of(wd, true);
            }
            dst[i] = z0;
            dst[i + 1] = z1;
        }
        __threadfence_block();  // other lanes of this wave read these values back
        __builtin_amdgcn_wave_barrier();
    }

    __device__ void push_ret(unsigned code) { ret = (ret << 2) | code; }
    __device__ void do_return()
    {
        pc = ret_to_pc((unsigned)(ret & 3u));
        ret >>= 2;
        level += 1;
    }
    __device__ void materialise_cur()
    {
        if (cur_idx >= 0) return;
        const int b = __ffs(free_mask) - 1;
        free_mask &= ~(1u << b);
        if (cur_idx == kInPrev) {
            store(pool(b), pth);
            if (lane == b) pool_logp = prev_logp;
        } else {
            store(pool(b), th);
            if (lane == b) pool_logp = edge_logp;
        }
        cur_idx = b;
    }
    __device__ uint32_t all_bufs() const { return (1u << (D + 2)) - 1u; }

    // logp = (1/2) sum theta_i g_i with g_i = -(theta_i w_i); every lane gets the same value
    __device__ double logp_of_registers() const
    {
        T w[kVpl];
        load(wvec(), w);
        double part = 0.0;
#pragma unroll
        for (int i = 0; i < kVpl; ++i) {
            const T g = -(th[i] * w[i]);
            part = fma((double)th[i], (double)g, part);
        }
        return 0.5 * wave_sum(part);
    }

    // U-turn test between the register end and a state (tx, rx) in memory; `reg_is_plus` says
    // which of the two is later in time.
    __device__ bool uturn_ok_regs(const T (&xt)[kVpl], const T (&xr)[kVpl], bool reg_is_plus) const
    {
        double da = 0.0, db = 0.0;
#pragma unroll
        for (int i = 0; i < kVpl; ++i) {
            const T delta = reg_is_plus ? th[i] - xt[i] : xt[i] - th[i];
            da = fma((double)delta, (double)xr[i], da);
            db = fma((double)delta, (double)r[i], db);
        }
        wave_sum2(da, db);
        return (da >= 0.0) && (db >= 0.0);
    }
    __device__ bool uturn_ok_with(const T* tx, const T* rx, bool reg_is_plus) const
    {
        T xt[kVpl], xr[kVpl];
        load(tx, xt);
        load(rx, xr);
        return uturn_ok_regs(xt, xr, reg_is_plus);
    }

    __device__ void block_fetch()
    {
        unsigned long long c = 0;
        if (lane == 0) c = atomicAdd(&sa.counters[kCtrQueue], 1ull);
        c = __shfl(c, 0, kWave);
        if ((long)c >= sa.n_chains) {
            pc = kPcHalt;
            return;
        }
        chain = (long)c;
        gchain = (uint32_t)(sa.first_chain + chain);
        iter = sa.iter_begin;
        top_idx = 0;
        free_mask = all_bufs() & ~1u;
        if (sa.init_states) {
            const T* src = (const T*)sa.init_states + (size_t)chain * d;
#pragma unroll
            for (int q = 0; q < kChunks; ++q)
#pragma unroll
                for (int e = 0; e < kW; ++e) th[q * kW + e] = elem(q, e) < d ? src[elem(q, e)] : T(0);
            store(pool(0), th);
        } else {
            draw_normals_to(kDrawInit, 0, pool(0));
            load(pool(0), th);
        }
        const double lp = logp_of_registers();  // the gradient at x0 is implicit: nothing to wait for
        if (lane == 0) pool_logp = lp;
        n_extra += 1;
        pc = kPcIterBegin;
    }

    __device__ void block_iter_begin()
    {
        load(pool(top_idx), th);
        draw_normals_to(kDrawMomentum, (uint32_t)iter, other(1));
        load(other(1), r);
        double kin = 0.0;
#pragma unroll
        for (int i = 0; i < kVpl; ++i) kin = fma((double)r[i], (double)r[i], kin);
        store(other(0), th);  // both ends of the trajectory start at the current point
        act = 1;
        H0 = -read_lane(pool_logp, uni(top_idx)) + 0.5 * wave_sum(kin);
        lw_tree = 0.0;
        if (sa.sampler == kSamplerSlice) {
            const Words4 ws = draw(key(), 0, kDrawSlice, 0, (uint32_t)iter, gchain);
            log_slice = log(uniform52(ws.w0, ws.w1));
            lw_tree = 1.0;  // the starting point is the first candidate
        }
        j = 0;
        nleap = 0;
        u_sub_leaf = -1;  // leaf counts restart
        pc = kPcDoubleBegin;
    }

    __device__ void block_double_begin()
    {
        const Words4 wd = draw(key(), (uint32_t)j, kDrawDirection, 0, (uint32_t)iter, gchain);
        v = (wd.w0 >> 31) ? 1 : -1;
        const int e = v > 0 ? 1 : 0;
        if (e != act) {  // bring the end that is to be extended into registers
            T xt[kVpl], xr[kVpl];
            load(other(0), xt);
            load(other(1), xr);
            store(other(0), th);
            store(other(1), r);
#pragma unroll
            for (int i = 0; i < kVpl; ++i) {
                th[i] = xt[i];
                r[i] = xr[i];
            }
            act = e;
        }
        m = 0;
        level = j;
        push_ret(kRetDoubleEnd);
        while (level > 0) {  // BUILD(level) -> BUILD(level-1) -> ... -> leaf
            level -= 1;
            push_ret(kRetAfterLeft);
        }
        pc = kPcLeaf;
    }

    __device__ void block_leaf()
    {
        const T half = (T)(0.5 * (v * sa.eps)), full = (T)(v * sa.eps);
        T w[kVpl];
        load(wvec(), w);
        // all but the last of the leaf's leapfrog steps: no energy is needed there
        for (int step = 1; step < sa.leaf_steps; ++step) {
#pragma unroll
            for (int i = 0; i < kVpl; ++i) {
                const T g0 = -(th[i] * w[i]);
                const T rh = r[i] + half * g0;
                const T tn = th[i] + full * rh;
                const T g1 = -(tn * w[i]);
                th[i] = tn;
                r[i] = rh + half * g1;
            }
        }
        double lp = 0.0, kin = 0.0;
#pragma unroll
        for (int i = 0; i < kVpl; ++i) {
            const T g0 = -(th[i] * w[i]);
            const T rh = r[i] + half * g0;
            const T tn = th[i] + full * rh;
            const T g1 = -(tn * w[i]);
            const T rn = rh + half * g1;
            th[i] = tn;
            r[i] = rn;
            lp = fma((double)tn, (double)g1, lp);
            kin = fma((double)rn, (double)rn, kin);
        }
        wave_sum2(lp, kin);
        edge_logp = 0.5 * lp;
        m += 1;
        nleap += sa.leaf_steps;
        n_leaf += sa.leaf_steps;
        double delta = (-edge_logp + 0.5 * kin) - H0;
        if (!(fabs(delta) < INFINITY)) delta = INFINITY;
        if (sa.sampler == kSamplerSlice) {
            cur_lw = (log_slice <= -delta) ? 1.0 : 0.0;
            cur_s = (log_slice < kDeltaMax - delta);
        } else {
            cur_lw = -delta;
            cur_s = (delta <= kDeltaMax);
        }
        cur_idx = kInEdge;
        if ((m & 1) && j >= 1) {
            // first leaf of every open subtree it starts: the two-leaf one reads it from registers, the
            // larger ones (if any) share one copy in memory
#pragma unroll
            for (int i = 0; i < kVpl; ++i) {
                pth[i] = th[i];
                pr[i] = r[i];
            }
            prev_logp = edge_logp;
            const int s = (m == 1) ? j : min(__ffs(m - 1) - 1, j);
            if (s >= 2) {
                store(first(s, 0), th);
                store(first(s, 1), r);
            }
        }
        do_return();
    }

    __device__ void block_after_left()
    {
        if (!cur_s) {
            do_return();
            return;
        }
        if (level == 1)
            cur_idx = kInPrev;  // the left leaf of a two-leaf subtree stays in registers until the merge
        else
            materialise_cur();
        if (lane == level) {
            frame_lw = cur_lw;
            frame_idx = cur_idx;
        }
        level -= 1;
        push_ret(kRetAfterRight);
        while (level > 0) {
            level -= 1;
            push_ret(kRetAfterLeft);
        }
        pc = kPcLeaf;
    }

    __device__ void block_after_right()
    {
        if (cur_s) {
            // the subtree's first leaf is asked for before anything else: its memory latency then runs under
            // the random draw and the weight arithmetic below
            const int f = m - (1 << level) + 1;
            const int s = (f == 1) ? j : min(__ffs(f - 1) - 1, j);
            const bool lowest = uni(level) == 1;  // two leaves: the first one is still in registers
            T xt[kVpl], xr[kVpl];
            if (!lowest) {
                load(first(s, 0), xt);
                load(first(s, 1), xr);
            }
            const double l_lw = read_lane(frame_lw, uni(level));  // the level is the same for the whole wave
            const int l_idx = __builtin_amdgcn_readlane(frame_idx, uni(level));
            const bool slice = sa.sampler == kSamplerSlice;
            if (uni(u_sub_leaf) != uni(nleap)) {
                // every merge this leaf completes draws at the same position: lane l draws for level l, once per leaf;
                // the values wait in LDS (they would cost registers this kernel does not have)
                const Words4 wd = draw(key(), (uint32_t)nleap, kDrawSubtree, (uint32_t)lane, (uint32_t)iter, gchain);
                usub[lane] = uniform52(wd.w0, wd.w1);
                u_sub_leaf = nleap;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
            }
            const double u = usub[uni(level)];
            double lw_new;
            bool take_right;
            if (slice) {
                lw_new = l_lw + cur_lw;
                take_right = u * lw_new < cur_lw;
            } else {  // both log-weights are finite here; u < w_R / (w_L + w_R) through the table
                double p_right;
                merge_logweights(l_lw, cur_lw, ftab, lw_new, p_right);
                take_right = u < p_right;
            }
            if (take_right) {
                if (l_idx >= 0) free_mask |= (1u << l_idx);
            } else {
                if (cur_idx >= 0) free_mask |= (1u << cur_idx);
                cur_idx = l_idx;
            }
            cur_lw = lw_new;
            cur_s = lowest ? uturn_ok_regs(pth, pr, v > 0) : uturn_ok_regs(xt, xr, v > 0);
        }
        do_return();
    }

    __device__ void block_double_end()
    {
        bool go_on = false;
        if (cur_s) {
            const Words4 wd = draw(key(), (uint32_t)j, kDrawTop, 0, (uint32_t)iter, gchain);
            const double u = uniform52(wd.w0, wd.w1);
            bool accept;
            if (sa.sampler == kSamplerSlice) {
                accept = u * lw_tree < cur_lw;
                lw_tree += cur_lw;
            } else {  // u < w_new / w_tree, with p = w_new / (w_tree + w_new) from the table
                double lw_new, p;
                merge_logweights(lw_tree, cur_lw, ftab, lw_new, p);
                accept = u * (1.0 - p) < p;
                lw_tree = lw_new;
            }
            if (accept) {
                materialise_cur();
                top_idx = cur_idx;
            }
            go_on = uturn_ok_with(other(0), other(1), act == 1);
        }
        // (an invalid new half ends the iteration: the tree's weight is not needed any more)
        j += 1;
        free_mask = all_bufs() & ~(1u << top_idx);
        pc = (go_on && j < D) ? kPcDoubleBegin : kPcIterEnd;
    }

    __device__ void block_iter_end()
    {
        const size_t row = (size_t)iter * (size_t)sa.n_chains + (size_t)chain;
        if (sa.out_states) {
            T x[kVpl];
            load(pool(top_idx), x);
            T* dst = (T*)sa.out_states + row * d;
#pragma unroll
            for (int q = 0; q < kChunks; ++q)
#pragma unroll
                for (int e = 0; e < kW; ++e)
                    if (elem(q, e) < d) dst[elem(q, e)] = x[q * kW + e];
        }
        if (lane == 0) {
            if (sa.out_depths) sa.out_depths[row] = j;
            if (sa.out_nleap) sa.out_nleap[row] = nleap;
        }
        iter += 1;
        pc = (iter < sa.iter_end) ? kPcIterBegin : kPcFetch;
    }

    __device__ void run()
    {
        for (;;) {
            switch (uni(pc)) {
            case kPcFetch: block_fetch(); break;
            case kPcIterBegin: block_iter_begin(); break;
            case kPcDoubleBegin: block_double_begin(); break;
            case kPcLeaf: block_leaf(); break;
            case kPcAfterLeft: block_after_left(); break;
            case kPcAfterRight: block_after_right(); break;
            case kPcDoubleEnd: block_double_end(); break;
            case kPcIterEnd: block_iter_end(); break;
            default: return;  // HALT
            }
        }
    }
};

template <typename T, int kVpl>
__global__ __launch_bounds__(256, 2) void nuts_elem_kernel(DevTarget<T> tg, DevSample sa, const double* ftab_global)
{
    __shared__ __align__(16) double s_ftab[kFtabDoubles];
    __shared__ __align__(16) T s_w[kElemMaxBytes / sizeof(T)];  // every leaf reads it: LDS, not a trip to L2
    __shared__ double s_usub[4][kWave];                         // per wave: the SUBTREE uniforms of the current leaf
    for (int i = threadIdx.x; i < kFtabDoubles; i += blockDim.x) s_ftab[i] = ftab_global[i];
    for (int i = threadIdx.x; i < tg.dstride; i += blockDim.x)
        s_w[i] = i < tg.d ? (tg.kind == kGaussDiag ? tg.inv_var[i] : T(1)) : T(0);
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    const size_t slot = (size_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    T* ws = reinterpret_cast<T*>(sa.workspace + slot * sa.slot_bytes);
    ElemChain<T, kVpl> ch(tg, sa, lane, ws, s_ftab, s_w, s_usub[(threadIdx.x / kWave) & 3]);
    ch.run();
    if (lane == 0) {
        // issued slots are charged by the host as slots x (largest count of one slot): see the wave kernel
        atomicMax(&sa.counters[kCtrSlotMax], ch.n_leaf + ch.n_extra);
        atomicAdd(&sa.counters[kCtrUseful], ch.n_leaf);
        atomicAdd(&sa.counters[kCtrExtra], ch.n_extra);
        atomicAdd(&sa.counters[kCtrRounds], ch.n_leaf + ch.n_extra);
    }
}

}  // namespace nuts
