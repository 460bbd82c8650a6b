// Wave-per-chain sampler kernel: the general path.
//
// One 64-lane wavefront owns one chain slot.  State vectors live in the
// workspace in HBM/L2 and are striped over the lanes (lane l owns components
// l, l+64, ...), so every vector operation is a coalesced stream and every
// reduction is a wavefront butterfly.  The chain's control state - program
// counter, return-address stack, tree scalars - is wave-uniform and sits in
// registers; the per-level frame scalars sit one level per lane.  Chains that
// finish hand their slot to the next chain of the queue, which keeps the slots
// full until the very end of the run (Section 4.2 of the paper: synchronise on
// gradients, not on trajectory boundaries).
//
// Handles every target kind, dtype, dimension and data size.  Dense
// contractions are done by the lanes of the wave itself here; the tile kernel
// batches them across chains on the matrix cores instead.
#pragma once
#include "nuts_dev.h"
#include "nuts_fastmath.h"
#include "nuts_rng.h"

namespace nuts {

// Workspace vectors of one slot (index -> vector number), D = max_tree_depth:
//   edges:        e*3 + c            e in {minus, plus}, c in {theta, r, grad}
//   proposal pool 6 + 2*b + c        b < D + 2, c in {theta, grad}
//   first-leaf    6 + 2*(D+2) + 2*s + c   s <= D, c in {theta, r}
__host__ __device__ inline int wave_num_vectors(int max_depth) { return 6 + 2 * (max_depth + 2) + 2 * (max_depth + 1); }

template <typename T>
struct WaveChain {
    const DevTarget<T>& tg;
    const DevSample& sa;
    const int lane;
    T* const ws;          // this slot's vectors
    T* const lds;         // d elements, this wave's broadcast buffer
    double* const resid;  // logistic regression: n residuals of this slot
    const int d, D;

    // control state (wave-uniform)
    int pc = kPcFetch;
    uint64_t ret = 0;
    int level = 0, j = 0, v = 1, m = 0, nleap = 0, iter = 0;
    int sub = 0;          // leapfrog steps already taken inside the current leaf
    long chain = 0;       // local index
    uint32_t gchain = 0;  // global id, enters the draw keys
    double H0 = 0, lw_tree = 0, cur_lw = 0, edge_logp = 0;
    double log_slice = 0;  // slice sampler: log(slice height / exp(-H0)) = log of a uniform
    int cur_s = 0, cur_idx = -1, top_idx = 0;
    uint32_t free_mask = 0;
    // lane-resident stacks: lane k holds the entry of level k / pool buffer k
    double frame_lw = 0, pool_logp = 0;
    int frame_idx = 0;
    // lane k: SUBTREE uniform of level k for the merges that leaf number `u_sub_leaf` of this iteration completes
    double u_sub = 0;
    int u_sub_leaf = -1;
    // table of the logistic function for the weight merges (global memory or LDS), or NULL: log and exp instead
    const double* ftab = nullptr;
    // statistics
    unsigned long long n_leaf = 0, n_extra = 0;

    __device__ WaveChain(const DevTarget<T>& tg_, const DevSample& sa_, int lane_, T* ws_, T* lds_, double* resid_)
        : tg(tg_), sa(sa_), lane(lane_), ws(ws_), lds(lds_), resid(resid_), d(tg_.d), D(sa_.max_depth) {}

    __device__ T* edge(int e, int c) const { return ws + (size_t)(e * 3 + c) * tg.dstride; }
    __device__ T* pool(int b, int c) const { return ws + (size_t)(6 + 2 * b + c) * tg.dstride; }
    __device__ T* first(int s, int c) const { return ws + (size_t)(6 + 2 * (D + 2) + 2 * s + c) * tg.dstride; }
    __device__ DrawKey key() const { return DrawKey{sa.key0, sa.key1}; }

    __device__ void push_ret(unsigned code) { ret = (ret << 2) | code; }
    __device__ void do_return()
    {
        pc = ret_to_pc((unsigned)(ret & 3u));
        ret >>= 2;
        level += 1;
    }
    __device__ int alloc_buf()
    {
        const int b = __ffs(free_mask) - 1;
        free_mask &= ~(1u << b);
        return b;
    }
    __device__ void free_buf(int b) { free_mask |= (1u << b); }
    __device__ void copy_vec(T* dst, const T* src) const
    {
        for (int i = lane; i < d; i += kWave) dst[i] = src[i];
    }

    // ---------------------------------------------------------------- target
    // (logp, grad) at th; every lane returns the same logp.
    __device__ double eval_target(const T* th, T* g)
    {
        double part = 0.0;
        switch (tg.kind) {
        case kStdNormal:
            for (int i = lane; i < d; i += kWave) {
                const T t = th[i], gi = -t;
                g[i] = gi;
                part = fma((double)t, (double)gi, part);
            }
            return 0.5 * wave_sum(part);
        case kGaussDiag:
            for (int i = lane; i < d; i += kWave) {
                const T t = th[i], gi = -(t * tg.inv_var[i]);
                g[i] = gi;
                part = fma((double)t, (double)gi, part);
            }
            return 0.5 * wave_sum(part);
        case kGaussDense: {
            for (int i = lane; i < d; i += kWave) lds[i] = th[i];
            __builtin_amdgcn_wave_barrier();
            for (int i = lane; i < d; i += kWave) {
                double acc = 0.0;
                for (int k = 0; k < d; ++k) acc = fma((double)tg.PT[(size_t)k * d + i], (double)lds[k], acc);
                g[i] = (T)(-acc);
                part = fma((double)lds[i], -acc, part);
            }
            __builtin_amdgcn_wave_barrier();
            return 0.5 * wave_sum(part);
        }
        case kLogReg: {
            const long n_rows = tg.n;
            for (int i = lane; i < d; i += kWave) lds[i] = th[i];
            __builtin_amdgcn_wave_barrier();
            // pass 1: lanes over data rows; z = X theta, log-likelihood terms, residuals
            for (long n = lane; n < n_rows; n += kWave) {
                double z = 0.0;
                for (int k = 0; k < d; ++k) z = fma((double)tg.XT[(size_t)k * n_rows + n], (double)lds[k], z);
                const double yn = (double)tg.y[n];
                const double e = exp(-fabs(z));
                part += yn * z - (fmax(z, 0.0) + log1p(e));
                const double sig = (z >= 0.0 ? 1.0 : e) / (1.0 + e);
                resid[n] = yn - sig;
            }
            __threadfence_block();
            __builtin_amdgcn_wave_barrier();
            // pass 2: grad = X' resid - theta / s^2; lanes = (feature, row-subgroup)
            const int KL = tg.kl, NS = kWave / KL;
            const int ks = lane & (KL - 1), ns = lane / KL;
            double sq = 0.0;
            for (int k0 = 0; k0 < d; k0 += KL) {
                const int k = k0 + ks;
                double acc = 0.0;
                if (k < d)
                    for (long n = ns; n < n_rows; n += NS) acc = fma((double)tg.X[(size_t)n * d + k], resid[n], acc);
                for (int o = KL; o < kWave; o <<= 1) acc += __shfl_xor(acc, o, kWave);
                if (k < d && ns == 0) {
                    const double t = (double)lds[k];
                    g[k] = (T)(acc - t * tg.prior_prec);
                    sq = fma(t, t, sq);
                }
            }
            __builtin_amdgcn_wave_barrier();
            wave_sum2(part, sq);
            return part - 0.5 * tg.prior_prec * sq;
        }
        default:
            return NAN;
        }
    }

    // True while the span from (tm, rm) to (tp, rp) has not turned back.
    __device__ bool uturn_ok(const T* tm, const T* rm, const T* tp, const T* rp) const
    {
        double dm = 0.0, dp = 0.0;
        for (int i = lane; i < d; i += kWave) {
            const T delta = tp[i] - tm[i];
            dm = fma((double)delta, (double)rm[i], dm);
            dp = fma((double)delta, (double)rp[i], dp);
        }
        wave_sum2(dm, dp);
        return (dm >= 0.0) && (dp >= 0.0);
    }

    // ---------------------------------------------------------------- blocks
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
        free_mask = ((D + 2) >= 32 ? 0xffffffffu : ((1u << (D + 2)) - 1u)) & ~1u;
        T* x0 = pool(0, 0);
        if (sa.init_states) {
            const T* src = (const T*)sa.init_states + (size_t)chain * d;
            for (int i = lane; i < d; i += kWave) x0[i] = src[i];
        } else {
            for (int i = lane; i < d; i += kWave) {
                const Words4 w = draw(key(), (uint32_t)(i >> 1), kDrawInit, 0, 0, gchain);
                x0[i] = (T)normal_of(w, i & 1);
            }
        }
        pc = kPcInitEval;
    }

    __device__ void block_iter_begin()
    {
        const T* th = pool(top_idx, 0);
        const T* g = pool(top_idx, 1);
        double kin = 0.0;
        // one draw gives two components: lane p makes components 2p and 2p + 1
        for (int p = lane; 2 * p < d; p += kWave) {
            const Words4 w = draw(key(), (uint32_t)p, kDrawMomentum, 0, (uint32_t)iter, gchain);
            double z[2];
            normal_pair(w, z[0], z[1]);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int i = 2 * p + q;
                if (i < d) {
                    const T r = (T)z[q];
                    const T t = th[i], gi = g[i];
                    edge(0, 0)[i] = t; edge(0, 1)[i] = r; edge(0, 2)[i] = gi;
                    edge(1, 0)[i] = t; edge(1, 1)[i] = r; edge(1, 2)[i] = gi;
                    kin = fma((double)r, (double)r, kin);
                }
            }
        }
        u_sub_leaf = -1;  // leaf counts restart: cached SUBTREE uniforms belong to the old iteration
        const double logp_top = read_lane(pool_logp, uni(top_idx));
        H0 = -logp_top + 0.5 * wave_sum(kin);
        lw_tree = 0.0;  // log of the starting point's weight
        if (sa.sampler == kSamplerSlice) {
            const Words4 w = draw(key(), 0, kDrawSlice, 0, (uint32_t)iter, gchain);
            log_slice = log(uniform52(w.w0, w.w1));
            lw_tree = 1.0;  // the starting point is the first candidate
        }
        j = 0;
        nleap = 0;
        pc = kPcDoubleBegin;
    }

    __device__ void block_double_begin()
    {
        const Words4 w = draw(key(), (uint32_t)j, kDrawDirection, 0, (uint32_t)iter, gchain);
        v = (w.w0 >> 31) ? 1 : -1;
        m = 0;
        level = j;
        push_ret(kRetDoubleEnd);
        pc = kPcBuild;
    }

    __device__ void block_build()
    {
        if (level == 0) {
            pc = kPcLeaf;
        } else {
            level -= 1;
            push_ret(kRetAfterLeft);
        }
    }

    // The gradient step of a chain standing at LEAF: kick, drift, gradient, kick; after the
    // last of the leaf's leaf_steps such steps, the leaf's weight and validity.  It is split at the gradient so that the
    // gradient can also come from outside (the grid kernels evaluate it for all chains
    // at once between two launches of the control kernel).
    __device__ T* leaf_position() const { return edge(v > 0 ? 1 : 0, 0); }
    __device__ T* leaf_gradient() const { return edge(v > 0 ? 1 : 0, 2); }
    __device__ void leaf_pre()
    {
        const int e = v > 0 ? 1 : 0;
        T *th = edge(e, 0), *r = edge(e, 1), *g = edge(e, 2);
        const T half = (T)(0.5 * (v * sa.eps)), full = (T)(v * sa.eps);
        for (int i = lane; i < d; i += kWave) {
            const T rh = r[i] + half * g[i];
            r[i] = rh;
            th[i] = th[i] + full * rh;
        }
    }
    __device__ void leaf_post(double logp)
    {
        const int e = v > 0 ? 1 : 0;
        T *r = edge(e, 1), *g = edge(e, 2);
        const T half = (T)(0.5 * (v * sa.eps));
        double kin = 0.0;
        for (int i = lane; i < d; i += kWave) {
            const T rn = r[i] + half * g[i];
            r[i] = rn;
            kin = fma((double)rn, (double)rn, kin);
        }
        leaf_finish(logp, wave_sum(kin));
    }
    // The rest of a leapfrog step once the second kick is done: kin = |r|^2 of the new momentum.
    __device__ void leaf_finish(double logp, double kin)
    {
        const int e = v > 0 ? 1 : 0;
        T *th = edge(e, 0), *r = edge(e, 1);
        edge_logp = logp;
        nleap += 1;
        n_leaf += 1;
        sub += 1;
        if (sub < sa.leaf_steps) return;  // the leaf is not finished: the chain stays at LEAF
        sub = 0;
        m += 1;
        double delta = (-edge_logp + 0.5 * kin) - H0;
        if (!(fabs(delta) < INFINITY)) delta = INFINITY;  // NaN or +-inf
        if (sa.sampler == kSamplerSlice) {
            cur_lw = (log_slice <= -delta) ? 1.0 : 0.0;
            cur_s = (log_slice < kDeltaMax - delta);
        } else {
            cur_lw = -delta;
            cur_s = (delta <= kDeltaMax);
        }
        cur_idx = -1;  // the proposal of a one-leaf subtree is the edge itself
        if ((m & 1) && j >= 1) {
            // first leaf of every open subtree it starts; one copy serves them all
            const int s = (m == 1) ? j : min(__ffs(m - 1) - 1, j);
            T *ft = first(s, 0), *fr = first(s, 1);
            for (int i = lane; i < d; i += kWave) {
                ft[i] = th[i];
                fr[i] = r[i];
            }
        }
        do_return();
    }
    __device__ void block_leaf()
    {
        leaf_pre();
        leaf_post(eval_target(leaf_position(), leaf_gradient()));
    }

    __device__ void init_post(double lp)
    {
        if (lane == top_idx) pool_logp = lp;
        n_extra += 1;
        pc = kPcIterBegin;
    }
    __device__ void block_init_eval() { init_post(eval_target(pool(top_idx, 0), pool(top_idx, 1))); }

    // Make sure the current proposal owns a pool buffer (a fresh leaf lives in the edge).
    __device__ void materialise_cur()
    {
        if (cur_idx >= 0) return;
        const int e = v > 0 ? 1 : 0;
        const int b = alloc_buf();
        copy_vec(pool(b, 0), edge(e, 0));
        copy_vec(pool(b, 1), edge(e, 2));
        if (lane == b) pool_logp = edge_logp;
        cur_idx = b;
    }

    __device__ void block_after_left()
    {
        if (!cur_s) {  // the right half is never built
            do_return();
            return;
        }
        materialise_cur();
        if (lane == level) {
            frame_lw = cur_lw;
            frame_idx = cur_idx;
        }
        level -= 1;
        push_ret(kRetAfterRight);
        pc = kPcBuild;
    }

    __device__ void block_after_right()
    {
        if (cur_s) {
            const double l_lw = read_lane(frame_lw, uni(level));  // the level is the same for the whole wave
            const int l_idx = __builtin_amdgcn_readlane(frame_idx, uni(level));
            const bool slice = sa.sampler == kSamplerSlice;
            if (u_sub_leaf != nleap) {
                // every merge this leaf can complete draws at the same position: lane l draws for level l
                const Words4 w = draw(key(), (uint32_t)nleap, kDrawSubtree, (uint32_t)lane, (uint32_t)iter, gchain);
                u_sub = uniform52(w.w0, w.w1);
                u_sub_leaf = nleap;
            }
            const double u = read_lane(u_sub, uni(level));
            double lw_new;
            bool take_right;
            if (slice) {
                lw_new = l_lw + cur_lw;
                take_right = u * lw_new < cur_lw;
            } else if (ftab) {  // both log-weights are finite here; u < w_R / (w_L + w_R) through the table
                double p_right;
                merge_logweights(l_lw, cur_lw, ftab, lw_new, p_right);
                take_right = u < p_right;
            } else {
                lw_new = logaddexp(l_lw, cur_lw);
                take_right = log(u) < cur_lw - lw_new;
            }
            if (take_right) {
                free_buf(l_idx);
            } else {
                if (cur_idx >= 0) free_buf(cur_idx);
                cur_idx = l_idx;
            }
            cur_lw = lw_new;
            const int f = m - (1 << level) + 1;  // first leaf of this subtree (1-based)
            const int s = (f == 1) ? j : min(__ffs(f - 1) - 1, j);
            const int e = v > 0 ? 1 : 0;
            const bool ok = v > 0 ? uturn_ok(first(s, 0), first(s, 1), edge(e, 0), edge(e, 1))
                                  : uturn_ok(edge(e, 0), edge(e, 1), first(s, 0), first(s, 1));
            cur_s = ok;
        }
        do_return();
    }

    __device__ void block_double_end()
    {
        bool go_on = false;
        if (cur_s) {
            const Words4 w = draw(key(), (uint32_t)j, kDrawTop, 0, (uint32_t)iter, gchain);
            const double u = uniform52(w.w0, w.w1);
            bool accept;
            if (sa.sampler == kSamplerSlice) {
                accept = u * lw_tree < cur_lw;
                lw_tree += cur_lw;
            } else if (ftab) {  // u < w_new / w_tree, with p = w_new / (w_tree + w_new) from the table
                double lw_new, p;
                merge_logweights(lw_tree, cur_lw, ftab, lw_new, p);
                accept = u * (1.0 - p) < p;
                lw_tree = lw_new;
            } else {
                accept = log(u) < cur_lw - lw_tree;
                lw_tree = logaddexp(lw_tree, cur_lw);
            }
            if (accept) {
                materialise_cur();
                top_idx = cur_idx;
            }
            go_on = uturn_ok(edge(0, 0), edge(0, 1), edge(1, 0), edge(1, 1));
        } else {
            // the trajectory ends here; keep the total for completeness (an invalid half may weigh -infinity or 0)
            lw_tree = sa.sampler == kSamplerSlice ? lw_tree + cur_lw : logaddexp(lw_tree, cur_lw);
        }
        j += 1;
        // after a doubling only the trajectory's proposal is live
        free_mask = ((D + 2) >= 32 ? 0xffffffffu : ((1u << (D + 2)) - 1u)) & ~(1u << top_idx);
        pc = (go_on && j < D) ? kPcDoubleBegin : kPcIterEnd;
    }

    __device__ void block_iter_end()
    {
        const size_t row = (size_t)iter * (size_t)sa.n_chains + (size_t)chain;
        if (sa.out_states) {
            T* dst = (T*)sa.out_states + row * d;
            const T* src = pool(top_idx, 0);
            for (int i = lane; i < d; i += kWave) dst[i] = src[i];
        }
        if (lane == 0) {
            if (sa.out_depths) sa.out_depths[row] = j;
            if (sa.out_nleap) sa.out_nleap[row] = nleap;
        }
        iter += 1;
        pc = (iter < sa.iter_end) ? kPcIterBegin : kPcFetch;
    }

    // Uniform control state <-> memory, for kernels that run the chain program in several launches.
    struct Saved {
        int pc, level, j, v, m, nleap, iter, sub, cur_s, cur_idx, top_idx;
        uint32_t gchain, free_mask;
        uint64_t ret;
        long chain;
        double H0, lw_tree, cur_lw, edge_logp, log_slice;
        unsigned long long n_leaf, n_extra;
        double frame_lw[kWave], pool_logp[kWave];
        int frame_idx[kWave];
    };
    __device__ void save(Saved* st) const
    {
        if (lane == 0) {
            st->pc = pc; st->level = level; st->j = j; st->v = v; st->m = m; st->nleap = nleap; st->iter = iter;
            st->sub = sub;
            st->cur_s = cur_s; st->cur_idx = cur_idx; st->top_idx = top_idx; st->gchain = gchain;
            st->free_mask = free_mask; st->ret = ret; st->chain = chain; st->H0 = H0; st->lw_tree = lw_tree;
            st->cur_lw = cur_lw; st->edge_logp = edge_logp; st->log_slice = log_slice; st->n_leaf = n_leaf; st->n_extra = n_extra;
        }
        st->frame_lw[lane] = frame_lw;
        st->pool_logp[lane] = pool_logp;
        st->frame_idx[lane] = frame_idx;
    }
    __device__ void restore(const Saved* st)
    {
        pc = st->pc; level = st->level; j = st->j; v = st->v; m = st->m; nleap = st->nleap; iter = st->iter;
        sub = st->sub;
        cur_s = st->cur_s; cur_idx = st->cur_idx; top_idx = st->top_idx; gchain = st->gchain;
        free_mask = st->free_mask; ret = st->ret; chain = st->chain; H0 = st->H0; lw_tree = st->lw_tree;
        cur_lw = st->cur_lw; edge_logp = st->edge_logp; log_slice = st->log_slice; n_leaf = st->n_leaf; n_extra = st->n_extra;
        frame_lw = st->frame_lw[lane];
        pool_logp = st->pool_logp[lane];
        frame_idx = st->frame_idx[lane];
        u_sub_leaf = -1;
    }

    // Run blocks until the chain needs a gradient (LEAF, INIT_EVAL) or has halted.
    __device__ void run_to_gradient_request()
    {
        for (;;) {
            const int p = uni(pc);
            switch (p) {
            case kPcFetch: block_fetch(); break;
            case kPcIterBegin: block_iter_begin(); break;
            case kPcDoubleBegin: block_double_begin(); break;
            case kPcBuild: block_build(); break;
            case kPcAfterLeft: block_after_left(); break;
            case kPcAfterRight: block_after_right(); break;
            case kPcDoubleEnd: block_double_end(); break;
            case kPcIterEnd: block_iter_end(); break;
            default: return;  // INIT_EVAL, LEAF, HALT
            }
        }
    }

    __device__ void run()
    {
        for (;;) {
            const int p = uni(pc);
            switch (p) {
            case kPcFetch: block_fetch(); break;
            case kPcIterBegin: block_iter_begin(); break;
            case kPcDoubleBegin: block_double_begin(); break;
            case kPcBuild: block_build(); break;
            case kPcAfterLeft: block_after_left(); break;
            case kPcAfterRight: block_after_right(); break;
            case kPcDoubleEnd: block_double_end(); break;
            case kPcIterEnd: block_iter_end(); break;
            case kPcInitEval: block_init_eval(); break;
            case kPcLeaf: block_leaf(); break;
            default: return;  // HALT
            }
        }
    }
};

template <typename T>
__global__ __launch_bounds__(256) void nuts_wave_kernel(DevTarget<T> tg, DevSample sa)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wib = threadIdx.x / kWave;
    const size_t slot = (size_t)blockIdx.x * (blockDim.x / kWave) + wib;
    T* lds = reinterpret_cast<T*>(smem) + (size_t)wib * tg.dstride;
    if (tg.lds_matrix) {
        // a dense precision matrix that fits is staged in LDS once and shared by the block's waves
        T* mat = reinterpret_cast<T*>(smem) + (size_t)(blockDim.x / kWave) * tg.dstride;
        for (size_t i = threadIdx.x; i < (size_t)tg.d * tg.d; i += blockDim.x) mat[i] = tg.PT[i];
        __syncthreads();
        tg.PT = mat;
    }
    char* base = sa.workspace + slot * sa.slot_bytes;
    T* ws = reinterpret_cast<T*>(base);
    const size_t vec_bytes = ((size_t)wave_num_vectors(sa.max_depth) * tg.dstride * sizeof(T) + 15) & ~(size_t)15;
    double* resid = reinterpret_cast<double*>(base + vec_bytes);
    WaveChain<T> ch(tg, sa, lane, ws, lds, resid);
    ch.run();
    if (lane == 0) {
        // a slot is held for the whole launch, which lasts as long as its busiest slot: the host
        // charges slots x (largest count) as issued once the launch is over
        atomicMax(&sa.counters[kCtrSlotMax], ch.n_leaf + ch.n_extra);
        atomicAdd(&sa.counters[kCtrUseful], ch.n_leaf);
        atomicAdd(&sa.counters[kCtrExtra], ch.n_extra);
        atomicAdd(&sa.counters[kCtrRounds], ch.n_leaf + ch.n_extra);
    }
}

}  // namespace nuts
