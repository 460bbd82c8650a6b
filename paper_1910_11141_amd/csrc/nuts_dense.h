// Register-resident kernel for a dense Gaussian of moderate dimension (d <= 128):
// configuration 2 of the benchmark, which is chain-poor (1024 chains) and so bound by
// the latency of one chain's step, not by throughput.
//
// One wavefront per chain slot.  The end of the trajectory that is being extended -
// position, momentum and gradient, two components per lane - stays in registers; the
// precision matrix is staged once per workgroup in LDS (row pitch 128, zero padded)
// and a gradient is one pass over it: the wave publishes its position in LDS, then
// every lane accumulates its two rows of P theta in ascending column order with one
// 16-byte matrix read and one broadcast read per column.  The tree's own storage
// (other end, proposal pool with gradients, first leaves) is in global memory as in
// the element-wise kernel.
#pragma once
#include "nuts_dev.h"
#include "nuts_fastmath.h"
#include "nuts_rng.h"

namespace nuts {

constexpr int kDenseMaxDim = 128;
constexpr int kDensePitch = 128;  // elements per workspace vector and per matrix row in LDS
constexpr int kDenseWaves = 4;    // waves (chain slots) per workgroup

// Workspace vectors of one slot (kDensePitch elements each), D = max_tree_depth:
//   0, 1, 2                   the trajectory end that is not in registers (theta, r, grad)
//   3 + 2*b + c               proposal pool, b < D + 2, c in {theta, grad}
//   3 + 2*(D+2) + 2*s + c     first-leaf slots, s <= D, c in {theta, r}
__host__ __device__ inline int dense_num_vectors(int max_depth) { return 3 + 2 * (max_depth + 2) + 2 * (max_depth + 1); }

template <typename T>
struct DenseVec;
template <>
struct DenseVec<float> {
    typedef float2 type;
};
template <>
struct DenseVec<double> {
    typedef double2 type;
};

// kBanded: the precision matrix has at most kBandHalf off-diagonals on each side (detected when the target is
// created); a lane then keeps the 2 x 9 coefficients of its two rows in registers and a gradient reads ten
// neighbouring components of the published position instead of a pass over the matrix.  Zero entries of a
// dense row add exact zeros, so the banded sum in ascending column order has the same value.
template <typename T, bool kBanded>
struct DenseChain {
    static constexpr int kVpl = 2, kW = 2, kChunks = 1;
    typedef typename DenseVec<T>::type Vec;

    const DevTarget<T>& tg;
    const DevSample& sa;
    const int lane, d, D;
    static constexpr int dstride = kDensePitch;
    T* const ws;
    const T* const mat;  // LDS: mat[k * kDensePitch + i] = P[i][k]
    T* const bcast;      // LDS: this wave's position, for the other lanes

    T th[kVpl], r[kVpl], g[kVpl];  // the register end of the trajectory
    T band0[2 * kBandHalf + 1], band1[2 * kBandHalf + 1];  // banded: coefficients of rows 2*lane and 2*lane+1

    int pc = kPcFetch, level = 0, j = 0, v = 1, m = 0, nleap = 0, iter = 0, act = 1;
    uint64_t ret = 0;
    long chain = 0;
    uint32_t gchain = 0, free_mask = 0;
    // Weights of trajectory points are numbers, not logarithms: a leaf weighs exp(H0 - H) / unit (slice sampler: 1 or 0),
    // a subtree the sum of its leaves, so a merge is an add and a selection one product and a comparison.  log_unit_w is
    // the logarithm of the unit: 0 until a leaf's energy falls more than 600 below what the unit can represent; then
    // that leaf becomes the unit and what the iteration holds is rescaled.
    double H0 = 0, w_tree = 0, cur_w = 0, log_unit_w = 0, edge_logp = 0, log_slice = 0;
    // Random numbers that do not depend on where the trajectory goes, one generator pass for many: lane j < 16 votes the
    // direction of doubling j into dirbits and lane 16 + j holds the TOP uniform of doubling j (once per iteration);
    // lane l < 16 holds the SUBTREE uniform of level l for the leaf that ends with leapfrog count u_sub_leaf and lane
    // 16 + l that of the next leaf that can complete a merge, two leaves on.
    double u_top = 0, u_sub = 0;
    uint32_t dirbits = 0;
    int u_sub_leaf = 0;
    int cur_s = 0, cur_idx = -1, top_idx = 0;
    double frame_w = 0, pool_logp = 0;  // lane k: level k / pool buffer k
    int frame_idx = 0;
    unsigned long long n_leaf = 0, n_extra = 0;

    __device__ DenseChain(const DevTarget<T>& tg_, const DevSample& sa_, int lane_, T* ws_, const T* mat_, T* bcast_)
        : tg(tg_), sa(sa_), lane(lane_), d(tg_.d), D(sa_.max_depth), ws(ws_), mat(mat_), bcast(bcast_) {}

    __device__ int elem(int q, int e) const { return (q * kWave + lane) * kW + e; }  // component of register q*kW+e
    __device__ T* other(int c) const { return ws + (size_t)c * dstride; }
    __device__ T* pool(int b, int c) const { return ws + (size_t)(3 + 2 * b + c) * dstride; }
    __device__ T* first(int s, int c) const { return ws + (size_t)(3 + 2 * (D + 2) + 2 * s + c) * dstride; }
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
        store(pool(b, 0), th);
        store(pool(b, 1), g);
        if (lane == b) pool_logp = edge_logp;
        cur_idx = b;
    }
    __device__ uint32_t all_bufs() const { return (1u << (D + 2)) - 1u; }

    // g = -P theta for the position in registers; returns the partial sum of theta_i g_i of this lane
    // (logp is half the wave's total).  Columns are taken in ascending order with a binary64 accumulator.
    __device__ double gradient()
    {
        *reinterpret_cast<Vec*>(bcast + 2 * lane) = Vec{th[0], th[1]};
        __builtin_amdgcn_wave_barrier();
        double acc0 = 0.0, acc1 = 0.0;
        if (kBanded) {
            // components 2*lane - 4 .. 2*lane + 5 (the buffer has kBandHalf zeros on either side)
            T x[2 * kBandHalf + 2];
#pragma unroll
            for (int u = 0; u < kBandHalf + 1; ++u) {
                const Vec p = *reinterpret_cast<const Vec*>(bcast + 2 * lane - kBandHalf + 2 * u);
                x[2 * u] = p.x;
                x[2 * u + 1] = p.y;
            }
#pragma unroll
            for (int k = 0; k < 2 * kBandHalf + 1; ++k) {
                acc0 = fma((double)band0[k], (double)x[k], acc0);
                acc1 = fma((double)band1[k], (double)x[k + 1], acc1);
            }
            __builtin_amdgcn_wave_barrier();
            g[0] = (T)(-acc0);
            g[1] = (T)(-acc1);
            return fma((double)th[0], -acc0, (double)th[1] * -acc1);
        }
        const T* row = mat + 2 * lane;
        // columns in batches of 20 so that the LDS reads of a batch are all in flight together
        constexpr int kBatch = 20;
        int k = 0;
        for (; k + kBatch <= d; k += kBatch) {
            Vec p[kBatch];
            T t[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                p[u] = *reinterpret_cast<const Vec*>(row + (size_t)(k + u) * kDensePitch);
                t[u] = bcast[k + u];
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                acc0 = fma((double)p[u].x, (double)t[u], acc0);
                acc1 = fma((double)p[u].y, (double)t[u], acc1);
            }
        }
        for (; k < d; ++k) {
            const Vec p = *reinterpret_cast<const Vec*>(row + (size_t)k * kDensePitch);
            const double t = (double)bcast[k];
            acc0 = fma((double)p.x, t, acc0);
            acc1 = fma((double)p.y, t, acc1);
        }
        __builtin_amdgcn_wave_barrier();
        g[0] = (T)(-acc0);
        g[1] = (T)(-acc1);
        return fma((double)th[0], -acc0, (double)th[1] * -acc1);
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
            store(pool(0, 0), th);
        } else {
            draw_normals_to(kDrawInit, 0, pool(0, 0));
            load(pool(0, 0), th);
        }
        const double lp = 0.5 * wave_sum(gradient());
        store(pool(0, 1), g);
        if (lane == 0) pool_logp = lp;
        n_extra += 1;
        pc = kPcIterBegin;
    }

    __device__ void block_iter_begin()
    {
        load(pool(top_idx, 0), th);
        load(pool(top_idx, 1), g);
        draw_normals_to(kDrawMomentum, (uint32_t)iter, other(1));
        load(other(1), r);
        double kin = 0.0;
#pragma unroll
        for (int i = 0; i < kVpl; ++i) kin = fma((double)r[i], (double)r[i], kin);
        store(other(0), th);  // both ends of the trajectory start at the current point
        store(other(2), g);
        act = 1;
        H0 = -read_lane(pool_logp, uni(top_idx)) + 0.5 * wave_sum(kin);
        w_tree = 1.0;  // the starting point: weight exp(0), or the first candidate
        log_unit_w = 0.0;
        if (sa.sampler == kSamplerSlice) {
            const Words4 ws = draw(key(), 0, kDrawSlice, 0, (uint32_t)iter, gchain);
            log_slice = log(uniform52(ws.w0, ws.w1));
        }
        {
            const Words4 wj = draw(key(), (uint32_t)(lane & 15), (lane & 16) ? kDrawTop : kDrawDirection, 0, (uint32_t)iter, gchain);
            dirbits = (uint32_t)__ballot(lane < 16 && (wj.w0 >> 31)) & 0xffffu;
            u_top = uniform52(wj.w0, wj.w1);
        }
        u_sub_leaf = kNoLeaf;
        j = 0;
        nleap = 0;
        pc = kPcDoubleBegin;
    }

    __device__ void block_double_begin()
    {
        v = ((dirbits >> j) & 1u) ? 1 : -1;
        const int e = v > 0 ? 1 : 0;
        if (e != act) {  // bring the end that is to be extended into registers
            T xt[kVpl], xr[kVpl], xg[kVpl];
            load(other(0), xt);
            load(other(1), xr);
            load(other(2), xg);
            store(other(0), th);
            store(other(1), r);
            store(other(2), g);
#pragma unroll
            for (int i = 0; i < kVpl; ++i) {
                th[i] = xt[i];
                r[i] = xr[i];
                g[i] = xg[i];
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
        double lp = 0.0, kin = 0.0;
        for (int step = 0; step < sa.leaf_steps; ++step) {
#pragma unroll
            for (int i = 0; i < kVpl; ++i) {
                r[i] = r[i] + half * g[i];
                th[i] = th[i] + full * r[i];
            }
            lp = gradient();
#pragma unroll
            for (int i = 0; i < kVpl; ++i) r[i] = r[i] + half * g[i];
        }
#pragma unroll
        for (int i = 0; i < kVpl; ++i) kin = fma((double)r[i], (double)r[i], kin);
        wave_sum2(lp, kin);
        edge_logp = 0.5 * lp;
        m += 1;
        nleap += sa.leaf_steps;
        n_leaf += sa.leaf_steps;
        double delta = (-edge_logp + 0.5 * kin) - H0;
        if (!(fabs(delta) < INFINITY)) delta = INFINITY;
        if (sa.sampler == kSamplerSlice) {
            cur_w = (log_slice <= -delta) ? 1.0 : 0.0;
            cur_s = (log_slice < kDeltaMax - delta);
        } else {
            double e = log_unit_w - delta;  // logarithm of the leaf's weight in the current unit
            if (e > 600.0) {  // the energy has fallen far: this leaf becomes the unit
                const double shrink = exp_bounded(-e);
                w_tree *= shrink;
                frame_w *= shrink;
                log_unit_w = delta;
                e = 0.0;
            }
            cur_w = exp_bounded(e);
            cur_s = (delta <= kDeltaMax);
        }
        cur_idx = -1;
        if ((m & 1) && j >= 1) {
            const int s = (m == 1) ? j : min(__ffs(m - 1) - 1, j);
            store(first(s, 0), th);
            store(first(s, 1), r);
        }
        do_return();
    }

    __device__ void block_after_left()
    {
        if (!cur_s) {
            do_return();
            return;
        }
        materialise_cur();
        if (lane == level) {
            frame_w = cur_w;
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
            T xt[kVpl], xr[kVpl];
            load(first(s, 0), xt);
            load(first(s, 1), xr);
            const double l_w = read_lane(frame_w, uni(level));  // the level is the same for the whole wave
            const int l_idx = __builtin_amdgcn_readlane(frame_idx, uni(level));
            // every merge that a leaf can complete draws at the same position (the leapfrog count), and only leaves
            // that close a right half complete merges, two leaves apart: one pass serves two of them
            const int leaf_gap = 2 * sa.leaf_steps;
            if (u_sub_leaf != nleap && u_sub_leaf + leaf_gap != nleap) {
                const Words4 wd = draw(key(), (uint32_t)(nleap + ((lane & 16) ? leaf_gap : 0)), kDrawSubtree, (uint32_t)(lane & 15),
                                       (uint32_t)iter, gchain);
                u_sub = uniform52(wd.w0, wd.w1);
                u_sub_leaf = nleap;
            }
            const double u = read_lane(u_sub, uni(level + (u_sub_leaf != nleap ? 16 : 0)));
            // right with probability w_R / (w_L + w_R) (never when both are zero)
            const double w_new = l_w + cur_w;
            if (u * w_new < cur_w) {
                free_mask |= (1u << l_idx);
            } else {
                if (cur_idx >= 0) free_mask |= (1u << cur_idx);
                cur_idx = l_idx;
            }
            cur_w = w_new;
            cur_s = uturn_ok_regs(xt, xr, v > 0);
        }
        do_return();
    }

    __device__ void block_double_end()
    {
        bool go_on = false;
        if (cur_s) {
            const double u = read_lane(u_top, uni(16 + j));
            const bool accept = u * w_tree < cur_w;  // with probability min(1, w_new / w_tree)
            w_tree += cur_w;
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
            load(pool(top_idx, 0), x);
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
        if (kBanded) {
#pragma unroll
            for (int k = 0; k < 2 * kBandHalf + 1; ++k) {
                band0[k] = tg.band[(size_t)(2 * lane) * (2 * kBandHalf + 1) + k];
                band1[k] = tg.band[(size_t)(2 * lane + 1) * (2 * kBandHalf + 1) + k];
            }
        }
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

template <typename T, bool kBanded>
__global__ __launch_bounds__(kDenseWaves* kWave) void nuts_dense_kernel(DevTarget<T> tg, DevSample sa)
{
    extern __shared__ __align__(16) unsigned char smem[];
    T* mat = reinterpret_cast<T*>(smem);  // dense: d rows of kDensePitch; banded: nothing
    const int mat_rows = kBanded ? 0 : tg.d;
    // per wave: kBandHalf zeros, the position, kBandHalf zeros
    constexpr int kBcast = kDensePitch + 2 * kBandHalf;
    T* bcast = mat + (size_t)mat_rows * kDensePitch + (size_t)(threadIdx.x / kWave) * kBcast + kBandHalf;
    for (int i = threadIdx.x; i < mat_rows * kDensePitch; i += blockDim.x) {
        const int k = i / kDensePitch, c = i % kDensePitch;
        mat[i] = c < tg.d ? tg.PT[(size_t)k * tg.d + c] : T(0);
    }
    for (int i = threadIdx.x; i < kDenseWaves * kBcast; i += blockDim.x) mat[(size_t)mat_rows * kDensePitch + i] = T(0);
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    const size_t slot = (size_t)blockIdx.x * kDenseWaves + threadIdx.x / kWave;
    T* ws = reinterpret_cast<T*>(sa.workspace + slot * sa.slot_bytes);
    DenseChain<T, kBanded> ch(tg, sa, lane, ws, mat, bcast);
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
