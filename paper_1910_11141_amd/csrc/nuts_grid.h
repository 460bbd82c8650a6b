// Grid kernels: logistic regression with many data rows and few chains
// (binary32, dim <= 128, up to 1024 chains resident at a time).
//
// Here one gradient evaluation of all chains is a pair of GEMMs that spans the
// whole chip - Z = X~ Theta with N rows, G = X~' sigma(-Z) - so the lock-step
// round of Algorithm 2 becomes two launches:
//   control   one workgroup per chain: its four waves sum the row slices' partial
//             gradients and log-likelihoods of the chain's last gradient in
//             binary64 in a fixed order; its first wave then finishes that
//             step, runs the chain program up to the next point that needs a
//             gradient, does the first half of the leapfrog step and publishes
//             the position as one column of Theta;
//   gradient  every workgroup takes a slice of the data rows; its 4 waves hold
//             32 chains each as the B operand of 32x32x2 binary32 MFMAs, bring
//             the packed rows of X~ into LDS once per workgroup (one row tile
//             ahead of the one being computed), apply the logistic functions to
//             the accumulator registers (whose layout is exactly the B-operand
//             layout of the second GEMM) and keep their slice's partial
//             gradient in accumulators.  Features are taken 32 at a time; when
//             at most 8 are left over (d = 100: 96 + 4) those go through
//             4x4x1 MFMAs of 16 blocks, four features at a time, whose B operand
//             is again the accumulator register as it stands (block = four
//             chains of one row) and which cost an eighth of a 32-feature tile.
// Chains step together in sets of 128 (one gradient workgroup's worth).  Sets are
// independent, so their rounds are enqueued on up to four streams: while one set
// is in its control launch another set's gradient keeps the matrix units busy,
// and two gradient workgroups (of different sets) fit on a compute unit together.
// The host enqueues rounds in batches and looks at a "who has halted" array one
// batch behind; rounds enqueued after the last chain of a set halted return at
// once.
//
// As in the tile kernel, X~ = diag(2y - 1) X, so the labels never reach the GPU
// arithmetic:  y z - log(1+e^z) = -log(1+e^{-z~}),  X'(y - sigma(z)) = X~' sigma(-z~).
#pragma once
#include <hip/hip_runtime.h>

#include <vector>

#include "nuts_dev.h"
#include "nuts_wave.h"

namespace nuts {

constexpr int kGridMaxDim = 128;
constexpr int kGridMaxChains = 1024;  // chain slots resident at a time (further chains wait in the queue)
constexpr int kGridMaxSlices = 256;  // row slices = gradient workgroups per launch
constexpr int kGridRows = 32;    // data rows per MFMA tile
constexpr int kGridGroup = 32;   // chains per wave
constexpr int kGridWaves = 4;                          // waves per gradient workgroup
constexpr int kGridSetChains = kGridGroup * kGridWaves;  // chains that step together
constexpr int kGridMaxSets = kGridMaxChains / kGridSetChains;
constexpr int kGridMaxStreams = 4;                     // the sets are dealt round-robin onto this many streams
constexpr int kGridSumParts = 8;                       // a chain's slices are summed in this many interleaved parts
constexpr int kGridFeatPad = 128;
constexpr int kGridBatch = 32;   // rounds enqueued between two looks at the halted flags

constexpr int kGridMaxTail = 2;  // left-over features go through the small MFMA in up to this many groups of 4

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct GridData {
    float* ops = nullptr;  // device: packed operands, grid_groups_per_tile() groups of 64 float4 per row tile
    int d = 0, ks1 = 0, mt = 0, tail = 0, n_tiles = 0;
    long n_rows = 0;
};

// Shape of the two GEMMs for d features: ks1 k-steps (of 2 features) in the first; in the second, mt
// tiles of 32 features and `tail` groups of 4 features after them.
inline void grid_shape(int64_t d, int* ks1, int* mt, int* tail)
{
    const int full = (int)(d / 32), left = (int)(d % 32);
    if (full >= 1 && left >= 1 && left <= 4 * kGridMaxTail) {
        *mt = full;
        *tail = (left + 3) / 4;
        *ks1 = 16 * full + 2 * *tail;
    } else {
        *mt = (int)((d + 31) / 32);
        *tail = 0;
        *ks1 = 16 * *mt;
    }
}

// Operand groups (of 4 k-steps: one float4 per lane) per row tile: ceil(ks1 / 4) for the first GEMM,
// 4*mt + 4*tail for the second, padded so that every wave of a workgroup fetches the same number.
__host__ __device__ constexpr int grid_groups_per_tile(int ks1, int mt, int tail)
{
    return ((ks1 + 3) / 4 + 4 * mt + 4 * tail + kGridWaves - 1) / kGridWaves * kGridWaves;
}

inline bool grid_supports_shape(int64_t d) { return d >= 1 && d <= kGridMaxDim; }

// Row i0(v) of accumulator register v in lane-half 0; lane-half 1 holds row i0(v) + 4.
__host__ __device__ inline int grid_acc_row(int v) { return 8 * (v / 4) + (v % 4); }

// Operand stream per 32-row tile t:
//   first GEMM:  ceil(ks1/4) groups of 4 k-steps; element [kg][lane][q] = X~[32t + lane%32][2(4kg+q) + lane/32]
//   second GEMM: mt feature tiles x 4 groups of 4 k-steps; k-step v contracts rows i0(v), i0(v)+4:
//                element [u][sg][lane][q] = X~[32t + i0(4sg+q) + 4(lane/32)][32u + lane%32]
//   tail:        per group g of 4 features, 4 groups of 4 steps; step v is one 4x4x1 MFMA whose block
//                lane/4 is row i0(v) + 4(lane/32) against four chains:
//                element [g][sg][lane][q] = X~[32t + i0(4sg+q) + 4(lane/32)][32mt + 4g + lane%4]
inline void grid_pack_operands(const float* X, const float* y, int64_t n, int64_t d, GridData* gd, std::vector<float>* out)
{
    gd->d = (int)d;
    grid_shape(d, &gd->ks1, &gd->mt, &gd->tail);
    const int kg1 = (gd->ks1 + 3) / 4;
    gd->n_rows = (long)n;
    gd->n_tiles = (int)((n + kGridRows - 1) / kGridRows);
    const size_t per_tile = (size_t)grid_groups_per_tile(gd->ks1, gd->mt, gd->tail) * 256;
    out->assign(per_tile * (gd->n_tiles + 1), 0.0f);  // one spare tile: the fetch runs one tile ahead
    auto xs = [&](int64_t row, int64_t feat) -> float {
        if (row >= n || feat >= d) return 0.0f;
        const float v = X[row * d + feat];
        return y[row] != 0.0f ? v : -v;
    };
    for (int t = 0; t < gd->n_tiles; ++t) {
        float* o = out->data() + per_tile * t;
        for (int kg = 0; kg < kg1; ++kg)
            for (int l = 0; l < 64; ++l)
                for (int q = 0; q < 4; ++q) o[(kg * 64 + l) * 4 + q] = xs((int64_t)t * 32 + (l & 31), 2 * (4 * kg + q) + (l >> 5));
        float* o2 = o + (size_t)kg1 * 256;
        for (int u = 0; u < gd->mt; ++u)
            for (int sg = 0; sg < 4; ++sg)
                for (int l = 0; l < 64; ++l)
                    for (int q = 0; q < 4; ++q)
                        o2[((u * 4 + sg) * 64 + l) * 4 + q] =
                            xs((int64_t)t * 32 + grid_acc_row(4 * sg + q) + 4 * (l >> 5), 32 * u + (l & 31));
        float* o3 = o2 + (size_t)gd->mt * 4 * 256;
        for (int g = 0; g < gd->tail; ++g)
            for (int sg = 0; sg < 4; ++sg)
                for (int l = 0; l < 64; ++l)
                    for (int q = 0; q < 4; ++q)
                        o3[((g * 4 + sg) * 64 + l) * 4 + q] =
                            xs((int64_t)t * 32 + grid_acc_row(4 * sg + q) + 4 * (l >> 5), 32 * gd->mt + 4 * g + (l & 3));
    }
}

// Device buffers of one sampling call (all inside the target's workspace).
struct GridBuffers {
    // (chain_stride = slots of this run, a multiple of 128)
    float* theta_t;        // [kGridFeatPad][chain_stride]: positions, one column per chain slot
    float* g_part;         // [slices][chain_stride][kGridFeatPad]: a chain's partial gradient is one 512-byte row per slice
    double* ll_part;       // [slices][chain_stride]
    int* active_all;       // [sets][kGridBatch]: does anybody of set k need a gradient in round r of the batch
    int* halted;           // [kGridMaxChains]
    void* saved;           // WaveChain<float>::Saved per slot
    char* chain_ws;        // wave-kernel style vectors per slot
    size_t chain_ws_bytes; // per slot
};

struct GridArgs {
    const float* ops;
    int d, ks1, mt, tail, n_tiles, n_slices;
    int chain_stride;            // slots of the run, rounded up to whole sets
    int slot_base, n_span_slots; // the consecutive sets of one stream: first slot, number of slots (a multiple of 4)
    long n_rows;
    unsigned long long* counters;
    const double* ftab;  // table of the logistic function for the weight merges, global memory
    GridBuffers b;
};

// ------------------------------------------------------------------ gradient
template <int kKs1, int kMt, int kTail>
__global__ __launch_bounds__(kGridWaves * kWave, 2) void nuts_grid_grad_kernel(GridArgs ga, int round)
{
    constexpr int kKg1 = (kKs1 + 3) / 4;
    // blockIdx.y: which of the stream's sets (the launch spans them all; ga describes the first)
    const int slot_base = ga.slot_base + (int)blockIdx.y * kGridSetChains;
    const int slots_left = ga.n_span_slots - (int)blockIdx.y * kGridSetChains;
    const int n_set_slots = slots_left < kGridSetChains ? slots_left : kGridSetChains;
    if (!ga.b.active_all[(slot_base / kGridSetChains) * kGridBatch + round]) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) {  // one gradient round of this set: every slot of the set is offered
        atomicAdd(&ga.counters[kCtrIssued], (unsigned long long)n_set_slots);
        atomicAdd(&ga.counters[kCtrRounds], 1ull);
    }
    const int lane = threadIdx.x & (kWave - 1), grp = threadIdx.x >> 6;
    const bool computes = grp * kGridGroup < n_set_slots;
    const int slice = blockIdx.x;
    const int t0 = (int)((long)ga.n_tiles * slice / ga.n_slices), t1 = (int)((long)ga.n_tiles * (slice + 1) / ga.n_slices);
    const int col = slot_base + grp * kGridGroup + (lane & 31), half = lane >> 5;

    float b1[4 * kKg1];  // B[k][j] = Theta[feature 2s + lane/32][chain col]  (only the first kKs1 are used)
#pragma unroll
    for (int s = 0; s < kKs1; ++s) b1[s] = ga.b.theta_t[(size_t)(2 * s + half) * ga.chain_stride + col];

    v16f G[kMt];
#pragma unroll
    for (int u = 0; u < kMt; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) G[u][v] = 0.0f;
    // tail group g, register i: feature 32 kMt + 4g + i of chain `col`, summed over this lane half's rows;
    // two accumulators per group, so that consecutive small MFMAs do not wait for each other
    v4f T[kTail > 0 ? kTail : 1][2];
#pragma unroll
    for (int g = 0; g < (kTail > 0 ? kTail : 1); ++g) T[g][0] = T[g][1] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    double ll = 0.0;
    // The operand groups of a tile are fetched once per workgroup, straight from global memory into LDS
    // (no registers in between): each wave requests its share of the next tile into the other stage
    // before it computes the current one, and waits for its requests before the barrier that ends the
    // tile, which also separates the two uses of a stage.
    constexpr int kGroups = grid_groups_per_tile(kKs1, kMt, kTail);
    constexpr int kShare = kGroups / kGridWaves;
    __shared__ float4 s_ops[2][kGroups * 64];
    const float4* src = reinterpret_cast<const float4*>(ga.ops) + ((size_t)t0 * kGroups + grp * kShare) * 64 + lane;
    auto fetch = [&](int stage) {
#pragma unroll
        for (int i = 0; i < kShare; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + i * 64),
                                             (__attribute__((address_space(3))) void*)(&s_ops[stage][(grp * kShare + i) * 64]), 16, 0, 0);
    };
    fetch(0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int t = t0; t < t1; ++t) {
        const int stage = (t - t0) & 1;
        src += kGroups * 64;  // the tile after the last one exists (a spare, all zeros)
        fetch(stage ^ 1);
        if (computes) {
            const float4* ops = &s_ops[stage][lane];
            v16f z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.0f;
#pragma unroll
            for (int kg = 0; kg < kKg1; ++kg) {
                const float4 a = ops[kg * 64];
                z = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b1[4 * kg + 0], z, 0, 0, 0);
                z = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b1[4 * kg + 1], z, 0, 0, 0);
                if (4 * kg + 2 < kKs1) {
                    z = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b1[4 * kg + 2], z, 0, 0, 0);
                    z = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b1[4 * kg + 3], z, 0, 0, 0);
                }
            }
            // logistic functions on the accumulator; rows past the end of the data contribute nothing.
            // Vector instructions do not overlap with MFMAs on this chip, so every one of them counts:
            // log(1 + e^-z) = max(-z, 0) + log(1 + e^-|z|), and the 16 second terms of a lane are taken as
            // one logarithm of the product of their arguments (each in [1, 2]).
            const bool ragged = (long)(t + 1) * kGridRows > ga.n_rows;
            float sg[16], prod = 1.0f, hinge = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float zt = z[v];
                // single hardware instructions: the arguments are in their safe ranges (2^x with x <= 0,
                // reciprocal of a number in [1, 2]); a NaN logit makes every result NaN
                const float e = __builtin_amdgcn_exp2f(fabsf(zt) * -1.44269504088896341f);
                float tt = 1.0f + e;
                const float inv = __builtin_amdgcn_rcpf(tt);
                float s = (zt < 0.0f ? 1.0f : e) * inv;
                if (ragged && (long)t * kGridRows + grid_acc_row(v) + 4 * half >= ga.n_rows) {
                    tt = 1.0f;  // the padded row has z = 0: no hinge term either
                    s = 0.0f;
                }
                prod *= tt;
                hinge += fmaxf(-zt, 0.0f);
                sg[v] = s;
            }
            ll -= (double)fmaf(__builtin_amdgcn_logf(prod), 0.69314718055994531f, hinge);
#pragma unroll
            for (int u = 0; u < kMt; ++u)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const float4 a = ops[(kKg1 + u * 4 + q4) * 64];
                    G[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, sg[4 * q4 + 0], G[u], 0, 0, 0);
                    G[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, sg[4 * q4 + 1], G[u], 0, 0, 0);
                    G[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, sg[4 * q4 + 2], G[u], 0, 0, 0);
                    G[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, sg[4 * q4 + 3], G[u], 0, 0, 0);
                }
#pragma unroll
            for (int g = 0; g < kTail; ++g)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const float4 a = ops[(kKg1 + (kMt + g) * 4 + q4) * 64];
                    T[g][0] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.x, sg[4 * q4 + 0], T[g][0], 0, 0, 0);
                    T[g][1] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.y, sg[4 * q4 + 1], T[g][1], 0, 0, 0);
                    T[g][0] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.z, sg[4 * q4 + 2], T[g][0], 0, 0, 0);
                    T[g][1] = __builtin_amdgcn_mfma_f32_4x4x1f32(a.w, sg[4 * q4 + 3], T[g][1], 0, 0, 0);
                }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }
    if (!computes) return;
    // accumulator register v = 4w + r of feature tile u is G[feature 32u + 8w + r + 4*half][chain col]:
    // four consecutive features per register quad
    float* gp = ga.b.g_part + ((size_t)slice * ga.chain_stride + col) * kGridFeatPad + 4 * half;
#pragma unroll
    for (int u = 0; u < kMt; ++u)
#pragma unroll
        for (int w = 0; w < 4; ++w)
            *reinterpret_cast<float4*>(gp + 32 * u + 8 * w) = make_float4(G[u][4 * w], G[u][4 * w + 1], G[u][4 * w + 2], G[u][4 * w + 3]);
#pragma unroll
    for (int g = 0; g < kTail; ++g) {  // the two lane halves hold the sums over their own rows
        float4 s;
        s.x = T[g][0][0] + T[g][1][0];
        s.y = T[g][0][1] + T[g][1][1];
        s.z = T[g][0][2] + T[g][1][2];
        s.w = T[g][0][3] + T[g][1][3];
        s.x += __shfl_xor(s.x, 32, kWave);
        s.y += __shfl_xor(s.y, 32, kWave);
        s.z += __shfl_xor(s.z, 32, kWave);
        s.w += __shfl_xor(s.w, 32, kWave);
        if (half == 0) *reinterpret_cast<float4*>(gp + 32 * kMt + 4 * g) = s;
    }
    ll += __shfl_xor(ll, 32, kWave);
    if (half == 0) ga.b.ll_part[(size_t)slice * ga.chain_stride + col] = ll;
}

// ------------------------------------------------------------------ control
// One workgroup per chain slot.  All four waves sum the slices' partial results of the chain's last
// gradient; the first wave then runs the chain.  After a kernel boundary every dependent access to
// global memory costs about a microsecond, so what the first wave needs to finish the step is
// requested before the sums.  first_launch: nothing is saved yet and nobody waits for a gradient.
__global__ __launch_bounds__(256) void nuts_grid_control_kernel(DevTarget<float> tg, DevSample sa, GridArgs ga, int round,
                                                                 int first_launch)
{
    typedef WaveChain<float> Chain;
    __builtin_amdgcn_s_setprio(3);  // ahead of the other set's gradient waves on the same SIMD: this launch is the short one
    __shared__ double s_g[kGridSumParts][kGridFeatPad];
    __shared__ double s_ll[kGridMaxSlices];
    const int lane = threadIdx.x & (kWave - 1);
    const int slot = ga.slot_base + blockIdx.x;  // the launch has one workgroup per slot, for all sets of its stream
    Chain::Saved* st = static_cast<Chain::Saved*>(ga.b.saved) + slot;
    float* ws = reinterpret_cast<float*>(ga.b.chain_ws + (size_t)slot * ga.b.chain_ws_bytes);
    Chain ch(tg, sa, lane, ws, nullptr, nullptr);
    ch.ftab = ga.ftab;
    const int d = tg.d;
    if (!first_launch) ch.restore(st);  // (every wave: the saved program counter decides what the workgroup does)
    const bool at_leaf = ch.pc == kPcLeaf, at_init = ch.pc == kPcInitEval;
    const bool waited = !first_launch && (at_leaf || at_init);  // a waiting chain made the last round active
    // d <= 128: two components per lane
    const float* th = at_leaf ? ch.leaf_position() : ch.pool(ch.top_idx, 0);
    float* g = at_leaf ? ch.leaf_gradient() : ch.pool(ch.top_idx, 1);
    float* rv = ch.edge(ch.v > 0 ? 1 : 0, 1);
    float th_reg[2] = {0.0f, 0.0f}, r_reg[2] = {0.0f, 0.0f};
    if (waited && threadIdx.x < kWave) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int i = lane + c * kWave;
            if (i < d) {
                th_reg[c] = th[i];
                if (at_leaf) r_reg[c] = rv[i];
            }
        }
    }
    if (waited) {
        // thread = (part, four features): slices part, part + 8, ... summed in that order, 16 loads in flight
        const int q = threadIdx.x & 31, part = threadIdx.x >> 5;
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        if (4 * q < d) {
            constexpr int P = kGridSumParts;
            const size_t stride = (size_t)ga.chain_stride * (kGridFeatPad / 4);  // float4 per slice
            const float4* p = reinterpret_cast<const float4*>(ga.b.g_part) + (size_t)slot * (kGridFeatPad / 4) + q;
            int s = part;
            for (; s + 15 * P < ga.n_slices; s += 16 * P) {
                float4 v[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) v[k] = p[(size_t)(s + k * P) * stride];
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    a0 += (double)v[k].x; a1 += (double)v[k].y; a2 += (double)v[k].z; a3 += (double)v[k].w;
                }
            }
            for (; s + 3 * P < ga.n_slices; s += 4 * P) {
                float4 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = p[(size_t)(s + k * P) * stride];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    a0 += (double)v[k].x; a1 += (double)v[k].y; a2 += (double)v[k].z; a3 += (double)v[k].w;
                }
            }
            for (; s < ga.n_slices; s += P) {
                const float4 v0 = p[(size_t)s * stride];
                a0 += (double)v0.x; a1 += (double)v0.y; a2 += (double)v0.z; a3 += (double)v0.w;
            }
        }
        s_g[part][4 * q + 0] = a0;
        s_g[part][4 * q + 1] = a1;
        s_g[part][4 * q + 2] = a2;
        s_g[part][4 * q + 3] = a3;
        s_ll[threadIdx.x] = (int)threadIdx.x < ga.n_slices ? ga.b.ll_part[(size_t)threadIdx.x * ga.chain_stride + slot] : 0.0;
    }
    __syncthreads();
    if (threadIdx.x >= kWave) return;

    if (waited) {
        // finish the step whose gradient the last round computed: gradient, second half-kick, energy
        const float half = (float)(0.5 * (ch.v * sa.eps));
        double sq = 0.0, kin = 0.0;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int i = lane + c * kWave;
            if (i < d) {
                const double t = (double)th_reg[c];
                const double gsum = ((s_g[0][i] + s_g[1][i]) + (s_g[2][i] + s_g[3][i])) + ((s_g[4][i] + s_g[5][i]) + (s_g[6][i] + s_g[7][i]));
                const float gi = (float)(gsum - t * tg.prior_prec);
                g[i] = gi;
                sq = fma(t, t, sq);
                if (at_leaf) {
                    const float rn = r_reg[c] + half * gi;
                    rv[i] = rn;
                    kin = fma((double)rn, (double)rn, kin);
                }
            }
        }
        double ll = (s_ll[lane] + s_ll[lane + 64]) + (s_ll[lane + 128] + s_ll[lane + 192]);
        wave_sum2(ll, sq);
        const double logp = ll - 0.5 * tg.prior_prec * sq;
        if (at_leaf)
            ch.leaf_finish(logp, wave_sum(kin));
        else
            ch.init_post(logp);
    }
    if (ch.pc != kPcHalt) ch.run_to_gradient_request();
    // publish the position the next gradient is wanted at (zeros if none)
    const float* pos = nullptr;
    if (ch.pc == kPcLeaf) {
        ch.leaf_pre();
        pos = ch.leaf_position();
    } else if (ch.pc == kPcInitEval) {
        pos = ch.pool(ch.top_idx, 0);
    }
    for (int i = lane; i < kGridFeatPad; i += kWave)
        ga.b.theta_t[(size_t)i * ga.chain_stride + slot] = (pos && i < d) ? pos[i] : 0.0f;
    if (lane == 0) {
        if (pos) ga.b.active_all[(slot / kGridSetChains) * kGridBatch + round] = 1;  // (a launch may span several sets)
        ga.b.halted[slot] = ch.pc == kPcHalt;
    }
    ch.save(st);
}

__global__ void nuts_grid_fill_kernel(int* p, int n, int value)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = value;
}

// counters of a finished run (the gradient launches have counted rounds and offered slots)
__global__ void nuts_grid_finish_kernel(GridArgs ga, DevSample sa, int n_slots)
{
    typedef WaveChain<float> Chain;
    for (int slot = threadIdx.x; slot < n_slots; slot += blockDim.x) {
        const Chain::Saved* st = static_cast<const Chain::Saved*>(ga.b.saved) + slot;
        atomicAdd(&sa.counters[kCtrUseful], st->n_leaf);
        atomicAdd(&sa.counters[kCtrExtra], st->n_extra);
    }
}

template <int kMt, int kTail>
inline void grid_launch_grad(const GridArgs& ga, int round, hipStream_t stream)
{
    const unsigned sets = (unsigned)((ga.n_span_slots + kGridSetChains - 1) / kGridSetChains);
    hipLaunchKernelGGL((nuts_grid_grad_kernel<16 * kMt + 2 * kTail, kMt, kTail>), dim3((unsigned)ga.n_slices, sets),
                       dim3(kGridWaves * kWave), 0, stream, ga, round);
}

// (the shapes grid_shape() can return)
inline void grid_launch_grad_any(const GridArgs& ga, int round, hipStream_t stream)
{
    switch (ga.mt * 4 + ga.tail) {
    case 4: grid_launch_grad<1, 0>(ga, round, stream); break;
    case 5: grid_launch_grad<1, 1>(ga, round, stream); break;
    case 6: grid_launch_grad<1, 2>(ga, round, stream); break;
    case 8: grid_launch_grad<2, 0>(ga, round, stream); break;
    case 9: grid_launch_grad<2, 1>(ga, round, stream); break;
    case 10: grid_launch_grad<2, 2>(ga, round, stream); break;
    case 12: grid_launch_grad<3, 0>(ga, round, stream); break;
    case 13: grid_launch_grad<3, 1>(ga, round, stream); break;
    case 14: grid_launch_grad<3, 2>(ga, round, stream); break;
    default: grid_launch_grad<4, 0>(ga, round, stream); break;
    }
}

}  // namespace nuts
