/*
 * nuts.h - C ABI of the MI355X lock-step NUTS sampler.
 *
 * The library runs many independent No-U-Turn-Sampler chains on one GPU.  The
 * recursive tree doubling of each chain is turned into an explicit per-chain
 * program counter and stack, and only chains that stand at the same program
 * point are stepped together - the program-counter batching of Radul et al.,
 * "Automatically batching control-intensive programs for modern accelerators"
 * (Section 3, Algorithm 2), specialised by hand to the sampler the paper
 * evaluates (Section 4).  The unit of work the paper counts is one evaluation
 * of the target's log-density gradient (Section 4.1); here that is one
 * leapfrog step, i.e. one leaf of a NUTS tree.
 *
 * All functions return 0 on success and a negative NUTS_E_* code otherwise; a
 * human-readable reason is then available from nuts_last_error().  No C++
 * exception crosses this boundary.  On an argument error nothing is written to
 * any output buffer.  The library never falls back to the CPU: without a GPU
 * every call that needs one fails with NUTS_E_DEVICE.
 */
#ifndef NUTS_H_
#define NUTS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { NUTS_OK = 0, NUTS_E_INVALID_ARG = -1, NUTS_E_ALLOC = -2, NUTS_E_DEVICE = -3, NUTS_E_UNSUPPORTED = -4 };

/* Arithmetic type of the target data, the chain states and out_states.  Energies,
 * log-weights and U-turn dot products are binary64 in both cases. */
enum { NUTS_F32 = 0, NUTS_F64 = 1 };

/* Target families (the paper's two test problems, Section 4, plus the two
 * element-wise Gaussians of the benchmark configurations). */
enum {
    NUTS_TARGET_STD_NORMAL = 0,            /* log p = -1/2 |x|^2                                   */
    NUTS_TARGET_GAUSS_DENSE_PRECISION = 1, /* log p = -1/2 x' P x                                  */
    NUTS_TARGET_GAUSS_DIAG = 2,            /* log p = -1/2 sum_i x_i^2 / sigma_i^2                 */
    NUTS_TARGET_LOGISTIC_REGRESSION = 3    /* sum_n [y_n z_n - log(1+e^{z_n})] - |x|^2/(2 s^2), z = X x */
};

/* Which kernel family nuts_sample_ex uses. */
enum {
    NUTS_VARIANT_AUTO = 0,
    NUTS_VARIANT_WAVE = 1,  /* one wavefront per chain, vectors striped over the 64 lanes; any target/shape */
    NUTS_VARIANT_TILE = 2,  /* 16 chains per workgroup in lock step, gradient as MFMA GEMMs (logistic
                               regression, binary64, dim <= 32, max_tree_depth <= 12); when dim = 1 mod 4
                               and a column of X is the same non-zero value in every row (an intercept),
                               that column's share of the logits is added ahead of the others' instead of
                               in its place among them: another order of the same sum                       */
    NUTS_VARIANT_ELEM = 3,  /* one wavefront per chain with the moving trajectory end held in registers
                               (standard normal / diagonal Gaussian, dim <= 1024 binary32, <= 512 binary64) */
    NUTS_VARIANT_GRID = 4,  /* every gradient round is a chip-wide binary32 MFMA GEMM over the data rows
                               (logistic regression, binary32, dim <= 128; up to 1024 chains are resident
                               at a time, further chains wait in a queue); this variant returns only when
                               sampling has finished; beyond 128 chains the resident ones are spread over
                               up to four streams, the caller's and three that the target owns, forked
                               from and joined to the caller's stream by events                            */
    NUTS_VARIANT_DENSE = 5, /* one wavefront per chain, moving trajectory end in registers, precision matrix in LDS
                               (dense Gaussian, dim <= 128)                                                 */
    NUTS_VARIANT_QUAD = 6   /* four chains per wavefront, their precision-matrix products together as MFMA blocks
                               with the matrix in LDS in operand order (dense Gaussian, binary64, dim <= 128,
                               max_tree_depth <= 12); chosen automatically for matrices that are not banded
                               from 2560 chains on                                                          */
};

typedef struct nuts_target nuts_target; /* opaque; owns device copies of its data */

/* All pointers in the descriptor are HOST pointers to arrays of `dtype`; they are
 * copied (and re-laid-out) during nuts_create_target and may be freed afterwards. */
typedef struct {
    int32_t kind;          /* NUTS_TARGET_*                                                    */
    int32_t dtype;         /* NUTS_F32 / NUTS_F64                                              */
    int64_t dim;           /* d >= 1                                                           */
    const void* precision; /* GAUSS_DENSE_PRECISION: d*d row-major, symmetric                  */
    const void* scales;    /* GAUSS_DIAG: sigma_i > 0, d values                                */
    const void* X;         /* LOGISTIC_REGRESSION: n_data*d row-major design matrix            */
    const void* y;         /* LOGISTIC_REGRESSION: n_data labels in {0,1}                      */
    int64_t n_data;        /* LOGISTIC_REGRESSION: n_data >= 1                                 */
    double prior_scale;    /* LOGISTIC_REGRESSION: prior N(0, prior_scale^2 I), > 0            */
} nuts_target_desc;

/* Counters of the last nuts_sample* call on a target (see nuts_get_stats). */
typedef struct {
    uint64_t leaf_slots_issued; /* chain slots handed to the batched gradient step over all lock-step
                                   rounds, idle and padded slots included.  Kernels whose chains do not
                                   step together (wave, element-wise) hold every slot for the whole
                                   launch: they charge, per launch, slots x the gradient count of the
                                   busiest slot                                                        */
    uint64_t leaf_slots_useful; /* of those, slots that carried a leapfrog step (= sum of out_n_leapfrog) */
    uint64_t extra_grad_evals;  /* gradient evaluations that are not leapfrog steps (initial points)   */
    uint64_t rounds;            /* lock-step rounds, summed over workgroups                            */
    double kernel_ms;           /* duration of the sampler kernel, from HIP events on its stream       */
    uint64_t phase_ticks[3];    /* tile kernel: shader-clock ticks spent in {control, batched gradient,
                                   step completion}, summed over workgroups (divide by `rounds`)       */
    int32_t variant;            /* NUTS_VARIANT_* that ran                                             */
    int32_t grid_blocks;        /* workgroups launched                                                 */
} nuts_stats;

/* When chains may start their next iteration (Section 4.2 of the paper compares the two).
 * FREE: a chain goes on as soon as its own trajectory is finished, so gradient steps of different
 *   iterations are batched together (what program-counter batching allows).
 * TRAJECTORY: no chain starts iteration i+1 before every chain of the call has finished iteration i
 *   (all a batching scheme that follows the control structure of the chain program can do).  One
 *   launch per iteration; the gradient at each iteration's starting point is evaluated again
 *   (counted in extra_grad_evals, never in out_n_leapfrog).
 * Both give bit-identical outputs. */
enum { NUTS_SCHEDULE_FREE = 0, NUTS_SCHEDULE_TRAJECTORY = 1 };

/* How the points of a trajectory are weighted when one of them is selected.
 * MULTINOMIAL (default): weight exp(H0 - H) per leaf, subtrees summarised by the log of their summed weights.
 * SLICE: the form of the No-U-Turn Sampler as first published (Hoffman & Gelman, JMLR 2014, Algorithm 3),
 *   which is what Section 4.1 of the paper batches: a height u is drawn uniformly below exp(-H0) once per
 *   iteration (draw purpose 5), a leaf is a candidate iff exp(-H) >= u and stays valid while
 *   exp(-H) > u exp(-1000); subtrees are summarised by their candidate counts; the right half's
 *   proposal is taken with probability count_R / (count_L + count_R), a new half with min(1, count_new / count_tree).
 * Everything else (doubling, U-turn tests, depth limit, leaf_steps, outputs) is shared. */
enum { NUTS_SAMPLER_MULTINOMIAL = 0, NUTS_SAMPLER_SLICE = 1 };

/* Options of nuts_sample_ex; zero-initialise for the defaults. */
typedef struct {
    const void* init_states; /* DEVICE, dtype, [n_chains][dim]; NULL: x0 ~ N(0, I) drawn from `seed`     */
    int64_t first_chain;     /* global id of chain 0 (enters the random-number keys); default 0.  A run
                                of chains [a, a+n) equals columns [a, a+n) of a larger run.              */
    int32_t variant;         /* NUTS_VARIANT_*                                                           */
    int32_t leaf_steps;      /* leapfrog steps per tree leaf, 1..NUTS_MAX_LEAF_STEPS; 0 means 1.  Section 4.1
                                of the paper takes 4 so that the control around a leaf is paid once per 4
                                gradients.  Only a leaf's end state is a candidate and enters the U-turn
                                and energy tests; out_n_leapfrog counts leapfrog steps (leaf_steps per
                                leaf); the subtree-selection draw is keyed by that count at the merge.   */
    int32_t schedule;        /* NUTS_SCHEDULE_*                                                          */
    int32_t sampler;         /* NUTS_SAMPLER_*                                                           */
} nuts_sample_options;
#define NUTS_MAX_LEAF_STEPS 64

/* Create a target, i.e. the fixed synthetic posterior the chains sample from (the
 * paper's test problems are of this kind: Section 4, logistic regression and a
 * correlated Gaussian): validates the descriptor, copies the data to the current
 * device in the layouts the kernels want.  STD_NORMAL needs no device.
 * Errors: INVALID_ARG (null/shape/kind/dtype, non-finite or non-positive scale),
 * DEVICE, ALLOC.  *out is set only on success. */
int nuts_create_target(const nuts_target_desc* desc, nuts_target** out);

/* Free a target and everything it owns (device data, cached workspace). NULL is allowed. */
int nuts_destroy_target(nuts_target* t);

/* The batched sampler itself: "the number of chains running in tandem" is the batch
 * size of Section 4.1, each chain is one batch member of Algorithm 2 with its own
 * program counter and stack.
 * Run n_iters NUTS iterations of n_chains chains (multinomial NUTS, one leapfrog
 * step per leaf, identity mass matrix, fixed step size; initial states
 * x0 ~ N(0, I) drawn from `seed`).  Every random number is a function of
 * (seed, chain, iteration, purpose, position) only, so results do not depend on
 * how chains are scheduled.
 *   out_states       DEVICE, dtype, [n_iters][n_chains][dim]: state after each iteration
 *   out_tree_depths  DEVICE, int32 [n_iters][n_chains]: doublings attempted (1..max_tree_depth)
 *   out_n_leapfrog   DEVICE, int32 [n_iters][n_chains]: leapfrog steps (= gradient evaluations
 *                    requested by the chain; the evaluation at x0 is not counted)
 * Any output may be NULL.  The caller owns the buffers.  The work is enqueued on
 * the stream given to nuts_set_stream (default: the null stream) and the call
 * returns without waiting; scratch memory is owned by the target and reused by
 * later calls, so calls on one target must not overlap.
 * Domain: n_chains >= 1, n_iters >= 1, step_size finite > 0, 1 <= max_tree_depth <= 20.
 * Errors: INVALID_ARG, DEVICE (no GPU / launch failure), ALLOC, UNSUPPORTED. */
int nuts_sample(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size,
                int32_t max_tree_depth, uint64_t seed, void* out_states, int32_t* out_tree_depths,
                int32_t* out_n_leapfrog);

/* nuts_sample with options (initial states, global chain offset, kernel variant). */
int nuts_sample_ex(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size,
                   int32_t max_tree_depth, uint64_t seed, const nuts_sample_options* options,
                   void* out_states, int32_t* out_tree_depths, int32_t* out_n_leapfrog);

/* nuts_sample_ex for callers that cannot allocate device memory while they call: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * outputs bit for bit; but the call allocates and frees nothing.  Its workspace and counters live in a
 * static device array of NUTS_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU
 * the library runs on holds one copy until the process ends).
 *   - The target must have been created with a GPU present (creation is where device data, tables, counters
 *     and events are set up, and where the array's device address is looked up).
 *   - A run whose workspace does not fit is refused with NUTS_E_UNSUPPORTED and a message that states the bytes
 *     needed and the maximum; nothing is written.  (The workspace grows with the resident chain slots, the
 *     dimension and max_tree_depth: configuration 3, 4096 chains of logistic regression, needs 46 MB.)
 *   - Also refused: NUTS_VARIANT_GRID (it owns streams and pinned host memory and waits on the host), and
 *     NUTS_SCHEDULE_TRAJECTORY without out_states (it would need a carry buffer).
 *   - All calls on one GPU share that GPU's array, whatever the target or host thread: two calls that overlap
 *     in time on one GPU race, also on different streams.  The array keeps the last call's contents; the call
 *     clears what it needs at zero with a small kernel (no memset node, so it can be captured).
 * nuts_get_stats afterwards reports this call. */
#define NUTS_STATIC_SCRATCH_BYTES (64u << 20)
int nuts_sample_static(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size,
                       int32_t max_tree_depth, uint64_t seed, const nuts_sample_options* options,
                       void* out_states, int32_t* out_tree_depths, int32_t* out_n_leapfrog);

/* Counters and kernel time of the last sampling call on `target`.  Waits for that
 * call to finish (synchronises on its stop event). */
int nuts_get_stats(const nuts_target* target, nuts_stats* out);

/* Stream (a hipStream_t) for subsequent nuts_sample* calls of this host thread. */
int nuts_set_stream(void* hip_stream);

/* Message for the last error on this host thread; valid until the next call. */
const char* nuts_last_error(void);

/* Host only (no device is touched): the operand stream that nuts_create_target lays out for the tile variant from a
 * binary64 logistic-regression data set (Section 4's logistic regression as the two GEMMs Z = X Theta, G = X' s on
 * 16-row tiles), for checking that layout without a GPU.  X is n x d row-major and y holds n labels (0 or not 0),
 * both host pointers.  `layout` is filled whenever the arguments and the shape are valid; the stream itself (layout->operand_doubles values) is copied to
 * `operands` if that is not NULL and `capacity` (in doubles) suffices, else INVALID_ARG when `operands` is not NULL.
 * Stream: per tile, operand pairs of 64 x 2 doubles; element (pair p, lane l, half h) is operand 2p + h as lane l
 * feeds it to v_mfma_f64_16x16x4: first GEMM operand s (0 .. ks1 - 1) holds X[16 t + l % 16][slot 4 s + l / 16],
 * second GEMM operand (u, s) (u < mt, s < 4; after the first GEMM's pairs, an odd ks1 leaves one half unused) holds
 * X[16 t + 4 s + l / 16][16 u + l % 16]; rows of y = 0 are negated unless a constant column stays out of the first
 * GEMM (const_col >= 0: then slot const_col carries feature d - 1 and slots from d - 1 on are zero). */
typedef struct {
    int32_t ks1, mt;             /* k-steps of the first GEMM, feature tiles of the second                */
    int32_t n_tiles;             /* row tiles that the kernel runs                                         */
    int32_t n_alloc_tiles;       /* row tiles in the stream (a multiple of 8)                              */
    int32_t const_col;           /* the constant column that is the first GEMM's initial value, or -1     */
    int32_t reserved;
    double const_val;            /* its value                                                              */
    int64_t n_pad;               /* rows of zeros that the kernel runs                                     */
    int64_t operand_doubles;     /* length of the stream                                                   */
} nuts_tile_layout;
int nuts_tile_pack(const double* X, const double* y, int64_t n, int64_t d, nuts_tile_layout* layout, double* operands,
                   int64_t capacity);

#ifdef __cplusplus
}
#endif
#endif /* NUTS_H_ */
