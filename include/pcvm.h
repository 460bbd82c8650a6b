/*
 * Program-counter virtual machine on one MI355X (C ABI).
 *
 * Runs a batch of independent executions of one program written in the control-flow-graph language of
 * Figure 4 of the paper (arxiv 1910.11141, Section 3): basic blocks of Push / Pop operations, each ended by
 * Jump, Branch, PushJump or Return.  The runtime is Algorithm 2 of the paper: every batch member has its own
 * program-counter stack and one stack per variable; at each step a group of members runs the earliest block
 * any of them waits for, under a mask.  A group is one 64-lane wavefront (the scheduler's "which block next"
 * freedom of Section 2 is taken per wavefront: members are independent, so results do not depend on it).
 *
 * Readings (the paper leaves them open): stack indexes count entries, the top is the last entry; a member
 * whose program-counter stack is empty has halted; variables are 64-bit integers with wrap-around arithmetic;
 * every primitive is total (x mod 0 = x mod -1 = 0, shift counts use their low 6 bits) because masked lanes
 * compute on junk; Update overwrites the top entry in place (a cancelled Pop/Push pair, Section 3.2); a
 * variable that is never pushed keeps index 0 and only ever uses its cached top.
 */
#ifndef PCVM_H
#define PCVM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PCVM_OK = 0,
    PCVM_E_INVALID_ARG = -1,     /* null pointer, size out of range, malformed program table          */
    PCVM_E_ALLOC = -2,
    PCVM_E_DEVICE = -3,          /* no HIP device, launch or copy failed (there is no CPU path)        */
    PCVM_E_STACK_OVERFLOW = -5,  /* a push beyond stack_depth (variable or program-counter stack)      */
    PCVM_E_STACK_UNDERFLOW = -6, /* a pop from an empty variable stack                                 */
    PCVM_E_STEP_LIMIT = -7       /* a group made max_steps steps without halting                       */
};

enum { PCVM_PUSH = 0, PCVM_UPDATE = 1, PCVM_POP = 2 };                      /* pcvm_op.kind  */
enum {                                                                      /* pcvm_op.fn: y = f(a, b, imm) */
    PCVM_CONST = 0, PCVM_COPY, PCVM_ADD, PCVM_SUB, PCVM_MUL, PCVM_ADDI, PCVM_MULI, PCVM_LE, PCVM_LT, PCVM_EQ,
    PCVM_LEI, PCVM_EQI, PCVM_MOD, PCVM_ANDI, PCVM_SHRI, PCVM_FN_COUNT
};
enum { PCVM_JUMP = 0, PCVM_BRANCH = 1, PCVM_PUSHJUMP = 2, PCVM_RETURN = 3 }; /* pcvm_block.term */

/* Which block a group runs next.  Any choice that starves nobody is correct (Section 2 of the paper).
 * EARLIEST: the lowest-numbered block anyone waits for (Algorithm 2 as printed).
 * MOST_WAITING: the block most lanes wait for (lowest on a tie): fewer, fuller steps; a lone lane can wait
 *   while the queue still feeds the others, but not beyond the end of the batch. */
enum { PCVM_SCHED_EARLIEST = 0, PCVM_SCHED_MOST_WAITING = 1 };

#define PCVM_MAX_VARS 16
#define PCVM_MAX_DEPTH 4096
#define PCVM_GROUP 64

/* One operation of a block.  PUSH: evaluate f on the tops of a and b, push the result on dst.  UPDATE: the same,
 * overwriting the top of dst.  POP: drop the top of dst (fn, a, b, imm ignored). */
typedef struct {
    int32_t kind, fn, dst, a, b, pad;
    int64_t imm;
} pcvm_op;

/* One basic block: operations [first_op, first_op + n_ops) then the terminator.
 * JUMP i | BRANCH x i j (to i if the top of x is non-zero, else j) | PUSHJUMP i j (enter i, resume at j) | RETURN.
 * `label` is free for the caller (e.g. a source line); the runtime ignores it. */
typedef struct {
    int32_t first_op, n_ops, term, x, i, j, label, pad;
} pcvm_block;

/* A program.  Variables 0 .. n_inputs-1 receive the inputs (one push each); every member starts at block 0;
 * the result is the top of output_var when the member halts.  `blocks` and `ops` are HOST arrays, read
 * during the call only. */
typedef struct {
    int32_t n_vars, n_inputs, output_var, n_blocks, n_ops, reserved;
    const pcvm_block* blocks;
    const pcvm_op* ops;
} pcvm_program;

typedef struct {
    uint64_t steps;               /* scheduler steps (one block executed by one group), summed over groups */
    uint64_t active_member_steps; /* members that really executed the block, summed over steps             */
    uint64_t issued_member_steps; /* steps x PCVM_GROUP: what the masked execution paid for                 */
    double kernel_ms;             /* duration of the interpreter kernel, from HIP events                    */
    int32_t n_groups, reserved;
} pcvm_stats;

/* Run `batch` executions to completion (synchronous: returns when the outputs are written).
 *   inputs   DEVICE, int64 [n_inputs][batch]
 *   outputs  DEVICE, int64 [batch]
 *   stack_depth  entries per stack, 1 .. PCVM_MAX_DEPTH; the call allocates (n_vars * 8 + 4) * stack_depth
 *            bytes per member of device memory and frees it before returning
 *   max_steps    per-group bound on scheduler steps (> 0): a program that does not halt ends with STEP_LIMIT
 *   trace    DEVICE int32 [2 * trace_capacity] or NULL: (block, number of active members) of the first
 *            trace_capacity steps of group 0 (members 0..63)
 *   stats    HOST or NULL
 * On a STACK_* or STEP_LIMIT error the outputs are unspecified.  The program table is validated on the host
 * first (every index in range), so a malformed table is INVALID_ARG and never reaches the device. */
int pcvm_run(const pcvm_program* program, int64_t batch, const int64_t* inputs, int32_t stack_depth,
             int64_t max_steps, int64_t* outputs, int32_t* trace, int64_t trace_capacity, pcvm_stats* stats);

/* The same, with members handed to lanes from a queue (Section 4.2 of the paper applied to the machine itself:
 * executions are batched across their boundaries).  At most as many groups as the chip holds at once are
 * started; a lane whose member has halted writes its output and takes the next unclaimed member, so the lanes
 * of a group stay busy until the batch runs dry, and the stacks need (n_vars * 8 + 4) * stack_depth bytes per
 * resident lane instead of per member.  Outputs are those of pcvm_run; which members share a group depends on
 * timing, so steps and utilisation vary a little from run to run and there is no trace.  max_steps bounds the
 * group steps one member may stay in flight; policy is PCVM_SCHED_*. */
int pcvm_run_queued(const pcvm_program* program, int64_t batch, const int64_t* inputs, int32_t stack_depth,
                    int64_t max_steps, int32_t policy, int64_t* outputs, pcvm_stats* stats);

/* HIP stream for pcvm_run's work (default: the null stream).  The call still waits for completion. */
int pcvm_set_stream(void* hip_stream);

/* Message of the last error on this thread. */
const char* pcvm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
