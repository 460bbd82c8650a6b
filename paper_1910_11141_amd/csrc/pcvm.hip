// Program-counter virtual machine: Algorithm 2 of the paper as a HIP interpreter.
//
// One batch member per lane, one lock-step group per 64-lane wavefront.  Per step the group takes the
// smallest block index any of its members waits for, and runs that block's operations for all lanes with
// the writes masked to the members that wait there (the masking style of Section 2).  The top entry of every
// stack is cached (LDS for the variables, a register for the program counter: the fourth optimisation of
// Section 3.2); the entries below it live in global memory as [variable][depth][member], so a push or pop of
// the whole group is one coalesced store or load.  Block and operation records are read through uniform
// indices.  There is no CPU path: without a device the entry point fails.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <vector>

#include "../../include/pcvm.h"

namespace {

thread_local char g_err[512] = "";
thread_local hipStream_t g_stream = nullptr;

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define PCVM_TRY(expr, code)                                                                    \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) return fail(code, "%s: %s", #expr, hipGetErrorString(e_));         \
    } while (0)

constexpr int kWave = PCVM_GROUP;
constexpr int kWavesPerBlock = 4;

struct VmArgs {
    const pcvm_block* blocks;
    const pcvm_op* ops;
    int n_vars, n_inputs, output_var, n_blocks;
    long batch, batch_pad;  // batch_pad: lanes launched = row pitch of the stacks (one stack column per lane)
    unsigned long long* queue;  // queued runs: index of the next member nobody has taken yet
    int policy;                 // queued runs: PCVM_SCHED_*
    int depth;
    long max_steps;
    const long long* inputs;
    long long* outputs;
    long long* var_stacks;  // [n_vars][depth][batch_pad]
    int* pc_stacks;         // [depth][batch_pad]
    int* trace;
    long trace_capacity;
    unsigned long long* counters;  // steps, active member steps
    int* error;                    // most severe error code seen (most negative)
};

// Minimum over the 64 lanes: rotations inside each row of 16 lanes (DPP, no LDS traffic), then the four
// row minima are read as scalars.
template <int kCtrl>
__device__ __forceinline__ int dpp_move(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, kCtrl, 0xf, 0xf, false);
}
__device__ __forceinline__ int wave_min(int x)
{
    x = min(x, dpp_move<0x128>(x));  // row_ror:8
    x = min(x, dpp_move<0x124>(x));  // row_ror:4
    x = min(x, dpp_move<0x122>(x));  // row_ror:2
    x = min(x, dpp_move<0x121>(x));  // row_ror:1
    return min(min(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
               min(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}

// The block most lanes wait for (the lowest such block on a tie); `halt` if nobody waits.
__device__ __forceinline__ int most_waiting(int pc_top, int halt)
{
    unsigned long long todo = __ballot(pc_top < halt);
    int best = halt, best_count = 0;
    while (todo) {
        const int b = __builtin_amdgcn_readlane(pc_top, (int)__builtin_ctzll(todo));
        const unsigned long long same = __ballot(pc_top == b);
        const int count = __popcll(same);
        if (count > best_count || (count == best_count && b < best)) {
            best = b;
            best_count = count;
        }
        todo &= ~same;
    }
    return best;
}

// y = f(a, b, imm): total functions on 64-bit integers, wrap-around.
__device__ __forceinline__ long long primitive(int fn, long long a, long long b, long long imm)
{
    typedef unsigned long long u64;
    switch (fn) {
    case PCVM_CONST: return imm;
    case PCVM_COPY: return a;
    case PCVM_ADD: return (long long)((u64)a + (u64)b);
    case PCVM_SUB: return (long long)((u64)a - (u64)b);
    case PCVM_MUL: return (long long)((u64)a * (u64)b);
    case PCVM_ADDI: return (long long)((u64)a + (u64)imm);
    case PCVM_MULI: return (long long)((u64)a * (u64)imm);
    case PCVM_LE: return a <= b;
    case PCVM_LT: return a < b;
    case PCVM_EQ: return a == b;
    case PCVM_LEI: return a <= imm;
    case PCVM_EQI: return a == imm;
    case PCVM_MOD: return (b == 0 || b == -1) ? 0 : a % b;
    case PCVM_ANDI: return a & imm;
    case PCVM_SHRI: return a >> (imm & 63);
    default: return 0;
    }
}

// kQueued = false: lane l of group g runs member 64 g + l and nothing else (Algorithm 2 on fixed groups).
// kQueued = true: a lane whose member has halted takes the next member from a global queue, so a group keeps
// all its lanes busy until the batch runs dry - members at the first block of a new execution are batched
// with members deep inside an old one, which is what the program-counter formulation makes possible.
template <bool kQueued>
__global__ __launch_bounds__(kWave* kWavesPerBlock) void pcvm_kernel(VmArgs va)
{
    __shared__ long long s_top[kWavesPerBlock][PCVM_MAX_VARS][kWave];
    __shared__ int s_sp[kWavesPerBlock][PCVM_MAX_VARS][kWave];
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    const long group = (long)blockIdx.x * kWavesPerBlock + w;
    const long slot = group * kWave + lane;  // this lane's column in the stack arrays
    long member = kQueued ? -1 : slot;
    bool valid = !kQueued && member < va.batch;
    const int halt = va.n_blocks;

    // "PUSH T onto x": a fresh execution has its inputs on the stacks, every other stack empty, and waits at block 0
    auto start_member = [&]() {
        for (int v = 0; v < va.n_vars; ++v) {
            const bool is_input = v < va.n_inputs;
            s_top[w][v][lane] = (is_input && valid) ? va.inputs[(size_t)v * va.batch + member] : 0;
            s_sp[w][v][lane] = is_input ? 1 : 0;
        }
    };
    start_member();
    int pc_top = valid ? 0 : halt;
    int pc_sp = valid ? 1 : 0;
    long steps = 0, member_steps = 0;
    unsigned long long active_steps = 0;
    int my_error = 0;
    // queued runs: the queue was empty when this lane asked, or its member failed - or the lane belongs to a wave of
    // the last workgroup beyond the last group, which has no stack columns and must not take a member
    bool retired = slot >= va.batch_pad;

    for (;;) {
        if (kQueued && pc_sp == 0 && !retired) {
            const long next = (long)atomicAdd(va.queue, 1ull);
            if (next < va.batch) {
                member = next;
                valid = true;
                start_member();
                pc_top = 0;
                pc_sp = 1;
                member_steps = 0;
            } else {
                retired = true;
            }
        }
        if (kQueued && pc_sp > 0 && member_steps >= va.max_steps) {  // this member does not halt: drop it
            my_error = PCVM_E_STEP_LIMIT;
            pc_top = halt;
            pc_sp = 0;
            retired = true;
        }
        // the earliest block anyone waits for (Algorithm 2), or the one most lanes wait for (a scalar either way)
        const int i = (kQueued && va.policy == PCVM_SCHED_MOST_WAITING) ? most_waiting(pc_top, halt) : wave_min(pc_top);
        if (i >= halt) break;
        if (!kQueued && steps >= va.max_steps) {
            my_error = PCVM_E_STEP_LIMIT;
            break;
        }
        const bool A = pc_top == i;  // locally active set
        const pcvm_block blk = va.blocks[i];
        for (int k = 0; k < blk.n_ops; ++k) {
            const pcvm_op op = va.ops[blk.first_op + k];
            long long& top = s_top[w][op.dst][lane];
            int& sp = s_sp[w][op.dst][lane];
            long long* stack = va.var_stacks + (size_t)op.dst * va.depth * va.batch_pad + slot;
            if (op.kind == PCVM_POP) {
                if (A) {
                    if (sp <= 0) {
                        my_error = min(my_error, (int)PCVM_E_STACK_UNDERFLOW);
                    } else {
                        sp -= 1;
                        if (sp >= 1) top = stack[(size_t)(sp - 1) * va.batch_pad];
                    }
                }
                continue;
            }
            const long long o = primitive(op.fn, s_top[w][op.a][lane], s_top[w][op.b][lane], op.imm);
            if (!A) continue;
            if (op.kind == PCVM_PUSH) {
                if (sp >= va.depth) {
                    my_error = min(my_error, (int)PCVM_E_STACK_OVERFLOW);
                } else {
                    if (sp >= 1) stack[(size_t)(sp - 1) * va.batch_pad] = top;  // the old top goes below
                    sp += 1;
                    top = o;
                }
            } else {
                top = o;
            }
        }
        if (A) {
            switch (blk.term) {
            case PCVM_JUMP: pc_top = blk.i; break;
            case PCVM_BRANCH: pc_top = s_top[w][blk.x][lane] != 0 ? blk.i : blk.j; break;
            case PCVM_PUSHJUMP:
                if (pc_sp >= va.depth) {
                    my_error = min(my_error, (int)PCVM_E_STACK_OVERFLOW);
                } else {
                    va.pc_stacks[(size_t)(pc_sp - 1) * va.batch_pad + slot] = blk.j;  // where this frame resumes
                    pc_sp += 1;
                    pc_top = blk.i;  // the callee's entry
                }
                break;
            default:  // PCVM_RETURN
                pc_sp -= 1;
                pc_top = pc_sp >= 1 ? va.pc_stacks[(size_t)(pc_sp - 1) * va.batch_pad + slot] : halt;
                if (kQueued && pc_sp == 0 && !my_error) va.outputs[member] = s_top[w][va.output_var][lane];
                break;
            }
            if (my_error) {  // a member in error stops; the others of its group go on
                pc_top = halt;
                pc_sp = 0;
                retired = true;
            }
        }
        member_steps += 1;
        const unsigned long long amask = __ballot(A);
        if (va.trace && group == 0 && lane == 0 && steps < va.trace_capacity) {
            va.trace[2 * steps] = i;
            va.trace[2 * steps + 1] = __popcll(amask);
        }
        steps += 1;
        active_steps += (unsigned long long)__popcll(amask);
    }

    if (!kQueued && valid) va.outputs[member] = s_top[w][va.output_var][lane];
    if (my_error) atomicMin(va.error, my_error);
    if (lane == 0) {
        atomicAdd(&va.counters[0], (unsigned long long)steps);
        atomicAdd(&va.counters[1], active_steps);
    }
}

int check_program(const pcvm_program* p)
{
    if (!p || !p->blocks || (!p->ops && p->n_ops > 0)) return fail(PCVM_E_INVALID_ARG, "program, blocks and ops must not be NULL");
    if (p->n_vars < 1 || p->n_vars > PCVM_MAX_VARS) return fail(PCVM_E_INVALID_ARG, "n_vars must be in [1, %d]", PCVM_MAX_VARS);
    if (p->n_inputs < 1 || p->n_inputs > p->n_vars) return fail(PCVM_E_INVALID_ARG, "n_inputs must be in [1, n_vars]");
    if (p->output_var < 0 || p->output_var >= p->n_vars) return fail(PCVM_E_INVALID_ARG, "output_var out of range");
    if (p->n_blocks < 1 || p->n_blocks > (1 << 20)) return fail(PCVM_E_INVALID_ARG, "n_blocks out of range");
    if (p->n_ops < 0 || p->n_ops > (1 << 24)) return fail(PCVM_E_INVALID_ARG, "n_ops out of range");
    auto var_ok = [&](int v) { return v >= 0 && v < p->n_vars; };
    auto blk_ok = [&](int b) { return b >= 0 && b < p->n_blocks; };
    for (int b = 0; b < p->n_blocks; ++b) {
        const pcvm_block& k = p->blocks[b];
        if (k.first_op < 0 || k.n_ops < 0 || (long)k.first_op + k.n_ops > p->n_ops)
            return fail(PCVM_E_INVALID_ARG, "block %d: operations out of range", b);
        switch (k.term) {
        case PCVM_JUMP:
            if (!blk_ok(k.i)) return fail(PCVM_E_INVALID_ARG, "block %d: jump target out of range", b);
            break;
        case PCVM_BRANCH:
            if (!blk_ok(k.i) || !blk_ok(k.j) || !var_ok(k.x)) return fail(PCVM_E_INVALID_ARG, "block %d: bad branch", b);
            break;
        case PCVM_PUSHJUMP:
            if (!blk_ok(k.i) || !blk_ok(k.j)) return fail(PCVM_E_INVALID_ARG, "block %d: bad call", b);
            break;
        case PCVM_RETURN: break;
        default: return fail(PCVM_E_INVALID_ARG, "block %d: unknown terminator %d", b, k.term);
        }
    }
    for (int o = 0; o < p->n_ops; ++o) {
        const pcvm_op& op = p->ops[o];
        if (op.kind < PCVM_PUSH || op.kind > PCVM_POP) return fail(PCVM_E_INVALID_ARG, "operation %d: unknown kind %d", o, op.kind);
        if (!var_ok(op.dst)) return fail(PCVM_E_INVALID_ARG, "operation %d: destination out of range", o);
        if (op.kind == PCVM_POP) continue;
        if (op.fn < 0 || op.fn >= PCVM_FN_COUNT) return fail(PCVM_E_INVALID_ARG, "operation %d: unknown function %d", o, op.fn);
        if (!var_ok(op.a) || !var_ok(op.b)) return fail(PCVM_E_INVALID_ARG, "operation %d: operand out of range", o);
    }
    return PCVM_OK;
}

// One device allocation per call, carved into the program tables, the stacks, the counters and the error word.
struct DeviceBuffers {
    void* base = nullptr;
    void* ptr[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    hipEvent_t ev[2] = {nullptr, nullptr};
    ~DeviceBuffers()
    {
        (void)hipFree(base);
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
    }
};

}  // namespace

extern "C" {

const char* pcvm_last_error(void) { return g_err; }

int pcvm_set_stream(void* hip_stream)
{
    g_stream = static_cast<hipStream_t>(hip_stream);
    return PCVM_OK;
}

static int run_impl(const pcvm_program* program, int64_t batch, const int64_t* inputs, int32_t stack_depth,
                    int64_t max_steps, int64_t* outputs, int32_t* trace, int64_t trace_capacity, pcvm_stats* stats,
                    bool queued, int policy)
{
    if (policy != PCVM_SCHED_EARLIEST && policy != PCVM_SCHED_MOST_WAITING) return fail(PCVM_E_INVALID_ARG, "unknown policy %d", policy);
    int rc = check_program(program);
    if (rc) return rc;
    if (batch < 1 || batch > (1ll << 28)) return fail(PCVM_E_INVALID_ARG, "batch must be in [1, 2^28]");
    if (!inputs || !outputs) return fail(PCVM_E_INVALID_ARG, "inputs and outputs must not be NULL");
    if (stack_depth < 1 || stack_depth > PCVM_MAX_DEPTH) return fail(PCVM_E_INVALID_ARG, "stack_depth must be in [1, %d]", PCVM_MAX_DEPTH);
    if (max_steps < 1) return fail(PCVM_E_INVALID_ARG, "max_steps must be > 0");
    if (trace && trace_capacity < 1) return fail(PCVM_E_INVALID_ARG, "trace_capacity must be > 0 with a trace buffer");
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count < 1)
        return fail(PCVM_E_DEVICE, "no HIP device available (this library has no CPU path)");

    long n_groups = (long)((batch + kWave - 1) / kWave);
    if (queued) {  // no more groups than the chip holds at once: the others' members come through the queue
        int per_cu = 0, cus = 0, dev = 0;
        PCVM_TRY(hipGetDevice(&dev), PCVM_E_DEVICE);
        PCVM_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pcvm_kernel<true>, kWave * kWavesPerBlock, 0), PCVM_E_DEVICE);
        PCVM_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), PCVM_E_DEVICE);
        const long resident = (long)(per_cu < 1 ? 1 : per_cu) * cus * kWavesPerBlock;
        if (n_groups > resident) n_groups = resident;
    }
    const long batch_pad = n_groups * kWave;
    const size_t var_bytes = (size_t)program->n_vars * stack_depth * batch_pad * sizeof(long long);
    const size_t pc_bytes = (size_t)stack_depth * batch_pad * sizeof(int);
    if (var_bytes + pc_bytes > (size_t)64 << 30) return fail(PCVM_E_ALLOC, "stacks would need %zu bytes", var_bytes + pc_bytes);

    DeviceBuffers buf;
    {
        const size_t part[6] = {sizeof(pcvm_block) * program->n_blocks, sizeof(pcvm_op) * (program->n_ops > 0 ? program->n_ops : 1),
                                var_bytes, pc_bytes, 3 * sizeof(unsigned long long), sizeof(int)};
        size_t off[6], total = 0;
        for (int i = 0; i < 6; ++i) {
            off[i] = total;
            total += (part[i] + 255) & ~(size_t)255;
        }
        PCVM_TRY(hipMalloc(&buf.base, total), PCVM_E_ALLOC);
        for (int i = 0; i < 6; ++i) buf.ptr[i] = static_cast<char*>(buf.base) + off[i];
    }
    PCVM_TRY(hipEventCreate(&buf.ev[0]), PCVM_E_DEVICE);
    PCVM_TRY(hipEventCreate(&buf.ev[1]), PCVM_E_DEVICE);
    PCVM_TRY(hipMemcpyAsync(buf.ptr[0], program->blocks, sizeof(pcvm_block) * program->n_blocks, hipMemcpyHostToDevice, g_stream), PCVM_E_DEVICE);
    if (program->n_ops > 0)
        PCVM_TRY(hipMemcpyAsync(buf.ptr[1], program->ops, sizeof(pcvm_op) * program->n_ops, hipMemcpyHostToDevice, g_stream), PCVM_E_DEVICE);
    PCVM_TRY(hipMemsetAsync(buf.ptr[4], 0, 3 * sizeof(unsigned long long), g_stream), PCVM_E_DEVICE);
    PCVM_TRY(hipMemsetAsync(buf.ptr[5], 0, sizeof(int), g_stream), PCVM_E_DEVICE);

    VmArgs va{};
    va.blocks = static_cast<const pcvm_block*>(buf.ptr[0]);
    va.ops = static_cast<const pcvm_op*>(buf.ptr[1]);
    va.n_vars = program->n_vars;
    va.n_inputs = program->n_inputs;
    va.output_var = program->output_var;
    va.n_blocks = program->n_blocks;
    va.batch = (long)batch;
    va.batch_pad = batch_pad;
    va.depth = stack_depth;
    va.max_steps = (long)max_steps;
    va.inputs = reinterpret_cast<const long long*>(inputs);
    va.outputs = reinterpret_cast<long long*>(outputs);
    va.var_stacks = static_cast<long long*>(buf.ptr[2]);
    va.pc_stacks = static_cast<int*>(buf.ptr[3]);
    va.trace = trace;
    va.trace_capacity = (long)trace_capacity;
    va.counters = static_cast<unsigned long long*>(buf.ptr[4]);
    va.queue = va.counters + 2;
    va.policy = policy;
    va.error = static_cast<int*>(buf.ptr[5]);

    const unsigned blocks = (unsigned)((n_groups + kWavesPerBlock - 1) / kWavesPerBlock);
    PCVM_TRY(hipEventRecord(buf.ev[0], g_stream), PCVM_E_DEVICE);
    if (queued)
        hipLaunchKernelGGL(pcvm_kernel<true>, dim3(blocks), dim3(kWave * kWavesPerBlock), 0, g_stream, va);
    else
        hipLaunchKernelGGL(pcvm_kernel<false>, dim3(blocks), dim3(kWave * kWavesPerBlock), 0, g_stream, va);
    PCVM_TRY(hipGetLastError(), PCVM_E_DEVICE);
    PCVM_TRY(hipEventRecord(buf.ev[1], g_stream), PCVM_E_DEVICE);
    unsigned long long counters[2] = {0, 0};
    int error = 0;
    PCVM_TRY(hipMemcpyAsync(counters, buf.ptr[4], sizeof(counters), hipMemcpyDeviceToHost, g_stream), PCVM_E_DEVICE);
    PCVM_TRY(hipMemcpyAsync(&error, buf.ptr[5], sizeof(error), hipMemcpyDeviceToHost, g_stream), PCVM_E_DEVICE);
    PCVM_TRY(hipStreamSynchronize(g_stream), PCVM_E_DEVICE);
    if (stats) {
        float ms = 0.f;
        PCVM_TRY(hipEventElapsedTime(&ms, buf.ev[0], buf.ev[1]), PCVM_E_DEVICE);
        stats->steps = counters[0];
        stats->active_member_steps = counters[1];
        stats->issued_member_steps = counters[0] * kWave;
        stats->kernel_ms = ms;
        stats->n_groups = (int32_t)n_groups;
        stats->reserved = 0;
    }
    if (error == PCVM_E_STACK_OVERFLOW) return fail(error, "a stack grew beyond stack_depth = %d entries", stack_depth);
    if (error == PCVM_E_STACK_UNDERFLOW) return fail(error, "pop from an empty variable stack");
    if (error == PCVM_E_STEP_LIMIT) return fail(error, "a group made %lld steps without halting", (long long)max_steps);
    if (error) return fail(PCVM_E_DEVICE, "unknown device error %d", error);
    return PCVM_OK;
}

int pcvm_run(const pcvm_program* program, int64_t batch, const int64_t* inputs, int32_t stack_depth,
             int64_t max_steps, int64_t* outputs, int32_t* trace, int64_t trace_capacity, pcvm_stats* stats)
{
    return run_impl(program, batch, inputs, stack_depth, max_steps, outputs, trace, trace_capacity, stats, false,
                    PCVM_SCHED_EARLIEST);
}

int pcvm_run_queued(const pcvm_program* program, int64_t batch, const int64_t* inputs, int32_t stack_depth,
                    int64_t max_steps, int32_t policy, int64_t* outputs, pcvm_stats* stats)
{
    return run_impl(program, batch, inputs, stack_depth, max_steps, outputs, nullptr, 0, stats, true, policy);
}

}  // extern "C"
