"""Parity of the HIP program-counter virtual machine with its oracle, through the C ABI, on a real MI355X.
Everything is 64-bit integer work: outputs, step counts, active-member counts and the schedule trace are
compared bit for bit."""
import numpy as np
import pytest

from oracle import pcvm_ref as V
from paper_1910_11141_amd import pcvm_programs as PP

pytestmark = pytest.mark.gpu


def gpu(program, inputs, depth, **kw):  # kw: max_steps, trace_capacity, queued
    import torch
    from paper_1910_11141_amd import pcvm
    ins = torch.as_tensor(np.ascontiguousarray(np.asarray(inputs, dtype=np.int64).reshape(program.n_inputs, -1))).cuda()
    out, stats, trace = pcvm.pcvm_run(program, ins, depth, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy(), stats, None if trace is None else trace.cpu().numpy()


def inputs_for(name, batch, seed):
    rng = np.random.default_rng(seed)
    if name == "fibonacci":
        return rng.integers(0, 15, size=(1, batch))
    if name == "collatz_steps":
        return rng.integers(1, 5000, size=(1, batch))
    if name == "gcd":
        return rng.integers(0, 10**9, size=(2, batch))
    if name == "parity":
        return rng.integers(0, 60, size=(1, batch))
    if name == "binomial":
        n = rng.integers(0, 11, size=batch)
        return np.stack([n, (rng.random(batch) * (n + 1)).astype(np.int64)])
    m = rng.integers(0, 3, size=batch)
    return np.stack([m, rng.integers(0, 5, size=batch)])


def test_fibonacci_worked_example_outputs_and_schedule():
    """The batch of Figure 3: same outputs and the same sequence of (block, active members) as Algorithm 2."""
    P = PP.fibonacci()
    want, st, trace = V.run(P, [6, 7, 8, 9], 12)
    out, stats, tr = gpu(P, [6, 7, 8, 9], 12, trace_capacity=1000)
    assert list(out) == [13, 21, 34, 55] == list(want)
    assert stats["steps"] == st["steps"] == 458 and stats["active_member_steps"] == st["active_member_steps"]
    assert [tuple(r) for r in tr[: st["steps"]]] == trace
    assert (tr[st["steps"]:] == -1).all()


@pytest.mark.parametrize("batch", [1, 63, 64, 65, 257, 1000])
@pytest.mark.parametrize("name", sorted(PP.ALL))
def test_programs_match_the_oracle_on_ragged_batches(name, batch):
    P = PP.ALL[name]()
    ins = inputs_for(name, batch, seed=batch)
    want, st, trace = V.run(P, ins, 80, group=64)
    out, stats, tr = gpu(P, ins, 80, trace_capacity=len(trace))
    assert np.array_equal(out, want)
    assert stats["steps"] == st["steps"] and stats["active_member_steps"] == st["active_member_steps"]
    assert stats["issued_member_steps"] == st["issued_member_steps"] and stats["n_groups"] == (batch + 63) // 64
    assert [tuple(r) for r in tr] == trace            # group 0 took the same blocks in the same order


def test_large_batch_against_the_closed_form_and_sampled_members():
    P = PP.fibonacci()
    rng = np.random.default_rng(5)
    ns = rng.integers(0, 21, size=200_000)
    out, stats, _ = gpu(P, ns, 32)
    fib = np.ones(22, dtype=np.int64)
    for i in range(2, 22):
        fib[i] = fib[i - 1] + fib[i - 2]
    assert np.array_equal(out, fib[ns])
    pick = rng.choice(ns.size, 64, replace=False)
    assert np.array_equal(out[pick], V.run(P, ns[pick], 32)[0])
    assert 0.0 < stats["utilization"] <= 1.0
    again, stats2, _ = gpu(P, ns, 32)
    assert np.array_equal(again, out) and stats2["steps"] == stats["steps"]


def test_equal_inputs_keep_every_lane_busy():
    out, stats, _ = gpu(PP.fibonacci(), [11] * 128, 16)
    assert (out == 144).all() and stats["utilization"] == 1.0


def test_limits_are_reported_not_trapped():
    from paper_1910_11141_amd import pcvm
    P = PP.fibonacci()
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(P, [3, 12, 2, 1], 6)
    assert e.value.code == pcvm.PCVM_E_STACK_OVERFLOW
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(PP.parity(), [100] * 70, 50)
    assert e.value.code == pcvm.PCVM_E_STACK_OVERFLOW
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(P, [15], 20, max_steps=100)
    assert e.value.code == pcvm.PCVM_E_STEP_LIMIT
    bad = PP.fibonacci()
    bad.ops["kind"][1] = PP.POP             # pops `ret`, which is never pushed
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(bad, [0, 5], 8)
    assert e.value.code == pcvm.PCVM_E_STACK_UNDERFLOW
    out, _, _ = gpu(P, [3, 4], 6)           # the library is still usable afterwards
    assert list(out) == [3, 5]


def test_maximum_stack_depth_and_variable_count():
    from paper_1910_11141_amd import pcvm
    P = PP.parity()
    ns = np.array([4094, 4095, 17, 0] * 20)       # 4095 nested calls need 4096 program-counter entries
    out, stats, _ = gpu(P, ns, pcvm.PCVM_MAX_DEPTH)
    assert list(out) == [1 - int(n) % 2 for n in ns]
    want, st, _ = V.run(P, ns[:8], pcvm.PCVM_MAX_DEPTH)
    assert np.array_equal(out[:8], want)
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(P, [4096], pcvm.PCVM_MAX_DEPTH)
    assert e.value.code == pcvm.PCVM_E_STACK_OVERFLOW
    # a program that uses all 16 variables: a chain of copies and additions through every one of them
    b = PP._Builder("wide", [f"v{i}" for i in range(16)], 1, "v15")
    ops = [PP.update(f"v{i}", PP.ADDI, f"v{i - 1}", imm=i) for i in range(1, 16)]
    b.block("only", 1, ops, (PP.RETURN,))
    wide = b.build()
    xs = np.arange(100)
    out, _, _ = gpu(wide, xs, 4)
    assert np.array_equal(out, xs + sum(range(1, 16)))
    assert np.array_equal(V.run(wide, xs, 4)[0], out)


# ------------------------------------------------------------------ members handed out from a queue

@pytest.mark.parametrize("batch", [1, 65, 1000, 70_000])
@pytest.mark.parametrize("name", sorted(PP.ALL))
def test_queued_runs_give_the_same_outputs(name, batch):
    P = PP.ALL[name]()
    ins = inputs_for(name, batch, seed=batch + 1)
    static, st_static, _ = gpu(P, ins, 80)
    queued, st_queued, _ = gpu(P, ins, 80, queued=True, policy=batch % 2)
    assert np.array_equal(queued, static)
    assert st_queued["active_member_steps"] == st_static["active_member_steps"]    # the same blocks per member
    if batch <= 1000:
        assert np.array_equal(static, V.run(P, ins, 80)[0])


def test_queue_keeps_lanes_busy_on_unequal_work():
    P = PP.fibonacci()
    ns = np.random.default_rng(9).integers(1, 21, size=1 << 20)
    static, st_static, _ = gpu(P, ns, 32)
    queued, st_queued, _ = gpu(P, ns, 32, queued=True)
    fuller, st_fuller, _ = gpu(P, ns, 32, queued=True, policy=1)
    assert np.array_equal(static, queued) and np.array_equal(static, fuller)
    assert st_static["utilization"] < st_queued["utilization"] < st_fuller["utilization"]
    assert st_fuller["active_member_steps"] == st_static["active_member_steps"]
    assert st_queued["n_groups"] < st_static["n_groups"]
    print("utilization static / queued / queued most-waiting:", st_static["utilization"], st_queued["utilization"],
          st_fuller["utilization"], "ms", st_static["kernel_ms"], st_queued["kernel_ms"], st_fuller["kernel_ms"])


def test_queued_limits_are_reported_and_other_members_finish():
    from paper_1910_11141_amd import pcvm
    P = PP.fibonacci()
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(P, [3, 12, 2, 1] * 50, 6, queued=True)
    assert e.value.code == pcvm.PCVM_E_STACK_OVERFLOW
    with pytest.raises(pcvm.PcvmError) as e:
        gpu(P, [15] * 300, 20, max_steps=100, queued=True)
    assert e.value.code == pcvm.PCVM_E_STEP_LIMIT
    out, _, _ = gpu(P, [3, 4] * 100, 6, queued=True)
    assert list(out) == [3, 5] * 100
