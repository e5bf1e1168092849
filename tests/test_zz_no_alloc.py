"""convert_replay_static (the replay entry point that allocates nothing: its scratch is a static device
array inside the library) against convert_replay, through the C ABI.

Two calls in a row share the static scratch array, the second on a smaller plan, so the array still holds
the first call's tile list when the second starts.  Results must equal convert_replay's bit for bit (same
kernels, same arithmetic) and the oracle's within 1e-6 relative (the FP32 Adam bar)."""
import numpy as np
import pytest
import torch

from paper_2412_15411_amd import binding as B
from paper_2412_15411_amd import workloads as W
from helpers import hp_of, model_of, np_of, state_of, max_rel_err

pytestmark = pytest.mark.gpu
KINDS = ("master", "m", "v", "compute")


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    return torch.device("cuda:0")


def _workload(seed, n_ops, max_numel):
    rng = np.random.default_rng(seed)
    tensors = []
    for e in range(n_ops):
        for _ in range(int(rng.integers(1, 4))):
            tensors.append((e, int(rng.integers(1, max_numel)) if rng.random() > 0.25 else int(rng.integers(0, 9))))
    return W.Workload(f"static{seed}", tensors, [e % 3 for e in range(n_ops)], 3)


def _device_table(tensors, dev):
    """Device array of device pointers (0 for None)."""
    return torch.tensor([0 if t is None else t.data_ptr() for t in tensors], dtype=torch.int64, device=dev)


def _bits(t):
    return t.view(torch.int16) if t.element_size() == 2 else t.view(torch.int32)


def _one_case(orc, dev, wl, seed, active_slots, steps):
    """Runs `steps` replay iterations on two copies of the same state: convert_replay on one, convert_replay_static
    on the other; frozen operators have no gradients (null entries)."""
    st_cpu = W.make_state(wl, seed=seed)
    ref_state = {k: [t.to(dev) for t in st_cpu[k]] for k in KINDS}
    new_state = {k: [t.to(dev) for t in st_cpu[k]] for k in KINDS}
    oracle_state = state_of(st_cpu)
    active = [1 if s in active_slots else 0 for s in wl.slot_of_op]
    mask = torch.tensor(active, dtype=torch.uint8, device=dev)
    plan_ref = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
    plan_new = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
    with pytest.raises(B.MoevError) as e:   # nothing resident yet: the call must not build tables by itself
        B.convert_replay_static(plan_new, wl.lr, wl.beta1, wl.beta2, wl.eps, 0.0, 11, mask, mask, mask)
    assert e.value.code == B.E_INVAL
    B.ckpt_plan_upload(plan_new)
    state_table = _device_table([t for k in KINDS for t in new_state[k]], dev)
    model, hp = model_of(wl), hp_of(wl)
    for step in steps:
        grads_cpu = W.make_grads(wl, step, seed=seed)
        grads = [g.to(dev) if active[wl.tensors[t][0]] else None for t, g in enumerate(grads_cpu)]
        grad_table = _device_table(grads, dev)
        B.convert_replay(plan_ref, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, step, mask, grads,
                         B.State(*[ref_state[k] for k in KINDS]))
        B.convert_replay_static(plan_new, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, step, mask, grad_table,
                                state_table)
        torch.cuda.synchronize()
        orc.replay_step(model, hp, step, np.array(active, dtype=np.uint8), [np_of(g) for g in grads_cpu], oracle_state)
    B.ckpt_plan_device_status(plan_ref)
    B.ckpt_plan_device_status(plan_new)
    changed = 0
    for k in KINDS:
        for t, (a, b) in enumerate(zip(ref_state[k], new_state[k])):
            assert torch.equal(_bits(a), _bits(b)), f"{wl.name}: {k}[{t}] differs from convert_replay"
            if not active[wl.tensors[t][0]]:
                assert torch.equal(_bits(b), _bits(st_cpu[k][t].to(dev))), f"{wl.name}: frozen {k}[{t}] was modified"
            elif b.numel():
                changed += int(not torch.equal(_bits(b), _bits(st_cpu[k][t].to(dev))))
    assert changed > 0
    worst = 0.0
    for name, ref in (("master", oracle_state.master), ("m", oracle_state.m), ("v", oracle_state.v)):
        for t, x in enumerate(new_state[name]):
            worst = max(worst, max_rel_err(np_of(x), ref[t]))
    assert worst <= 1e-6, f"{wl.name}: relative error {worst} against the oracle"
    return worst


def test_static_replay_equals_convert_replay_on_two_calls_in_a_row(orc, dev):
    big = _workload(5, n_ops=40, max_numel=90000)       # ~80 tensors, ragged lengths, empty tensors
    small = _workload(6, n_ops=4, max_numel=3000)       # fewer, shorter tensors: the scratch still holds the big tile list
    assert small.n_tensors < big.n_tensors
    w1 = _one_case(orc, dev, big, seed=21, active_slots=(0, 1), steps=(11, 12))
    w2 = _one_case(orc, dev, small, seed=22, active_slots=(0, 2), steps=(11,))
    w3 = _one_case(orc, dev, big, seed=23, active_slots=(2,), steps=(13,))
    print(f"static replay: worst relative error against the oracle {max(w1, w2, w3):.3g}")


@pytest.mark.parametrize("regime", ["fp8_fp32_fp32+fp32", "fp8_fp16_fp32+fp32", "fp8_fp8_fp8+fp16"])
def test_static_replay_on_low_precision_state(dev, regime):
    """State stored in the formats of a low-precision regime (master weights of 4, 2 and 1 bytes; the first two run the
    paired 64 x 1 shape, whose grid the static call sizes without knowing the pointers): same codes as convert_replay,
    whose parity with the oracle the low-precision tests establish."""
    from test_gpu_low_precision import LIB_FMT_OF_DTYPE
    dtypes = W.LOW_PRECISION_REGIMES[regime]
    wl = _workload(9, n_ops=12, max_numel=60000)
    per_kind = W.default_scales(dtypes)
    st_cpu = W.make_low_precision_state(wl, dtypes, per_kind, seed=4)
    ref_state = {k: [t.to(dev) for t in st_cpu[k]] for k in KINDS}
    new_state = {k: [t.to(dev) for t in st_cpu[k]] for k in KINDS}
    d_scales = torch.tensor([[x] * wl.n_tensors for x in per_kind], dtype=torch.float32, device=dev)
    active = [1 if s != 1 else 0 for s in wl.slot_of_op]
    mask = torch.tensor(active, dtype=torch.uint8, device=dev)
    formats = [LIB_FMT_OF_DTYPE[d] for d in dtypes]
    plan_ref = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, formats=formats)
    plan_new = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, formats=formats)
    B.ckpt_plan_upload(plan_new)
    state_table = _device_table([t for k in KINDS for t in new_state[k]], dev)
    for step in (7, 8):
        grads_cpu = W.make_grads(wl, step, seed=4)
        grads = [g.to(dev) if active[wl.tensors[t][0]] else None for t, g in enumerate(grads_cpu)]
        B.convert_replay(plan_ref, 1e-3, 0.9, 0.95, 1e-8, 0.01, step, mask, grads, B.State(*[ref_state[k] for k in KINDS]),
                         d_scales=d_scales)
        B.convert_replay_static(plan_new, 1e-3, 0.9, 0.95, 1e-8, 0.01, step, mask, _device_table(grads, dev), state_table,
                                d_scales=d_scales)
        torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan_ref)
    B.ckpt_plan_device_status(plan_new)
    changed = 0
    for k in KINDS:
        for t, (a, b) in enumerate(zip(ref_state[k], new_state[k])):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"{regime}: {k}[{t}] differs from convert_replay"
            changed += int(b.numel() > 0 and not torch.equal(b.view(torch.uint8), st_cpu[k][t].to(dev).view(torch.uint8)))
    assert changed > 0


def test_static_replay_refuses_plans_beyond_its_scratch(dev):
    n = 65536 + 1
    plan = B.ckpt_plan([(e, 4) for e in range(n)], B.EXPLICIT, window=1, slot_of_op=[0] * n)
    x = torch.zeros(8, dtype=torch.int64, device=dev)
    with pytest.raises(B.MoevError) as e:
        B.convert_replay_static(plan, 1e-4, 0.9, 0.95, 1e-8, 0.0, 1, x, x, x)
    assert e.value.code == B.E_RANGE
