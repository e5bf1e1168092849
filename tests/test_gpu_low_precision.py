"""GPU parity of the replay on low-precision state (Sec. 5.6 regimes) against the CPU oracle.

Stored state is integer codes, so the comparison is bit for bit: both sides widen the same codes to
FP32, take the same FP32 step (operation order pinned on both sides) and narrow with round to nearest
even.  NaN results are compared as "NaN on both sides" (the sign of a generated NaN is the machine's).
"""
import numpy as np
import pytest
import torch

from paper_2412_15411_amd import binding as B
from paper_2412_15411_amd import workloads as W
from helpers import ORACLE_FMT_OF_DTYPE, hp_of, model_of, np_of
from test_gpu_parity import DeviceState, KINDS, packed_buffer, ragged_workload

pytestmark = pytest.mark.gpu

LIB_FMT_OF_DTYPE = {torch.float32: B.FMT_F32, torch.float16: B.FMT_F16, torch.bfloat16: B.FMT_BF16,
                    torch.float8_e4m3fn: B.FMT_E4M3, torch.float8_e5m2: B.FMT_E5M2}
REGIMES = dict(W.LOW_PRECISION_REGIMES)
# the same width combinations with the other format of each width, and FP16 compute weights on FP32 state
# (the precision the paper's own runs use for compute weights)
VARIANTS = dict(REGIMES)
VARIANTS["bf16_everywhere"] = (torch.bfloat16,) * 4
VARIANTS["fp16_state_bf16_compute"] = (torch.float16, torch.float16, torch.float16, torch.bfloat16)
VARIANTS["fp32_state_fp16_compute"] = (torch.float32, torch.float32, torch.float32, torch.float16)
VARIANTS["e5m2_m_and_compute"] = (torch.float16, torch.float8_e5m2, torch.float16, torch.float8_e5m2)
VARIANTS["e5m2_master"] = (torch.float8_e5m2, torch.float8_e4m3fn, torch.bfloat16, torch.float8_e5m2)


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    return torch.device("cuda:0")


def lp_plan(wl, dtypes, align=0, adam_shape=None):
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, align=align,
                       formats=[LIB_FMT_OF_DTYPE[d] for d in dtypes])
    if adam_shape:
        B.moev_tune(plan, B.TUNE_ADAM_UNROLL, 1)
        B.moev_tune(plan, B.TUNE_ADAM_THREADS, adam_shape[0])
        B.moev_tune(plan, B.TUNE_ADAM_UNROLL, adam_shape[1])
    return plan


def scale_table(wl, dtypes, seed, odd=False):
    """[4, n_tensors] per-tensor scales: the kind's default times a per-tensor power of two (odd: times 1.37)."""
    rng = np.random.default_rng(seed)
    base = np.array(W.default_scales(dtypes), dtype=np.float32)[:, None]
    table = base * np.exp2(rng.integers(-1, 2, size=(4, wl.n_tensors))).astype(np.float32)
    if odd:
        table = (table * np.float32(1.37)).astype(np.float32)
    return np.ascontiguousarray(table, dtype=np.float32)


def codes_equal_up_to_nan(got: np.ndarray, ref: np.ndarray, fmt, orc):
    """Bitwise equal, except that both may hold (possibly differently signed) NaN codes at a position."""
    if got.tobytes() == ref.tobytes():
        return True
    if got.dtype == np.float32:
        g, r = got.reshape(-1).view(np.uint32), ref.reshape(-1).view(np.uint32)
    else:
        g, r = got.reshape(-1), ref.reshape(-1)
    for i in np.flatnonzero(g != r):
        if not (np.isnan(orc.decode(fmt, int(g[i]))) and np.isnan(orc.decode(fmt, int(r[i])))):
            return False
    return True


def run_both(orc, dev, wl, dtypes, st_cpu, table, grads_cpu, mask_np, hp, step, plan):
    """One replay step on the GPU and in the oracle; returns (device state, oracle state)."""
    fmts = tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes)
    model = model_of(wl, formats=fmts)
    ref = orc.State(*[[np_of(t) for t in st_cpu[k]] for k in KINDS])
    orc.replay_step(model, hp, step, mask_np, [g.numpy() for g in grads_cpu], ref, table)
    ds = DeviceState(st_cpu, dev)
    d_scales = torch.from_numpy(table).to(dev) if table is not None else None
    mask = torch.from_numpy(mask_np).to(dev)
    grads = [g.to(dev) if mask_np[wl.tensors[t][0]] else None for t, g in enumerate(grads_cpu)]
    B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, step, mask, grads, ds.state,
                     d_scales=d_scales)
    torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)  # raises if the kernels flagged anything
    return ds, ref, fmts


def assert_states_match(orc, ds, ref, fmts):
    got = ds.to_oracle()
    for k, kind in enumerate(KINDS):
        for t, (x, y) in enumerate(zip(got.kinds()[kind], ref.kinds()[kind])):
            assert codes_equal_up_to_nan(x, y, fmts[k], orc), (kind, t)
    assert ds.guards_intact()


@pytest.mark.parametrize("name", list(VARIANTS))
def test_low_precision_replay_matches_oracle(orc, dev, name):
    """Ragged tensors (tails of 1-3 elements, an empty tensor, several tiles), per-tensor scales, a mask
    with frozen operators (whose gradients are NULL): every stored code equals the oracle's."""
    dtypes = VARIANTS[name]
    wl = ragged_workload(31 + len(name), max_numel=50000)
    table = scale_table(wl, dtypes, seed=1)
    st_cpu = W.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=8)
    grads = W.make_grads(wl, 12, seed=8)
    rng = np.random.default_rng(4)
    mask_np = (rng.random(wl.n_ops) < 0.7).astype(np.uint8)
    mask_np[0] = 1
    mask_np[1] = 0
    hp = orc.AdamHP(lr=1e-3, weight_decay=0.01)
    plan = lp_plan(wl, dtypes)
    for k in range(4):
        assert B.ckpt_plan_format(plan, k) == LIB_FMT_OF_DTYPE[dtypes[k]]
        assert B.ckpt_plan_width(plan, k) == torch.empty(0, dtype=dtypes[k]).element_size()
    ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, table, grads, mask_np, hp, 12, plan)
    assert_states_match(orc, ds, ref, fmts)
    # frozen operators were not touched at all
    start = DeviceState(st_cpu, dev).to_oracle()
    after = ds.to_oracle()
    for t, (op, _) in enumerate(wl.tensors):
        if not mask_np[op]:
            for kind in KINDS:
                assert after.kinds()[kind][t].tobytes() == start.kinds()[kind][t].tobytes()


@pytest.mark.parametrize("distance", [0, 512, 16384, 65536, 1 << 20], ids=["consecutive", "512B", "16KiB", "64KiB", "1MiB"])
@pytest.mark.parametrize("name", ["fp16_fp16_fp16+fp16", "fp8_fp16_fp32+fp32", "fp8_fp8_fp8+fp16"])
def test_low_precision_replay_paired_tile_distances(orc, dev, name, distance):
    """The paired tiles of the 64 x 1 shape (default distance: test_low_precision_replay_matches_oracle) at other piece
    distances and switched off, with master weights of 2, 2 and 1 bytes: the tile grid follows the master pointers, which
    sit at arbitrary 16-byte offsets in the arena."""
    dtypes = REGIMES[name]
    wl = ragged_workload(55, max_numel=70000)
    table = scale_table(wl, dtypes, seed=3)
    st_cpu = W.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=5)
    grads = W.make_grads(wl, 9, seed=5)
    mask_np = np.ones(wl.n_ops, dtype=np.uint8)
    mask_np[2] = 0
    hp = orc.AdamHP(lr=1e-3, weight_decay=0.01)
    plan = lp_plan(wl, dtypes)
    assert B.moev_tune_get(plan, B.TUNE_PAIRED_TILES) == 32768
    B.moev_tune(plan, B.TUNE_PAIRED_TILES, distance)
    ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, table, grads, mask_np, hp, 9, plan)
    assert_states_match(orc, ds, ref, fmts)
    assert ds.guards_intact()


@pytest.mark.parametrize("shape", [(64, 2), (128, 1), (128, 2), (256, 1), (256, 2)])
def test_low_precision_replay_launch_shapes(orc, dev, shape):
    dtypes = REGIMES["fp8_fp8_fp8+fp16"]
    wl = ragged_workload(77, max_numel=30000)
    table = scale_table(wl, dtypes, seed=2, odd=True)   # scales that are not powers of two
    st_cpu = W.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=1)
    grads = W.make_grads(wl, 30, seed=1)
    mask_np = np.ones(wl.n_ops, dtype=np.uint8)
    hp = orc.AdamHP(lr=3e-3)
    ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, table, grads, mask_np, hp, 30, lp_plan(wl, dtypes, adam_shape=shape))
    assert_states_match(orc, ds, ref, fmts)


def test_low_precision_replay_without_scales_and_fixed_grid_knob(orc, dev):
    """d_scales = NULL means all ones; the fixed-grid knob does not apply to these regimes (same result)."""
    dtypes = REGIMES["fp16_fp16_fp16+fp16"]
    wl = ragged_workload(5, max_numel=20000)
    st_cpu = W.make_low_precision_state(wl, dtypes, [1.0, 1.0, 1.0, 1.0], seed=2)
    grads = W.make_grads(wl, 11, seed=2)
    mask_np = np.ones(wl.n_ops, dtype=np.uint8)
    hp = orc.AdamHP(lr=1e-2)
    for persistent in (0, 1):
        plan = lp_plan(wl, dtypes)
        B.moev_tune(plan, B.TUNE_PERSISTENT, persistent)
        ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, None, grads, mask_np, hp, 11, plan)
        assert_states_match(orc, ds, ref, fmts)


def _probe_values(orc, fmt, bits, rng):
    """FP32 inputs that exercise a narrowing conversion: every representable value, every midpoint between
    neighbours and its two FP32 neighbours, the overflow boundary, FP32 subnormals, random patterns."""
    n_codes = 1 << (bits - 1)
    vals = np.array([orc.decode(fmt, c) for c in range(n_codes)])
    vals = vals[np.isfinite(vals)]
    if len(vals) > 5000:
        keep = np.unique(np.concatenate([np.arange(1500), np.arange(len(vals) - 1500, len(vals)), rng.integers(0, len(vals), 3000)]))
        mids = ((vals[keep[:-1]] + vals[keep[:-1] + 1]) / 2).astype(np.float32)
        vals = vals[keep]
    else:
        mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    top = np.float32(vals[-1])
    step = np.float32(vals[-1] - vals[-2])
    with np.errstate(over="ignore"):
        extra = np.array([top + step / 2, np.nextafter(top + step / 2, np.float32(0)), top + step, 3e38, 1e-45, 1e-40, 0.0],
                         dtype=np.float32)
    x = np.concatenate([vals.astype(np.float32), mids, np.nextafter(mids, np.float32(0)),
                        np.nextafter(mids, np.float32(np.inf)), extra,
                        rng.integers(0, 0x7F800000, 20000).astype(np.uint32).view(np.float32)])
    x = x[np.isfinite(x)]
    return np.concatenate([x, -x]).astype(np.float32)


@pytest.mark.parametrize("name,fmt_bits", [("fp16_fp16_fp16+fp16", 16), ("bf16_everywhere", 16),
                                           ("fp8_fp16_fp8+fp16", 8), ("e5m2_m_and_compute", 8)])
def test_narrowing_conversions_on_crafted_values(orc, dev, name, fmt_bits):
    """With beta1 = beta2 = 0 and lr = 0 the step stores m = narrow(g), v = narrow(g*g), and leaves the master
    weights alone (compute = narrow(widen(master))): the gradient carries crafted FP32 values (ties, values one
    FP32 step off a tie, overflow boundary, subnormals) straight into the kernel's conversions."""
    dtypes = VARIANTS[name]
    fmts = tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes)
    rng = np.random.default_rng(6)
    g = _probe_values(orc, fmts[1], fmt_bits, rng)
    g2 = _probe_values(orc, fmts[2], 16, rng)
    with np.errstate(over="ignore", invalid="ignore"):
        roots = np.sqrt(np.abs(g2)).astype(np.float32)   # squares land near (not on) the probes: fine, more values
    g = np.concatenate([g, roots, g2[:20000]])
    n = g.size
    wl = W.Workload("probe", [(0, n), (1, 7)], [0, 0], 1)
    st_cpu = W.make_low_precision_state(wl, dtypes, [1.0, 1.0, 1.0, 1.0], seed=3)
    # master: every code of its format, so that widen() and the compute cast see all of them
    wbytes = st_cpu["master"][0].element_size()
    if wbytes == 1:
        st_cpu["master"][0] = torch.from_numpy((np.arange(n) % 256).astype(np.uint8)).view(dtypes[0])
    elif wbytes == 2:
        st_cpu["master"][0] = torch.from_numpy((np.arange(n) % 65536).astype(np.uint16).view(np.int16)).view(dtypes[0])
    grads = [torch.from_numpy(g.copy()), torch.zeros(7)]
    hp = orc.AdamHP(lr=0.0, beta1=0.0, beta2=0.0, eps=1e-8)
    mask_np = np.ones(2, dtype=np.uint8)
    ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, None, grads, mask_np, hp, 3, lp_plan(wl, dtypes))
    assert_states_match(orc, ds, ref, fmts)


@pytest.mark.parametrize("name", ["fp8_fp16_fp8+fp16", "e5m2_m_and_compute", "fp16_fp16_fp16+fp16", "bf16_everywhere"])
def test_non_finite_gradients_through_the_narrowing_conversions(orc, dev, name):
    """NaN stays NaN in every format; infinities saturate in the 8-bit formats and stay infinite in the 16-bit
    ones (beta1 = 0: m = narrow(g))."""
    dtypes = VARIANTS[name]
    inf = float("inf")
    g = np.array([np.nan, -np.nan, inf, -inf, 3e38, -3e38, 500.0, -500.0, 6e4, -6e4, 7e4, 0.0, -0.0, 1.0] * 3, dtype=np.float32)
    wl = W.Workload("probe", [(0, g.size)], [0], 1)
    st_cpu = W.make_low_precision_state(wl, dtypes, [1.0, 1.0, 1.0, 1.0], seed=3)
    hp = orc.AdamHP(lr=0.0, beta1=0.0, beta2=0.0)
    ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, None, [torch.from_numpy(g.copy())], np.ones(1, np.uint8), hp, 3,
                             lp_plan(wl, dtypes))
    assert_states_match(orc, ds, ref, fmts)
    m = ds.to_oracle().m[0]
    vals = [orc.decode(fmts[1], int(c)) for c in m[:14]]
    assert np.isnan(vals[0]) and np.isnan(vals[1])
    top = {orc.FMT_E4M3: 448.0, orc.FMT_E5M2: 57344.0}.get(fmts[1], inf)
    assert vals[2] == top and vals[3] == -top
    if fmts[1] != orc.FMT_BF16:   # 3e38 is beyond every format's range except bfloat16's
        assert vals[4] == top and vals[5] == -top


def test_fp8_compute_cast_of_fp32_master_on_crafted_values(orc, dev):
    """FP32 master weights and 8-bit compute weights (lr = 0: master unchanged, compute = narrow(master * s))."""
    dtypes = REGIMES["fp8_fp32_fp32+fp32"]
    rng = np.random.default_rng(16)
    p = _probe_values(orc, orc.FMT_E4M3, 8, rng)
    wl = W.Workload("probe", [(0, p.size)], [0], 1)
    st_cpu = W.make_low_precision_state(wl, dtypes, [1.0, 1.0, 1.0, 1.0], seed=3)
    st_cpu["master"][0] = torch.from_numpy(p.copy())
    for s_c in (1.0, 0.5, 3.0):
        table = np.ones((4, 1), dtype=np.float32)
        table[3, 0] = s_c
        grads = [torch.zeros(p.size)]
        hp = orc.AdamHP(lr=0.0)
        ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, table, grads, np.ones(1, np.uint8), hp, 2, lp_plan(wl, dtypes))
        assert_states_match(orc, ds, ref, fmts)


@pytest.mark.parametrize("name", list(REGIMES))
def test_low_precision_conversion_equals_dense_run(orc, dev, name):
    """Sec. 3.3 on the GPU in every Sec. 5.6 regime: snapshots taken along a dense run, then load + replay per
    slot from a poisoned state; the result equals the dense run's final state, and both equal the oracle's."""
    dtypes = REGIMES[name]
    fmts = tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes)
    wl = ragged_workload(3, n_ops=9, window=3, max_numel=40000, with_empty=False)
    table = scale_table(wl, dtypes, seed=9)
    st_cpu = W.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=6)
    hp = hp_of(wl)
    plan = lp_plan(wl, dtypes)
    d_scales = torch.from_numpy(table).to(dev)
    ds = DeviceState(st_cpu, dev)
    everyone = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    snaps = []
    for k in range(wl.window):
        buf = packed_buffer(plan, dev, k)
        B.snapshot_pack(plan, k, wl.t0 + k, ds.state, buf)
        snaps.append(buf)
        grads = [g.to(dev) for g in W.make_grads(wl, wl.t0 + k + 1, seed=6)]
        B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, wl.t0 + k + 1, everyone, grads,
                         ds.state, d_scales=d_scales)
    torch.cuda.synchronize()
    rebuilt = DeviceState(st_cpu, dev)
    for kind in KINDS:
        for v in rebuilt.views[kind]:
            v.view(torch.uint8).fill_(0xFF)
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    for i in range(wl.window):
        grads = W.make_grads(wl, wl.t0 + i + 1, seed=6)
        dg = [g.to(dev) if wl.slot_of_op[wl.tensors[t][0]] <= i else None for t, g in enumerate(grads)]
        if i % 2 == 0:
            B.restore_unpack(plan, i, None, snaps[i], rebuilt.state, mask)
            B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, wl.t0 + i + 1, mask, dg,
                             rebuilt.state, d_scales=d_scales)
        else:  # the combined call runs the same two kernels in these regimes
            B.convert_window_step(plan, i, None, snaps[i], hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay,
                                  wl.t0 + i + 1, mask, dg, rebuilt.state, d_scales=d_scales)
    torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)
    assert bool(mask.cpu().all())
    a, b = rebuilt.to_oracle(), ds.to_oracle()
    for kind in KINDS:
        for x, y in zip(a.kinds()[kind], b.kinds()[kind]):
            assert x.tobytes() == y.tobytes()
    # the oracle's dense run from the same start
    model = model_of(wl, formats=fmts)
    ref = orc.State(*[[np_of(t) for t in st_cpu[k]] for k in KINDS])
    ones = np.ones(wl.n_ops, dtype=np.uint8)
    for k in range(wl.window):
        orc.replay_step(model, hp, wl.t0 + k + 1, ones, [g.numpy() for g in W.make_grads(wl, wl.t0 + k + 1, seed=6)], ref, table)
    assert_states_match(orc, ds, ref, fmts)
    assert rebuilt.guards_intact()


def test_plain_division_and_square_root_equal_the_full_sequences(dev):
    """The replay takes its divisions and its square root without the rescaling / special-case steps of the
    IEEE expansions where the operands are in a middle exponent range.  On the GPU, against the compiler's
    full expansions: the square root for EVERY FP32 value of [2^-60, 2^60); the division by a bias
    correction for EVERY numerator of that range (both signs) and 40 divisors; 2^32 random pairs for the
    division by the per-element denominator."""
    lo, n = (127 - 60) << 23, 120 << 23
    assert B.moev_arith_selfcheck(1, 1.0, lo, n) == 0
    divisors = [float(np.float32(1.0 - beta ** step)) for beta in (0.9, 0.95, 0.99, 0.999, 0.9999)
                for step in (1, 2, 3, 11, 100, 1000, 100000)]
    divisors += [1.0, 2.0 ** -20, float(np.nextafter(np.float32(2.0 ** -20), np.float32(1))), float(np.nextafter(np.float32(1), np.float32(0))),
                 float(np.float32(1.0 / 3.0))]
    for d in divisors:
        assert 2.0 ** -20 <= d <= 1.0
        assert B.moev_arith_selfcheck(0, d, lo, n) == 0, d
    assert B.moev_arith_selfcheck(2, 1.0, 0, 1 << 32, seed=7) == 0
    assert B.moev_arith_selfcheck(2, 1.0, 0, 1 << 30, seed=8) == 0
    with pytest.raises(B.MoevError) as e:
        B.moev_arith_selfcheck(1, 1.0, 0x7F000000, 1 << 30)
    assert e.value.code == B.E_RANGE


@pytest.mark.parametrize("name", ["fp8_fp8_fp8+fp16", "fp16_fp16_fp16+fp16"])
def test_low_precision_replay_with_and_without_the_plain_sequences(orc, dev, name):
    """Same inputs, knob on and off: both equal the oracle.  Values are in range for most wavefronts (plain
    sequences) and a few tensors carry zeros, denormals and huge values (full sequences)."""
    dtypes = VARIANTS[name]
    wl = ragged_workload(19, max_numel=60000, with_empty=False)
    table = scale_table(wl, dtypes, seed=3)
    st_cpu = W.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=2)
    grads = W.make_grads(wl, 40, seed=2)
    grads[0][::7] = 0.0            # zero gradients next to ordinary ones
    grads[1][::5] = 1e-30          # squares underflow to zero / denormals
    grads[2][::3] = 3e19           # squares overflow
    st_cpu["m"][0].view(torch.uint8)[: st_cpu["m"][0].numel() * st_cpu["m"][0].element_size() // 2] = 0   # zero moments
    mask_np = np.ones(wl.n_ops, dtype=np.uint8)
    hp = orc.AdamHP(lr=1e-3, weight_decay=0.01)
    for knob in (1, 0):
        plan = lp_plan(wl, dtypes)
        B.moev_tune(plan, B.TUNE_PLAIN_DIVIDE_SQRT, knob)
        assert B.moev_tune_get(plan, B.TUNE_PLAIN_DIVIDE_SQRT) == knob
        ds, ref, fmts = run_both(orc, dev, wl, dtypes, st_cpu, table, grads, mask_np, hp, 40, plan)
        assert_states_match(orc, ds, ref, fmts)


def test_low_precision_replay_argument_errors(dev):
    wl = ragged_workload(2, max_numel=1000)
    mask = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    # a width combination without a kernel
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, widths=(4, 2, 2, 2))
    dummy = [torch.zeros(max(n, 1) * 4, dtype=torch.uint8, device=dev) for _, n in wl.tensors]
    st = B.State(dummy, dummy, dummy, dummy)
    with pytest.raises(B.MoevError) as e:
        B.convert_replay(plan, 1e-4, 0.9, 0.95, 1e-8, 0.0, 11, mask, [None] * wl.n_tensors, st)
    assert e.value.code == B.E_INVAL
    # a launch shape the low-precision kernel does not have
    plan = lp_plan(wl, REGIMES["fp16_fp16_fp16+fp16"])
    B.moev_tune(plan, B.TUNE_ADAM_THREADS, 512)
    with pytest.raises(B.MoevError) as e:
        B.convert_replay(plan, 1e-4, 0.9, 0.95, 1e-8, 0.0, 11, mask, [None] * wl.n_tensors, st)
    assert e.value.code == B.E_INVAL


@pytest.mark.parametrize("seed", list(range(16)))
def test_random_plans_whole_window(orc, dev, seed):
    """Seeded random plans: operator count, tensor sizes (ragged, some empty), window, schedule order, segment
    alignment, storage formats (FP32 regime or one of the low-precision combinations), launch shapes, scales.
    Dense run with snapshots, then conversion from a poisoned state: equals the dense run and the oracle."""
    rng = np.random.default_rng(1000 + seed)
    n_ops = int(rng.integers(1, 14))
    window = min(n_ops, 1 + seed % 4)
    tensors = []
    for e in range(n_ops):
        for _ in range(int(rng.integers(1, 4))):
            n = int(rng.choice([0, 1, 3, 4, 5, 63, 64, 257, 1000, 4097, 20000, 70001]))
            tensors.append((e, n))
    slots = [int(x) for x in rng.integers(0, window, size=n_ops)]
    for k in range(window):                       # every slot of the window is used
        slots[int(rng.integers(0, n_ops))] = k if n_ops >= window else slots[0]
    window = max(slots) + 1
    order = sorted(range(n_ops), key=lambda e: (slots[e], int(rng.integers(0, 1000))))
    wl = W.Workload(f"random{seed}", tensors, slots, window, order=order, lr=float(rng.choice([1e-4, 1e-2])),
                    weight_decay=float(rng.choice([0.0, 0.05])))
    names = [None] + list(VARIANTS)
    name = names[int(rng.integers(0, len(names)))]
    align = int(rng.choice([16, 64, 256, 1024]))
    hp = hp_of(wl)
    if name is None:
        dtypes = (torch.float32, torch.float32, torch.float32, torch.bfloat16)
        st_cpu, table = W.make_state(wl, seed=seed), None
        plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, align=align)
        model = model_of(wl, align=align)
    else:
        dtypes = VARIANTS[name]
        table = scale_table(wl, dtypes, seed=seed, odd=bool(rng.integers(0, 2)))
        st_cpu = W.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=seed)
        plan = lp_plan(wl, dtypes, align=align)
        model = model_of(wl, align=align, formats=tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes))
    fmts = tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes)
    shapes = [(64, 1), (64, 2), (128, 1), (128, 2), (256, 1), (256, 2)]
    th, un = shapes[int(rng.integers(0, len(shapes)))]
    B.moev_tune(plan, B.TUNE_ADAM_UNROLL, 1)
    B.moev_tune(plan, B.TUNE_ADAM_THREADS, th)
    B.moev_tune(plan, B.TUNE_ADAM_UNROLL, un)
    B.moev_tune(plan, B.TUNE_XCD_REGIONS, int(rng.integers(0, 2)))
    d_scales = torch.from_numpy(table).to(dev) if table is not None else None
    live = DeviceState(st_cpu, dev)
    ref = orc.State(*[[np_of(t) for t in st_cpu[k]] for k in KINDS])
    everyone = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    ones = np.ones(wl.n_ops, dtype=np.uint8)
    bufs = []
    for k in range(wl.window):
        bufs.append(packed_buffer(plan, dev, k))
        B.snapshot_pack(plan, k, wl.t0 + k, live.state, bufs[k])
        torch.cuda.synchronize()
        exp = orc.pack(model, k, wl.t0 + k, ref)
        assert bufs[k].cpu().numpy()[:exp.size].tobytes() == exp.tobytes(), f"snapshot {k}"
        g = W.make_grads(wl, wl.t0 + k + 1, seed=seed)
        B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, wl.t0 + k + 1, everyone,
                         [x.to(dev) for x in g], live.state, d_scales=d_scales)
        orc.replay_step(model, hp, wl.t0 + k + 1, ones, [x.numpy() for x in g], ref, table)
    torch.cuda.synchronize()
    assert_states_match(orc, live, ref, fmts)
    rebuilt = DeviceState(st_cpu, dev)
    for kind in KINDS:
        for v in rebuilt.views[kind]:
            v.view(torch.uint8).fill_(0xFF)
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    for i in range(wl.window):
        g = W.make_grads(wl, wl.t0 + i + 1, seed=seed)
        dg = [x.to(dev) if wl.slot_of_op[wl.tensors[t][0]] <= i else None for t, x in enumerate(g)]
        if int(rng.integers(0, 2)):
            B.convert_window_step(plan, i, None, bufs[i], hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay,
                                  wl.t0 + i + 1, mask, dg, rebuilt.state, d_scales=d_scales)
        else:
            B.restore_unpack(plan, i, None, bufs[i], rebuilt.state, mask)
            B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, wl.t0 + i + 1, mask, dg,
                             rebuilt.state, d_scales=d_scales)
    torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)
    assert bool(mask.cpu().all())
    a, b = rebuilt.to_oracle(), live.to_oracle()
    for kind in KINDS:
        for t, (x, y) in enumerate(zip(a.kinds()[kind], b.kinds()[kind])):
            assert x.tobytes() == y.tobytes(), (kind, t)
    assert rebuilt.guards_intact() and live.guards_intact()
