"""CPU tests of the HIP library's host side: it loads, exports every declared symbol, and its
plan (schedule, segment tables, sizes, hash) agrees with the oracle.  No GPU compute calls."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_2412_15411_amd import binding as B
from paper_2412_15411_amd import workloads as W
from helpers import model_of

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "moev.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text))
    declared -= {"defined"}
    assert {"ckpt_plan", "snapshot_pack", "snapshot_drain", "restore_unpack", "convert_replay"} <= declared
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in moev.h but not exported"
    assert declared == set(B.EXPORTS)


def _plan_of(wl, mode="explicit", align=0, widths=(0, 0, 0, 0), n_active=0):
    if mode == "explicit":
        return B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, align=align,
                           widths=widths)
    return B.ckpt_plan(wl.tensors, B.FIXED, n_active=n_active, order=wl.order, align=align, widths=widths)


def _cases():
    rng = np.random.default_rng(12)
    ragged_tensors = []
    for e in range(9):
        for _ in range(int(rng.integers(1, 4))):
            ragged_tensors.append((e, int(rng.integers(0, 5000))))
    ragged = W.Workload("ragged", ragged_tensors, [int(x) for x in rng.integers(0, 4, size=9)], 4)
    return [
        W.tiny_moe(),
        W.mixtral_layer(d_model=64, d_ff=224),
        W.fine_grained_stack(n_layers=2, n_routed=16, n_shared=2, d_model=32, d_ff=22, per_slot=4),
        W.ep_rank_share(n_layers=3, n_experts=8, d_model=16, d_ff=8, per_slot=2),
        ragged,
        W.fine_grained_stack(),   # full-size configs: table sizes only, nothing is allocated
        W.ep_rank_share(),
    ]


@pytest.mark.parametrize("wl", _cases(), ids=lambda w: w.name)
@pytest.mark.parametrize("align", [16, 256, 4096])
def test_plan_matches_oracle(orc, wl, align):
    plan = _plan_of(wl, align=align)
    model = model_of(wl, align=align)
    assert B.ckpt_plan_window(plan) == wl.window
    assert B.ckpt_plan_n_ops(plan) == wl.n_ops and B.ckpt_plan_n_tensors(plan) == wl.n_tensors
    assert B.ckpt_plan_slot_of_op(plan) == list(wl.slot_of_op)
    assert B.ckpt_plan_order(plan) == list(wl.order)
    assert orc.check_schedule(B.ckpt_plan_order(plan), B.ckpt_plan_slot_of_op(plan), wl.window) == orc.OK
    assert B.ckpt_plan_hash(plan) == orc.plan_hash(model)
    biggest = 0
    for k in range(wl.window):
        segs, total = orc.layout(model, k)
        assert B.ckpt_plan_segments(plan, k) == segs
        assert B.ckpt_plan_n_segments(plan, k) == len(segs)
        assert B.ckpt_plan_packed_bytes(plan, k) == total
        biggest = max(biggest, total)
        assert B.ckpt_plan_active_params(plan, k) == wl.active_params_at(k)
    assert B.ckpt_plan_max_packed_bytes(plan) == biggest
    assert B.ckpt_plan_packed_bytes(plan, wl.window) == 0


# (compute, master, optimizer) regimes of Sec. 5.6 as element widths (master, m, v, compute)
REGIMES = {
    "fp16/fp32/fp32+fp32 (default)": (4, 4, 4, 2),
    "fp16/fp16/fp16+fp16": (2, 2, 2, 2),
    "fp8/fp32/fp32+fp32": (4, 4, 4, 1),
    "fp8/fp16/fp32+fp32": (2, 4, 4, 1),
    "fp8/fp16/fp8+fp16": (2, 1, 2, 1),
    "fp8/fp8/fp8+fp16": (1, 1, 2, 1),
}


@pytest.mark.parametrize("widths", list(REGIMES.values()), ids=list(REGIMES))
def test_low_precision_layouts_match_oracle(orc, widths):
    """Sec. 5.6: other precisions of compute weights, master weights and optimizer state only change
    the element widths of the snapshot layout."""
    wl = W.fine_grained_stack(n_layers=1, n_routed=8, n_shared=2, d_model=24, d_ff=13, per_slot=2)
    plan, model = _plan_of(wl, widths=widths), model_of(wl, widths=widths)
    assert B.ckpt_plan_hash(plan) == orc.plan_hash(model)
    full = widths[0] + widths[1] + widths[2]
    for k in range(wl.window):
        segs, total = orc.layout(model, k)
        assert B.ckpt_plan_segments(plan, k) == segs and B.ckpt_plan_packed_bytes(plan, k) == total
        assert sum(s[2] for s in segs) == wl.slot_payload_bytes(k, widths=widths)
    # "reduces the snapshot size by as much as 66%": FP8 master + FP8/FP16 moments against FP32 everywhere
    if widths == (1, 1, 2, 1):
        assert round(100 * (1 - full / 12)) in (66, 67)


def test_storage_formats_and_widths_resolve_each_other():
    """Formats and widths of the Sec. 5.6 regimes: either may be left to the other; a contradiction is refused."""
    tensors = [(0, 10), (1, 20)]
    kw = dict(mode=B.EXPLICIT, window=2, slot_of_op=[0, 1])
    plan = B.ckpt_plan(tensors, **kw)
    assert [B.ckpt_plan_width(plan, k) for k in range(4)] == [4, 4, 4, 2]
    assert [B.ckpt_plan_format(plan, k) for k in range(4)] == [B.FMT_F32, B.FMT_F32, B.FMT_F32, B.FMT_BF16]
    plan = B.ckpt_plan(tensors, widths=(1, 1, 2, 1), **kw)   # widths only: FP16 for 2 bytes, E4M3 for 1 byte
    assert [B.ckpt_plan_format(plan, k) for k in range(4)] == [B.FMT_E4M3, B.FMT_E4M3, B.FMT_F16, B.FMT_E4M3]
    plan = B.ckpt_plan(tensors, widths=(2, 2, 2, 2), **kw)   # 2-byte compute weights default to bfloat16
    assert [B.ckpt_plan_format(plan, k) for k in range(4)] == [B.FMT_F16, B.FMT_F16, B.FMT_F16, B.FMT_BF16]
    plan = B.ckpt_plan(tensors, formats=(B.FMT_F16, B.FMT_E5M2, B.FMT_BF16, B.FMT_E4M3), **kw)  # formats only
    assert [B.ckpt_plan_width(plan, k) for k in range(4)] == [2, 1, 2, 1]
    assert [B.ckpt_plan_format(plan, k) for k in range(4)] == [B.FMT_F16, B.FMT_E5M2, B.FMT_BF16, B.FMT_E4M3]
    plan = B.ckpt_plan(tensors, widths=(8, 8, 8, 8), **kw)   # copy-only state: no format
    assert [B.ckpt_plan_format(plan, k) for k in range(4)] == [0, 0, 0, 0]
    assert B.ckpt_plan_width(plan, 4) == 0 and B.ckpt_plan_format(plan, 7) == 0
    for bad in (dict(widths=(4, 4, 4, 2), formats=(B.FMT_F16, 0, 0, 0)), dict(formats=(0, 0, 0, 6)),
                dict(widths=(3, 4, 4, 2))):
        with pytest.raises(B.MoevError) as e:
            B.ckpt_plan(tensors, **kw, **bad)
        assert e.value.code == B.E_INVAL


def test_fixed_mode_matches_generate_schedule(orc):
    for n, a, seed in [(6, 2, 0), (13, 4, 1), (8, 1, 2), (66, 66, 3), (7, 3, 4)]:
        order = W.seeded_permutation(n, seed)
        tensors = [(e, 10 + e) for e in range(n)]
        plan = B.ckpt_plan(tensors, B.FIXED, n_active=a, order=order)
        slots, window = orc.generate_schedule(order, a)
        assert B.ckpt_plan_window(plan) == window and B.ckpt_plan_slot_of_op(plan) == slots
        assert B.ckpt_plan_order(plan) == order and B.ckpt_plan_n_active(plan) == a
        model = orc.Model(tensors, order, slots, window)
        assert B.ckpt_plan_hash(plan) == orc.plan_hash(model)
        for k in range(window):
            assert B.ckpt_plan_segments(plan, k) == orc.layout(model, k)[0]


def test_auto_mode_follows_algorithm_1(orc):
    rng = np.random.default_rng(8)
    for _ in range(100):
        n = int(rng.integers(1, 70))
        bw = float(rng.uniform(1e9, 6e10))
        t_iter = float(rng.uniform(1e-3, 3.0))
        per_op = int(rng.integers(1000, 5_000_000))
        w, a = B.moev_find_window_size(n, t_iter, 2.0 * per_op, 4.0 * per_op, 8.0 * per_op, bw)
        assert (w, a) == orc.find_window_size(n, t_iter, 2.0 * per_op, 4.0 * per_op, 8.0 * per_op, bw)
        plan = B.ckpt_plan([(e, per_op) for e in range(n)], B.AUTO, t_iter_s=t_iter, host_link_Bps=bw)
        assert B.ckpt_plan_window(plan) == w and B.ckpt_plan_n_active(plan) == a
        assert B.ckpt_plan_slot_of_op(plan) == orc.generate_schedule(list(range(n)), a)[0]


def test_order_operators_and_reorder_trigger(orc):
    rng = np.random.default_rng(2)
    for _ in range(30):
        pop = [float(x) for x in rng.integers(0, 7, size=int(rng.integers(1, 50)))]
        assert B.moev_order_operators(pop) == orc.order_by_popularity(pop)
    # Sec. 3.5: re-order when the frequency moved by more than 10% for at least 25% of the experts
    old = [100.0] * 8
    assert not B.moev_reorder_needed(old, [100.0] * 6 + [120.0, 80.0][:1] + [100.0])   # 1 of 8 moved
    assert B.moev_reorder_needed(old, [100.0] * 6 + [120.0, 80.0])                      # 2 of 8 = 25%
    assert not B.moev_reorder_needed(old, [109.0] * 8)                                   # all within 10%
    assert B.moev_reorder_needed(old, [111.0] * 8)


def test_plan_rejects_bad_configurations():
    t = [(0, 10), (1, 10), (2, 10)]
    bad = [
        dict(tensors=[(0, 10), (2, 10)], mode=B.EXPLICIT, window=2, slot_of_op=[0, 1, 1]),   # operator 1 has no tensor
        dict(tensors=[(1, 10), (0, 10)], mode=B.EXPLICIT, window=2, slot_of_op=[0, 1]),      # not grouped ascending
        dict(tensors=t, mode=B.EXPLICIT, window=2, slot_of_op=[0, 1, 2]),                    # slot outside the window
        dict(tensors=t, mode=B.EXPLICIT, window=0, slot_of_op=[0, 0, 0]),
        dict(tensors=t, mode=B.EXPLICIT, window=3, slot_of_op=[0, 1, 2], order=[2, 1, 0]),   # order walks back
        dict(tensors=t, mode=B.FIXED, n_active=0),
        dict(tensors=t, mode=B.FIXED, n_active=2, order=[0, 1, 1]),                          # not a permutation
        dict(tensors=t, mode=B.AUTO, t_iter_s=1.0, host_link_Bps=0.0),
        dict(tensors=t, mode=B.EXPLICIT, window=1, slot_of_op=[0, 0, 0], align=48),          # not a power of two
        dict(tensors=t, mode=B.EXPLICIT, window=1, slot_of_op=[0, 0, 0], align=8),
        dict(tensors=t, mode=B.EXPLICIT, window=1, slot_of_op=[0, 0, 0], widths=(3, 4, 4, 2)),
        dict(tensors=t, mode=7),
    ]
    for kw in bad:
        with pytest.raises(B.MoevError) as e:
            B.ckpt_plan(**kw)
        assert e.value.code == B.E_INVAL, kw


def test_tune_knobs_validate():
    plan = _plan_of(W.tiny_moe())
    assert B.moev_tune_get(plan, B.TUNE_COPY_TILE_BYTES) % 4096 == 0
    B.moev_tune(plan, B.TUNE_COPY_TILE_BYTES, 65536)
    assert B.moev_tune_get(plan, B.TUNE_COPY_TILE_BYTES) == 65536
    B.moev_tune(plan, B.TUNE_COPY_THREADS, 512)
    B.moev_tune(plan, B.TUNE_COPY_UNROLL, 2)
    for knob, value in [(B.TUNE_COPY_TILE_BYTES, 1000), (B.TUNE_ADAM_TILE_ELEMS, 100), (B.TUNE_COPY_MAX_BLOCKS, -1), (99, 1),
                        (B.TUNE_COPY_UNROLL, 4), (B.TUNE_COPY_THREADS, 100), (B.TUNE_ADAM_UNROLL, 3), (B.TUNE_COPY_UNROLL, 8)]:
        with pytest.raises(B.MoevError):
            B.moev_tune(plan, knob, value)


def test_mapping_and_pairing_knobs_validate():
    """Workgroup -> tile mapping (0 off, 1 an eighth of the tiles per XCD, a power of two up to 65536 = chunk size) and
    the piece distance of the paired replay tiles (0 off, 1 = the default 32 KiB, a power of two in [512, 4 MiB])."""
    plan = _plan_of(W.tiny_moe())
    assert B.moev_tune_get(plan, B.TUNE_XCD_REGIONS) == 1
    assert B.moev_tune_get(plan, B.TUNE_COPY_XCD_REGIONS) == 64
    assert B.moev_tune_get(plan, B.TUNE_PAIRED_TILES) == 32768
    for knob in (B.TUNE_XCD_REGIONS, B.TUNE_COPY_XCD_REGIONS):
        for good in (0, 1, 2, 64, 65536):
            B.moev_tune(plan, knob, good)
            assert B.moev_tune_get(plan, knob) == good
        for bad in (-1, 3, 48, 131072):
            with pytest.raises(B.MoevError) as e:
                B.moev_tune(plan, knob, bad)
            assert e.value.code == B.E_INVAL
            assert B.moev_tune_get(plan, knob) == 65536     # a refused value changes nothing
    for good, stored in ((0, 0), (1, 32768), (512, 512), (4 << 20, 4 << 20)):
        B.moev_tune(plan, B.TUNE_PAIRED_TILES, good)
        assert B.moev_tune_get(plan, B.TUNE_PAIRED_TILES) == stored
    for bad in (-8, 2, 256, 3000, 8 << 20):
        with pytest.raises(B.MoevError) as e:
            B.moev_tune(plan, B.TUNE_PAIRED_TILES, bad)
        assert e.value.code == B.E_INVAL


def test_snapshot_peek_accepts_oracle_snapshot_and_rejects_others(orc):
    """The header the oracle writes is the header the library expects (format is shared by definition)."""
    import torch
    from helpers import state_of
    wl = W.tiny_moe(d_in=8, d_hidden=16)
    plan, model = _plan_of(wl), model_of(wl)
    st = state_of(W.make_state(wl, seed=1))
    snap = orc.pack(model, 1, 77, st)
    buf = torch.from_numpy(snap)
    hd = B.snapshot_peek(plan, 1, buf)
    assert hd["iter"] == 77 and hd["slot"] == 1 and hd["n_segments"] == len(orc.layout(model, 1)[0])
    with pytest.raises(B.MoevError) as e:
        B.snapshot_peek(plan, 0, buf)
    assert e.value.code == B.E_MISMATCH
    other = _plan_of(wl, align=512)
    with pytest.raises(B.MoevError):
        B.snapshot_peek(other, 1, buf)


def test_gpu_calls_fail_loudly_without_a_gpu():
    """No silent fallback: on a machine without a usable GPU the hot-path calls raise."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    wl = W.tiny_moe(d_in=8, d_hidden=16)
    plan = _plan_of(wl)
    st = W.make_state(wl, seed=0)
    state = B.State(st["master"], st["m"], st["v"], st["compute"])
    packed = torch.zeros(B.ckpt_plan_max_packed_bytes(plan) + 512, dtype=torch.uint8)
    addr = (packed.data_ptr() + 255) // 256 * 256
    with pytest.raises(B.MoevError) as e:
        B.snapshot_pack(plan, 0, 10, state, addr, cap=B.ckpt_plan_max_packed_bytes(plan))
    assert e.value.code == B.E_HIP


def test_plan_hash_covers_the_storage_formats(orc):
    """A snapshot taken under one precision regime must not pass the header check of a plan with the same element
    widths and other storage formats: the formats are part of the hash, on both sides alike."""
    wl = W.fine_grained_stack(n_layers=1, n_routed=8, n_shared=2, d_model=24, d_ff=13, per_slot=2)
    lib_of = {orc.FMT_F32: B.FMT_F32, orc.FMT_F16: B.FMT_F16, orc.FMT_BF16: B.FMT_BF16, orc.FMT_E4M3: B.FMT_E4M3,
              orc.FMT_E5M2: B.FMT_E5M2}
    seen = set()
    for fmts in ((orc.FMT_F16,) * 4, (orc.FMT_BF16,) * 4, (orc.FMT_F16, orc.FMT_F16, orc.FMT_F16, orc.FMT_BF16),
                 (orc.FMT_F16, orc.FMT_E4M3, orc.FMT_F16, orc.FMT_E4M3), (orc.FMT_F16, orc.FMT_E5M2, orc.FMT_F16, orc.FMT_E5M2),
                 (orc.FMT_F32, orc.FMT_F32, orc.FMT_F32, orc.FMT_E4M3)):
        plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order,
                           formats=[lib_of[f] for f in fmts])
        h = B.ckpt_plan_hash(plan)
        assert h == orc.plan_hash(model_of(wl, formats=fmts))
        assert h not in seen
        seen.add(h)
    # formats left open are filled in by width before hashing
    by_width = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, widths=(2, 2, 2, 2))
    assert B.ckpt_plan_hash(by_width) == orc.plan_hash(model_of(wl, formats=(orc.FMT_F16, orc.FMT_F16, orc.FMT_F16, orc.FMT_BF16)))
    # and a host snapshot of one regime is refused by the other's plan
    f16 = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, formats=[B.FMT_F16] * 4)
    bf16 = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, formats=[B.FMT_BF16] * 4)
    model = model_of(wl, formats=(orc.FMT_F16,) * 4)
    st = W.make_low_precision_state(wl, (torch.float16,) * 4, (1.0, 64.0, 65536.0, 1.0), seed=1)
    snap = orc.pack(model, 1, 77, orc.State(*[[t.view(torch.int16).numpy().view(np.uint16) for t in st[k]]
                                              for k in ("master", "m", "v", "compute")]))
    assert B.snapshot_peek(f16, 1, torch.from_numpy(snap))["iter"] == 77
    with pytest.raises(B.MoevError) as e:
        B.snapshot_peek(bf16, 1, torch.from_numpy(snap))
    assert e.value.code == B.E_MISMATCH


def test_bias_corrections_agree_with_the_oracle_up_to_100000_steps(orc):
    """1 - beta^step in double precision, rounded to FP32 once: the library raises beta to the power with the math
    library, the oracle multiplies step times.  The two must land on the same FP32 value for every step a run can
    reach (the GPU parity tests only visit small step numbers).  Every step up to 20,000 (beyond ~17,500 even
    0.999^step is below half an FP32 unit of 1 and both corrections are exactly 1), then 1,000 steps spread up to
    100,000 (the oracle's product costs `step` multiplications per call)."""
    rng = np.random.default_rng(3)
    far = sorted(set(int(x) for x in rng.integers(20_001, 100_001, size=990)) | set(range(99_991, 100_001)))
    for beta1, beta2 in ((0.9, 0.95), (0.95, 0.999), (0.999, 0.9)):
        hp = orc.AdamHP(1e-4, beta1, beta2, 1e-8, 0.0)
        distinct = set()
        for step in list(range(1, 20_001)) + far:
            got = B.moev_bias_corrections(beta1, beta2, step)
            assert got == orc.bias_corrections(hp, step), (beta1, beta2, step)
            distinct.add(got)
        assert len(distinct) > 100 and B.moev_bias_corrections(beta1, beta2, 100_000) == (1.0, 1.0)
    # the closed form's ends
    assert B.moev_bias_corrections(0.9, 0.999, 10 ** 9) == (1.0, 1.0)
    b1, _ = B.moev_bias_corrections(0.9, 0.999, 1)
    assert b1 == float(np.float32(1.0 - float(np.float32(0.9))))
    with pytest.raises(B.MoevError):
        B.moev_bias_corrections(0.9, 0.999, 0)
