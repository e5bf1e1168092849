"""GPU parity at the benchmark configurations' FULL sizes, in the launch configuration bench.py times.

The oracle cannot hold or finish these sizes, so the checks are (a) sampled outputs the oracle
computes one by one (windows of every segment / tensor, including first and last bytes), and (b)
properties that hold at any size: the wrapping 64-bit word sum of a packed snapshot equals the sum
over its source segments (padding is zero), pack followed by unpack restores every word sum, and
whatever is not named by the slot keeps its poison pattern.
"""
import gc

import numpy as np
import pytest
import torch

from paper_2412_15411_amd import binding as B
from paper_2412_15411_amd import workloads as W
from helpers import hp_of, model_of, np_of

pytestmark = pytest.mark.gpu
KINDS = ("master", "m", "v", "compute")
KIND_ID = {0: "master", 1: "m", 2: "v", 3: "compute"}


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    return torch.device("cuda:0")


def _release():
    gc.collect()
    torch.cuda.empty_cache()


def word_sum(t: torch.Tensor) -> int:
    """Wrapping sum of the tensor's bytes read as little-endian 64-bit words (tail zero-extended)."""
    raw = t.reshape(-1).view(torch.uint8)
    n8 = raw.numel() // 8 * 8
    total = int(raw[:n8].view(torch.int64).sum().item()) if n8 else 0
    if raw.numel() > n8:
        tail = raw[n8:].cpu().numpy().tobytes() + b"\0" * (8 - (raw.numel() - n8))
        total += int(np.frombuffer(tail, dtype="<i8")[0])
    return total & ((1 << 64) - 1)


def sample_windows(nbytes: int, rng, n_random: int, width: int):
    """Byte windows of a segment: its first and last `width` bytes plus random interior ones."""
    if nbytes <= 2 * width:
        return [(0, nbytes)]
    wins = [(0, width), (nbytes - width, nbytes)]
    for _ in range(n_random):
        a = int(rng.integers(0, nbytes - width))
        wins.append((a, a + width))
    return wins


def check_packed_against_oracle(orc, wl, model, plan, k, it, st, buf, rng, n_random=2, width=8192):
    segs, total = orc.layout(model, k)
    assert total == B.ckpt_plan_packed_bytes(plan, k)
    header = buf[:256].cpu().numpy()
    # the oracle writes the header of an empty-tensor twin of this plan: same integers, no data needed
    assert header[:8].tobytes() == b"MOEVSNAP"
    assert int.from_bytes(header[12:16].tobytes(), "little") == k
    assert int.from_bytes(header[16:24].tobytes(), "little") == orc.plan_hash(model)
    assert int.from_bytes(header[24:32].tobytes(), "little") == it
    assert int.from_bytes(header[32:40].tobytes(), "little") == len(segs)
    assert int.from_bytes(header[40:48].tobytes(), "little") == total - 256
    assert not header[52:].any()
    expect_sum = word_sum(buf[:256])
    for kind, t, nbytes, off in segs:
        src = st[KIND_ID[kind]][t].view(torch.uint8)
        expect_sum = (expect_sum + word_sum(src)) & ((1 << 64) - 1)
        for a, b in sample_windows(nbytes, rng, n_random, width):
            assert torch.equal(buf[off + a: off + b], src[a:b]), f"slot {k} segment ({kind},{t}) window {a}"
        padded = -(-nbytes // model.align) * model.align
        assert not buf[off + nbytes: off + padded].any().item()
    assert word_sum(buf[:total]) == expect_sum, f"slot {k}: packed word sum differs"


def run_pack_unpack_fullsize(orc, dev, wl, slots, seed=0, keep_copy=True):
    model = model_of(wl)
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
    st = W.make_state(wl, seed=seed, device=dev)
    state = B.State(*[st[k] for k in KINDS])
    sums = {k: [word_sum(t) for t in st[k]] for k in KINDS}
    rng = np.random.default_rng(seed)
    buf = torch.empty(B.ckpt_plan_max_packed_bytes(plan), dtype=torch.uint8, device=dev)
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    for pos, k in enumerate(slots):
        buf.fill_(0xA5)
        B.snapshot_pack(plan, k, 100 + k, state, buf)
        torch.cuda.synchronize()
        check_packed_against_oracle(orc, wl, model, plan, k, 100 + k, st, buf, rng)
        # poison the whole state, restore the slot, check sums / poison
        for kind in KINDS:
            for t in st[kind]:
                t.view(torch.int16).fill_(0x7BAD)
        mask.fill_(9)
        B.restore_unpack(plan, k, None, buf, state, mask)
        torch.cuda.synchronize()
        B.ckpt_plan_device_status(plan)
        m = mask.cpu().numpy()
        for t, (op, numel) in enumerate(wl.tensors):
            s = wl.slot_of_op[op]
            assert m[op] == (1 if s == k else 0 if s > k else 9)
            for kind in KINDS:
                restored = (s == k and kind != "compute") or (s > k and kind == "compute")
                if restored:
                    assert word_sum(st[kind][t]) == sums[kind][t], f"slot {k} {kind}[{t}] not restored"
                elif s == k and kind == "compute":
                    # derived from the restored master weights: spot-check against the oracle's cast
                    idx = rng.integers(0, numel, size=64)
                    got = st["compute"][t].view(torch.int16)[idx].cpu().numpy().view(np.uint16)
                    exp = orc.bf16_rne_array(st["master"][t][idx].cpu().numpy())
                    assert np.array_equal(got, exp)
                else:
                    probe = st[kind][t].view(torch.int16)
                    assert probe[0].item() == 0x7BAD and probe[-1].item() == 0x7BAD
                    assert probe[int(rng.integers(0, probe.numel()))].item() == 0x7BAD
        if pos + 1 < len(slots):  # bring the state back for the next slot: regenerate
            del st, state
            _release()
            st = W.make_state(wl, seed=seed, device=dev)
            state = B.State(*[st[k] for k in KINDS])
    del st, state, buf
    _release()


def test_fullsize_mixtral_layer_pack_unpack(orc, dev):
    """configs[1]: 19.7 GB of state, slots 0 (30 segments), 3 and 7."""
    run_pack_unpack_fullsize(orc, dev, W.mixtral_layer(), slots=(0, 3, 7))


def test_fullsize_fine_grained_pack_unpack(orc, dev):
    """configs[2]: 264 operators, 888 segments in slot 0, permuted schedule, shared experts in slot 15."""
    run_pack_unpack_fullsize(orc, dev, W.fine_grained_stack(), slots=(0, 15))


def _replay_sampled(orc, dev, wl, it_index, extra_windows=()):
    """convert_replay at full size with the mask of replay iteration `it_index`; sampled element windows of
    every tensor (first / last / random / the given extra ones) against the oracle's Adam."""
    hp = hp_of(wl)
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
    st = W.make_state(wl, seed=3, device=dev)
    state = B.State(*[st[k] for k in KINDS])
    step = wl.t0 + it_index + 1
    active = [1 if s <= it_index else 0 for s in wl.slot_of_op]
    mask = torch.tensor(active, dtype=torch.uint8, device=dev)
    full = W.make_grads(wl, step, seed=3, device=dev)
    grads = [g if active[wl.tensors[t][0]] else None for t, g in enumerate(full)]
    rng = np.random.default_rng(1)
    width = 4096
    before = {}
    for t, (op, numel) in enumerate(wl.tensors):
        wins = [(a // 4, b // 4) for a, b in sample_windows(numel * 4, rng, 1 if wl.n_tensors > 100 else 6, width * 4)]
        wins += [(a, b) for a, b in extra_windows if b <= numel]
        before[t] = [(a, b, {k: st[k][t][a:b].clone() for k in KINDS}, full[t][a:b].clone()) for a, b in wins]
    B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, step, mask, grads, state)
    torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)
    worst = 0.0
    for t, (op, numel) in enumerate(wl.tensors):
        for a, b, old, g in before[t]:
            now = {k: np_of(st[k][t][a:b]) for k in KINDS}
            if not active[op]:
                for k in KINDS:
                    assert now[k].tobytes() == np_of(old[k]).tobytes(), f"frozen tensor {t} changed"
                continue
            p, m, v, c = np_of(old["master"]), np_of(old["m"]), np_of(old["v"]), np_of(old["compute"])
            orc.adam_tensor(p, m, v, np_of(g), c, hp, step)
            for name, ref in (("master", p), ("m", m), ("v", v)):
                err = np.max(np.abs(now[name].astype(np.float64) - ref.astype(np.float64)) /
                             np.maximum(np.abs(ref.astype(np.float64)), 1e-30))
                worst = max(worst, float(err))
                assert err <= 1e-6, f"{wl.name} tensor {t} {name} window {a}: rel err {err}"
            same = now["master"].view(np.uint32) == p.view(np.uint32)
            assert np.array_equal(now["compute"][same], c[same])
    print(f"{wl.name}: worst relative error over sampled windows {worst:.3g}")
    del st, state, full, grads, before
    _release()


def test_fullsize_replay_sampled(orc, dev):
    """configs[1] and configs[4] shapes: convert_replay at full size with the mask of a mid-window
    iteration; sampled windows of every tensor (first / last / random) against the oracle's Adam."""
    for wl, it_index in ((W.mixtral_layer(), 5), (W.conversion_stress(), 9)):
        _replay_sampled(orc, dev, wl, it_index)


def test_tensors_beyond_4_GiB(orc, dev):
    """Maximum sizes: single tensors of 5.0 and 4.4 GB per FP32 kind (ragged lengths), so that byte offsets
    INSIDE one segment pass 2^32 and element indices pass 2^30: pack / unpack (sampled windows, word sums,
    poison) and the replay on windows around those boundaries and at the ragged tails."""
    wl = W.Workload("huge", [(0, 1_250_000_003), (1, 1_100_000_001)], [0, 1], 2)
    run_pack_unpack_fullsize(orc, dev, wl, slots=(0, 1), seed=2)
    edge = 1 << 30
    _replay_sampled(orc, dev, wl, 1, extra_windows=[(edge - 2048, edge + 2048), (edge - 3, edge + 5),
                                                    (1_100_000_001 - 9, 1_100_000_001), (1_250_000_003 - 7, 1_250_000_003)])


@pytest.mark.parametrize("regime", ["fp8_fp8_fp8+fp16", "fp16_fp16_fp16+fp16", "fp8_fp16_fp32+fp32"])
def test_fullsize_low_precision_replay_sampled(orc, dev, regime):
    """configs[1] at full size with the state stored as a Sec. 5.6 regime, in the launch configuration
    `bench.py --regime` times: sampled windows of every tensor against the oracle's low-precision step,
    code for code; frozen tensors keep their bits."""
    from helpers import ORACLE_FMT_OF_DTYPE
    lib_fmt = {torch.float32: B.FMT_F32, torch.float16: B.FMT_F16, torch.bfloat16: B.FMT_BF16,
               torch.float8_e4m3fn: B.FMT_E4M3, torch.float8_e5m2: B.FMT_E5M2}
    wl, it_index = W.mixtral_layer(), 5
    dtypes = W.LOW_PRECISION_REGIMES[regime]
    fmts = tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes)
    hp = hp_of(wl)
    per_kind = W.default_scales(dtypes)
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order,
                       formats=[lib_fmt[d] for d in dtypes])
    st = W.make_low_precision_state(wl, dtypes, per_kind, seed=3, device=dev)
    state = B.State(*[st[k] for k in KINDS])
    d_scales = torch.tensor([[x] * wl.n_tensors for x in per_kind], dtype=torch.float32, device=dev)
    step = wl.t0 + it_index + 1
    active = [1 if s <= it_index else 0 for s in wl.slot_of_op]
    mask = torch.tensor(active, dtype=torch.uint8, device=dev)
    full = W.make_grads(wl, step, seed=3, device=dev)
    grads = [g if active[wl.tensors[t][0]] else None for t, g in enumerate(full)]
    rng = np.random.default_rng(1)
    before = {}
    for t, (op, numel) in enumerate(wl.tensors):
        wins = [(a // 4, b // 4) for a, b in sample_windows(numel * 4, rng, 4, 4096 * 4)]
        before[t] = [(a, b, {k: st[k][t][a:b].clone() for k in KINDS}, full[t][a:b].clone()) for a, b in wins]
    B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, step, mask, grads, state, d_scales=d_scales)
    torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)
    checked = 0
    for t, (op, numel) in enumerate(wl.tensors):
        for a, b, old, g in before[t]:
            now = {k: np_of(st[k][t][a:b]) for k in KINDS}
            ref = {k: np_of(old[k]) for k in KINDS}
            if active[op]:
                orc.adam_tensor_lp(ref["master"], ref["m"], ref["v"], np_of(g), ref["compute"], hp, step, fmts, per_kind)
            for k in KINDS:
                assert now[k].tobytes() == ref[k].tobytes(), f"{regime} tensor {t} {k} window {a}"
            checked += b - a
    print(f"{regime}: {checked} sampled parameters match the oracle code for code")
    del st, state, full, grads, before
    _release()


def test_fullsize_ep_rank_share_pack(orc, dev):
    """configs[3]: 180 GB of state resident in HBM, slot 0 (1,920 segments, 41.9 GB packed): sampled
    windows of every segment plus the word-sum property; then restore into the poisoned state."""
    free, total = torch.cuda.mem_get_info()
    wl = W.ep_rank_share()
    need = wl.n_params * 14 + wl.slot_payload_bytes(0) + (8 << 30)
    if free < need:
        pytest.skip(f"needs {need / 1e9:.0f} GB of free HBM, {free / 1e9:.0f} GB available")
    run_pack_unpack_fullsize(orc, dev, wl, slots=(0,))
