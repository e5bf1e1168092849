"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical seeded inputs.

Copies (pack, drain, unpack) must agree bit for bit; replayed FP32 Adam state within a max
relative error of 1e-6 (max |x - ref| / max(|ref|, 1e-30)); the bf16 compute weights must be
the round-to-nearest-even cast of the GPU's own master weights and equal the oracle's wherever
the master weights agree bitwise.
"""
import numpy as np
import pytest
import torch

from paper_2412_15411_amd import binding as B
from paper_2412_15411_amd import workloads as W
from helpers import hp_of, model_of, np_of, state_of, states_equal, max_rel_err

pytestmark = pytest.mark.gpu

REL_TOL = 1e-6
KINDS = ("master", "m", "v", "compute")


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    return torch.device("cuda:0")


# ---------------------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------------------
GUARD = 64  # bytes of sentinel between neighbouring tensors


class DeviceState:
    """The workload's tensors carved out of one device arena per kind, with sentinel-filled
    guard gaps between neighbours so that any stray write shows."""

    def __init__(self, st_cpu, dev):
        self.arena, self.views, self.spans = {}, {k: [] for k in KINDS}, {k: [] for k in KINDS}
        for kind in KINDS:
            offs, cursor = [], GUARD
            for t in st_cpu[kind]:
                cursor = (cursor + 15) // 16 * 16
                offs.append(cursor)
                cursor += t.numel() * t.element_size() + GUARD
            arena = torch.full((cursor + 16,), 0x5A, dtype=torch.uint8, device=dev)
            base = (-arena.data_ptr()) % 16  # torch allocations are far more aligned; keep it general
            for t, o in zip(st_cpu[kind], offs):
                nbytes = t.numel() * t.element_size()
                view = arena[base + o: base + o + nbytes].view(t.dtype)
                view.copy_(t)
                self.views[kind].append(view)
                self.spans[kind].append((base + o, nbytes))
            self.arena[kind] = arena
        self.state = B.State(*[self.views[k] for k in KINDS])

    def guards_intact(self):
        for kind in KINDS:
            a = self.arena[kind].cpu().numpy()
            keep = np.ones(a.size, dtype=bool)
            for o, n in self.spans[kind]:
                keep[o:o + n] = False
            if not (a[keep] == 0x5A).all():
                return False
        return True

    def to_oracle(self):
        import oracle
        return oracle.State(*[[np_of(v) for v in self.views[k]] for k in KINDS])

    def poison(self):
        for k in ("master", "m", "v"):
            for v in self.views[k]:
                v.view(torch.int32).fill_(0x7FC0DEAD)
        for v in self.views["compute"]:
            v.view(torch.int16).fill_(-1)


def make_plan(wl, align=0, tile=None, blocks=None, adam_tile=None, adam_blocks=None, nt=None,
              copy_shape=None, adam_shape=None, xcd_regions=None, paired=None):
    """tile / blocks / adam_tile / adam_blocks select the fixed-grid launch shape with those values;
    copy_shape / adam_shape = (threads, unroll) select a one-tile-per-workgroup shape (the default)."""
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order,
                       align=align)
    if tile or blocks or adam_tile or adam_blocks:
        B.moev_tune(plan, B.TUNE_PERSISTENT, 1)
    for knob, value in ((B.TUNE_COPY_TILE_BYTES, tile), (B.TUNE_COPY_MAX_BLOCKS, blocks),
                        (B.TUNE_ADAM_TILE_ELEMS, adam_tile), (B.TUNE_ADAM_MAX_BLOCKS, adam_blocks)):
        if value:
            B.moev_tune(plan, knob, value)
    for shape, k_threads, k_unroll in ((copy_shape, B.TUNE_COPY_THREADS, B.TUNE_COPY_UNROLL),
                                       (copy_shape, B.TUNE_UNPACK_THREADS, B.TUNE_UNPACK_UNROLL),
                                       (adam_shape, B.TUNE_ADAM_THREADS, B.TUNE_ADAM_UNROLL)):
        if shape:
            B.moev_tune(plan, k_unroll, 1)
            B.moev_tune(plan, k_threads, shape[0])
            B.moev_tune(plan, k_unroll, shape[1])
    if nt is not None:
        B.moev_tune(plan, B.TUNE_NONTEMPORAL, nt)
    if xcd_regions is not None:
        B.moev_tune(plan, B.TUNE_XCD_REGIONS, xcd_regions)
        B.moev_tune(plan, B.TUNE_COPY_XCD_REGIONS, xcd_regions)
    if paired is not None:
        B.moev_tune(plan, B.TUNE_PAIRED_TILES, paired)
    return plan


def packed_buffer(plan, dev, slot=None):
    n = B.ckpt_plan_max_packed_bytes(plan) if slot is None else B.ckpt_plan_packed_bytes(plan, slot)
    buf = torch.full((n + 256,), 0xA5, dtype=torch.uint8, device=dev)
    assert buf.data_ptr() % 256 == 0
    return buf


def ragged_workload(seed, n_ops=11, window=4, max_numel=70000, with_empty=True):
    rng = np.random.default_rng(seed)
    tensors = []
    for e in range(n_ops):
        for _ in range(int(rng.integers(1, 4))):
            n = int(rng.integers(1, max_numel))
            if rng.random() < 0.3:
                n = int(rng.integers(1, 40))          # tiny tensors: many sub-vector tails
            tensors.append((e, n))
    if with_empty:
        tensors[3] = (tensors[3][0], 0)
    slots = [int(x) for x in rng.integers(0, window, size=n_ops)]
    slots[0], slots[1] = 0, window - 1
    return W.Workload(f"ragged{seed}", tensors, slots, window)


# ---------------------------------------------------------------------------------------
# layout scan
# ---------------------------------------------------------------------------------------
def _many_segments():
    n_ops = 9000
    rng = np.random.default_rng(0)
    return W.Workload("many", [(e, int(rng.integers(1, 40))) for e in range(n_ops)], [e % 2 for e in range(n_ops)], 2)


@pytest.mark.parametrize("wl,align,tile", [
    (ragged_workload(1), 16, 4096), (ragged_workload(2), 256, 32768), (ragged_workload(3), 4096, 8192),
    (W.fine_grained_stack(n_layers=2, n_routed=64, n_shared=2, d_model=16, d_ff=11), 256, 4096),
    (_many_segments(), 64, 4096), (ragged_workload(4), 256, None),
], ids=["ragged16", "ragged256", "ragged4096", "c2_small_888seg", "18000seg", "default_shape"])
def test_device_layout_scan_matches_oracle(orc, dev, wl, align, tile):
    """The wavefront prefix sums on the device reproduce the oracle's serial layout exactly."""
    plan = make_plan(wl, align=align, tile=tile)
    model = model_of(wl, align=align)
    per_slot = tile is None
    for k in range(wl.window):
        if per_slot:   # default shape: 256 threads x 16 bytes x (1 or 2 accesses per lane, chosen per slot)
            tile = B.ckpt_plan_pack_tile_bytes(plan, k)
            assert tile in (4096, 8192)
        segs, total = orc.layout(model, k)
        off, tiles, dev_total = B.ckpt_plan_device_layout(plan, k)
        assert off == [s[3] for s in segs]
        assert dev_total == total == B.ckpt_plan_packed_bytes(plan, k)
        exp_tiles = [0]
        for s in segs:
            padded = -(-s[2] // align) * align
            exp_tiles.append(exp_tiles[-1] + -(-padded // tile))
        assert tiles == exp_tiles


# ---------------------------------------------------------------------------------------
# pack / drain / unpack
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed,align,tile,blocks,nt,shape", [
    (1, 256, None, None, 1, None), (2, 16, None, None, 0, (64, 1)), (3, 4096, None, None, 1, (512, 2)),
    (4, 64, None, None, 1, (256, 4)), (5, 256, None, None, 0, (1024, 1)), (6, 16, None, None, 1, (128, 1)),
    (1, 256, 32768, None, 1, None), (2, 16, 4096, 3, 1, None), (3, 4096, 8192, 7, 0, None), (4, 64, 65536, 1, 1, None),
])
def test_pack_bit_exact(orc, dev, seed, align, tile, blocks, nt, shape):
    """Ragged tensors with arbitrary bit patterns: GPU packed buffer == oracle packed buffer, byte
    for byte (header, segments, zero padding), for every slot; the source state is not modified."""
    wl = ragged_workload(seed)
    st_cpu = W.random_bits_state(wl, seed=seed)
    ds = DeviceState(st_cpu, dev)
    ref_state = state_of(st_cpu)
    plan, model = make_plan(wl, align=align, tile=tile, blocks=blocks, nt=nt, copy_shape=shape), model_of(wl, align=align)
    buf = packed_buffer(plan, dev)
    for k in range(wl.window):
        buf.fill_(0xA5)
        B.snapshot_pack(plan, k, 100 + k, ds.state, buf, cap=B.ckpt_plan_packed_bytes(plan, k))
        torch.cuda.synchronize()
        exp = orc.pack(model, k, 100 + k, ref_state)
        got = buf.cpu().numpy()
        assert got[:exp.size].tobytes() == exp.tobytes(), f"slot {k}"
        assert (got[exp.size:] == 0xA5).all()           # nothing written past the snapshot
    assert states_equal(ds.to_oracle(), ref_state) == [] and ds.guards_intact()


@pytest.mark.parametrize("seed,align,tile,blocks,shape", [
    (11, 256, None, None, None), (12, 16, None, None, (64, 1)), (13, 4096, None, None, (512, 2)), (14, 64, None, None, (256, 4)),
    (15, 256, None, None, (1024, 1)), (11, 256, 32768, None, None), (12, 16, 4096, 5, None), (13, 4096, 16384, 2, None)])
def test_unpack_bit_exact_with_sentinels(orc, dev, seed, align, tile, blocks, shape):
    """restore_unpack of an ORACLE-made snapshot into a poisoned device state equals the oracle's
    unpack: restored tensors, derived bf16 weights of the newly active operators, untouched
    tensors, guard gaps and the active mask."""
    wl = ragged_workload(seed)
    model = model_of(wl, align=align)
    truth = state_of(W.random_bits_state(wl, seed=seed))
    plan = make_plan(wl, align=align, tile=tile, blocks=blocks, copy_shape=shape)
    st_cpu = W.random_bits_state(wl, seed=seed + 100)
    for k in range(wl.window):
        ds = DeviceState(st_cpu, dev)
        ds.poison()
        ref = ds.to_oracle()
        snap = orc.pack(model, k, 50 + k, truth)
        ref_mask = np.full(wl.n_ops, 9, dtype=np.uint8)
        orc.unpack(model, k, snap, ref, ref_mask)
        buf = packed_buffer(plan, dev, k)
        buf[:snap.size].copy_(torch.from_numpy(snap))
        mask = torch.full((wl.n_ops,), 9, dtype=torch.uint8, device=dev)
        B.restore_unpack(plan, k, None, buf, ds.state, mask)
        torch.cuda.synchronize()
        B.ckpt_plan_device_status(plan)
        assert states_equal(ds.to_oracle(), ref) == [], f"slot {k}"
        assert ds.guards_intact()
        assert np.array_equal(mask.cpu().numpy(), ref_mask)


@pytest.mark.parametrize("persistent", [False, True], ids=["direct", "fixed_grid_global_table"])
def test_pack_unpack_many_tiny_segments(orc, dev, persistent):
    """18,000 segments in a slot (beyond what the fixed-grid shape stages in LDS): every tensor is a
    few elements long, so nearly every tile is a ragged tail."""
    wl = _many_segments()
    model = model_of(wl, align=16)
    st_cpu = W.random_bits_state(wl, seed=3)
    ref_state = state_of(st_cpu)
    ds = DeviceState(st_cpu, dev)
    plan = make_plan(wl, align=16, tile=4096 if persistent else None, blocks=64 if persistent else None)
    buf = packed_buffer(plan, dev)
    for k in range(wl.window):
        buf.fill_(0xA5)
        B.snapshot_pack(plan, k, 3, ds.state, buf)
        torch.cuda.synchronize()
        exp = orc.pack(model, k, 3, ref_state)
        assert buf.cpu().numpy()[:exp.size].tobytes() == exp.tobytes()
        target = DeviceState(st_cpu, dev)
        target.poison()
        ref = target.to_oracle()
        ref_mask = np.zeros(wl.n_ops, dtype=np.uint8)
        orc.unpack(model, k, exp, ref, ref_mask)
        mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
        B.restore_unpack(plan, k, None, buf, target.state, mask)
        torch.cuda.synchronize()
        assert states_equal(target.to_oracle(), ref) == [] and target.guards_intact()
        assert np.array_equal(mask.cpu().numpy(), ref_mask)


def test_degenerate_slots(orc, dev):
    """Slots with no active operator (only compute weights), with nothing at all (header only), a
    window of one slot (dense checkpoint) and an alignment above the header size."""
    cases = [
        W.Workload("gap", [(0, 5000), (1, 33), (2, 70001)], [0, 3, 3], 5),      # slots 1, 2 compute-only; 4 empty
        W.Workload("dense", [(0, 4097), (1, 12)], [0, 0], 1),
    ]
    for wl in cases:
        for align in (16, 4096):
            model, plan = model_of(wl, align=align), make_plan(wl, align=align)
            st_cpu = W.random_bits_state(wl, seed=8)
            ref_state = state_of(st_cpu)
            ds = DeviceState(st_cpu, dev)
            buf = packed_buffer(plan, dev)
            for k in range(wl.window):
                buf.fill_(0xA5)
                B.snapshot_pack(plan, k, 9, ds.state, buf)
                torch.cuda.synchronize()
                exp = orc.pack(model, k, 9, ref_state)
                got = buf.cpu().numpy()
                assert got[:exp.size].tobytes() == exp.tobytes(), (wl.name, align, k)
                assert (got[exp.size:] == 0xA5).all()
                target = DeviceState(st_cpu, dev)
                target.poison()
                ref = target.to_oracle()
                ref_mask = np.full(wl.n_ops, 5, dtype=np.uint8)
                orc.unpack(model, k, exp, ref, ref_mask)
                mask = torch.full((wl.n_ops,), 5, dtype=torch.uint8, device=dev)
                B.restore_unpack(plan, k, None, buf, target.state, mask)
                torch.cuda.synchronize()
                B.ckpt_plan_device_status(plan)
                assert states_equal(target.to_oracle(), ref) == [] and target.guards_intact()
                assert np.array_equal(mask.cpu().numpy(), ref_mask)


@pytest.mark.parametrize("widths", [(2, 2, 2, 2), (4, 4, 4, 1), (2, 1, 2, 1), (1, 1, 2, 1)],
                         ids=["fp16_state", "fp8_compute", "fp8_m_fp16_v", "fp8_master"])
def test_low_precision_regimes_pack_unpack(orc, dev, widths):
    """Sec. 5.6 regimes: pack and unpack are byte copies whatever the element widths are (odd byte
    counts, 1-byte elements); no compute weights are derived outside the FP32-master regime."""
    wl = ragged_workload(60 + sum(widths), max_numel=30000)
    kinds_w = dict(zip(KINDS, widths))
    g = torch.Generator().manual_seed(7)
    st_cpu = {k: [torch.randint(0, 256, (n * kinds_w[k],), dtype=torch.uint8, generator=g) for _, n in wl.tensors]
              for k in KINDS}
    model = orc.Model(list(wl.tensors), list(wl.order), list(wl.slot_of_op), wl.window, 64, widths)
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order,
                       align=64, widths=widths)
    import oracle
    ref_state = oracle.State(*[[t.numpy().copy() for t in st_cpu[k]] for k in KINDS])
    ds = DeviceState(st_cpu, dev)
    buf = packed_buffer(plan, dev)
    for k in range(wl.window):
        buf.fill_(0xA5)
        B.snapshot_pack(plan, k, 4, ds.state, buf)
        torch.cuda.synchronize()
        exp = orc.pack(model, k, 4, ref_state)
        assert buf.cpu().numpy()[:exp.size].tobytes() == exp.tobytes()
        target = DeviceState(st_cpu, dev)
        for kind in KINDS:
            for v in target.views[kind]:
                v.fill_(0xEE)
        ref = oracle.State(*[[v.cpu().numpy().copy() for v in target.views[kk]] for kk in KINDS])
        ref_mask = np.zeros(wl.n_ops, dtype=np.uint8)
        orc.unpack(model, k, exp, ref, ref_mask)
        mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
        B.restore_unpack(plan, k, None, buf, target.state, mask)
        torch.cuda.synchronize()
        got = oracle.State(*[[v.cpu().numpy().copy() for v in target.views[kk]] for kk in KINDS])
        assert states_equal(got, ref) == [] and target.guards_intact()
        assert np.array_equal(mask.cpu().numpy(), ref_mask)


def test_pack_drain_restore_roundtrip_through_pinned_host(orc, dev):
    """pack -> drain (side stream, event-ordered) -> host bytes equal the oracle's snapshot;
    restore from the pinned copy (H2D + scatter) brings a poisoned state back: identity."""
    wl = ragged_workload(21, max_numel=200000)
    model = model_of(wl)
    st_cpu = W.make_state(wl, seed=3)
    ds = DeviceState(st_cpu, dev)
    ref_state = state_of(st_cpu)
    plan = make_plan(wl)
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    buf = packed_buffer(plan, dev)
    host = torch.empty(B.ckpt_plan_max_packed_bytes(plan), dtype=torch.uint8).pin_memory()
    for k in range(wl.window):
        packed_done, drained = torch.cuda.Event(), torch.cuda.Event()
        with torch.cuda.stream(main):
            B.snapshot_pack(plan, k, 7 + k, ds.state, buf, stream=main)
            packed_done.record(main)
        drained.record(side)  # create the event handle before handing it to the library
        B.snapshot_drain(plan, k, buf, host, side_stream=side, pack_done=packed_done, drained=drained)
        drained.synchronize()
        n = B.ckpt_plan_packed_bytes(plan, k)
        exp = orc.pack(model, k, 7 + k, ref_state)
        assert host.numpy()[:n].tobytes() == exp.tobytes()
        assert B.snapshot_peek(plan, k, host)["iter"] == 7 + k
        # restore into a poisoned copy through the host path
        target = DeviceState(st_cpu, dev)
        target.poison()
        ref = target.to_oracle()
        ref_mask = np.zeros(wl.n_ops, dtype=np.uint8)
        orc.unpack(model, k, exp, ref, ref_mask)
        mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
        buf2 = packed_buffer(plan, dev, k)
        B.restore_unpack(plan, k, host, buf2, target.state, mask, stream=main)
        main.synchronize()
        assert states_equal(target.to_oracle(), ref) == [] and target.guards_intact()
        assert np.array_equal(mask.cpu().numpy(), ref_mask)
        main.synchronize()
        side.synchronize()


def test_drain_through_a_ring_of_pinned_chunks(orc, dev):
    """A host that cannot pin a whole slot drains it in ranges through a small ring of pinned chunks; the
    reassembled bytes equal the oracle's snapshot (ragged last chunk, empty range, ranges outside the slot)."""
    wl = ragged_workload(27, max_numel=150000)
    model, plan = model_of(wl), make_plan(wl)
    st_cpu = W.make_state(wl, seed=9)
    ds, ref_state = DeviceState(st_cpu, dev), state_of(st_cpu)
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    chunk, n_chunks = 100_000, 3                     # not a multiple of anything
    ring = [torch.empty(chunk, dtype=torch.uint8).pin_memory() for _ in range(n_chunks)]
    events = [torch.cuda.Event() for _ in range(n_chunks)]
    buf = packed_buffer(plan, dev)
    for k in (0, wl.window - 1):
        packed_done = torch.cuda.Event()
        B.snapshot_pack(plan, k, 3, ds.state, buf, stream=main)
        packed_done.record(main)
        total = B.ckpt_plan_packed_bytes(plan, k)
        out = np.empty(total, dtype=np.uint8)
        offsets = list(range(0, total, chunk))
        for i, off in enumerate(offsets):
            slot_in_ring = i % n_chunks
            if i >= n_chunks:                        # consume the chunk that is about to be reused
                events[slot_in_ring].synchronize()
                prev = offsets[i - n_chunks]
                out[prev:prev + chunk] = ring[slot_in_ring].numpy()[:min(chunk, total - prev)]
            n = min(chunk, total - off)
            events[slot_in_ring].record(side)
            B.snapshot_drain_range(plan, k, buf, off, ring[slot_in_ring], n, side_stream=side,
                                   pack_done=packed_done if i == 0 else None, drained=events[slot_in_ring])
        side.synchronize()
        for i in range(max(0, len(offsets) - n_chunks), len(offsets)):
            off = offsets[i]
            out[off:off + chunk] = ring[i % n_chunks].numpy()[:min(chunk, total - off)]
        assert out.tobytes() == orc.pack(model, k, 3, ref_state).tobytes()
        B.snapshot_drain_range(plan, k, buf, total, None, 0, side_stream=side)          # empty range at the end
        for off, n in ((total, 1), (0, total + 1), (total + 5, 0)):
            with pytest.raises(B.MoevError) as e:
                B.snapshot_drain_range(plan, k, buf, off, ring[0], n, side_stream=side)
            assert e.value.code == B.E_RANGE


def test_fresh_plan_used_on_two_streams_without_host_synchronisation(orc, dev):
    """The plan's device tables are built by its first call, on that call's stream; the next call runs on
    another stream, ordered only by the caller's event on the data.  Pack on stream A, unpack (into another
    state, so the pointer table is rewritten) and replay on stream B: results equal the oracle's."""
    wl = ragged_workload(41, max_numel=300000)
    model, hp = model_of(wl), hp_of(wl)
    st_cpu = W.make_state(wl, seed=12)
    truth = state_of(st_cpu)
    grads_cpu = W.make_grads(wl, 11, seed=12)
    for k in (0, wl.window - 1):
        plan = make_plan(wl)                      # fresh: nothing uploaded yet
        src, dst = DeviceState(st_cpu, dev), DeviceState(st_cpu, dev)
        dst.poison()
        ref = dst.to_oracle()
        buf = packed_buffer(plan, dev, k)
        mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
        grads = [g.to(dev) for g in grads_cpu]
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        packed_ready = torch.cuda.Event()
        B.snapshot_pack(plan, k, 10, src.state, buf, stream=a)
        packed_ready.record(a)
        b.wait_event(packed_ready)
        B.restore_unpack(plan, k, None, buf, dst.state, mask, stream=b)
        B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, 11, mask,
                         [g if wl.slot_of_op[wl.tensors[t][0]] == k else None for t, g in enumerate(grads)], dst.state, stream=b)
        torch.cuda.synchronize()
        B.ckpt_plan_device_status(plan)
        ref_mask = np.zeros(wl.n_ops, dtype=np.uint8)
        orc.unpack(model, k, orc.pack(model, k, 10, truth), ref, ref_mask)
        orc.replay_step(model, hp, 11, ref_mask, [g.numpy() for g in grads_cpu], ref)
        assert states_equal(dst.to_oracle(), ref) == [] and dst.guards_intact()
        assert np.array_equal(mask.cpu().numpy(), ref_mask)


def test_conversion_window_captured_in_a_graph(orc, dev):
    """Launch-bound windows (configs[0]) can be replayed from a HIP graph: with resident tables the calls
    enqueue kernels only.  The graph is replayed several times with eager work and synchronisations in
    between, and every replay must reproduce the eager conversion; a call that would have to upload a table
    during capture is refused and records nothing."""
    wl = W.tiny_moe()
    hp = hp_of(wl)
    st_cpu = W.make_state(wl, seed=5)
    plan = make_plan(wl)
    live = DeviceState(st_cpu, dev)
    everyone = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    per_iter = {t: [g.to(dev) for g in W.make_grads(wl, t, seed=5)] for t in range(wl.t0 + 1, wl.t0 + wl.window + 1)}
    gbuf = [torch.empty_like(g) for g in per_iter[wl.t0 + 1]]     # persistent gradient buffers: constant pointers
    bufs = []
    for k in range(wl.window):
        bufs.append(packed_buffer(plan, dev, k))
        B.snapshot_pack(plan, k, wl.t0 + k, live.state, bufs[k])
        B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, wl.t0 + k + 1, everyone,
                         per_iter[wl.t0 + k + 1], live.state)
    torch.cuda.synchronize()
    rebuilt = DeviceState(st_cpu, dev)
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)

    def window():
        mask.zero_()
        for i in range(wl.window):
            for dst, src in zip(gbuf, per_iter[wl.t0 + i + 1]):
                dst.copy_(src)
            B.restore_unpack(plan, i, None, bufs[i], rebuilt.state, mask, stream=torch.cuda.current_stream())
            B.convert_replay(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, wl.t0 + i + 1, mask, gbuf,
                             rebuilt.state, stream=torch.cuda.current_stream())

    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        rebuilt.poison()
        window()                                   # eager: also makes the plan's tables resident
        s.synchronize()
        eager = rebuilt.to_oracle()
        assert states_equal(eager, live.to_oracle()) == []
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            window()
        for rep in range(3):
            rebuilt.poison()                       # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert states_equal(rebuilt.to_oracle(), eager) == [], f"replay {rep}"
            assert bool(mask.cpu().all()) and rebuilt.guards_intact()
        B.ckpt_plan_device_status(plan, s)
        # another state (other pointers) inside a capture: refused, nothing recorded, the capture stays valid
        other = DeviceState(st_cpu, dev)
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2, stream=s):
            with pytest.raises(B.MoevError) as e:
                B.restore_unpack(plan, 0, None, bufs[0], other.state, mask, stream=torch.cuda.current_stream())
            assert e.value.code == B.E_INVAL
            mask.zero_()
        g2.replay()
        torch.cuda.synchronize()
        assert states_equal(other.to_oracle(), state_of(st_cpu)) == []


def test_foreign_snapshots_are_refused(orc, dev):
    """Host path: MISMATCH before anything is enqueued.  Device path: the kernel skips the scatter
    and raises the status word; the state stays as it was."""
    wl = ragged_workload(31)
    model, plan = model_of(wl), make_plan(wl)
    st_cpu = W.random_bits_state(wl, seed=1)
    ds = DeviceState(st_cpu, dev)
    before = ds.to_oracle()
    snap1 = orc.pack(model, 1, 5, state_of(st_cpu))
    host = torch.from_numpy(snap1.copy()).pin_memory()
    buf = packed_buffer(plan, dev)
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    with pytest.raises(B.MoevError) as e:
        B.restore_unpack(plan, 0, host, buf, ds.state, mask)      # slot-1 snapshot offered as slot 0
    assert e.value.code == B.E_MISMATCH
    buf.zero_()
    buf[:snap1.size].copy_(torch.from_numpy(snap1))
    B.restore_unpack(plan, 2, None, buf, ds.state, mask)          # device-resident, wrong slot
    torch.cuda.synchronize()
    with pytest.raises(B.MoevError) as e:
        B.ckpt_plan_device_status(plan)
    assert e.value.code == B.E_MISMATCH
    B.ckpt_plan_device_status(plan)                               # reading cleared it
    assert states_equal(ds.to_oracle(), before) == [] and not mask.any().item()


def test_host_side_argument_checks(dev):
    wl = W.tiny_moe(d_in=8, d_hidden=16)
    plan = make_plan(wl)
    st = W.make_state(wl, seed=0, device=dev)
    state = B.State(st["master"], st["m"], st["v"], st["compute"])
    buf = packed_buffer(plan, dev)
    with pytest.raises(B.MoevError) as e:
        B.snapshot_pack(plan, wl.window, 0, state, buf)
    assert e.value.code == B.E_RANGE
    with pytest.raises(B.MoevError) as e:
        B.snapshot_pack(plan, 0, 0, state, buf, cap=B.ckpt_plan_packed_bytes(plan, 0) - 1)
    assert e.value.code == B.E_RANGE
    with pytest.raises(B.MoevError) as e:
        B.snapshot_pack(plan, 0, 0, state, buf.data_ptr() + 16, cap=buf.numel() - 16)
    assert e.value.code == B.E_INVAL
    skew = [t for t in st["master"]]
    skew[0] = torch.empty(skew[0].numel() + 4, dtype=torch.float32, device=dev)[1:1 + skew[0].numel()]
    with pytest.raises(B.MoevError) as e:
        B.snapshot_pack(plan, 0, 0, B.State(skew, st["m"], st["v"], st["compute"]), buf)
    assert e.value.code == B.E_INVAL
    mask = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    grads = W.make_grads(wl, 11, device=dev)
    with pytest.raises(B.MoevError) as e:
        B.convert_replay(plan, 1e-4, 0.9, 0.95, 1e-8, 0.0, 0, mask, grads, state)   # step counts from 1
    assert e.value.code == B.E_INVAL
    # an active operator without gradients is skipped and reported, never dereferenced
    grads[0] = None
    before = st["master"][0].clone()
    B.convert_replay(plan, 1e-4, 0.9, 0.95, 1e-8, 0.0, 11, mask, grads, state)
    torch.cuda.synchronize()
    with pytest.raises(B.MoevError) as e:
        B.ckpt_plan_device_status(plan)
    assert e.value.code == B.E_INVAL and torch.equal(before, st["master"][0])


def test_measurement_probes_move_what_they_say(dev):
    """The copy / read-only / write-only / paired-copy probes (the yardsticks of bench.py): the copy is exact including a ragged
    last tile, the write probe fills exactly its range, the read probe leaves its sink alone, bad arguments are refused."""
    n = (1 << 20) + 4096 + 48
    src = torch.randint(0, 255, (n + 64,), dtype=torch.uint8, device=dev)
    dst = torch.full((n + 64,), 0xEE, dtype=torch.uint8, device=dev)
    for blocks in (0, 7):
        dst.fill_(0xEE)
        B.moev_copy_probe(dst, src, n, blocks, 1)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src[:n]) and bool((dst[n:] == 0xEE).all())
    dst.fill_(0xEE)
    B.moev_stream_probe(2, dst, None, n, 0x04030201, 0)
    torch.cuda.synchronize()
    want = torch.tensor([1, 2, 3, 4], dtype=torch.uint8, device=dev).repeat(n // 4)
    assert torch.equal(dst[:n], want) and bool((dst[n:] == 0xEE).all())
    dst.fill_(0xEE)
    B.moev_stream_probe(1, dst, src, n, 0, 1)
    torch.cuda.synchronize()
    assert bool((dst == 0xEE).all())
    # paired copy: two 512-byte pieces per wavefront instruction, `value` bytes apart; blocks of twice that, aligned
    arena_s = torch.randint(0, 255, ((1 << 20) * 3,), dtype=torch.uint8, device=dev)
    arena_d = torch.full(((1 << 20) * 3,), 0xEE, dtype=torch.uint8, device=dev)
    bs, bd = (-arena_s.data_ptr()) % (1 << 20), (-arena_d.data_ptr()) % (1 << 20)
    for dist, size in ((512, 5 * 1024), (32768, 1 << 20), (32768, 3 << 16), (1 << 19, 1 << 20)):
        arena_d.fill_(0xEE)
        B.moev_stream_probe(3, arena_d[bd:], arena_s[bs:], size, dist, 1)
        torch.cuda.synchronize()
        assert torch.equal(arena_d[bd:bd + size], arena_s[bs:bs + size]), (dist, size)
        assert bool((arena_d[:bd] == 0xEE).all()) and bool((arena_d[bd + size:] == 0xEE).all())
    for bad in (lambda: B.moev_stream_probe(4, dst, src, n), lambda: B.moev_stream_probe(1, dst, src, n + 1),
                lambda: B.moev_stream_probe(3, arena_d[bd:], arena_s[bs:], 1 << 20, 3000),
                lambda: B.moev_stream_probe(3, arena_d[bd:], arena_s[bs:], 1 << 20, 256),
                lambda: B.moev_stream_probe(3, arena_d[bd:], arena_s[bs:], (1 << 20) + 4096, 32768),
                lambda: B.moev_stream_probe(3, arena_d[bd + 4096:], arena_s[bs:], 1 << 16, 32768),
                lambda: B.moev_stream_probe(1, dst, None, n), lambda: B.moev_stream_probe(2, dst[1:], None, n)):
        with pytest.raises(B.MoevError) as e:
            bad()
        assert e.value.code == B.E_INVAL


# ---------------------------------------------------------------------------------------
# Adam replay
# ---------------------------------------------------------------------------------------
def _compare_adam(ds, ref, label=""):
    got = ds.to_oracle()
    worst = 0.0
    for kind in ("master", "m", "v"):
        for t, (x, y) in enumerate(zip(got.kinds()[kind], ref.kinds()[kind])):
            err = max_rel_err(x, y)
            assert err <= REL_TOL, f"{label} {kind}[{t}] max rel err {err}"
            worst = max(worst, err)
    import oracle
    for t, (c, p, cr, pr) in enumerate(zip(got.compute, got.master, ref.compute, ref.master)):
        same = p.view(np.uint32) == pr.view(np.uint32)
        assert np.array_equal(c[same], cr[same]), f"{label} compute[{t}]"
        if not same.all():  # where the master differs in the last bits, compute must be the cast of the GPU's own master
            idx = np.nonzero(~same)[0][:64]
            assert np.array_equal(c[idx], oracle.bf16_rne_array(p[idx]))
    return worst


@pytest.mark.parametrize("paired", [1, 0], ids=["paired_tiles", "consecutive_tiles"])
@pytest.mark.parametrize("plain", [1, 0], ids=["plain_divide_sqrt", "full_divide_sqrt"])
@pytest.mark.parametrize("seed,wd,heavy,adam_tile,blocks,nt,shape", [
    (1, 0.0, False, None, None, 1, None), (2, 0.1, True, None, None, 0, (64, 1)), (3, 0.0, True, None, None, 1, (512, 2)),
    (4, 0.01, False, None, None, 1, (256, 4)), (5, 0.0, False, None, None, 0, (1024, 1)),
    (1, 0.0, False, 8192, None, 1, None), (2, 0.1, True, 1024, 3, 1, None), (3, 0.0, True, 4096, 1, 0, None),
    (4, 0.01, False, 16384, 9, 0, None),
])
def test_adam_replay_matches_oracle(orc, dev, seed, wd, heavy, adam_tile, blocks, nt, shape, plain, paired):
    """One replayed iteration on ragged tensors with a mixed active/frozen mask: FP32 state within
    1e-6 relative of the oracle (expected bit-identical), frozen tensors and guards untouched.  Both
    with the plain division / square-root sequences where the operands allow them (the default) and
    with the compiler's full IEEE sequences everywhere."""
    wl = ragged_workload(40 + seed)
    wl.weight_decay, wl.heavy_tail = wd, heavy
    model, hp = model_of(wl), hp_of(wl)
    st_cpu = W.make_state(wl, seed=seed)
    ds = DeviceState(st_cpu, dev)
    ref = state_of(st_cpu)
    if not paired and (shape not in (None, (64, 1)) or adam_tile):
        pytest.skip("the paired tiles exist for the 64 x 1 one-tile-per-workgroup shape only: nothing to switch off")
    plan = make_plan(wl, adam_tile=adam_tile, adam_blocks=blocks, nt=nt, adam_shape=shape, paired=paired)
    B.moev_tune(plan, B.TUNE_PLAIN_DIVIDE_SQRT, plain)
    rng = np.random.default_rng(seed)
    mask_np = (rng.random(wl.n_ops) < 0.6).astype(np.uint8)
    mask_np[0] = 1
    mask = torch.from_numpy(mask_np).to(dev)
    for step in (11, 12, 13):
        grads_cpu = W.make_grads(wl, step, seed=seed)
        grads_dev = [g.to(dev) for g in grads_cpu]
        if step == 12:  # frozen operators have no weight gradients: their entries may be missing
            grads_dev = [g if mask_np[wl.tensors[t][0]] else None for t, g in enumerate(grads_dev)]
        B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, step, mask, grads_dev, ds.state)
        torch.cuda.synchronize()
        orc.replay_step(model, hp, step, mask_np, [np_of(g) for g in grads_cpu], ref)
    B.ckpt_plan_device_status(plan)
    worst = _compare_adam(ds, ref, "ragged")
    assert ds.guards_intact()
    exact = states_equal(ds.to_oracle(), ref) == []
    print(f"adam seed {seed}: worst rel err {worst:.3g}, bit-identical={exact}")


@pytest.mark.parametrize("plain", [1, 0], ids=["plain_divide_sqrt", "full_divide_sqrt"])
def test_adam_special_values(orc, dev, plain):
    """NaN / Inf / denormal / zero inputs propagate exactly as in the oracle (no flushing)."""
    n = 4096 + 3
    wl = W.Workload("special", [(0, n)], [0], 1)
    model, hp = model_of(wl), hp_of(wl)
    st_cpu = W.make_state(wl, seed=9)
    specials = torch.tensor([0.0, -0.0, float("inf"), -float("inf"), float("nan"), 1e-45, -1e-45, 1e-39, 3e38, -3e38,
                             1.17549435e-38, 1e-20], dtype=torch.float32)
    g = W.make_grads(wl, 11, seed=9)[0]
    k = specials.numel()
    st_cpu["master"][0][:k] = specials
    st_cpu["m"][0][k:2 * k] = specials
    st_cpu["v"][0][2 * k:3 * k] = specials.abs()
    g[3 * k:4 * k] = specials
    g[4 * k:5 * k] = 0.0
    st_cpu["v"][0][4 * k:5 * k] = 0.0
    st_cpu["m"][0][4 * k:5 * k] = 0.0        # 0/(0+eps) = 0
    ds = DeviceState(st_cpu, dev)
    ref = state_of(st_cpu)
    plan = make_plan(wl)
    B.moev_tune(plan, B.TUNE_PLAIN_DIVIDE_SQRT, plain)
    mask = torch.ones(1, dtype=torch.uint8, device=dev)
    B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, 0.0, 11, mask, [g.to(dev)], ds.state)
    torch.cuda.synchronize()
    orc.replay_step(model, hp, 11, np.ones(1, dtype=np.uint8), [np_of(g)], ref)
    _compare_adam(ds, ref, "special")
    got = ds.to_oracle()
    for kind in ("master", "m", "v"):
        assert np.array_equal(np.isnan(got.kinds()[kind][0]), np.isnan(ref.kinds()[kind][0]))


# ---------------------------------------------------------------------------------------
# whole window: snapshots during a dense run, then sparse-to-dense conversion
# ---------------------------------------------------------------------------------------
def _gpu_window(orc, dev, wl, seed, align=256, via_host=False, fused=False, **tune):
    """Dense GPU run with per-iteration snapshots, then GPU conversion from them; returns the GPU's
    converted state, the oracle's dense-run state and the oracle's snapshots."""
    model, hp = model_of(wl, align=align), hp_of(wl)
    st_cpu = W.make_state(wl, seed=seed)
    grads_cpu = {t: W.make_grads(wl, t, seed=seed) for t in range(wl.t0 + 1, wl.t0 + wl.window + 1)}
    grads_dev = {t: [g.to(dev) for g in gs] for t, gs in grads_cpu.items()}
    # oracle: dense truth + snapshots
    dense = state_of(st_cpu)
    snaps = orc.dense_run(model, dense, hp, lambda t: [np_of(g) for g in grads_cpu[t]], wl.t0, wl.window, snapshots=True)
    # GPU: same dense run, snapshot SS_{t0+k} packed from the state after step t0+k
    plan = make_plan(wl, align=align, **tune)
    live = DeviceState(st_cpu, dev)
    everyone = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    bufs = []
    for k in range(wl.window):
        buf = packed_buffer(plan, dev, k)
        B.snapshot_pack(plan, k, wl.t0 + k, live.state, buf)
        bufs.append(buf)
        B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.t0 + k + 1, everyone,
                         grads_dev[wl.t0 + k + 1], live.state)
    torch.cuda.synchronize()
    for k in range(wl.window):
        assert bufs[k].cpu().numpy()[:snaps[k].size].tobytes() == snaps[k].tobytes(), f"snapshot {k}"
    # GPU: conversion into a poisoned state
    rebuilt = DeviceState(st_cpu, dev)
    rebuilt.poison()
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    for i in range(wl.window):
        host = None
        if via_host:
            host = bufs[i].cpu().pin_memory()
            bufs[i].fill_(0)
        if fused:
            # frozen operators have no gradients; the fused call reads the new operators' FP32 state from the snapshot
            g = [x if wl.slot_of_op[wl.tensors[t][0]] <= i else None for t, x in enumerate(grads_dev[wl.t0 + i + 1])]
            B.convert_window_step(plan, i, host, bufs[i], wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay,
                                  wl.t0 + i + 1, mask, g, rebuilt.state)
        else:
            B.restore_unpack(plan, i, host, bufs[i], rebuilt.state, mask)
            B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.t0 + i + 1, mask,
                             grads_dev[wl.t0 + i + 1], rebuilt.state)
        torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)
    assert mask.all().item()
    return rebuilt, live, dense


@pytest.mark.parametrize("fused", [False, True], ids=["two_calls", "fused_step"])
def test_window_tiny_config(orc, dev, fused):
    """configs[0]: snapshots bit-exact, converted state == the GPU's own dense run bitwise and
    within 1e-6 relative of the oracle's brute-force dense Adam run."""
    wl = W.tiny_moe()
    rebuilt, live, dense = _gpu_window(orc, dev, wl, seed=0, fused=fused)
    assert states_equal(rebuilt.to_oracle(), live.to_oracle()) == []
    _compare_adam(rebuilt, dense, "c0")
    assert rebuilt.guards_intact() and live.guards_intact()


@pytest.mark.parametrize("fused", [False, True], ids=["two_calls", "fused_step"])
def test_window_conversion_stress_small(orc, dev, fused):
    """A shrunken configs[4]: 2 layers x (16 routed + 2 shared), W = 8, permuted schedule, heavy-tailed
    gradients, restore through pinned host memory."""
    wl = W.conversion_stress(n_layers=2, n_routed=16, n_shared=2, d_model=64, d_ff=44, per_slot=2)
    assert wl.window == 8
    tune = {} if fused else dict(tile=4096, adam_tile=1024)
    rebuilt, live, dense = _gpu_window(orc, dev, wl, seed=4, via_host=True, fused=fused, **tune)
    assert states_equal(rebuilt.to_oracle(), live.to_oracle()) == []
    _compare_adam(rebuilt, dense, "c4-small")


@pytest.mark.parametrize("fused", [False, True], ids=["two_calls", "fused_step"])
def test_window_ragged_direct_shapes(orc, dev, fused):
    wl = ragged_workload(78, n_ops=9, window=3, with_empty=True)
    rebuilt, live, dense = _gpu_window(orc, dev, wl, seed=6, align=64, fused=fused, copy_shape=(512, 2), adam_shape=(128, 1))
    assert states_equal(rebuilt.to_oracle(), live.to_oracle()) == []
    _compare_adam(rebuilt, dense, "ragged-window-direct")
    assert rebuilt.guards_intact()


def test_fused_step_refuses_foreign_snapshot_and_missing_gradients(orc, dev):
    """The fused step modifies nothing when the device-resident snapshot is not the slot's, and
    insists on gradients for the operators it activates."""
    wl = ragged_workload(33)
    model, plan = model_of(wl), make_plan(wl)
    st_cpu = W.make_state(wl, seed=2)
    ds = DeviceState(st_cpu, dev)
    before = ds.to_oracle()
    snap = orc.pack(model, 1, 5, state_of(st_cpu))
    buf = packed_buffer(plan, dev)
    buf.zero_()
    buf[:snap.size].copy_(torch.from_numpy(snap))
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    grads = [g.to(dev) for g in W.make_grads(wl, 6, seed=2)]
    B.convert_window_step(plan, 2, None, buf, wl.lr, wl.beta1, wl.beta2, wl.eps, 0.0, 6, mask, grads, ds.state)
    torch.cuda.synchronize()
    with pytest.raises(B.MoevError) as e:
        B.ckpt_plan_device_status(plan)
    assert e.value.code == B.E_MISMATCH
    assert states_equal(ds.to_oracle(), before) == [] and not mask.any().item() and ds.guards_intact()
    first_active = next(t for t, (op, n) in enumerate(wl.tensors) if wl.slot_of_op[op] == 1 and n)
    grads[first_active] = None
    with pytest.raises(B.MoevError) as e:
        B.convert_window_step(plan, 1, None, buf, wl.lr, wl.beta1, wl.beta2, wl.eps, 0.0, 6, mask, grads, ds.state)
    assert e.value.code == B.E_INVAL


@pytest.mark.parametrize("regions", [0, 1, 2, 64, 4096, 65536], ids=["off", "eighths", "chunk2", "chunk64", "chunk4096", "chunk65536"])
@pytest.mark.parametrize("fused", [False, True], ids=["two_calls", "fused_step"])
def test_window_with_every_xcd_mapping(orc, dev, fused, regions):
    """The workgroup -> tile mappings of the one-tile-per-workgroup kernels: consecutive, an eighth of the tiles per XCD,
    chunks of G tiles dealt round robin (smaller and far larger than the launches of this workload)."""
    wl = ragged_workload(79, n_ops=10, window=4, with_empty=True)
    rebuilt, live, dense = _gpu_window(orc, dev, wl, seed=7, align=256, fused=fused, xcd_regions=regions)
    assert states_equal(rebuilt.to_oracle(), live.to_oracle()) == []
    _compare_adam(rebuilt, dense, "ragged-window-no-regions")
    assert rebuilt.guards_intact()


@pytest.mark.parametrize("fused", [False, True], ids=["two_calls", "fused_step"])
def test_window_with_consecutive_tiles(orc, dev, fused):
    """The replay's paired tiles switched off (every wavefront takes 1 KB of consecutive bytes per stream)."""
    wl = ragged_workload(80, n_ops=10, window=4, with_empty=True)
    rebuilt, live, dense = _gpu_window(orc, dev, wl, seed=8, align=256, fused=fused, paired=0)
    assert states_equal(rebuilt.to_oracle(), live.to_oracle()) == []
    _compare_adam(rebuilt, dense, "ragged-window-consecutive")
    assert rebuilt.guards_intact()


@pytest.mark.parametrize("distance", [None, 512, 2048, 65536, 1 << 20], ids=["default_32KiB", "512B", "2KiB", "64KiB", "1MiB"])
def test_paired_tiles_cover_every_element_for_any_pointer_alignment(orc, dev, distance):
    """The paired tile grid follows the address of the master weights: tensors of block-multiple and ragged lengths at
    every kind of offset inside a 64 KiB block (0, 16 bytes, just below 32 KiB, just above, just below 64 KiB), with the
    other streams at other offsets: every element is updated exactly once, nothing outside is touched.  Also for the
    other piece distances the knob accepts (they exist for sweeps)."""
    lengths = [16384 * 3, 16384 * 2 + 8192, 16384 + 1, 8191, 257, 3, 40000, 1]
    offsets = [0, 16, 32768 - 16, 32768 + 512, 65536 - 16, 4096, 16384, 49152 + 48]
    wl = W.Workload("aligned", [(e, n) for e, n in enumerate(lengths)], [0] * len(lengths), 1)
    model, hp = model_of(wl), hp_of(wl)
    st_cpu = W.make_state(wl, seed=31)
    grads_cpu = W.make_grads(wl, 11, seed=31)
    ref = state_of(st_cpu)
    orc.replay_step(model, hp, 11, np.ones(wl.n_ops, dtype=np.uint8), [np_of(g) for g in grads_cpu], ref)
    guard = 256
    views, arenas = {k: [] for k in KINDS}, []
    for t, n in enumerate(lengths):
        for q, kind in enumerate(KINDS + ("grad",)):
            width = 2 if kind == "compute" else 4
            off = offsets[(t + 3 * q) % len(offsets)] if kind != "master" else offsets[t]
            arena = torch.full((65536 * 2 + off + n * width + guard,), 0x5A, dtype=torch.uint8, device=dev)
            base = (-arena.data_ptr()) % 65536 + off           # the tensor starts `off` bytes into a 64 KiB block
            src = grads_cpu[t] if kind == "grad" else st_cpu[kind][t]
            view = arena[base: base + n * width].view(src.dtype)
            view.copy_(src)
            assert view.data_ptr() % 65536 == off
            arenas.append((arena, base, n * width))
            if kind == "grad":
                views.setdefault("grad", []).append(view)
            else:
                views[kind].append(view)
    plan = make_plan(wl, paired=distance)
    assert B.moev_tune_get(plan, B.TUNE_PAIRED_TILES) == (distance or 32768)
    for bad in (3, 256, 48 * 1024, 8 << 20, -4):
        with pytest.raises(B.MoevError) as e:
            B.moev_tune(plan, B.TUNE_PAIRED_TILES, bad)
        assert e.value.code == B.E_INVAL
    mask = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, 11, mask, views["grad"],
                     B.State(*[views[k] for k in KINDS]))
    torch.cuda.synchronize()
    B.ckpt_plan_device_status(plan)
    import oracle
    got = oracle.State(*[[np_of(v) for v in views[k]] for k in KINDS])
    for k in ("master", "m", "v"):
        for t, (x, y) in enumerate(zip(got.kinds()[k], ref.kinds()[k])):
            assert max_rel_err(x, y) <= REL_TOL, f"{k}[{t}] (length {lengths[t]}, offset {offsets[t]})"
    for t, (c, p, cr, pr) in enumerate(zip(got.compute, got.master, ref.compute, ref.master)):
        same = p.view(np.uint32) == pr.view(np.uint32)
        assert np.array_equal(c[same], cr[same]), f"compute[{t}]"
    for arena, base, nbytes in arenas:
        a = arena.cpu().numpy()
        assert (a[:base] == 0x5A).all() and (a[base + nbytes:] == 0x5A).all()


def test_window_ragged_small_grid(orc, dev):
    wl = ragged_workload(77, n_ops=9, window=3, with_empty=True)
    rebuilt, live, dense = _gpu_window(orc, dev, wl, seed=5, align=16, tile=4096, blocks=2, adam_tile=1024, adam_blocks=2)
    assert states_equal(rebuilt.to_oracle(), live.to_oracle()) == []
    _compare_adam(rebuilt, dense, "ragged-window")


def test_recovery_from_a_failure_mid_run(orc, dev):
    """Sec. 3.6 end to end on the GPU: snapshots every iteration (slot (t - t0) mod W) packed and
    drained to pinned host memory while the run goes on; at a failure the live state is discarded,
    the last complete window is converted from the host copies (fused load + replay), the remaining
    iterations are re-executed, and the result equals the uninterrupted run bit for bit (and the
    oracle's uninterrupted run within 1e-6)."""
    wl = ragged_workload(91, n_ops=8, window=3, max_numel=40000, with_empty=False)
    model, hp = model_of(wl), hp_of(wl)
    w, t0 = wl.window, wl.t0
    last = t0 + 3 * w + 1
    st_cpu = W.make_state(wl, seed=11)
    grads_cpu = {t: W.make_grads(wl, t, seed=11) for t in range(t0 + 1, last + 1)}
    grads_dev = {t: [g.to(dev) for g in gs] for t, gs in grads_cpu.items()}
    # oracle: uninterrupted run
    ref = state_of(st_cpu)
    ref_states = {}
    everyone_np = np.ones(wl.n_ops, dtype=np.uint8)
    for t in range(t0, last):
        orc.replay_step(model, hp, t + 1, everyone_np, [np_of(g) for g in grads_cpu[t + 1]], ref)
        ref_states[t + 1] = ref.clone()
    # GPU: uninterrupted run with a snapshot + drain per iteration
    plan = make_plan(wl)
    live = DeviceState(st_cpu, dev)
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    everyone = torch.ones(wl.n_ops, dtype=torch.uint8, device=dev)
    cap = B.ckpt_plan_max_packed_bytes(plan)
    d_buf = [torch.empty(cap, dtype=torch.uint8, device=dev) for _ in range(2)]   # double buffer
    buf_free = [torch.cuda.Event(), torch.cuda.Event()]
    host, gpu_states = {}, {}
    for t in range(t0, last):
        b = (t - t0) % 2
        host[t] = torch.empty(cap, dtype=torch.uint8).pin_memory()
        if t - t0 >= 2:
            main.wait_event(buf_free[b])     # the drain of two iterations ago has released the buffer
        packed_done = torch.cuda.Event()
        B.snapshot_pack(plan, (t - t0) % w, t, live.state, d_buf[b], stream=main)
        packed_done.record(main)
        B.snapshot_drain(plan, (t - t0) % w, d_buf[b], host[t], side_stream=side, pack_done=packed_done)
        buf_free[b].record(side)
        B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, t + 1, everyone, grads_dev[t + 1],
                         live.state, stream=main)
        main.synchronize()
        gpu_states[t + 1] = live.to_oracle()
    side.synchronize()
    for fail_at in (t0 + w, t0 + 2 * w - 1, t0 + 2 * w + 1, last):
        s = t0 + ((fail_at - t0) // w - 1) * w
        rebuilt = DeviceState(st_cpu, dev)
        rebuilt.poison()
        mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
        scratch = torch.empty(cap, dtype=torch.uint8, device=dev)
        for i in range(w):
            assert B.snapshot_peek(plan, i, host[s + i])["iter"] == s + i
            g = [x if wl.slot_of_op[wl.tensors[k][0]] <= i else None for k, x in enumerate(grads_dev[s + i + 1])]
            B.convert_window_step(plan, i, host[s + i], scratch, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay,
                                  s + i + 1, mask, g, rebuilt.state, stream=main)
            main.synchronize()
        for t in range(s + w, fail_at):
            B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, t + 1, everyone,
                             grads_dev[t + 1], rebuilt.state, stream=main)
        main.synchronize()
        B.ckpt_plan_device_status(plan)
        assert states_equal(rebuilt.to_oracle(), gpu_states[fail_at]) == [], f"failure at {fail_at}"
        _compare_adam(rebuilt, ref_states[fail_at], f"recovery at {fail_at}")
        assert rebuilt.guards_intact()
