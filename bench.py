#!/usr/bin/env python3
"""bench.py -- throughput of the sparse-snapshot / sparse-to-dense hot path on one MI355X.

One "step" is one pass of the whole HBM-resident hot path over one window of the workload:
    for every slot k:  snapshot_pack(k)                       (Sec. 3.2)
    for every slot i:  restore_unpack(i); convert_replay(t0+i+1)   (Sec. 3.3)
with the state, the gradients and the packed snapshots resident in HBM.  `value` is the
algorithmic HBM bytes of a step divided by its wall time.  The device-to-host drain is bound by
the host link, not by HBM; it is measured right after the timed steps and reported in its own
object (it never enters `value`).

Prints ONE JSON line.  Default: configs[1] (Mixtral-8x7B-shaped MoE layer; FP32 master weights and moments with bf16
compute weights) as the headline, then configs[2], [3] and [4] as complete results under `configs`; --config runs one
workload alone, --regime stores the state as one of the low-precision regimes of Sec. 5.6.  Besides the contract's
fields the line carries per-kernel figures (`kernels`), the fused conversion, the copy probe, the drain (whole and
chunked), the upstream-log ring, a what-if (Algorithm 1 / recovery bounds / ETTR from the measured rates) and the
oracle's CPU baseline.  --knob-sweep, --paired-tiles-sweep and --pair-distance-sweep add comparisons of the launch knobs
made inside this one process (same tensors, same physical placement).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# vector-ALU issue peak: 256 compute units x 4 SIMDs x 16 lanes per clock x 2.4 GHz (lane-instructions per second);
# the published 157.3 TFLOP/s of FP32 vector math is this figure x 2 (a fused multiply-add) x 2 (packed pairs)
VALU_PEAK_GOPS = 256 * 4 * 16 * 2.4
METRIC = "snapshot pack/restore GB/s (% HBM peak) + convert_replay iters/s, 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="all", choices=["all", "c0", "c1", "c2", "c3", "c4"],
                    help="all (default): configs[1] is the headline (the contract's fields describe it) and the line also "
                         "carries configs[2], configs[3] and configs[4] under `configs`; cN: that workload alone")
    ap.add_argument("--sub-steps", type=int, default=10, help="timed steps of each workload under `configs` (3 warm-up steps)")
    ap.add_argument("--regime", default="fp32", help="precision regime of the training state: fp32 (FP32 master weights and "
                    "moments, bf16 compute weights; the default) or one of the low-precision regimes of Sec. 5.6: "
                    "fp16_fp16_fp16+fp16, fp8_fp32_fp32+fp32, fp8_fp16_fp32+fp32, fp8_fp16_fp8+fp16, fp8_fp8_fp8+fp16 "
                    "(compute_master_optimizer)")
    ap.add_argument("--no-drain", action="store_true", help="skip the host-link drain measurement")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--overlap", action="store_true", help="also time the drain under a concurrent bf16 GEMM loop")
    ap.add_argument("--overlap-slot", type=int, default=-1, help="configs[3]: slot of the overlap / drain measurements; default the "
                    "last one (19.3 GB, what this box can pin in one piece; slot 0 is 41.9 GB)")
    ap.add_argument("--cu-mask-sweep", action="store_true", help="configs[3]: also run the pack on side streams restricted to "
                    "192, 128, 96, 64 and 32 compute units (hipExtStreamCreateWithCUMask) against the GEMM loop")
    ap.add_argument("--persistent", action="store_true", help="fixed-grid launch shape (LDS-staged tile table)")
    ap.add_argument("--copy-tile", type=int, default=0)
    ap.add_argument("--adam-tile", type=int, default=0)
    ap.add_argument("--copy-blocks", type=int, default=0)
    ap.add_argument("--adam-blocks", type=int, default=0)
    ap.add_argument("--alloc", default="tensor", choices=["flat", "tensor", "skewed"], help="how the bench allocates the training state and the "
                    "gradients: flat = one flat buffer per kind / per iteration with the tensors as views (what flat-partition "
                    "optimizers do), tensor = every tensor its own allocation (the default), skewed = flat with every kind starting at "
                    "another offset inside a 64 KiB block.  The library sees pointers either way")
    ap.add_argument("--adam-shape", default="", help="one-tile-per-workgroup shape of the replay as THREADSxUNROLL, e.g. 64x2 "
                    "(default: the library's choice, 64x1 in the fp32 regime)")
    ap.add_argument("--nontemporal", type=int, default=-1)
    ap.add_argument("--xcd-regions", type=int, default=-1, help="replay: 0 consecutive workgroups take consecutive tiles, 1 every XCD sweeps an "
                    "eighth of the tiles (default), G >= 2: chunks of G tiles dealt to the XCDs round robin")
    ap.add_argument("--copy-xcd-regions", type=int, default=-1, help="the same for pack and unpack (default 64)")
    ap.add_argument("--paired-tiles", type=int, default=-1, help="replay: distance in bytes between the two 512-byte pieces a wavefront "
                    "takes per stream (default 32768; a power of two in [512, 4 MiB]); 0: 1 KB of consecutive bytes")
    ap.add_argument("--paired-tiles-sweep", action="store_true", help="after the timed steps: the replay of the last window iteration "
                    "timed at every piece distance from 512 B to 4 MiB in this process (same tensors, same placement)")
    ap.add_argument("--knob-sweep", action="store_true", help="after the timed steps: pack, unpack and replay timed under every launch knob "
                    "and one-tile-per-workgroup shape in this process (same tensors, same placement)")
    ap.add_argument("--pair-distance-sweep", action="store_true", help="copy probe with two 512-byte pieces per wavefront instruction, "
                    "swept over their distance (512 B .. 2 MiB): shows the address bit the paired tiles exploit")
    ap.add_argument("--plain-divide-sqrt", type=int, default=-1, help="0: always the full IEEE division / square-root sequences in the replay")
    ap.add_argument("--seed", type=int, default=0)
    return ap.parse_args()


# ---------------------------------------------------------------------------------------
# algorithmic bytes: what the method itself must move per slot and per replayed iteration
# ---------------------------------------------------------------------------------------
FP32_WIDTHS = (4, 4, 4, 2)                         # bytes per element of master, Adam m, Adam v, compute


ALLOC_TEXT = {"tensor": "one allocation per tensor", "flat": "one flat buffer per kind",
              "skewed": "one flat buffer per kind, the kinds at different offsets modulo 64 KiB"}


def pack_bytes(wl, k, widths=FP32_WIDTHS):
    return 2 * wl.slot_payload_bytes(k, widths)    # read every payload byte once, write it once


def unpack_bytes(wl, k, widths=FP32_WIDTHS):
    total = 2 * wl.slot_payload_bytes(k, widths)
    if widths == FP32_WIDTHS:                      # + derived bf16 weights of the new operators (this regime only;
        total += 2 * sum(p for e, p in enumerate(wl.params_of_op()) if wl.slot_of_op[e] == k)  # otherwise the replay writes them)
    return total


def replay_bytes(wl, i, widths=FP32_WIDTHS):
    # read p, m, v and the FP32 gradient, write p, m, v and the compute weight: 16 + 12 + 2 = 30 B in the FP32 regime
    return (2 * (widths[0] + widths[1] + widths[2]) + 4 + widths[3]) * wl.active_params_at(i)


def kernel_table(timings, wl, widths):
    """timings: (kind, algorithmic bytes, start event, end event) of every timed launch, each kind in slot / iteration order
    0 .. W-1 step after step.  -> ({kind: bytes, ms, launches}, the `kernels` object of the JSON line: per kind the rate of
    algorithmic bytes over all launches, per slot (pack, unpack) or per replay iteration, and for the two copies the
    payload rate (snapshot bytes / time: half of the pack's traffic))."""
    per_kind, per_slot = {}, {}
    for kind, nbytes, e0, e1 in timings:
        ms = e0.elapsed_time(e1)
        d = per_kind.setdefault(kind, {"bytes": 0, "ms": 0.0, "launches": 0})
        slot = d["launches"] % wl.window
        d["bytes"] += nbytes
        d["ms"] += ms
        d["launches"] += 1
        ps = per_slot.setdefault(kind, [[0, 0.0] for _ in range(wl.window)])
        ps[slot][0] += nbytes
        ps[slot][1] += ms
    kernels = {}
    for kind, d in per_kind.items():
        gbs = d["bytes"] / (d["ms"] / 1e3) / 1e9
        kernels[kind] = {"GBs": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                         "avg_ms_per_launch": round(d["ms"] / d["launches"], 4),
                         "avg_bytes_per_launch": d["bytes"] // d["launches"], "launches": d["launches"],
                         ("per_iteration_GBs" if kind == "replay" else "per_slot_GBs"):
                             [round(b / (ms / 1e3) / 1e9, 1) if ms else None for b, ms in per_slot[kind]]}
        if kind in ("pack", "unpack"):
            payload = sum(wl.slot_payload_bytes(k, widths) for k in range(wl.window)) * (d["launches"] // wl.window)
            kernels[kind]["payload_GBs"] = round(payload / (d["ms"] / 1e3) / 1e9, 1)
    return per_kind, kernels


def read_valu_count(kernel, regime):
    """Vector-ALU instructions per parameter of a kernel, from the SQ_INSTS_VALU counter run summarised in
    profiles/valu_instructions.txt, or None."""
    path = os.path.join(ROOT, "profiles", "valu_instructions.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 3 and not line.startswith("#") and parts[0] == kernel and parts[1] == regime:
            return float(parts[2])
    return None


def read_traffic(kernel, workload):
    """HBM traffic per launch measured with rocprofv3 --pmc (profiles/hbm_traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 4 and not line.startswith("#") and parts[0] == kernel and parts[1] == workload:
            return float(parts[2]) + float(parts[3])
    return None


# ---------------------------------------------------------------------------------------
def regime_of(name, torch, W):
    """-> (storage dtypes or None for the FP32 regime, element widths)."""
    if name == "fp32":
        return None, FP32_WIDTHS
    if name not in W.LOW_PRECISION_REGIMES:
        print(f"bench.py: unknown --regime {name}; one of fp32, " + ", ".join(W.LOW_PRECISION_REGIMES), file=sys.stderr)
        sys.exit(2)
    dtypes = W.LOW_PRECISION_REGIMES[name]
    return dtypes, tuple(torch.empty(0, dtype=d).element_size() for d in dtypes)


def _oracle_sample(cfg_name, parts, W):
    """The bounded sample of a workload the oracle is timed on, cut into `parts` equal shares: every share has all
    the operators and the whole schedule of the sample and 1/parts of the columns of every tensor."""
    if cfg_name == "c1":
        return (W.mixtral_layer(d_ff=14336 // 8 // parts),
                "configs[1] with d_ff 1792 (1/8 of the columns): 8 experts, W=8, whole window pack+unpack+replay")
    if cfg_name in ("c2", "c4"):
        return (W.fine_grained_stack(n_layers=1, n_routed=16, n_shared=2, per_slot=4, d_ff=704 // parts,
                                     heavy_tail=cfg_name == "c4"),
                "one layer of 16 routed + 2 shared experts with d_ff 704 (half of the columns), W=4, whole window "
                "pack+unpack+replay")
    if cfg_name == "c3":
        return (W.ep_rank_share(n_layers=1, n_experts=32, d_ff=512 // parts),
                "one of the 16 layers (32 experts, W=8) with d_ff 512 (1/4 of the columns): W x (pack + unpack), no replay")
    return W.tiny_moe(d_hidden=1024 // parts), "configs[0], whole window"


def _oracle_leg(cfg_name, seed, regime, parts, share, barrier, queue):
    """One process of an oracle timing leg: the unchanged single-threaded oracle over one share of the sample."""
    try:
        import numpy as np
        import torch
        if parts > 1:
            torch.set_num_threads(1)   # input generation only; the oracle itself is single-threaded C

        import oracle
        from paper_2412_15411_amd import workloads as W

        wl, sample = _oracle_sample(cfg_name, parts, W)
        if regime != "fp32" and cfg_name == "c1" and parts == 1:   # the oracle converts element by element there
            wl = W.mixtral_layer(d_ff=14336 // 64)
            sample = "configs[1] with d_ff 224 (1/64 of the columns): 8 experts, W=8, whole window pack+unpack+replay"
        seed = seed + 7919 * share

        def np_of(t):
            if t.element_size() == 2:
                return t.view(torch.int16).numpy().view(np.uint16)
            return t.view(torch.uint8).numpy() if t.element_size() == 1 else t.numpy()

        dtypes, widths = regime_of(regime, torch, W)
        formats = scales = None
        if dtypes is None:
            st = W.make_state(wl, seed=seed)
        else:
            fmt_of = {torch.float32: oracle.FMT_F32, torch.float16: oracle.FMT_F16, torch.bfloat16: oracle.FMT_BF16,
                      torch.float8_e4m3fn: oracle.FMT_E4M3, torch.float8_e5m2: oracle.FMT_E5M2}
            formats = tuple(fmt_of[d] for d in dtypes)
            per_kind = W.default_scales(dtypes)
            st = W.make_low_precision_state(wl, dtypes, per_kind, seed=seed)
            scales = np.ascontiguousarray(np.array([[x] * wl.n_tensors for x in per_kind], dtype=np.float32))
            sample += f"; state stored as {regime}"
        state = oracle.State(*[[np_of(t) for t in st[k]] for k in ("master", "m", "v", "compute")])
        model = oracle.Model(list(wl.tensors), list(wl.order), list(wl.slot_of_op), wl.window, 256, widths, formats)
        hp = oracle.AdamHP(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay)
        replay = cfg_name != "c3"
        grads = [np_of(g) for g in W.make_grads(wl, wl.t0 + 1, seed=seed)] if replay else None
        snaps = [np.empty(oracle.layout(model, k)[1], dtype=np.uint8) for k in range(wl.window)]
        for sn in snaps:
            sn.fill(0)  # touch the pages before timing
        mask = np.zeros(wl.n_ops, dtype=np.uint8)
        barrier.wait()
        t_begin = time.monotonic()
        t_pack = t_unpack = t_replay = 0.0
        b_pack = b_unpack = b_replay = 0
        for k in range(wl.window):
            t0 = time.monotonic()
            oracle.pack(model, k, wl.t0 + k, state, out=snaps[k])
            t_pack += time.monotonic() - t0
            b_pack += pack_bytes(wl, k, widths)
        for i in range(wl.window):
            t0 = time.monotonic()
            oracle.unpack(model, i, snaps[i], state, mask)
            t1 = time.monotonic()
            if replay:
                oracle.replay_step(model, hp, wl.t0 + i + 1, mask, grads, state, scales)
                b_replay += replay_bytes(wl, i, widths)
            t2 = time.monotonic()
            t_unpack += t1 - t0
            t_replay += t2 - t1
            b_unpack += unpack_bytes(wl, i, widths)
        queue.put({"share": share, "begin": t_begin, "end": time.monotonic(), "sample": sample, "window": wl.window,
                   "t": (t_pack, t_unpack, t_replay), "b": (b_pack, b_unpack, b_replay)})
    except BaseException as e:  # the parent must not wait for ever
        try:
            barrier.abort()
        except Exception:
            pass
        queue.put({"share": share, "error": repr(e)})


def _oracle_legs(cfg_name, seed, regime, parts):
    """Runs `parts` forked processes (fork: nothing here has touched the GPU yet), each timing the oracle on its
    share between a common barrier and its own end; returns the aggregate figures."""
    import multiprocessing as mp

    import oracle
    oracle.build()
    ctx = mp.get_context("fork")
    barrier, queue = ctx.Barrier(parts), ctx.Queue()
    procs = [ctx.Process(target=_oracle_leg, args=(cfg_name, seed, regime, parts, w, barrier, queue)) for w in range(parts)]
    for pr in procs:
        pr.start()
    results = [queue.get(timeout=600) for _ in procs]
    for pr in procs:
        pr.join(timeout=60)
    bad = [r["error"] for r in results if "error" in r]
    if bad:
        raise RuntimeError("oracle timing leg failed: " + "; ".join(bad))
    wall = max(r["end"] for r in results) - min(r["begin"] for r in results)
    b = [sum(r["b"][k] for r in results) for k in range(3)]
    # per phase: the bytes of all shares over the longest share's time in that phase
    t = [max(r["t"][k] for r in results) for k in range(3)]
    out = {"value": round(sum(b) / wall / 1e9, 3), "unit": "GB/s", "cores": parts, "kind": "oracle",
           "sample": results[0]["sample"], "seconds": round(wall, 2),
           "pack_GBs": round(b[0] / t[0] / 1e9, 3), "unpack_GBs": round(b[1] / t[1] / 1e9, 3)}
    if b[2]:
        out["replay_GBs"] = round(b[2] / t[2] / 1e9, 3)
        out["replay_iters_per_s"] = round(results[0]["window"] / t[2], 3)
    return out


def cpu_baseline(cfg_name, seed, regime="fp32"):
    """The oracle, as it stands, on a bounded sample of the same workload: (i) single-threaded, on one core;
    (ii) the same unchanged code in one process per host core (at most 16, this box's share), each on an equal
    share of the sample's columns, started together.  Must be called before the process touches the GPU."""
    single = _oracle_legs(cfg_name, seed, regime, 1)
    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    if cores > 1:
        every = _oracle_legs(cfg_name, seed, regime, cores)
        every["sample"] = f"the same sample, {cores} processes, each the unchanged oracle on 1/{cores} of the columns of every tensor"
        single["all_cores"] = every
    return single


# ---------------------------------------------------------------------------------------
def apply_launch_knobs(args, plan, B):
    """The launch-shape flags of the command line, set on a fresh plan."""
    if args.persistent:
        B.moev_tune(plan, B.TUNE_PERSISTENT, 1)
    for knob, val in ((B.TUNE_COPY_TILE_BYTES, args.copy_tile), (B.TUNE_ADAM_TILE_ELEMS, args.adam_tile),
                      (B.TUNE_COPY_MAX_BLOCKS, args.copy_blocks), (B.TUNE_ADAM_MAX_BLOCKS, args.adam_blocks)):
        if val:
            B.moev_tune(plan, knob, val)
    if args.adam_shape:
        threads, unroll = (int(x) for x in args.adam_shape.split("x"))
        B.moev_tune(plan, B.TUNE_ADAM_UNROLL, 1)
        B.moev_tune(plan, B.TUNE_ADAM_THREADS, threads)
        B.moev_tune(plan, B.TUNE_ADAM_UNROLL, unroll)
    if args.nontemporal >= 0:
        B.moev_tune(plan, B.TUNE_NONTEMPORAL, args.nontemporal)
    if args.xcd_regions >= 0:
        B.moev_tune(plan, B.TUNE_XCD_REGIONS, args.xcd_regions)
    if args.copy_xcd_regions >= 0:
        B.moev_tune(plan, B.TUNE_COPY_XCD_REGIONS, args.copy_xcd_regions)
    if args.plain_divide_sqrt >= 0:
        B.moev_tune(plan, B.TUNE_PLAIN_DIVIDE_SQRT, args.plain_divide_sqrt)
    if args.paired_tiles >= 0:
        B.moev_tune(plan, B.TUNE_PAIRED_TILES, args.paired_tiles)


def knob_sweep(args, wl, state, grads, packed, mask, stream, widths, torch, B):
    """Every launch knob in turn, in THIS process and on the tensors of the timed steps, so that the physical placement of
    the tensors (which alone moves the rates by several per cent between processes) is the same for every line: GB/s of the
    pack (all W slots), the unpack (all W slots) and the replay (last iteration of the window: every operator active).
    packed: one buffer per slot, or one buffer all slots go through; grads None: no replay (configs[3])."""
    def shape(t, u):
        knobs = []
        for k_threads, k_unroll in ((B.TUNE_COPY_THREADS, B.TUNE_COPY_UNROLL), (B.TUNE_UNPACK_THREADS, B.TUNE_UNPACK_UNROLL),
                                    (B.TUNE_ADAM_THREADS, B.TUNE_ADAM_UNROLL)):
            knobs += [(k_unroll, 1), (k_threads, t), (k_unroll, u)]
        return knobs

    def regions(v):
        return [(B.TUNE_XCD_REGIONS, v), (B.TUNE_COPY_XCD_REGIONS, v)]

    variants = [("defaults", []), ("defaults again", []), ("xcd regions off", regions(0)), ("xcd regions: eighths", regions(1)),
                ("nontemporal 0", [(B.TUNE_NONTEMPORAL, 0)]), ("paired_tiles 0", [(B.TUNE_PAIRED_TILES, 0)]),
                ("persistent", [(B.TUNE_PERSISTENT, 1)])]
    variants += [(f"xcd chunks of {g} tiles", regions(g)) for g in (2, 4, 8, 16, 32, 64, 128, 256, 1024, 4096, 16384, 65536)]
    variants += [(f"shape {t}x{u}", shape(t, u)) for u in (1, 2, 4) for t in (64, 128, 256, 512, 1024) if t * u <= 1024]
    buf = (lambda k: packed[k]) if isinstance(packed, (list, tuple)) else (lambda k: packed)
    last = wl.window - 1
    rows = {}
    for label, knobs in variants:
        plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
        apply_launch_knobs(args, plan, B)
        for knob, value in knobs:
            B.moev_tune(plan, knob, value)
        B.ckpt_plan_upload(plan, stream)
        marks = {"pack": [], "unpack": [], "replay": []}

        def timed(kind, fn):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            marks[kind].append((e0, e1))

        for rep in range(4):      # the first repetition warms up
            if rep == 1:
                marks = {"pack": [], "unpack": [], "replay": []}
            for k in range(wl.window):
                timed("pack", lambda: B.snapshot_pack(plan, k, wl.t0 + k, state, buf(k), stream=stream))
                timed("unpack", lambda: B.restore_unpack(plan, k, None, buf(k), state, mask, stream=stream))
            if grads is not None:   # the mask now marks every operator active
                for _ in range(2):
                    timed("replay", lambda: B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.t0 + wl.window,
                                                             mask, grads[wl.t0 + wl.window], state, stream=stream))
        stream.synchronize()
        B.ckpt_plan_device_status(plan, stream)
        nbytes = {"pack": 3 * sum(pack_bytes(wl, k, widths) for k in range(wl.window)),
                  "unpack": 3 * sum(unpack_bytes(wl, k, widths) for k in range(wl.window)),
                  "replay": 6 * replay_bytes(wl, last, widths)}
        rows[label] = {kind: round(nbytes[kind] / (sum(e0.elapsed_time(e1) for e0, e1 in ev) / 1e3) / 1e9, 1)
                       for kind, ev in marks.items() if ev}
        del plan
    return {"what": "GB/s of algorithmic bytes per launch knob, same process and tensors: pack and unpack over all W slots, "
                    "replay with every operator active", "GBs": rows}


def rank_share_bench(args, steps, warmup, torch, B, W, dev):
    """configs[3]: one GPU's share of a large MoE (180 GB of state resident in HBM).  The packed
    snapshots of a window (245 GB) cannot be resident next to the state, so a step here is
    W x (snapshot_pack into one reused buffer, restore_unpack from it); the replay is not part of
    this configuration.  Also measured: the pack and the drain while a bf16 GEMM loop runs on the
    main stream (the overlap the method relies on, Sec. 3.2 / Sec. 4)."""
    wl = W.ep_rank_share()
    t_setup = time.time()
    log(f"[bench] workload {wl.name}: {wl.n_ops} operators, {wl.n_tensors} tensors, {wl.n_params / 1e9:.3f} B params, W={wl.window}")
    st = W.make_state(wl, seed=args.seed, device=dev, flat=args.alloc == "flat", skew=args.alloc == "skewed")
    state = B.State(st["master"], st["m"], st["v"], st["compute"])
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
    apply_launch_knobs(args, plan, B)
    packed = torch.empty(B.ckpt_plan_max_packed_bytes(plan), dtype=torch.uint8, device=dev)
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    B.ckpt_plan_upload(plan, main)
    torch.cuda.synchronize()
    log(f"[bench] inputs resident in HBM after {time.time() - t_setup:.1f} s; {torch.cuda.memory_allocated() / 1e9:.1f} GB allocated")

    timings = []

    def timed(kind, nbytes, fn, record, stream):
        if record:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            timings.append((kind, nbytes, e0, e1))
        else:
            fn()

    def one_step(record):
        for k in range(wl.window):
            timed("pack", pack_bytes(wl, k), lambda: B.snapshot_pack(plan, k, wl.t0 + k, state, packed, stream=main), record, main)
            timed("unpack", unpack_bytes(wl, k), lambda: B.restore_unpack(plan, k, None, packed, state, mask, stream=main), record, main)

    step_bytes = sum(pack_bytes(wl, k) + unpack_bytes(wl, k) for k in range(wl.window))
    for _ in range(warmup):
        one_step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.ckpt_plan_device_status(plan, main)
    per_kind, kernels = kernel_table(timings, wl, FP32_WIDTHS)
    value = step_bytes / (elapsed / steps) / 1e9
    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"configs[3] {wl.name}", "state_allocation": ALLOC_TEXT[args.alloc], "n_ops": wl.n_ops, "n_params": wl.n_params, "window": wl.window,
                   "step": "W x (snapshot_pack + restore_unpack) through one reused packed buffer, HBM-resident; no replay",
                   "step_algorithmic_bytes": step_bytes},
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4), "kernels": kernels,
        "roofline": {"bound": "hbm", "kernel": "k_unpack_direct", "achieved": kernels["unpack"]["GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": kernels["unpack"]["frac_hbm_peak"], "traffic": read_traffic("k_unpack_direct", "c3")},
    }

    # ---- overlap: pack and drain of slot `k` against a bf16 GEMM loop on the main stream -------
    k = args.overlap_slot if 0 <= args.overlap_slot < wl.window else wl.window - 1
    nbytes = B.ckpt_plan_packed_bytes(plan, k)
    a = torch.randn(8192, 4096, dtype=torch.bfloat16, device=dev)
    b = torch.randn(4096, 2048, dtype=torch.bfloat16, device=dev)
    c = torch.empty(8192, 2048, dtype=torch.bfloat16, device=dev)

    def gemm_loop(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(main):
            e0.record(main)
            for _ in range(n):
                torch.mm(a, b, out=c)
            e1.record(main)
        return e0, e1

    gemm_loop(50)                      # warm-up: library initialisation and kernel selection
    torch.cuda.synchronize()
    g0, g1 = gemm_loop(200)
    torch.cuda.synchronize()
    per_gemm_ms = g0.elapsed_time(g1) / 200
    gemm_tflops = 2 * 8192 * 4096 * 2048 / (per_gemm_ms / 1e3) / 1e12

    def pack_on_side(p):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)          # `side` is looked up at call time (the CU-mask sweep rebinds it)
        B.snapshot_pack(p, k, wl.t0 + k, state, packed, stream=side)
        e1.record(side)
        return e0, e1

    # the default shape floods the dispatcher with small workgroups; the fixed-grid shape with a cap
    # on its workgroups leaves compute units to the GEMM
    overlap = []
    for label, cap in (("one tile per workgroup (default)", None), ("fixed grid, 1024 workgroups", 1024),
                       ("fixed grid, 256 workgroups", 256)):
        p = plan
        if cap is not None:
            p = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order)
            B.moev_tune(p, B.TUNE_PERSISTENT, 1)
            B.moev_tune(p, B.TUNE_COPY_MAX_BLOCKS, cap)
        p0, p1 = pack_on_side(p)
        torch.cuda.synchronize()
        p0, p1 = pack_on_side(p)
        torch.cuda.synchronize()
        pack_alone_ms = p0.elapsed_time(p1)
        n_gemm = max(50, int(3 * pack_alone_ms / per_gemm_ms))
        g0, g1 = gemm_loop(n_gemm)
        torch.cuda.synchronize()
        gemm_alone_ms = g0.elapsed_time(g1)
        g0, g1 = gemm_loop(n_gemm)
        p0, p1 = pack_on_side(p)
        torch.cuda.synchronize()
        overlap.append({
            "pack_shape": label, "n_gemm": n_gemm,
            "pack_ms_alone": round(pack_alone_ms, 3), "pack_ms_with_gemm": round(p0.elapsed_time(p1), 3),
            "pack_GBs_alone": round(pack_bytes(wl, k) / (pack_alone_ms / 1e3) / 1e9, 1),
            "pack_GBs_with_gemm": round(pack_bytes(wl, k) / (p0.elapsed_time(p1) / 1e3) / 1e9, 1),
            "gemm_ms_alone": round(gemm_alone_ms, 3), "gemm_ms_with_pack": round(g0.elapsed_time(g1), 3),
            "gemm_ms_lost": round(g0.elapsed_time(g1) - gemm_alone_ms, 3)})
        del p
    out["pack_under_gemm"] = {"slot": k, "gemm": "bf16 [8192x4096]x[4096x2048] back to back on the main stream",
                              "gemm_TFLOPs_alone": round(gemm_tflops, 1), "runs": overlap}

    # The same pack (default shape) on a side stream that may only use the first n compute units: does leaving
    # compute units to the GEMM reduce what the GEMM loses?
    if args.cu_mask_sweep:
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        hip.hipExtStreamCreateWithCUMask.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32)]
        hip.hipStreamDestroy.argtypes = [ctypes.c_void_p]
        default_side, masked = side, []
        for n_cu in (192, 128, 96, 64, 32):
            words = (ctypes.c_uint32 * 8)(*[(1 << min(32, max(0, n_cu - 32 * w))) - 1 for w in range(8)])
            raw = ctypes.c_void_p()
            rc = hip.hipExtStreamCreateWithCUMask(ctypes.byref(raw), 8, words)
            if rc != 0:
                masked.append({"compute_units": n_cu, "error": f"hipExtStreamCreateWithCUMask returned {rc}"})
                continue
            side = torch.cuda.ExternalStream(raw.value)     # pack_on_side() launches on `side`
            pack_on_side(plan)
            torch.cuda.synchronize()
            p0, p1 = pack_on_side(plan)
            torch.cuda.synchronize()
            pack_alone_ms = p0.elapsed_time(p1)
            n_gemm = max(50, int(3 * pack_alone_ms / per_gemm_ms))
            g0, g1 = gemm_loop(n_gemm)
            torch.cuda.synchronize()
            gemm_alone_ms = g0.elapsed_time(g1)
            g0, g1 = gemm_loop(n_gemm)
            p0, p1 = pack_on_side(plan)
            torch.cuda.synchronize()
            masked.append({"compute_units": n_cu, "n_gemm": n_gemm, "pack_ms_alone": round(pack_alone_ms, 3),
                           "pack_GBs_alone": round(pack_bytes(wl, k) / (pack_alone_ms / 1e3) / 1e9, 1),
                           "pack_ms_with_gemm": round(p0.elapsed_time(p1), 3), "gemm_ms_alone": round(gemm_alone_ms, 3),
                           "gemm_ms_lost": round(g0.elapsed_time(g1) - gemm_alone_ms, 3)})
            side = default_side
            hip.hipStreamDestroy(raw)
        out["pack_under_gemm"]["cu_masked_side_stream"] = masked

    if not args.no_drain:
        t_pin = time.time()
        host = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
        log(f"[bench] pinned {nbytes / 1e9:.1f} GB of host memory in {time.time() - t_pin:.1f} s")
        done = torch.cuda.Event()
        B.snapshot_pack(plan, k, wl.t0 + k, state, packed, stream=main)
        done.record(main)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        B.snapshot_drain(plan, k, packed, host, side_stream=side, pack_done=done)
        e1.record(side)
        torch.cuda.synchronize()
        drain_alone_ms = e0.elapsed_time(e1)
        n_gemm = max(20, int(1.2 * drain_alone_ms / per_gemm_ms))
        g0, g1 = gemm_loop(n_gemm)
        torch.cuda.synchronize()
        gemm_alone_ms = g0.elapsed_time(g1)
        # the GEMM loop again with the drain on the side stream; events after every 1/12 of the loop put both on one
        # time axis (milliseconds since the loop's start)
        batch = max(1, n_gemm // 12)
        marks = []
        origin = torch.cuda.Event(enable_timing=True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(main):
            origin.record(main)
            side.wait_event(origin)
            e0.record(side)
            B.snapshot_drain(plan, k, packed, host, side_stream=side)
            e1.record(side)
            for i in range(n_gemm):
                torch.mm(a, b, out=c)
                if (i + 1) % batch == 0 or i + 1 == n_gemm:
                    ev = torch.cuda.Event(enable_timing=True)
                    ev.record(main)
                    marks.append((i + 1, ev))
        torch.cuda.synchronize()
        t_drain = (origin.elapsed_time(e0), origin.elapsed_time(e1))
        ends = [(n, origin.elapsed_time(ev)) for n, ev in marks]
        during = [(n, t) for n, t in ends if t_drain[0] <= t <= t_drain[1]]
        out["drain"] = {"bound": "host-link", "link": "PCIe Gen5 x16, 64 GB/s per direction in theory", "slot": k, "bytes": nbytes, "ms": round(drain_alone_ms, 2),
                        "GBs": round(nbytes / (drain_alone_ms / 1e3) / 1e9, 2),
                        "header_ok": B.snapshot_peek(plan, k, host)["slot"] == k}
        out["drain_under_gemm"] = {
            "gemm": "bf16 [8192x4096]x[4096x2048], %d back to back on the main stream" % n_gemm,
            "drain_ms": round(t_drain[1] - t_drain[0], 2),
            "drain_GBs": round(nbytes / ((t_drain[1] - t_drain[0]) / 1e3) / 1e9, 2),
            "gemm_ms_alone": round(gemm_alone_ms, 2), "gemm_ms_with_drain": round(ends[-1][1], 2),
            "gemm_slowdown_pct": round((ends[-1][1] / gemm_alone_ms - 1) * 100, 2),
            "gemm_us_per_kernel_alone": round(gemm_alone_ms / n_gemm * 1e3, 2),
            "gemm_us_per_kernel_while_draining": (round((during[-1][1] - during[0][1]) / (during[-1][0] - during[0][0]) * 1e3, 2)
                                                  if len(during) > 1 else None),
            "timeline_ms": {"drain_start": round(t_drain[0], 2), "drain_end": round(t_drain[1], 2),
                            "gemm_kernels_done_at": [[n, round(t, 2)] for n, t in ends]}}
        del host
    if args.knob_sweep:
        out["knob_sweep"] = knob_sweep(args, wl, state, None, packed, mask, main, FP32_WIDTHS, torch, B)
    del st, state, packed, a, b, c
    return out


# ---------------------------------------------------------------------------------------
def window_bench(args, cfg, steps, warmup, extras, torch, B, W, dev):
    """One workload with a replay (configs[0], [1], [2], [4]): W x snapshot_pack, then W x (restore_unpack +
    convert_replay), everything resident in HBM.  extras: also the copy probe, the drain, the upstream-log ring and
    the what-if (the headline workload); otherwise the step, its kernels and the fused conversion only."""
    dtypes, widths = regime_of(args.regime, torch, W)
    wl = W.CONFIGS[cfg]()
    t_setup = time.time()
    log(f"[bench] workload {wl.name}: {wl.n_ops} operators, {wl.n_tensors} tensors, {wl.n_params / 1e9:.3f} B params, W={wl.window}")
    formats, d_scales = (0, 0, 0, 0), None
    if dtypes is None:
        st = W.make_state(wl, seed=args.seed, device=dev, flat=args.alloc == "flat", skew=args.alloc == "skewed")
    else:
        lib_fmt = {torch.float32: B.FMT_F32, torch.float16: B.FMT_F16, torch.bfloat16: B.FMT_BF16,
                   torch.float8_e4m3fn: B.FMT_E4M3, torch.float8_e5m2: B.FMT_E5M2}
        formats = tuple(lib_fmt[d] for d in dtypes)
        per_kind = W.default_scales(dtypes)
        st = W.make_low_precision_state(wl, dtypes, per_kind, seed=args.seed, device=dev)
        d_scales = torch.tensor([[x] * wl.n_tensors for x in per_kind], dtype=torch.float32, device=dev)
    state = B.State(st["master"], st["m"], st["v"], st["compute"])
    # Gradients of replay iteration i exist only for the operators that are active in it: frozen
    # operators skip their weight-gradient computation (Sec. 3.3), so their entries are None.
    grads = {}
    for i in range(wl.window):
        grads[wl.t0 + i + 1] = W.make_grads(wl, wl.t0 + i + 1, seed=args.seed, device=dev, flat=args.alloc == "flat", skew=args.alloc == "skewed",
                                            only=[wl.slot_of_op[op] <= i for op, _ in wl.tensors])
    plan = B.ckpt_plan(wl.tensors, B.EXPLICIT, window=wl.window, slot_of_op=wl.slot_of_op, order=wl.order, formats=formats)
    apply_launch_knobs(args, plan, B)
    packed = [torch.empty(B.ckpt_plan_packed_bytes(plan, k), dtype=torch.uint8, device=dev) for k in range(wl.window)]
    mask = torch.zeros(wl.n_ops, dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    B.ckpt_plan_upload(plan, stream)
    torch.cuda.synchronize()
    log(f"[bench] inputs resident in HBM after {time.time() - t_setup:.1f} s; "
        f"{torch.cuda.memory_allocated() / 1e9:.1f} GB allocated")

    timings = []  # (kind, algorithmic bytes, start event, end event)

    def timed(kind, nbytes, fn, record):
        if record:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            timings.append((kind, nbytes, e0, e1))
        else:
            fn()

    def one_step(record):
        for k in range(wl.window):
            timed("pack", pack_bytes(wl, k, widths),
                  lambda: B.snapshot_pack(plan, k, wl.t0 + k, state, packed[k], stream=stream), record)
        mask.zero_()  # on torch's current stream == `stream` inside the with-block below
        for i in range(wl.window):
            timed("unpack", unpack_bytes(wl, i, widths),
                  lambda: B.restore_unpack(plan, i, None, packed[i], state, mask, stream=stream), record)
            timed("replay", replay_bytes(wl, i, widths),
                  lambda: B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.t0 + i + 1, mask,
                                           grads[wl.t0 + i + 1], state, stream=stream, d_scales=d_scales), record)

    step_bytes = sum(pack_bytes(wl, k, widths) + unpack_bytes(wl, k, widths) + replay_bytes(wl, k, widths)
                     for k in range(wl.window))
    with torch.cuda.stream(stream):
        for _ in range(warmup):
            one_step(False)
        torch.cuda.synchronize()
        step_marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        step_marks[0].record(stream)
        for n in range(steps):
            one_step(True)
            step_marks[n + 1].record(stream)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    B.ckpt_plan_device_status(plan, stream)
    ms_per_step = elapsed / steps * 1e3
    value = step_bytes / (elapsed / steps) / 1e9
    per_step_ms = sorted(step_marks[n].elapsed_time(step_marks[n + 1]) for n in range(steps))

    per_kind, kernels = kernel_table(timings, wl, widths)
    dominant = max(per_kind, key=lambda k: per_kind[k]["ms"])
    suffix = "_persistent" if args.persistent else "_direct"
    kname = {"pack": "k_pack", "unpack": "k_unpack", "replay": "k_adam"}[dominant] + suffix
    if dominant == "replay" and dtypes is not None:
        kname = "k_adam_lp"
    roofline = {"bound": "hbm", "kernel": kname, "achieved": kernels[dominant]["GBs"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kernels[dominant]["frac_hbm_peak"],
                "traffic": read_traffic(kname, cfg if dtypes is None else cfg + ":" + args.regime)}
    # The replay of state stored in 1-byte formats moves so few bytes per parameter that the vector ALU, not HBM,
    # bounds it (three correctly rounded divisions and a square root per parameter): then the roofline is the ALU's.
    valu_per_param = read_valu_count("k_adam_lp", args.regime) if dtypes is not None else None
    if kname == "k_adam_lp" and valu_per_param:
        params_per_s = sum(wl.active_params_at(i) for i in range(wl.window)) * steps / (per_kind["replay"]["ms"] / 1e3)
        valu_gops = valu_per_param * params_per_s / 1e9
        if valu_gops / VALU_PEAK_GOPS > roofline["frac"]:
            roofline = {"bound": "alu", "kernel": kname, "achieved": round(valu_gops, 1), "peak": VALU_PEAK_GOPS,
                        "unit": "G lane-instructions/s", "frac": round(valu_gops / VALU_PEAK_GOPS, 4), "traffic": None,
                        "valu_instructions_per_param": valu_per_param, "hbm_GBs": kernels[dominant]["GBs"],
                        "hbm_frac": kernels[dominant]["frac_hbm_peak"]}
    replay_iters_per_s = per_kind["replay"]["launches"] / (per_kind["replay"]["ms"] / 1e3)

    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{cfg[1]}] {wl.name}", "regime": args.regime, "element_bytes": list(widths),
                   "state_allocation": ALLOC_TEXT[args.alloc],
                   "n_ops": wl.n_ops, "n_params": wl.n_params,
                   "window": wl.window, "step": "W x snapshot_pack + W x (restore_unpack + convert_replay), HBM-resident",
                   "step_algorithmic_bytes": step_bytes},
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "ms_per_step_median": round(per_step_ms[len(per_step_ms) // 2], 3), "ms_per_step_min": round(per_step_ms[0], 3),
        "replay_iters_per_s": round(replay_iters_per_s, 2),
        "kernels": kernels,
        "roofline": roofline,
    }

    # ---- the same conversion with the fused load-and-replay call (convert_window_step) ----------
    def fused_window():
        mask.zero_()
        for i in range(wl.window):
            B.convert_window_step(plan, i, None, packed[i], wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay,
                                  wl.t0 + i + 1, mask, grads[wl.t0 + i + 1], state, stream=stream)

    def measure_fused():
        fused_bytes = 0
        for i in range(wl.window):
            frozen = sum(p for e, p in enumerate(wl.params_of_op()) if wl.slot_of_op[e] > i)
            fused_bytes += 2 * 2 * frozen + replay_bytes(wl, i)   # compute-weight copies + 30 B per active parameter
        with torch.cuda.stream(stream):
            fused_window()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(steps):
                fused_window()
            e1.record(stream)
            torch.cuda.synchronize()
        B.ckpt_plan_device_status(plan, stream)
        fused_ms = e0.elapsed_time(e1) / steps
        two_call_ms = (per_kind["unpack"]["ms"] + per_kind["replay"]["ms"]) / steps
        return {
            "call": "convert_window_step (restore_unpack + convert_replay in one pass, same results)",
            "ms_per_window": round(fused_ms, 3), "two_call_ms_per_window": round(two_call_ms, 3),
            "iters_per_s": round(wl.window / (fused_ms / 1e3), 2),
            "algorithmic_bytes": fused_bytes, "GBs": round(fused_bytes / (fused_ms / 1e3) / 1e9, 1)}

    if dtypes is None:   # the fused kernel exists for the FP32 regime; elsewhere the call runs the two kernels unfused
        out["fused_conversion"] = measure_fused()

    # ---- the replay at every piece distance of the paired tiles, same process and tensors ---------------------
    if args.paired_tiles_sweep and not args.persistent:
        last = wl.window - 1   # every operator active (the mask is in that state after a window)
        sweep = {}
        for dist in [0] + [1 << b for b in range(9, 23)]:
            B.moev_tune(plan, B.TUNE_PAIRED_TILES, dist)
            run = lambda: B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.t0 + wl.window, mask,
                                           grads[wl.t0 + wl.window], state, stream=stream, d_scales=d_scales)
            for _ in range(2):
                run()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(8):
                run()
            e1.record(stream)
            stream.synchronize()
            sweep[str(dist)] = round(8 * replay_bytes(wl, last, widths) / (e0.elapsed_time(e1) / 1e3) / 1e9, 1)
        B.ckpt_plan_device_status(plan, stream)
        B.moev_tune(plan, B.TUNE_PAIRED_TILES, args.paired_tiles if args.paired_tiles >= 0 else 1)
        out["paired_tiles_sweep"] = {"what": "replay GB/s, all operators active, by distance in bytes (of an FP32 stream; narrower "
                                     "streams proportionally less) between the two pieces of 128 elements a wavefront takes per "
                                     "stream (0 and 512: consecutive bytes)", "GBs": sweep}

    if args.knob_sweep and dtypes is None:
        out["knob_sweep"] = knob_sweep(args, wl, state, grads, packed, mask, stream, widths, torch, B)

    # ---- launch-bound windows: the same step replayed from a HIP graph -------------------------------------
    # (with resident tables every call enqueues kernels only; all gradient pointers are passed in every
    # iteration so that the pointer table stays the same)
    if cfg == "c0":
        all_grads = W.make_grads(wl, wl.t0 + 1, seed=args.seed, device=dev)

        def whole_step():
            for k in range(wl.window):
                B.snapshot_pack(plan, k, wl.t0 + k, state, packed[k], stream=stream)
            mask.zero_()
            for i in range(wl.window):
                B.restore_unpack(plan, i, None, packed[i], state, mask, stream=stream)
                B.convert_replay(plan, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.t0 + i + 1, mask,
                                 all_grads, state, stream=stream, d_scales=d_scales)

        with torch.cuda.stream(stream):
            whole_step()
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                whole_step()
            reps = max(steps, 20)
            e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            e0.record(stream)
            for _ in range(reps):
                whole_step()
            e1.record(stream)
            for _ in range(reps):
                graph.replay()
            e2.record(stream)
            torch.cuda.synchronize()
        B.ckpt_plan_device_status(plan, stream)
        out["graph_replay"] = {"what": "the whole step (W packs, W x (unpack + replay)) captured once in a HIP graph",
                               "kernels_per_step": 4 * wl.window + 1, "eager_us_per_step": round(e0.elapsed_time(e1) / reps * 1e3, 1),
                               "graph_us_per_step": round(e1.elapsed_time(e2) / reps * 1e3, 1)}

    if not extras:
        del state, st, grads, packed
        return out

    # ---- plain contiguous copy of known size: the box's practical copy ceiling, and the kernel
    # against which the rocprofv3 HBM counters are calibrated ----------------------------------
    probe_bytes = 4 << 30
    src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()

    def best_of(fn, reps=4):
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            stream.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best

    best = best_of(lambda: B.moev_copy_probe(dst, src, probe_bytes, 0, 1, stream))
    read_ms = best_of(lambda: B.moev_stream_probe(1, dst, src, probe_bytes, 0, 1, stream))
    write_ms = best_of(lambda: B.moev_stream_probe(2, dst, None, probe_bytes, 0x01010101, 1, stream))
    read_gbs, write_gbs = probe_bytes / (read_ms / 1e3) / 1e9, probe_bytes / (write_ms / 1e3) / 1e9
    out["copy_probe"] = {"bytes_each_way": probe_bytes, "ms": round(best, 4),
                         "GBs": round(2 * probe_bytes / (best / 1e3) / 1e9, 1),
                         "frac_hbm_peak": round(2 * probe_bytes / (best / 1e3) / 1e9 / HBM_PEAK_GBS, 4),
                         "read_only_GBs": round(read_gbs, 1), "write_only_GBs": round(write_gbs, 1)}
    # The box's own yardstick for mixed traffic is the plain copy (one-directional streams run faster than any mix of
    # the two directions); `frac` stays relative to the published 8 TB/s.
    if roofline["bound"] == "hbm":
        out["roofline"]["achieved_over_copy_probe"] = round(roofline["achieved"] / out["copy_probe"]["GBs"], 4)
        # what the box's one-directional streams would allow for this kernel's read : write mix if the two directions did not
        # disturb each other: bytes / (read bytes / read-only rate + written bytes / write-only rate)
        if dominant == "replay":
            rd = 4 + widths[0] + widths[1] + widths[2]
            wr = widths[0] + widths[1] + widths[2] + widths[3]
        else:
            rd = wr = 1
        mix = (rd + wr) / (rd / read_gbs + wr / write_gbs)
        out["roofline"]["read_write_mix_bound_GBs"] = round(mix, 1)
        out["roofline"]["achieved_over_read_write_mix_bound"] = round(roofline["achieved"] / mix, 4)
    if args.pair_distance_sweep:
        # the same copy with every wavefront instruction covering two 512-byte pieces D bytes apart (D = 512: consecutive)
        sweep = {}
        for log2 in range(9, 23):
            dist = 1 << log2
            if src.data_ptr() % (2 * dist) or dst.data_ptr() % (2 * dist):
                break
            ms = best_of(lambda: B.moev_stream_probe(3, dst, src, probe_bytes, dist, 1, stream))
            sweep[str(dist)] = round(2 * probe_bytes / (ms / 1e3) / 1e9, 1)
        assert torch.equal(dst[-(1 << 20):], src[-(1 << 20):])
        out["copy_probe"]["piece_distance_sweep_GBs"] = sweep
    del src, dst

    # ---- drain: host link, measured outside the timed steps --------------------------------
    if not args.no_drain:
        k = 0
        nbytes = B.ckpt_plan_packed_bytes(plan, k)
        host = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
        side = torch.cuda.Stream()
        B.snapshot_pack(plan, k, wl.t0, state, packed[k], stream=stream)
        done = torch.cuda.Event()
        done.record(stream)
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(side)
            B.snapshot_drain(plan, k, packed[k], host, side_stream=side, pack_done=done)
            e1.record(side)
            side.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        out["drain"] = {"bound": "host-link", "link": "PCIe Gen5 x16, 64 GB/s per direction in theory", "slot": k, "bytes": nbytes, "ms": round(best, 3),
                        "GBs": round(nbytes / (best / 1e3) / 1e9, 2)}
        ok = B.snapshot_peek(plan, k, host)["slot"] == k
        out["drain"]["header_ok"] = bool(ok)
        # the same slot through a ring of four 64 MiB pinned chunks (hosts that cannot pin a whole slot)
        chunk = 64 << 20
        ring = [torch.empty(chunk, dtype=torch.uint8).pin_memory() for _ in range(4)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        for i, off in enumerate(range(0, nbytes, chunk)):
            B.snapshot_drain_range(plan, k, packed[k], off, ring[i % 4], min(chunk, nbytes - off), side_stream=side)
        e1.record(side)
        side.synchronize()
        out["drain"]["chunked_64MiB_GBs"] = round(nbytes / (e0.elapsed_time(e1) / 1e3) / 1e9, 2)
        del ring
        if args.overlap:
            a = torch.randn(8192, 4096, dtype=torch.bfloat16, device=dev)
            b = torch.randn(4096, 2048, dtype=torch.bfloat16, device=dev)
            n_gemm = 2000

            def gemm_loop():
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                with torch.cuda.stream(stream):
                    e0.record(stream)
                    for _ in range(n_gemm):
                        torch.mm(a, b)
                    e1.record(stream)
                return e0, e1
            g0, g1 = gemm_loop()
            torch.cuda.synchronize()
            alone_ms = g0.elapsed_time(g1)
            g0, g1 = gemm_loop()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(side)
            B.snapshot_drain(plan, k, packed[k], host, side_stream=side)
            e1.record(side)
            torch.cuda.synchronize()
            out["drain_under_gemm"] = {
                "gemm": "bf16 [8192x4096]x[4096x2048] x %d on the main stream" % n_gemm,
                "drain_GBs": round(nbytes / (e0.elapsed_time(e1) / 1e3) / 1e9, 2),
                "gemm_ms_alone": round(alone_ms, 2), "gemm_ms_with_drain": round(g0.elapsed_time(g1), 2)}
        del host

    # ---- upstream logging (Sec. 3.4): boundary tensors into the pinned ring and back, host link --------------
    if not args.no_drain:
        entry_bytes, n_entries = 256 << 20, 8        # a [32 x 2048 x 2048] 2-byte activation; 8 micro-batches
        ring = torch.empty(n_entries * entry_bytes, dtype=torch.uint8).pin_memory()
        log_ring = B.uplog_create(ring, max_entries=64)
        acts = torch.empty(entry_bytes, dtype=torch.uint8, device=dev).fill_(7)
        back = torch.empty_like(acts)
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record(side)
        for mb in range(n_entries):
            with torch.cuda.stream(side):
                acts.fill_(mb + 1)                   # every entry differs (stream-ordered with the copies)
            B.uplog_append(log_ring, wl.t0, mb, B.ACTIVATION, acts, side_stream=side)
        e1.record(side)
        for mb in range(n_entries):
            B.uplog_replay(log_ring, wl.t0, mb, B.ACTIVATION, back, stream=side)
        e2.record(side)
        side.synchronize()
        live = B.uplog_stats(log_ring)[0]
        dropped = B.uplog_gc(log_ring, wl.t0 + 1)
        out["upstream_log"] = {"bound": "host-link", "entries": n_entries, "entry_bytes": entry_bytes,
                               "append_GBs": round(n_entries * entry_bytes / (e0.elapsed_time(e1) / 1e3) / 1e9, 2),
                               "replay_GBs": round(n_entries * entry_bytes / (e1.elapsed_time(e2) / 1e3) / 1e9, 2),
                               "round_trip_ok": bool((back == n_entries).all().item()) and live == n_entries and dropped == n_entries}
        del ring, log_ring, acts, back

    # ---- what the measured rates mean for the method's own model (Algorithm 1, Sec. 3.6, App. C) -----------
    # Inputs that are MEASURED here: the host-link rate of the drain (B_PCIe), the time the state is held for
    # a snapshot (the pack of the largest slot; the drain runs under the next iteration), the conversion time
    # of a window.  Inputs that are ASSUMED: the iteration time (this bench trains nothing; the paper's runs
    # imply 1-3 s) and the MTBF values of the paper's tables.  All formulas are the library's host helpers.
    if "drain" in out:
        per_op = wl.n_params / wl.n_ops
        link = out["drain"]["GBs"] * 1e9
        stall_s = max(e0.elapsed_time(e1) for kind, _, e0, e1 in timings if kind == "pack") / 1e3
        convert_s = (out["fused_conversion"]["ms_per_window"] if "fused_conversion" in out else
                     (per_kind["unpack"]["ms"] + per_kind["replay"]["ms"]) / steps) / 1e3
        rows = []
        for t_iter in (0.25, 0.5, 1.0, 2.0):
            w, a = B.moev_find_window_size(wl.n_ops, t_iter, widths[3] * per_op, widths[0] * per_op,
                                           (widths[1] + widths[2]) * per_op, link)
            expected, worst = B.moev_recovery_time(True, w, t_iter)
            rows.append({"t_iter_s": t_iter, "window": w, "active_per_slot": a,
                         "expected_recovery_s": round(expected + convert_s, 3), "worst_recovery_s": round(worst + convert_s, 3),
                         "ettr": {f"mtbf_{m}s": round(B.moev_ettr(stall_s, t_iter, 1.0, expected + convert_s, m), 4)
                                  for m in (600, 1800, 3600)}})
        out["what_if"] = {"assumed": "t_iter_s, mtbf", "measured": {"host_link_GBs": out["drain"]["GBs"],
                          "snapshot_stall_s": round(stall_s, 5), "window_conversion_s": round(convert_s, 4)},
                          "note": "FindWindowSize on this GPU's operators with the measured link rate; recovery = 1.5 W T_iter "
                                  "(expected) / 2 W T_iter (worst) plus the measured conversion; ETTR with a snapshot every iteration",
                          "rows": rows}

    del state, st, grads, packed
    return out


# ---------------------------------------------------------------------------------------
def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (each expert-parallel rank snapshots and converts its own "
              "experts independently; there is nothing to exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    todo = ["c1", "c2", "c3", "c4"] if args.config == "all" else [args.config]
    if args.regime != "fp32" and "c3" in todo:
        if args.config == "c3":
            print("bench.py: --config c3 runs in the fp32 regime only", file=sys.stderr)
            sys.exit(2)
        todo.remove("c3")

    # The oracle's CPU legs run FIRST: their worker processes are forked before anything touches the GPU.
    cpu = {}
    if not args.no_cpu_baseline:
        for cfg in todo:
            t0 = time.time()
            cpu[cfg] = cpu_baseline(cfg, args.seed, args.regime)
            log(f"[bench] oracle legs of {cfg}: {time.time() - t0:.1f} s")

    import torch
    from paper_2412_15411_amd import binding as B
    from paper_2412_15411_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    regime_of(args.regime, torch, W)   # exits on an unknown regime

    def run(cfg, steps, warmup, extras):
        if cfg == "c3":
            res = rank_share_bench(args, steps, warmup, torch, B, W, dev)
        else:
            res = window_bench(args, cfg, steps, warmup, extras, torch, B, W, dev)
        if cfg in cpu:
            res["cpu_baseline"] = cpu[cfg]
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        return res

    out = run(todo[0], args.steps, args.warmup, True)
    if args.config == "all":
        # the other workloads, timed by the same run: each entry is a complete result of its own
        # (its step, kernels, roofline; configs[3] also the overlap with compute and the drain)
        out["configs"] = {}
        for cfg in todo[1:]:
            t0 = time.time()
            sub = run(cfg, args.sub_steps, 3, False)
            for key in ("metric", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "data"):
                sub.pop(key, None)
            out["configs"][cfg] = sub
            log(f"[bench] {cfg} done in {time.time() - t0:.1f} s")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
