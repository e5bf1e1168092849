"""ctypes binding of libmoev.so: the same names as include/moev.h, argument marshalling only.

Every step of the hot path runs inside the HIP library.  There is no fallback: importing
this module without the built library raises, and GPU calls raise MoevError when no GPU is
usable.  PyTorch appears only as the owner of device memory and streams: functions accept
torch tensors (their data_ptr is passed) or raw integer addresses.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoev.so")

OK, E_INVAL, E_NOMEM, E_RANGE, E_MISMATCH, E_HIP = 0, -1, -2, -3, -4, -5
KIND_MASTER, KIND_ADAM_M, KIND_ADAM_V, KIND_COMPUTE = 0, 1, 2, 3
EXPLICIT, FIXED, AUTO = 0, 1, 2
FMT_DEFAULT, FMT_F32, FMT_F16, FMT_BF16, FMT_E4M3, FMT_E5M2 = range(6)
HEADER_BYTES = 256
(TUNE_COPY_TILE_BYTES, TUNE_COPY_MAX_BLOCKS, TUNE_ADAM_TILE_ELEMS, TUNE_ADAM_MAX_BLOCKS, TUNE_NONTEMPORAL,
 TUNE_PERSISTENT, TUNE_COPY_THREADS, TUNE_COPY_UNROLL, TUNE_ADAM_THREADS, TUNE_ADAM_UNROLL,
 TUNE_UNPACK_THREADS, TUNE_UNPACK_UNROLL, TUNE_XCD_REGIONS, TUNE_PLAIN_DIVIDE_SQRT, TUNE_PAIRED_TILES,
 TUNE_COPY_XCD_REGIONS) = range(16)

EXPORTS = [
    "moev_last_error", "ckpt_plan", "ckpt_plan_free", "moev_find_window_size", "moev_order_operators",
    "moev_reorder_needed", "moev_popularity_time_decayed", "moev_popularity_capacity_aware", "moev_ettr",
    "moev_recovery_time", "moev_bias_corrections", "ckpt_plan_window", "ckpt_plan_n_ops", "ckpt_plan_n_tensors", "ckpt_plan_n_active",
    "ckpt_plan_hash", "ckpt_plan_width", "ckpt_plan_format", "ckpt_plan_slot_of_op", "ckpt_plan_order", "ckpt_plan_packed_bytes",
    "ckpt_plan_max_packed_bytes", "ckpt_plan_n_segments", "ckpt_plan_segments", "ckpt_plan_active_params",
    "ckpt_plan_pack_tile_bytes",
    "moev_tune", "moev_tune_get", "ckpt_plan_upload", "ckpt_plan_device_layout", "ckpt_plan_device_status",
    "snapshot_pack", "snapshot_drain", "snapshot_drain_range", "snapshot_peek", "restore_unpack", "convert_replay", "convert_replay_static", "convert_window_step",
    "moev_copy_probe", "moev_stream_probe", "moev_arith_selfcheck", "uplog_create", "uplog_free", "uplog_reserve", "uplog_append", "uplog_find", "uplog_replay",
    "uplog_gc", "uplog_stats",
]


class MoevError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libmoev error {code}: {message}")
        self.code = code


class _Tensor(C.Structure):
    _fields_ = [("op", C.c_uint32), ("numel", C.c_uint64)]


class _PlanCfg(C.Structure):
    _fields_ = [("n_ops", C.c_uint32), ("n_tensors", C.c_uint32), ("tensors", C.POINTER(_Tensor)),
                ("mode", C.c_int), ("window", C.c_uint32), ("n_active", C.c_uint32),
                ("order", C.POINTER(C.c_uint32)), ("slot_of_op", C.POINTER(C.c_uint32)),
                ("t_iter_s", C.c_double), ("host_link_Bps", C.c_double), ("align", C.c_uint32),
                ("master_bytes", C.c_uint8), ("m_bytes", C.c_uint8), ("v_bytes", C.c_uint8), ("compute_bytes", C.c_uint8),
                ("master_fmt", C.c_uint8), ("m_fmt", C.c_uint8), ("v_fmt", C.c_uint8), ("compute_fmt", C.c_uint8)]


class _Segment(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("tensor", C.c_uint32), ("nbytes", C.c_uint64), ("dst_off", C.c_uint64)]


class _State(C.Structure):
    _fields_ = [("master", C.POINTER(C.c_void_p)), ("m", C.POINTER(C.c_void_p)),
                ("v", C.POINTER(C.c_void_p)), ("compute", C.POINTER(C.c_void_p))]


class _Adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_uint64), ("d_scales", C.c_void_p)]


class _Header(C.Structure):
    _fields_ = [("magic", C.c_uint64), ("version", C.c_uint32), ("slot", C.c_uint32), ("plan_hash", C.c_uint64),
                ("iter", C.c_uint64), ("n_segments", C.c_uint64), ("payload_bytes", C.c_uint64),
                ("align", C.c_uint32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, u32, u64, i64 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int64
    lib.moev_last_error.restype = C.c_char_p
    lib.ckpt_plan.argtypes = [C.POINTER(_PlanCfg), C.POINTER(vp)]
    lib.ckpt_plan_free.argtypes = [vp]
    lib.ckpt_plan_free.restype = None
    lib.moev_find_window_size.argtypes = [u32, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double,
                                          C.POINTER(u32), C.POINTER(u32)]
    lib.moev_order_operators.argtypes = [u32, C.POINTER(C.c_double), C.POINTER(u32)]
    lib.moev_reorder_needed.argtypes = [u32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_double, C.c_double]
    dp = C.POINTER(C.c_double)
    lib.moev_popularity_time_decayed.argtypes = [u32, C.c_double, dp, dp, dp]
    lib.moev_popularity_capacity_aware.argtypes = [u32, dp, dp, dp]
    lib.moev_ettr.argtypes = [C.c_double] * 5
    lib.moev_ettr.restype = C.c_double
    lib.moev_recovery_time.argtypes = [C.c_int, C.c_double, C.c_double, dp, dp]
    lib.moev_bias_corrections.argtypes = [C.c_float, C.c_float, u64, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    for name in ("ckpt_plan_window", "ckpt_plan_n_ops", "ckpt_plan_n_tensors", "ckpt_plan_n_active"):
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = u32
    lib.ckpt_plan_hash.argtypes = [vp]
    lib.ckpt_plan_hash.restype = u64
    lib.ckpt_plan_pack_tile_bytes.argtypes = [vp, u32]
    lib.ckpt_plan_pack_tile_bytes.restype = u64
    for name in ("ckpt_plan_width", "ckpt_plan_format"):
        getattr(lib, name).argtypes = [vp, u32]
        getattr(lib, name).restype = u32
    lib.ckpt_plan_slot_of_op.argtypes = [vp, C.POINTER(u32)]
    lib.ckpt_plan_order.argtypes = [vp, C.POINTER(u32)]
    lib.ckpt_plan_packed_bytes.argtypes = [vp, u32]
    lib.ckpt_plan_packed_bytes.restype = u64
    lib.ckpt_plan_max_packed_bytes.argtypes = [vp]
    lib.ckpt_plan_max_packed_bytes.restype = u64
    lib.ckpt_plan_n_segments.argtypes = [vp, u32]
    lib.ckpt_plan_n_segments.restype = u32
    lib.ckpt_plan_segments.argtypes = [vp, u32, C.POINTER(_Segment), u64]
    lib.ckpt_plan_segments.restype = i64
    lib.ckpt_plan_active_params.argtypes = [vp, u32]
    lib.ckpt_plan_active_params.restype = u64
    lib.moev_tune.argtypes = [vp, C.c_int, i64]
    lib.moev_tune_get.argtypes = [vp, C.c_int]
    lib.moev_tune_get.restype = i64
    lib.ckpt_plan_upload.argtypes = [vp, vp]
    lib.ckpt_plan_device_layout.argtypes = [vp, u32, C.POINTER(u64), C.POINTER(u32), C.POINTER(u64), vp]
    lib.ckpt_plan_device_status.argtypes = [vp, vp]
    lib.snapshot_pack.argtypes = [vp, u32, u64, C.POINTER(_State), vp, C.c_size_t, vp]
    lib.snapshot_drain.argtypes = [vp, u32, vp, vp, C.c_size_t, vp, vp, vp]
    lib.snapshot_drain_range.argtypes = [vp, u32, vp, u64, vp, C.c_size_t, vp, vp, vp]
    lib.snapshot_peek.argtypes = [vp, u32, vp, C.POINTER(_Header)]
    lib.restore_unpack.argtypes = [vp, u32, vp, vp, C.POINTER(_State), vp, vp]
    lib.convert_replay.argtypes = [vp, C.POINTER(_Adam), vp, C.POINTER(vp), C.POINTER(_State), vp]
    lib.convert_replay_static.argtypes = [vp, C.POINTER(_Adam), vp, vp, vp, vp]
    lib.convert_window_step.argtypes = [vp, u32, vp, vp, C.POINTER(_Adam), vp, C.POINTER(vp), C.POINTER(_State), vp]
    lib.moev_copy_probe.argtypes = [vp, vp, C.c_size_t, u32, C.c_int, vp]
    lib.moev_stream_probe.argtypes = [C.c_int, vp, vp, C.c_size_t, u32, C.c_int, vp]
    lib.moev_arith_selfcheck.argtypes = [C.c_int, C.c_float, u32, u64, u64, C.POINTER(u64), vp]
    lib.uplog_create.argtypes = [vp, C.c_size_t, u32, C.POINTER(vp)]
    lib.uplog_free.argtypes = [vp]
    lib.uplog_free.restype = None
    lib.uplog_reserve.argtypes = [vp, u64, u32, u32, C.c_size_t, C.POINTER(u64)]
    lib.uplog_append.argtypes = [vp, u64, u32, u32, vp, C.c_size_t, vp, vp]
    lib.uplog_find.argtypes = [vp, u64, u32, u32, C.POINTER(vp), C.POINTER(C.c_size_t)]
    lib.uplog_replay.argtypes = [vp, u64, u32, u32, vp, C.c_size_t, vp]
    lib.uplog_gc.argtypes = [vp, u64]
    lib.uplog_gc.restype = i64
    lib.uplog_stats.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64)]
    return lib


_lib = _load()


def _check(rc: int):
    if rc < 0:
        raise MoevError(rc, (_lib.moev_last_error() or b"").decode())
    return rc


def _addr(x) -> Optional[int]:
    """Address of a torch tensor / object with data_ptr(), or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream  # torch.cuda.Stream


def _event(e) -> Optional[int]:
    if e is None:
        return None
    if isinstance(e, int):
        return e
    return e.cuda_event  # torch.cuda.Event (must have been recorded or created eagerly)


def _ptr_array(items: Sequence) -> C.Array:
    return (C.c_void_p * len(items))(*[_addr(t) for t in items])


class State:
    """moev_state: four host arrays of device pointers (torch tensors are kept alive here)."""

    def __init__(self, master: Sequence, m: Sequence, v: Sequence, compute: Sequence):
        self.tensors = (list(master), list(m), list(v), list(compute))
        self._arrays = [_ptr_array(g) for g in self.tensors]
        self.c = _State(*self._arrays)


# ---- Algorithm 1 helpers -----------------------------------------------------------------
def moev_find_window_size(n_ops, t_iter_s, compute_bytes_per_op, master_bytes_per_op, optim_bytes_per_op,
                          host_link_Bps):
    w, a = C.c_uint32(), C.c_uint32()
    _check(_lib.moev_find_window_size(n_ops, t_iter_s, compute_bytes_per_op, master_bytes_per_op,
                                      optim_bytes_per_op, host_link_Bps, C.byref(w), C.byref(a)))
    return w.value, a.value


def moev_order_operators(popularity: Sequence[float]) -> List[int]:
    n = len(popularity)
    out = (C.c_uint32 * n)()
    _check(_lib.moev_order_operators(n, (C.c_double * n)(*popularity), out))
    return list(out)


def moev_reorder_needed(old_freq: Sequence[float], new_freq: Sequence[float], rel_change=0.10,
                        min_fraction=0.25) -> bool:
    n = len(old_freq)
    return bool(_check(_lib.moev_reorder_needed(n, (C.c_double * n)(*old_freq), (C.c_double * n)(*new_freq),
                                                rel_change, min_fraction)))


def moev_popularity_time_decayed(alpha: float, previous: Sequence[float], batch_count: Sequence[float]) -> List[float]:
    n = len(previous)
    out = (C.c_double * n)()
    _check(_lib.moev_popularity_time_decayed(n, alpha, (C.c_double * n)(*previous), (C.c_double * n)(*batch_count), out))
    return list(out)


def moev_popularity_capacity_aware(popularity: Sequence[float], capacity: Sequence[float]) -> List[float]:
    n = len(popularity)
    out = (C.c_double * n)()
    _check(_lib.moev_popularity_capacity_aware(n, (C.c_double * n)(*popularity), (C.c_double * n)(*capacity), out))
    return list(out)


def moev_ettr(t_ckpt_s, t_iter_s, ckpt_interval_iters, expected_recovery_s, mtbf_s) -> float:
    return _lib.moev_ettr(t_ckpt_s, t_iter_s, ckpt_interval_iters, expected_recovery_s, mtbf_s)


def moev_recovery_time(sparse: bool, interval_or_window: float, t_iter_s: float):
    e, w = C.c_double(), C.c_double()
    _check(_lib.moev_recovery_time(int(bool(sparse)), interval_or_window, t_iter_s, C.byref(e), C.byref(w)))
    return e.value, w.value


# ---- plan --------------------------------------------------------------------------------
def moev_bias_corrections(beta1: float, beta2: float, step: int):
    b1, b2 = C.c_float(), C.c_float()
    _check(_lib.moev_bias_corrections(beta1, beta2, step, C.byref(b1), C.byref(b2)))
    return b1.value, b2.value


class Plan:
    """Owner of a moev_plan* (freed with the object)."""

    def __init__(self, handle: int):
        self.handle = C.c_void_p(handle)

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:  # at interpreter shutdown the module globals may already be gone
            _lib.ckpt_plan_free(h)


def ckpt_plan(tensors: Sequence, mode: int = EXPLICIT, window: int = 0, n_active: int = 0,
              order: Optional[Sequence[int]] = None, slot_of_op: Optional[Sequence[int]] = None,
              t_iter_s: float = 0.0, host_link_Bps: float = 0.0, align: int = 0,
              widths=(0, 0, 0, 0), n_ops: Optional[int] = None, formats=(0, 0, 0, 0)) -> Plan:
    nt = len(tensors)
    if n_ops is None:
        n_ops = (max(op for op, _ in tensors) + 1) if nt else 0
    ts = (_Tensor * max(nt, 1))(*[_Tensor(int(o), int(n)) for o, n in tensors])
    order_a = (C.c_uint32 * len(order))(*order) if order is not None else None
    slots_a = (C.c_uint32 * len(slot_of_op))(*slot_of_op) if slot_of_op is not None else None
    if len(widths) == 3:  # (master, both moments, compute)
        widths = (widths[0], widths[1], widths[1], widths[2])
    cfg = _PlanCfg(n_ops, nt, ts, mode, window, n_active, order_a, slots_a, t_iter_s, host_link_Bps, align,
                   widths[0], widths[1], widths[2], widths[3], formats[0], formats[1], formats[2], formats[3])
    out = C.c_void_p()
    _check(_lib.ckpt_plan(C.byref(cfg), C.byref(out)))
    return Plan(out.value)


def ckpt_plan_free(plan: Plan) -> None:
    h, plan.handle = plan.handle, None
    if h:
        _lib.ckpt_plan_free(h)


def ckpt_plan_window(plan): return _lib.ckpt_plan_window(plan.handle)
def ckpt_plan_n_ops(plan): return _lib.ckpt_plan_n_ops(plan.handle)
def ckpt_plan_n_tensors(plan): return _lib.ckpt_plan_n_tensors(plan.handle)
def ckpt_plan_n_active(plan): return _lib.ckpt_plan_n_active(plan.handle)
def ckpt_plan_hash(plan): return _lib.ckpt_plan_hash(plan.handle)
def ckpt_plan_pack_tile_bytes(plan, slot): return _lib.ckpt_plan_pack_tile_bytes(plan.handle, slot)
def ckpt_plan_width(plan, kind): return _lib.ckpt_plan_width(plan.handle, kind)
def ckpt_plan_format(plan, kind): return _lib.ckpt_plan_format(plan.handle, kind)
def ckpt_plan_packed_bytes(plan, slot): return _lib.ckpt_plan_packed_bytes(plan.handle, slot)
def ckpt_plan_max_packed_bytes(plan): return _lib.ckpt_plan_max_packed_bytes(plan.handle)
def ckpt_plan_n_segments(plan, slot): return _lib.ckpt_plan_n_segments(plan.handle, slot)
def ckpt_plan_active_params(plan, i): return _lib.ckpt_plan_active_params(plan.handle, i)


def ckpt_plan_slot_of_op(plan) -> List[int]:
    out = (C.c_uint32 * ckpt_plan_n_ops(plan))()
    _check(_lib.ckpt_plan_slot_of_op(plan.handle, out))
    return list(out)


def ckpt_plan_order(plan) -> List[int]:
    out = (C.c_uint32 * ckpt_plan_n_ops(plan))()
    _check(_lib.ckpt_plan_order(plan.handle, out))
    return list(out)


def ckpt_plan_segments(plan, slot):
    """-> [(kind, tensor, nbytes, dst_off)] of the slot (host-computed offsets)."""
    n = _check(_lib.ckpt_plan_segments(plan.handle, slot, None, 0))
    segs = (_Segment * max(n, 1))()
    _check(_lib.ckpt_plan_segments(plan.handle, slot, segs, n))
    return [(s.kind, s.tensor, s.nbytes, s.dst_off) for s in segs[:n]]


def moev_tune(plan, knob: int, value: int) -> None:
    _check(_lib.moev_tune(plan.handle, knob, value))


def moev_tune_get(plan, knob: int) -> int:
    return _lib.moev_tune_get(plan.handle, knob)


def ckpt_plan_upload(plan, stream=None) -> None:
    _check(_lib.ckpt_plan_upload(plan.handle, _stream(stream)))


def ckpt_plan_device_layout(plan, slot, stream=None):
    """-> (dst_off list, tile_start list, packed_bytes) as computed by the on-device scan."""
    n = ckpt_plan_n_segments(plan, slot)
    off = (C.c_uint64 * max(n, 1))()
    tiles = (C.c_uint32 * (n + 1))()
    total = C.c_uint64()
    _check(_lib.ckpt_plan_device_layout(plan.handle, slot, off, tiles, C.byref(total), _stream(stream)))
    return list(off[:n]), list(tiles), total.value


def ckpt_plan_device_status(plan, stream=None) -> None:
    _check(_lib.ckpt_plan_device_status(plan.handle, _stream(stream)))


# ---- snapshot / conversion ---------------------------------------------------------------
def snapshot_pack(plan, slot: int, it: int, state: State, d_packed, cap: Optional[int] = None, stream=None):
    if cap is None:
        cap = d_packed.numel() * d_packed.element_size()
    _check(_lib.snapshot_pack(plan.handle, slot, it, C.byref(state.c), _addr(d_packed), cap, _stream(stream)))


def snapshot_drain(plan, slot: int, d_packed, h_pinned, cap: Optional[int] = None, side_stream=None,
                   pack_done=None, drained=None):
    if cap is None:
        cap = h_pinned.numel() * h_pinned.element_size()
    _check(_lib.snapshot_drain(plan.handle, slot, _addr(d_packed), _addr(h_pinned), cap, _stream(side_stream),
                               _event(pack_done), _event(drained)))


def snapshot_drain_range(plan, slot: int, d_packed, offset: int, h_pinned, nbytes: int, side_stream=None,
                         pack_done=None, drained=None):
    _check(_lib.snapshot_drain_range(plan.handle, slot, _addr(d_packed), offset, _addr(h_pinned), nbytes,
                                     _stream(side_stream), _event(pack_done), _event(drained)))


def snapshot_peek(plan, slot: int, h_packed) -> dict:
    hd = _Header()
    _check(_lib.snapshot_peek(plan.handle, slot, _addr(h_packed), C.byref(hd)))
    return {f: getattr(hd, f) for f, _ in _Header._fields_}


def restore_unpack(plan, slot: int, h_pinned, d_packed, state: State, d_active_mask, stream=None):
    _check(_lib.restore_unpack(plan.handle, slot, _addr(h_pinned), _addr(d_packed), C.byref(state.c),
                               _addr(d_active_mask), _stream(stream)))


def convert_replay(plan, lr, beta1, beta2, eps, weight_decay, step: int, d_active_mask, grads: Sequence,
                   state: State, stream=None, d_scales=None):
    adam = _Adam(lr, beta1, beta2, eps, weight_decay, step, _addr(d_scales))
    g = _ptr_array(grads)
    _check(_lib.convert_replay(plan.handle, C.byref(adam), _addr(d_active_mask), g, C.byref(state.c),
                               _stream(stream)))


def convert_replay_static(plan, lr, beta1, beta2, eps, weight_decay, step: int, d_active_mask, d_grad_table,
                          d_state_table, stream=None, d_scales=None):
    """d_grad_table / d_state_table: DEVICE arrays of device pointers ([n_tensors] and [4 * n_tensors] kind-major)."""
    adam = _Adam(lr, beta1, beta2, eps, weight_decay, step, _addr(d_scales))
    _check(_lib.convert_replay_static(plan.handle, C.byref(adam), _addr(d_active_mask), _addr(d_grad_table),
                                      _addr(d_state_table), _stream(stream)))


def convert_window_step(plan, slot: int, h_pinned, d_packed, lr, beta1, beta2, eps, weight_decay, step: int,
                        d_active_mask, grads: Sequence, state: State, stream=None, d_scales=None):
    adam = _Adam(lr, beta1, beta2, eps, weight_decay, step, _addr(d_scales))
    g = _ptr_array(grads)
    _check(_lib.convert_window_step(plan.handle, slot, _addr(h_pinned), _addr(d_packed), C.byref(adam),
                                    _addr(d_active_mask), g, C.byref(state.c), _stream(stream)))


def moev_arith_selfcheck(what: int, divisor: float, first_bits: int, count: int, seed: int = 0, stream=None) -> int:
    """-> number of inputs on which the plain division / square root differ from the full IEEE sequences."""
    out = C.c_uint64()
    _check(_lib.moev_arith_selfcheck(what, C.c_float(divisor), C.c_uint32(first_bits), C.c_uint64(count), C.c_uint64(seed),
                                     C.byref(out), _stream(stream)))
    return out.value


def moev_copy_probe(d_dst, d_src, nbytes: int, blocks: int = 0, nontemporal: int = 1, stream=None):
    _check(_lib.moev_copy_probe(_addr(d_dst), _addr(d_src), nbytes, blocks, nontemporal, _stream(stream)))


# ---- upstream logging ring -----------------------------------------------------------------
ACTIVATION, GRADIENT = 0, 1


def moev_stream_probe(mode: int, d_dst, d_src, nbytes: int, value: int = 0, nontemporal: int = 1, stream=None):
    """mode 1: read d_src[nbytes] only; mode 2: fill d_dst[nbytes] with the 32-bit value; mode 3: copy with two 512-byte
    pieces `value` bytes apart per wavefront instruction (size and pointers multiples of 2 x value)."""
    _check(_lib.moev_stream_probe(mode, _addr(d_dst), _addr(d_src), nbytes, value, nontemporal, _stream(stream)))


class UpLog:
    """Owner of a moev_uplog* over a caller-owned pinned host buffer (kept alive here)."""

    def __init__(self, handle: int, ring):
        self.handle = C.c_void_p(handle)
        self.ring = ring

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.uplog_free(h)


def uplog_create(h_pinned_ring, ring_bytes: Optional[int] = None, max_entries: int = 4096) -> UpLog:
    if ring_bytes is None:
        ring_bytes = h_pinned_ring.numel() * h_pinned_ring.element_size()
    out = C.c_void_p()
    _check(_lib.uplog_create(_addr(h_pinned_ring), ring_bytes, max_entries, C.byref(out)))
    return UpLog(out.value, h_pinned_ring)


def uplog_reserve(log: UpLog, it: int, micro_batch: int, kind: int, nbytes: int) -> int:
    off = C.c_uint64()
    _check(_lib.uplog_reserve(log.handle, it, micro_batch, kind, nbytes, C.byref(off)))
    return off.value


def uplog_append(log: UpLog, it: int, micro_batch: int, kind: int, d_tensor, nbytes: Optional[int] = None,
                 side_stream=None, ready=None) -> None:
    if nbytes is None:
        nbytes = d_tensor.numel() * d_tensor.element_size()
    _check(_lib.uplog_append(log.handle, it, micro_batch, kind, _addr(d_tensor), nbytes, _stream(side_stream),
                             _event(ready)))


def uplog_find(log: UpLog, it: int, micro_batch: int, kind: int):
    """-> (host address, nbytes)."""
    p, n = C.c_void_p(), C.c_size_t()
    _check(_lib.uplog_find(log.handle, it, micro_batch, kind, C.byref(p), C.byref(n)))
    return p.value, n.value


def uplog_replay(log: UpLog, it: int, micro_batch: int, kind: int, d_dst, cap: Optional[int] = None, stream=None):
    if cap is None:
        cap = d_dst.numel() * d_dst.element_size()
    _check(_lib.uplog_replay(log.handle, it, micro_batch, kind, _addr(d_dst), cap, _stream(stream)))


def uplog_gc(log: UpLog, first_kept_iter: int) -> int:
    return _check(_lib.uplog_gc(log.handle, first_kept_iter))


def uplog_stats(log: UpLog):
    """-> (live entries, bytes in use, capacity)."""
    e, b, c = C.c_uint64(), C.c_uint64(), C.c_uint64()
    _check(_lib.uplog_stats(log.handle, C.byref(e), C.byref(b), C.byref(c)))
    return e.value, b.value, c.value
