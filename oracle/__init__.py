"""CPU oracle for the sparse-snapshot / sparse-to-dense hot path (MoEvement, arXiv 2412.15411).

TEST INFRASTRUCTURE ONLY.  The arithmetic lives in ``moev_oracle.c`` (plain C, written from
the paper); this module is its ctypes face plus the window-level drivers (dense run,
snapshot taking, conversion) that follow Sec. 3.2 / Sec. 3.3 step by step.  Nothing here
imports, loads or shares code with the HIP library, and the library never imports this.
Only tests, the smoke check and the bench's cpu_baseline leg may use it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moev_oracle.c")
_LIB = os.path.join(_HERE, "libmoev_oracle.so")

MASTER, ADAM_M, ADAM_V, COMPUTE = 0, 1, 2, 3
HEADER_BYTES = 256
OK, BAD_ARG, NOT_A_SCHEDULE, TOO_SMALL, BAD_SNAPSHOT = 0, -1, -2, -3, -4
FMT_F32, FMT_F16, FMT_BF16, FMT_E4M3, FMT_E5M2 = 1, 2, 3, 4, 5
FMT_BYTES = {FMT_F32: 4, FMT_F16: 2, FMT_BF16: 2, FMT_E4M3: 1, FMT_E5M2: 1}
FMT_DTYPE = {FMT_F32: np.float32, FMT_F16: np.uint16, FMT_BF16: np.uint16, FMT_E4M3: np.uint8, FMT_E5M2: np.uint8}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, so fp32 op order is as written)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "moev_oracle.h")))
    if force or stale:
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-math-errno", "-Wall", "-Wextra",
             "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Tensor(C.Structure):
    _fields_ = [("op", C.c_uint32), ("numel", C.c_uint64)]


class _Widths(C.Structure):
    _fields_ = [("master", C.c_uint32), ("m", C.c_uint32), ("v", C.c_uint32), ("compute", C.c_uint32)]


class _Segment(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("tensor", C.c_uint32), ("nbytes", C.c_uint64),
                ("dst_off", C.c_uint64)]


class _Model(C.Structure):
    _fields_ = [("n_ops", C.c_uint32), ("n_tensors", C.c_uint32), ("tensors", C.POINTER(_Tensor)),
                ("order", C.POINTER(C.c_uint32)), ("slot_of_op", C.POINTER(C.c_uint32)),
                ("window", C.c_uint32), ("align", C.c_uint32), ("width", _Widths), ("fmt", C.c_uint32 * 4)]


class _State(C.Structure):
    _fields_ = [("master", C.POINTER(C.c_void_p)), ("m", C.POINTER(C.c_void_p)),
                ("v", C.POINTER(C.c_void_p)), ("compute", C.POINTER(C.c_void_p))]


class _AdamHP(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_layout.restype = C.c_int64
        _lib.orc_plan_hash.restype = C.c_uint64
        _lib.orc_fnv1a64.restype = C.c_uint64
        _lib.orc_fnv1a64.argtypes = [C.c_char_p, C.c_uint64]
        _lib.orc_bf16_rne.restype = C.c_uint16
        _lib.orc_bf16_rne.argtypes = [C.c_float]
        _lib.orc_adam_tensor.restype = None
        _lib.orc_bias_corrections.restype = None
        _lib.orc_decode.restype = C.c_double
        _lib.orc_decode.argtypes = [C.c_uint32, C.c_uint32]
        _lib.orc_encode.restype = C.c_uint32
        _lib.orc_encode.argtypes = [C.c_uint32, C.c_float]
        _lib.orc_fmt_bytes.restype = C.c_uint32
        _lib.orc_fmt_bytes.argtypes = [C.c_uint32]
        _lib.orc_find_window_size.argtypes = [C.c_uint32, C.c_double, C.c_double, C.c_double,
                                              C.c_double, C.c_double, C.POINTER(C.c_uint32),
                                              C.POINTER(C.c_uint32)]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


# --------------------------------------------------------------------------------------
# model / state containers
# --------------------------------------------------------------------------------------
@dataclass
class Model:
    """Operators, their tensors and the window schedule (Algorithm 1's O, O_Ordered, W_sparse)."""
    tensors: List[Tuple[int, int]]            # (op, numel), grouped by ascending op
    order: Sequence[int]                      # O_Ordered
    slot_of_op: Sequence[int]
    window: int
    align: int = 256
    widths: Tuple[int, ...] = (4, 4, 4, 2)   # bytes per element: master, Adam m, Adam v, compute
    formats: Optional[Tuple[int, int, int, int]] = None  # FMT_* per kind (low-precision regimes, Sec. 5.6)
    _keep: list = field(default_factory=list, repr=False)

    @property
    def n_ops(self) -> int:
        return len(self.slot_of_op)

    @property
    def n_tensors(self) -> int:
        return len(self.tensors)

    def c(self) -> _Model:
        ts = (_Tensor * self.n_tensors)(*[_Tensor(int(o), int(n)) for o, n in self.tensors])
        order = (C.c_uint32 * self.n_ops)(*[int(x) for x in self.order])
        slots = (C.c_uint32 * self.n_ops)(*[int(x) for x in self.slot_of_op])
        self._keep = [ts, order, slots]
        w = tuple(int(x) for x in self.widths)
        if len(w) == 3:  # (master, both moments, compute)
            w = (w[0], w[1], w[1], w[2])
        fmt = (C.c_uint32 * 4)(*(self.formats if self.formats is not None else (0, 0, 0, 0)))
        return _Model(self.n_ops, self.n_tensors, ts, order, slots, int(self.window), int(self.align), _Widths(*w), fmt)


@dataclass
class State:
    """Dense training state: one contiguous numpy array per tensor and kind."""
    master: List[np.ndarray]
    m: List[np.ndarray]
    v: List[np.ndarray]
    compute: List[np.ndarray]
    _keep: list = field(default_factory=list, repr=False)

    def c(self) -> _State:
        arrs = []
        for group in (self.master, self.m, self.v, self.compute):
            for a in group:
                assert a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
            arrs.append((C.c_void_p * len(group))(*[a.ctypes.data for a in group]))
        self._keep = arrs
        return _State(*arrs)

    def clone(self) -> "State":
        return State(*[[a.copy() for a in g] for g in (self.master, self.m, self.v, self.compute)])

    def kinds(self):
        return {"master": self.master, "m": self.m, "v": self.v, "compute": self.compute}


@dataclass
class AdamHP:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.0

    def c(self) -> _AdamHP:
        return _AdamHP(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay)


# --------------------------------------------------------------------------------------
# schedule (Algorithm 1)
# --------------------------------------------------------------------------------------
def find_window_size(o_total, t_iter, s_compute, s_master, s_optim, b_pcie):
    w, a = C.c_uint32(), C.c_uint32()
    rc = lib().orc_find_window_size(o_total, t_iter, s_compute, s_master, s_optim, b_pcie,
                                    C.byref(w), C.byref(a))
    if rc:
        raise OracleError(rc, "find_window_size")
    return w.value, a.value


def generate_schedule(order: Sequence[int], o_active: int):
    n = len(order)
    o = (C.c_uint32 * n)(*[int(x) for x in order])
    slots = (C.c_uint32 * n)()
    w = C.c_uint32()
    rc = lib().orc_generate_schedule(C.c_uint32(n), o, C.c_uint32(o_active), slots, C.byref(w))
    if rc:
        raise OracleError(rc, "generate_schedule")
    return list(slots), w.value


def order_by_popularity(popularity: Sequence[float]):
    n = len(popularity)
    pop = (C.c_double * n)(*[float(x) for x in popularity])
    order = (C.c_uint32 * n)()
    rc = lib().orc_order_by_popularity(C.c_uint32(n), pop, order)
    if rc:
        raise OracleError(rc, "order_by_popularity")
    return list(order)


def order_from_slots(slot_of_op: Sequence[int]):
    """O_Ordered for an explicitly given slot assignment: by slot, then by operator id."""
    return sorted(range(len(slot_of_op)), key=lambda e: (slot_of_op[e], e))


def check_schedule(order, slot_of_op, window) -> int:
    n = len(slot_of_op)
    o = (C.c_uint32 * n)(*[int(x) for x in order])
    s = (C.c_uint32 * n)(*[int(x) for x in slot_of_op])
    return lib().orc_check_schedule(C.c_uint32(n), o, s, C.c_uint32(window))


def popularity_time_decayed(alpha, previous, batch_count):
    n = len(previous)
    out = (C.c_double * n)()
    lib().orc_popularity_time_decayed(C.c_uint32(n), C.c_double(alpha), (C.c_double * n)(*previous),
                                      (C.c_double * n)(*batch_count), out)
    return list(out)


def popularity_capacity_aware(popularity, capacity):
    n = len(popularity)
    out = (C.c_double * n)()
    lib().orc_popularity_capacity_aware(C.c_uint32(n), (C.c_double * n)(*popularity), (C.c_double * n)(*capacity), out)
    return list(out)


def ettr(t_ckpt, t_iter, ckpt_interval, expected_recovery, mtbf):
    f = lib().orc_ettr
    f.restype = C.c_double
    f.argtypes = [C.c_double] * 5
    return f(t_ckpt, t_iter, ckpt_interval, expected_recovery, mtbf)


def recovery(kind, interval_or_window, t_iter):
    """kind = 'dense' or 'sparse' -> (expected, worst) recovery time in seconds (Sec. 3.6)."""
    e, w = C.c_double(), C.c_double()
    f = lib().orc_recovery_dense if kind == "dense" else lib().orc_recovery_sparse
    f.restype = None
    f.argtypes = [C.c_double, C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    f(interval_or_window, t_iter, C.byref(e), C.byref(w))
    return e.value, w.value


# --------------------------------------------------------------------------------------
# layout / pack / unpack
# --------------------------------------------------------------------------------------
def fnv1a64(data: bytes) -> int:
    return lib().orc_fnv1a64(data, C.c_uint64(len(data)))


def plan_hash(model: Model) -> int:
    cm = model.c()
    return lib().orc_plan_hash(C.byref(cm))


def layout(model: Model, slot: int):
    """-> ([(kind, tensor, nbytes, dst_off)], packed_bytes)."""
    cm = model.c()
    total = C.c_uint64()
    n = lib().orc_layout(C.byref(cm), C.c_uint32(slot), None, C.c_uint64(0), C.byref(total))
    if n < 0:
        raise OracleError(n, "layout")
    segs = (_Segment * max(n, 1))()
    lib().orc_layout(C.byref(cm), C.c_uint32(slot), segs, C.c_uint64(n), C.byref(total))
    return [(s.kind, s.tensor, s.nbytes, s.dst_off) for s in segs[:n]], total.value


def pack(model: Model, slot: int, it: int, state: State, out: Optional[np.ndarray] = None) -> np.ndarray:
    _, total = layout(model, slot)
    if out is None:
        out = np.full(total, 0xA5, dtype=np.uint8)  # poisoned, so missing writes show
    cm, cs = model.c(), state.c()
    rc = lib().orc_pack(C.byref(cm), C.c_uint32(slot), C.c_uint64(it), C.byref(cs),
                        C.c_void_p(out.ctypes.data), C.c_uint64(out.nbytes))
    if rc:
        raise OracleError(rc, "pack")
    return out


def unpack(model: Model, slot: int, packed: np.ndarray, state: State, mask: np.ndarray) -> int:
    assert mask.dtype == np.uint8 and mask.size == model.n_ops
    assert packed.dtype == np.uint8 and packed.flags["C_CONTIGUOUS"]
    cm, cs = model.c(), state.c()
    it = C.c_uint64()
    rc = lib().orc_unpack(C.byref(cm), C.c_uint32(slot), C.c_void_p(packed.ctypes.data),
                          C.c_uint64(packed.nbytes), C.byref(cs), C.c_void_p(mask.ctypes.data),
                          C.byref(it))
    if rc:
        raise OracleError(rc, "unpack")
    return it.value


# --------------------------------------------------------------------------------------
# Adam replay
# --------------------------------------------------------------------------------------
def bf16_rne(x: float) -> int:
    return lib().orc_bf16_rne(C.c_float(x))


def bf16_rne_array(x: np.ndarray) -> np.ndarray:
    """Elementwise through the C routine's loop (adam_tensor with lr=0 would also change m, v)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return np.array([lib().orc_bf16_rne(C.c_float(float(v))) for v in x.ravel()], dtype=np.uint16).reshape(x.shape)


def bias_corrections(hp: AdamHP, step: int):
    b1, b2 = C.c_float(), C.c_float()
    chp = hp.c()
    lib().orc_bias_corrections(C.byref(chp), C.c_uint64(step), C.byref(b1), C.byref(b2))
    return b1.value, b2.value


def adam_tensor(p, m, v, g, c, hp: AdamHP, step: int) -> None:
    """In-place Adam step of iteration `step` on one tensor (fp32 p, m, v, g; uint16 bf16 c or None)."""
    for a in (p, m, v, g):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.size == p.size
    cptr = None
    if c is not None:
        assert c.dtype == np.uint16 and c.size == p.size
        cptr = C.c_void_p(c.ctypes.data)
    chp = hp.c()
    lib().orc_adam_tensor(C.c_void_p(p.ctypes.data), C.c_void_p(m.ctypes.data), C.c_void_p(v.ctypes.data),
                          C.c_void_p(g.ctypes.data), cptr, C.c_uint64(p.size), C.byref(chp),
                          C.c_uint64(step))


def decode(fmt: int, bits: int) -> float:
    """Value of a bit pattern of storage format `fmt` (Sec. 5.6 regimes)."""
    return lib().orc_decode(fmt, int(bits))


def encode(fmt: int, x: float) -> int:
    """Bit pattern of the value of format `fmt` nearest to the FP32 number x (ties to even)."""
    return lib().orc_encode(fmt, C.c_float(x))


def adam_tensor_lp(p, m, v, g, c, hp: AdamHP, step: int, formats, scales=(1.0, 1.0, 1.0, 1.0)) -> None:
    """In-place optimizer step on one tensor stored in `formats` (master, m, v, compute)."""
    for a, f in zip((p, m, v, c), formats):
        if a is not None:
            assert a.dtype == FMT_DTYPE[f] and a.flags["C_CONTIGUOUS"] and a.size == p.size
    assert g.dtype == np.float32 and g.size == p.size and g.flags["C_CONTIGUOUS"]
    chp = hp.c()
    rc = lib().orc_adam_tensor_lp(C.c_void_p(p.ctypes.data), C.c_void_p(m.ctypes.data), C.c_void_p(v.ctypes.data),
                                  C.c_void_p(g.ctypes.data), None if c is None else C.c_void_p(c.ctypes.data),
                                  C.c_uint64(p.size), C.byref(chp), C.c_uint64(step),
                                  (C.c_uint32 * 4)(*formats), (C.c_float * 4)(*scales))
    if rc:
        raise OracleError(rc, "adam_tensor_lp")


def replay_step(model: Model, hp: AdamHP, step: int, mask: np.ndarray, grads: List[np.ndarray],
                state: State, scales: Optional[np.ndarray] = None) -> None:
    """scales: float32 array [4, n_tensors] (kind-major) for models with `formats`, or None."""
    assert mask.dtype == np.uint8 and mask.size == model.n_ops
    cm, cs, chp = model.c(), state.c(), hp.c()
    for g, (_, n) in zip(grads, model.tensors):
        assert g.dtype == np.float32 and g.size == n and g.flags["C_CONTIGUOUS"]
    gp = (C.c_void_p * len(grads))(*[g.ctypes.data for g in grads])
    if model.formats is not None:
        sp = None
        if scales is not None:
            assert scales.dtype == np.float32 and scales.shape == (4, model.n_tensors) and scales.flags["C_CONTIGUOUS"]
            sp = C.c_void_p(scales.ctypes.data)
        rc = lib().orc_replay_step_lp(C.byref(cm), (C.c_uint32 * 4)(*model.formats), C.byref(chp), C.c_uint64(step),
                                      C.c_void_p(mask.ctypes.data), gp, C.byref(cs), sp)
        if rc:
            raise OracleError(rc, "replay_step_lp")
        return
    rc = lib().orc_replay_step(C.byref(cm), C.byref(chp), C.c_uint64(step), C.c_void_p(mask.ctypes.data),
                               gp, C.byref(cs))
    if rc:
        raise OracleError(rc, "replay_step")


# --------------------------------------------------------------------------------------
# window-level drivers (Sec. 3.2 worked example, Sec. 3.3 walk-through)
# --------------------------------------------------------------------------------------
def dense_run(model: Model, state: State, hp: AdamHP, grads_of_step, t0: int, n_steps: int,
              snapshots: bool = False):
    """Fault-free training from the state after iteration t0: every operator takes every
    optimizer step (nothing is frozen outside recovery).  With snapshots=True, sparse snapshot
    SS_{t0+k} (slot k) is taken from the state after step t0+k, i.e. while iteration t0+k+1
    would be running (Sec. 3.2: "iteration 11 ... SS_10").  Returns the list of snapshots.
    grads_of_step(t) -> list of per-tensor fp32 gradient arrays of iteration t."""
    everyone = np.ones(model.n_ops, dtype=np.uint8)
    snaps = []
    for k in range(n_steps):
        if snapshots and k < model.window:
            snaps.append(pack(model, k, t0 + k, state))
        replay_step(model, hp, t0 + k + 1, everyone, grads_of_step(t0 + k + 1), state)
    return snaps


def poisoned_like(state: State) -> State:
    """A state holding NaN / 0xFFFF patterns everywhere: whatever conversion does not restore shows."""
    out = state.clone()
    for g in (out.master, out.m, out.v, out.compute):
        for a in g:
            if a.dtype == np.float32:
                a.view(np.uint32)[...] = 0x7FC0DEAD
            else:
                a.view(np.uint8)[...] = 0xFF
    return out


def convert(model: Model, snaps: List[np.ndarray], hp: AdamHP, grads_of_step, state: State,
            trace: Optional[list] = None) -> np.ndarray:
    """Sparse-to-dense conversion (Sec. 3.3 walk-through): for i = 0..W-1 load SS_{t0+i}, which
    activates the operators whose FP32 state it carries, then replay iteration t0+i+1 on the
    active operators only.  `state` is overwritten in place; returns the final active mask.
    If `trace` is a list, the mask after every load and the mask used by every replay are
    appended as ("load", i, mask) / ("replay", step, mask)."""
    mask = np.zeros(model.n_ops, dtype=np.uint8)
    for i in range(model.window):
        it = unpack(model, i, snaps[i], state, mask)
        if trace is not None:
            trace.append(("load", it, mask.copy()))
        replay_step(model, hp, it + 1, mask, grads_of_step(it + 1), state)
        if trace is not None:
            trace.append(("replay", it + 1, mask.copy()))
    return mask


# --------------------------------------------------------------------------------------
# upstream logging (Sec. 3.4)
# --------------------------------------------------------------------------------------
class UpstreamLog:
    """What upstream logging keeps (Sec. 3.4): stage-boundary tensors, activations of the forward
    pass (kind 0) and gradients of the backward pass (kind 1), tagged with the iteration and the
    micro-batch; logs older than the latest persisted sparse checkpoint are dropped."""

    def __init__(self):
        self.store = {}

    def append(self, it: int, micro_batch: int, kind: int, data: bytes) -> None:
        assert kind in (0, 1) and (it, micro_batch, kind) not in self.store
        self.store[(it, micro_batch, kind)] = bytes(data)

    def find(self, it: int, micro_batch: int, kind: int):
        return self.store.get((it, micro_batch, kind))

    def gc(self, first_kept_iter: int) -> int:
        stale = [k for k in self.store if k[0] < first_kept_iter]
        for k in stale:
            del self.store[k]
        return len(stale)
