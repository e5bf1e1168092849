"""Seeded synthetic workloads: shapes, schedules and value generators.

This module only describes inputs (which operators exist, how large their tensors are,
which window slot each operator is scheduled in) and draws seeded random values with the
stated distributions.  It holds none of the method's arithmetic and is used both by the
HIP path's callers and by the tests that feed the CPU oracle, so both see the same bits.

Shapes stand in for the MoE models of the paper's evaluation (Sec. 5.1, model table):
a Mixtral-8x7B-shaped layer, fine-grained layers with shared experts (DeepSeek-MoE-like)
and one expert-parallel rank's share of a large MoE.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

T0 = 10  # iteration after which the first snapshot of a window is taken (the paper's example uses 10)


@dataclass
class Workload:
    name: str
    tensors: List[Tuple[int, int]]        # (op, numel) grouped by ascending op
    slot_of_op: List[int]                 # slot in which each operator is checkpointed with full state
    window: int
    order: List[int] = field(default_factory=list)  # O_Ordered; derived from slots when empty
    heavy_tail: bool = False              # gradients: 5% of entries scaled by 100
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.0
    t0: int = T0

    def __post_init__(self):
        if not self.order:
            self.order = sorted(range(len(self.slot_of_op)), key=lambda e: (self.slot_of_op[e], e))

    @property
    def n_ops(self) -> int:
        return len(self.slot_of_op)

    @property
    def n_tensors(self) -> int:
        return len(self.tensors)

    @property
    def n_params(self) -> int:
        return sum(n for _, n in self.tensors)

    def params_of_op(self) -> List[int]:
        out = [0] * self.n_ops
        for op, n in self.tensors:
            out[op] += n
        return out

    def slot_payload_bytes(self, slot: int, widths=(4, 4, 4, 2)) -> int:
        """Unpadded bytes a snapshot of `slot` carries: full state of the operators scheduled
        in the slot plus compute weights of the operators scheduled later.
        widths = bytes per element of master, Adam m, Adam v, compute."""
        full = widths[0] + widths[1] + widths[2]
        total = 0
        for e, p in enumerate(self.params_of_op()):
            if self.slot_of_op[e] == slot:
                total += full * p
            elif self.slot_of_op[e] > slot:
                total += widths[3] * p
        return total

    def active_params_at(self, i: int) -> int:
        """Parameters updated by replay iteration i of a conversion (operators with slot <= i)."""
        return sum(p for e, p in enumerate(self.params_of_op()) if self.slot_of_op[e] <= i)


# ---------------------------------------------------------------------------------------
# small integer hashing used for seeds and permutations (no floating point involved)
# ---------------------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def mix64(x: int) -> int:
    """splitmix64 finaliser."""
    x = (x + 0x9E3779B97F4A7C15) & _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def stream_seed(seed: int, stream: int, tensor: int, step: int = 0) -> int:
    h = mix64(seed)
    for part in (stream, tensor, step):
        h = mix64(h ^ mix64(part + 0x51ED27))
    return h & ((1 << 63) - 1)


def seeded_permutation(n: int, seed: int) -> List[int]:
    """Fisher-Yates shuffle driven by the counter hash above."""
    perm = list(range(n))
    for i in range(n - 1, 0, -1):
        j = mix64((seed << 20) ^ i) % (i + 1)
        perm[i], perm[j] = perm[j], perm[i]
    return perm


# ---------------------------------------------------------------------------------------
# the benchmark configurations
# ---------------------------------------------------------------------------------------
def _swiglu(d_model: int, d_ff: int) -> List[int]:
    return [d_model * d_ff, d_model * d_ff, d_ff * d_model]  # w1, w3, w2


def tiny_moe(n_experts=8, d_in=256, d_hidden=1024, window=4, n_active=2) -> Workload:
    """configs[0]: 8 experts, W_in 256x1024 and W_out 1024x256, W=4, 2 active per slot, round robin."""
    tensors = []
    for e in range(n_experts):
        tensors += [(e, d_in * d_hidden), (e, d_hidden * d_in)]
    slots = [e // n_active for e in range(n_experts)]
    assert max(slots) + 1 == window
    return Workload("c0_tiny_moe", tensors, slots, window, order=list(range(n_experts)))


def mixtral_layer(n_experts=8, d_model=4096, d_ff=14336, n_active=1) -> Workload:
    """configs[1]: one Mixtral-8x7B-shaped MoE layer, W=8, one expert active per slot."""
    tensors = []
    for e in range(n_experts):
        tensors += [(e, n) for n in _swiglu(d_model, d_ff)]
    slots = [e // n_active for e in range(n_experts)]
    return Workload("c1_mixtral_layer", tensors, slots, max(slots) + 1, order=list(range(n_experts)))


def fine_grained_stack(n_layers=4, n_routed=64, n_shared=2, d_model=2048, d_ff=1408, per_slot=4,
                       seed=0, heavy_tail=False, name="c2_fine_grained") -> Workload:
    """configs[2] / configs[4]: per layer, the routed experts are checkpointed in the order of a
    seeded permutation, `per_slot` of them per layer per slot; the always-routed shared experts
    are the most popular operators and therefore come last (they join the final slot)."""
    window = (n_routed + per_slot - 1) // per_slot
    per_layer = n_routed + n_shared
    tensors, slots = [], []
    for layer in range(n_layers):
        perm = seeded_permutation(n_routed, seed + layer)
        pos = {e: q for q, e in enumerate(perm)}
        for j in range(per_layer):
            op = layer * per_layer + j
            tensors += [(op, n) for n in _swiglu(d_model, d_ff)]
            slots.append(pos[j] // per_slot if j < n_routed else window - 1)
    return Workload(name, tensors, slots, window, heavy_tail=heavy_tail)


def ep_rank_share(n_layers=16, n_experts=32, d_model=4096, d_ff=2048, per_slot=4) -> Workload:
    """configs[3]: one GPU's share of a large MoE, uniform experts, W=8, 4 per layer per slot."""
    tensors, slots = [], []
    for layer in range(n_layers):
        for j in range(n_experts):
            op = layer * n_experts + j
            tensors += [(op, n) for n in _swiglu(d_model, d_ff)]
            slots.append(j // per_slot)
    return Workload("c3_ep_rank_share", tensors, slots, max(slots) + 1)


def conversion_stress(**kw) -> Workload:
    """configs[4]: configs[2] shapes with heavy-tailed gradients."""
    kw.setdefault("heavy_tail", True)
    kw.setdefault("name", "c4_conversion_stress")
    return fine_grained_stack(**kw)


CONFIGS = {
    "c0": tiny_moe,
    "c1": mixtral_layer,
    "c2": fine_grained_stack,
    "c3": ep_rank_share,
    "c4": conversion_stress,
}


# ---------------------------------------------------------------------------------------
# value generators
# ---------------------------------------------------------------------------------------
_STREAM = {"master": 1, "m": 2, "v": 3, "grad": 4, "tail": 5}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_state_tensor(wl: Workload, kind: str, t: int, seed: int = 0, device="cpu") -> torch.Tensor:
    """Tensor `t` of one kind of the state make_state() builds, regenerated on its own (same bits): lets a
    caller whose state does not fit twice compare one tensor at a time."""
    n = wl.tensors[t][1]
    src = "master" if kind == "compute" else kind
    std = 0.02 if src == "master" else 1e-3
    x = torch.empty(n, dtype=torch.float32, device=device)
    x.normal_(0.0, std, generator=_gen(device, stream_seed(seed, _STREAM[src], t)))
    if kind == "v":
        x.square_()
    return x.to(torch.bfloat16) if kind == "compute" else x


# Byte offsets (inside a 64 KiB block) at which the kinds of a `skew`ed state start: no two kinds are congruent modulo
# 64 KiB, the situation of small tensors carved out of shared allocator blocks.
SKEW_LEAD = {"master": 0, "m": 20 * 1024, "v": 40 * 1024 + 512, "compute": 12 * 1024, "grad": 52 * 1024 + 256}


def _flat_views(numels: Sequence[int], dtype: torch.dtype, device, lead: int = 0) -> List[torch.Tensor]:
    """Views into ONE allocation, one per tensor, each starting on a 4 KiB boundary (plus `lead` bytes): the way
    flat-partition optimizers (ZeRO-style) keep a kind of state.  Separate allocations per tensor and one flat buffer
    per kind are the same to the library (it sees pointers); what differs is where the memory lands physically."""
    width = torch.empty(0, dtype=dtype).element_size()
    seg = [(n * width + 4095) // 4096 * 4096 for n in numels]
    flat = torch.empty(max(sum(seg), 1) + lead, dtype=torch.uint8, device=device)
    out, off = [], lead
    for n, sz in zip(numels, seg):
        out.append(flat[off: off + n * width].view(dtype))
        off += sz
    return out


def make_state(wl: Workload, seed: int = 0, device="cpu", flat: bool = False, skew: bool = False) -> Dict[str, List[torch.Tensor]]:
    """master ~ N(0, std 0.02), m ~ N(0, std 1e-3), v = N(0, std 1e-3)^2 (so v >= 0),
    compute = bfloat16 copy of master.  One generator stream per (kind, tensor).  flat: every kind lives in one
    flat buffer (same values); skew: flat, and every kind starts at another offset inside a 64 KiB block (SKEW_LEAD)."""
    st: Dict[str, List[torch.Tensor]] = {"master": [], "m": [], "v": [], "compute": []}
    if flat or skew:
        numels = [n for _, n in wl.tensors]
        st = {k: _flat_views(numels, torch.bfloat16 if k == "compute" else torch.float32, device,
                             SKEW_LEAD[k] if skew else 0) for k in st}
        for t in range(wl.n_tensors):
            for k in ("master", "m", "v"):
                st[k][t].copy_(make_state_tensor(wl, k, t, seed, device))
            st["compute"][t].copy_(st["master"][t])
        return st
    for t in range(wl.n_tensors):
        p = make_state_tensor(wl, "master", t, seed, device)
        st["master"].append(p)
        st["m"].append(make_state_tensor(wl, "m", t, seed, device))
        st["v"].append(make_state_tensor(wl, "v", t, seed, device))
        st["compute"].append(p.to(torch.bfloat16))
    return st


def make_grads(wl: Workload, step: int, seed: int = 0, device="cpu", flat: bool = False,
               only: Optional[Sequence[bool]] = None, skew: bool = False) -> List[Optional[torch.Tensor]]:
    """Gradients of iteration `step`: N(0, std 1e-3), fresh per (step, tensor).  With
    wl.heavy_tail an independent uniform draw marks 5% of the entries, which are scaled by 100.
    only[t] False: no gradient for tensor t (None in the result); flat: the gradients share one flat buffer."""
    want = [True] * wl.n_tensors if only is None else list(only)
    views = None
    if flat or skew:
        views = iter(_flat_views([n for (_, n), w in zip(wl.tensors, want) if w], torch.float32, device,
                                 SKEW_LEAD["grad"] if skew else 0))
    out: List[Optional[torch.Tensor]] = []
    for t, (_, n) in enumerate(wl.tensors):
        if not want[t]:
            out.append(None)
            continue
        g = torch.empty(n, dtype=torch.float32, device=device)
        g.normal_(0.0, 1e-3, generator=_gen(device, stream_seed(seed, _STREAM["grad"], t, step)))
        if wl.heavy_tail:
            u = torch.empty(n, dtype=torch.float32, device=device)
            u.uniform_(0.0, 1.0, generator=_gen(device, stream_seed(seed, _STREAM["tail"], t, step)))
            g = torch.where(u < 0.05, g * 100.0, g)
        if views is not None:
            dst = next(views)
            dst.copy_(g)
            g = dst
        out.append(g)
    return out


def random_bits_state(wl: Workload, seed: int = 0, device="cpu") -> Dict[str, List[torch.Tensor]]:
    """State filled with arbitrary bit patterns (for pure byte-movement tests: compute weights
    are NOT the rounded master weights here, NaN / Inf / denormal patterns occur)."""
    st: Dict[str, List[torch.Tensor]] = {"master": [], "m": [], "v": [], "compute": []}
    for t, (_, n) in enumerate(wl.tensors):
        for k, kind in enumerate(("master", "m", "v")):
            bits = torch.randint(-(1 << 31), (1 << 31) - 1, (n,), dtype=torch.int32, device=device,
                                 generator=_gen(device, stream_seed(seed, 10 + k, t)))
            st[kind].append(bits.view(torch.float32))
        bits = torch.randint(-(1 << 15), (1 << 15) - 1, (n,), dtype=torch.int16, device=device,
                             generator=_gen(device, stream_seed(seed, 13, t)))
        st["compute"].append(bits.view(torch.bfloat16))
    return st


# ---------------------------------------------------------------------------------------
# low-precision training state (the regimes of Sec. 5.6)
# ---------------------------------------------------------------------------------------
# (compute, master, optimizer) precisions of the five evaluated regimes, as torch dtypes in the order
# master, Adam m, Adam v, compute
LOW_PRECISION_REGIMES = {
    "fp16_fp16_fp16+fp16": (torch.float16, torch.float16, torch.float16, torch.float16),
    "fp8_fp32_fp32+fp32": (torch.float32, torch.float32, torch.float32, torch.float8_e4m3fn),
    "fp8_fp16_fp32+fp32": (torch.float16, torch.float32, torch.float32, torch.float8_e4m3fn),
    "fp8_fp16_fp8+fp16": (torch.float16, torch.float8_e4m3fn, torch.float16, torch.float8_e4m3fn),
    "fp8_fp8_fp8+fp16": (torch.float8_e4m3fn, torch.float8_e4m3fn, torch.float16, torch.float8_e4m3fn),
}

# per-kind scale that brings the value distributions of make_state into the middle of the narrow
# formats' ranges (powers of two): master std 0.02, m std 1e-3, v ~1e-6
DEFAULT_SCALES = {
    torch.float32: (1.0, 1.0, 1.0, 1.0),
    torch.float16: (1.0, 64.0, 65536.0, 1.0),
    torch.bfloat16: (1.0, 1.0, 1.0, 1.0),
    torch.float8_e4m3fn: (1024.0, 4096.0, 2.0 ** 24, 1024.0),
    torch.float8_e5m2: (1024.0, 4096.0, 2.0 ** 24, 1024.0),
}


def default_scales(dtypes) -> List[float]:
    """One scale per kind (master, m, v, compute) for the given storage dtypes."""
    return [DEFAULT_SCALES[d][k] for k, d in enumerate(dtypes)]


def make_low_precision_state(wl: Workload, dtypes, scales, seed: int = 0, device="cpu") -> Dict[str, List[torch.Tensor]]:
    """The state of make_state stored in the given dtypes: every tensor is multiplied by its kind's
    scale and cast with torch (any valid bit pattern is a legitimate input; the cast only makes the
    values plausible).  scales: [4] per kind, or [4][n_tensors]."""
    st = make_state(wl, seed, device)
    out: Dict[str, List[torch.Tensor]] = {}
    for k, kind in enumerate(("master", "m", "v", "compute")):
        src = st["master"] if kind == "compute" else st[kind]
        out[kind] = []
        for t, x in enumerate(src):
            s = scales[k][t] if isinstance(scales[k], (list, tuple)) else scales[k]
            out[kind].append((x.float() * float(s)).to(dtypes[k]))
    return out
