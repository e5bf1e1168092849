"""Glue shared by the tests: move seeded workload tensors into the oracle's numpy containers."""
import numpy as np
import torch

import oracle


def model_of(wl, align=256, widths=(4, 4, 4, 2), formats=None):
    if formats is not None:
        widths = tuple(oracle.FMT_BYTES[f] for f in formats)
    return oracle.Model(list(wl.tensors), list(wl.order), list(wl.slot_of_op), wl.window, align, widths, formats)


ORACLE_FMT_OF_DTYPE = {torch.float32: oracle.FMT_F32, torch.float16: oracle.FMT_F16, torch.bfloat16: oracle.FMT_BF16,
                       torch.float8_e4m3fn: oracle.FMT_E4M3, torch.float8_e5m2: oracle.FMT_E5M2}


def hp_of(wl):
    return oracle.AdamHP(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay)


def np_of(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    if t.dtype in (torch.float8_e4m3fn, torch.float8_e5m2):
        return t.view(torch.uint8).numpy().copy()
    return t.numpy().copy()


def state_of(st) -> "oracle.State":
    return oracle.State(*[[np_of(t) for t in st[k]] for k in ("master", "m", "v", "compute")])


def states_equal(a: "oracle.State", b: "oracle.State"):
    """Bitwise comparison; returns the list of (kind, tensor) that differ."""
    bad = []
    for kind in ("master", "m", "v", "compute"):
        for t, (x, y) in enumerate(zip(a.kinds()[kind], b.kinds()[kind])):
            if x.tobytes() != y.tobytes():
                bad.append((kind, t))
    return bad


def max_rel_err(x: np.ndarray, ref: np.ndarray) -> float:
    """max |x - ref| / max(|ref|, 1e-30) over the finite reference values; NaN positions and
    infinities must coincide exactly (otherwise the error is infinite)."""
    x = x.astype(np.float64)
    ref = ref.astype(np.float64)
    nan_x, nan_r = np.isnan(x), np.isnan(ref)
    if not np.array_equal(nan_x, nan_r):
        return float("inf")
    inf_r = np.isinf(ref)
    if not np.array_equal(x[inf_r], ref[inf_r]):
        return float("inf")
    ok = ~nan_r & ~inf_r
    if not ok.any():
        return 0.0
    with np.errstate(invalid="ignore"):
        err = np.abs(x[ok] - ref[ok]) / np.maximum(np.abs(ref[ok]), 1e-30)
    return float(np.max(np.nan_to_num(err, nan=np.inf)))
