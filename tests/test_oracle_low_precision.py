"""Pins for the oracle's low-precision state handling (Sec. 5.6 regimes): the storage formats against
the facts their specifications fix, numpy's binary16 and brute-force nearest-value search; the
low-precision optimizer step against the FP32 step it reduces to and against a composition of the
separately pinned pieces; and the window property (conversion == dense run, Sec. 3.3) in every regime."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import ORACLE_FMT_OF_DTYPE, hp_of, model_of, state_of, states_equal
from paper_2412_15411_amd import workloads as wk

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "narrow_float_formats.txt")
FMT = {"F16": oracle.FMT_F16, "BF16": oracle.FMT_BF16, "E4M3": oracle.FMT_E4M3, "E5M2": oracle.FMT_E5M2}
BITS = {oracle.FMT_F16: 16, oracle.FMT_BF16: 16, oracle.FMT_E4M3: 8, oracle.FMT_E5M2: 8}
SATURATING = {oracle.FMT_E4M3, oracle.FMT_E5M2}


def _value(text):
    if text in ("nan", "inf", "-inf"):
        return float(text)
    if text == "-0":
        return -0.0
    a, b = text.split("*2^")
    return float(a) * 2.0 ** int(b)


def test_format_facts():
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, _, pattern, value = line.split()
        got = oracle.decode(FMT[name], int(pattern, 16))
        want = _value(value)
        if math.isnan(want):
            assert math.isnan(got), line
        else:
            assert got == want and math.copysign(1, got) == math.copysign(1, want), line
            if not (math.isinf(want) and FMT[name] in SATURATING):  # conversions saturate: nothing encodes to it
                assert oracle.encode(FMT[name], want) == int(pattern, 16), line


def test_binary16_decode_is_numpys():
    codes = np.arange(65536, dtype=np.uint16)
    want = codes.view(np.float16).astype(np.float64)
    got = np.array([oracle.decode(oracle.FMT_F16, int(c)) for c in codes])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan]) and np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bfloat16_decode_is_the_upper_half_of_binary32():
    codes = np.arange(65536, dtype=np.uint32)
    want = (codes << 16).view(np.float32).astype(np.float64)
    got = np.array([oracle.decode(oracle.FMT_BF16, int(c)) for c in codes])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], want[~nan])


def test_e5m2_is_binary16_cut_after_two_mantissa_bits():
    for b in range(256):
        x, y = oracle.decode(oracle.FMT_E5M2, b), oracle.decode(oracle.FMT_F16, b << 8)
        assert (math.isnan(x) and math.isnan(y)) or x == y


def _positive_table(fmt):
    """(values, codes) of the non-negative finite codes, ascending."""
    n = 1 << (BITS[fmt] - 1)
    vals = np.array([oracle.decode(fmt, c) for c in range(n)])
    keep = np.isfinite(vals)
    codes = np.arange(n)[keep]
    vals = vals[keep]
    assert np.all(np.diff(vals) > 0)  # codes of one sign are ordered like their values
    return vals, codes


def _nearest_by_search(fmt, x, table):
    """Definition of round-to-nearest-even by search over all finite values of the format."""
    vals, codes = table
    sign = (1 << (BITS[fmt] - 1)) if math.copysign(1.0, x) < 0 else 0
    a = abs(float(x))
    top_val, top_code = vals[-1], int(codes[-1])
    if a >= top_val:
        if fmt in SATURATING:
            return sign | top_code
        # IEEE: the value one spacing above the largest finite one is where infinity sits for rounding purposes
        beyond = top_val + (top_val - vals[-2])
        mid = (top_val + beyond) / 2
        return sign | (top_code + 1 if a >= mid else top_code)  # tie goes to the even mantissa = infinity's code
    hi = int(np.searchsorted(vals, a, side="right"))
    lo = hi - 1
    d_lo, d_hi = a - vals[lo], vals[hi] - a
    if d_lo < d_hi:
        return sign | int(codes[lo])
    if d_hi < d_lo:
        return sign | int(codes[hi])
    return sign | int(codes[lo] if codes[lo] % 2 == 0 else codes[hi])


@pytest.mark.parametrize("name", ["E4M3", "E5M2", "F16", "BF16"])
def test_encode_is_nearest_even_by_brute_force(name):
    fmt = FMT[name]
    table = _positive_table(fmt)
    vals = table[0]
    rng = np.random.default_rng(5)
    pick = np.arange(len(vals)) if len(vals) <= 4096 else np.unique(
        np.concatenate([np.arange(0, 2100), np.arange(len(vals) - 2100, len(vals)), rng.integers(0, len(vals), 4000)]))
    xs = []
    for i in pick:
        v = np.float32(vals[i])
        xs.append(v)
        if i + 1 < len(vals):
            mid = np.float32((vals[i] + vals[i + 1]) / 2)  # exact in FP32 for all these formats
            assert float(mid) == (vals[i] + vals[i + 1]) / 2
            xs += [mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(np.inf))]
    top = np.float32(vals[-1])
    spacing = np.float32(vals[-1] - vals[-2])
    xs += [top + spacing / 2, np.nextafter(top + spacing / 2, np.float32(0)), top + spacing, top * 2, np.float32(3e38)]
    lo, hi = math.log2(vals[1]) - 3, math.log2(vals[-1]) + 2
    xs += list(np.exp2(rng.uniform(lo, min(hi, 127.9), 20000)).astype(np.float32))
    for x in xs:
        x = np.float32(x)
        if not np.isfinite(x):
            continue
        for s in (x, -x):
            assert oracle.encode(fmt, float(s)) == _nearest_by_search(fmt, s, table), (name, float(s))


def test_encode_special_values():
    inf, nan = float("inf"), float("nan")
    assert oracle.encode(oracle.FMT_F16, inf) == 0x7C00 and oracle.encode(oracle.FMT_F16, -inf) == 0xFC00
    assert oracle.encode(oracle.FMT_E5M2, inf) == 0x7B and oracle.encode(oracle.FMT_E5M2, -inf) == 0xFB  # saturating
    assert oracle.encode(oracle.FMT_E4M3, inf) == 0x7E and oracle.encode(oracle.FMT_E4M3, -1e9) == 0xFE
    assert math.isnan(oracle.decode(oracle.FMT_F16, oracle.encode(oracle.FMT_F16, nan)))
    assert math.isnan(oracle.decode(oracle.FMT_E5M2, oracle.encode(oracle.FMT_E5M2, nan)))
    assert oracle.encode(oracle.FMT_E4M3, nan) & 0x7F == 0x7F
    for fmt in FMT.values():
        assert oracle.encode(fmt, 0.0) == 0 and oracle.encode(fmt, -0.0) == 1 << (BITS[fmt] - 1)


def test_binary16_encode_is_numpys():
    rng = np.random.default_rng(11)
    x = np.concatenate([
        np.exp2(rng.uniform(-30, 17, 200000)) * rng.choice([-1.0, 1.0], 200000),
        rng.normal(0, 1e-6, 50000), [65504.0, 65519.99, 65520.0, 65536.0, 1e-8, 2.98e-8, 2.9802322387695312e-08],
    ]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.encode(oracle.FMT_F16, float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("name", ["E4M3", "E5M2", "F16", "BF16"])
def test_roundtrip_of_every_code(name):
    fmt = FMT[name]
    for code in range(1 << BITS[fmt]):
        v = oracle.decode(fmt, code)
        if math.isnan(v):
            assert math.isnan(oracle.decode(fmt, oracle.encode(fmt, v)))
        elif math.isinf(v) and fmt in SATURATING:
            assert oracle.decode(fmt, oracle.encode(fmt, v)) == math.copysign(57344.0, v)
        else:
            assert oracle.encode(fmt, v) == code


# --------------------------------------------------------------------------------------
# optimizer step on low-precision state
# --------------------------------------------------------------------------------------
F32, F16, BF16, E4M3, E5M2 = oracle.FMT_F32, oracle.FMT_F16, oracle.FMT_BF16, oracle.FMT_E4M3, oracle.FMT_E5M2
REGIMES = {name: tuple(ORACLE_FMT_OF_DTYPE[d] for d in dtypes) for name, dtypes in wk.LOW_PRECISION_REGIMES.items()}


def _random_codes(fmt, n, rng, scale_hint):
    """Bit patterns of plausible values: a normal draw times the hint, encoded by torch/numpy-free search."""
    x = (rng.normal(0, 1, n) * scale_hint).astype(np.float32)
    if fmt == F32:
        return x
    return np.array([oracle.encode(fmt, float(v)) for v in x], dtype=oracle.FMT_DTYPE[fmt])


def test_fp32_formats_reduce_to_the_fp32_step():
    rng = np.random.default_rng(1)
    n = 5000
    p, m, v = (rng.normal(0, s, n).astype(np.float32) for s in (0.02, 1e-3, 1e-3))
    v = v * v
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    hp = oracle.AdamHP(weight_decay=0.01)
    p2, m2, v2 = p.copy(), m.copy(), v.copy()
    c, c2 = np.zeros(n, np.uint16), np.zeros(n, np.uint16)
    oracle.adam_tensor(p, m, v, g, c, hp, 17)
    oracle.adam_tensor_lp(p2, m2, v2, g, c2, hp, 17, (F32, F32, F32, BF16), (3.0, 5.0, 7.0, 1.0))  # FP32 kinds ignore scales
    for a, b in ((p, p2), (m, m2), (v, v2), (c, c2)):
        assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("regime", list(REGIMES))
@pytest.mark.parametrize("scales", [(1.0, 1.0, 1.0, 1.0), (1024.0, 4096.0, 65536.0, 512.0), (3.0, 1000.0, 12345.0, 0.7)])
def test_low_precision_step_is_widen_step_narrow(regime, scales):
    """The step equals: decode every stored value (pinned above), multiply by the scale's reciprocal, take the FP32
    step (pinned in test_oracle_adam_conversion), multiply by the scale, encode; compute weights from
    the master weights as stored.  Composed here element by element from the separately pinned pieces."""
    fmts = REGIMES[regime]
    rng = np.random.default_rng(3)
    n = 700
    hints = (0.02 * scales[0], 1e-3 * scales[1], 1e-6 * scales[2])
    P, M = _random_codes(fmts[0], n, rng, hints[0]), _random_codes(fmts[1], n, rng, hints[1])
    V = _random_codes(fmts[2], n, rng, hints[2])
    if fmts[2] == F32:
        V = np.abs(V)
    else:
        V = V & ((1 << (8 * V.itemsize - 1)) - 1)  # clear the sign: second moments are not negative
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    Cw = np.zeros(n, oracle.FMT_DTYPE[fmts[3]])
    hp = oracle.AdamHP(lr=1e-3)
    want = [P.copy(), M.copy(), V.copy(), Cw.copy()]
    f32 = np.float32

    def widen(arr, k, i):
        if fmts[k] == F32:
            return f32(arr[i])
        return f32(f32(oracle.decode(fmts[k], int(arr[i]))) * (f32(1) / f32(scales[k])))

    def narrow(k, x):
        if fmts[k] == F32:
            return f32(x)
        return oracle.encode(fmts[k], float(f32(x) * f32(scales[k])))

    for i in range(n):
        p, m, v = (np.array([widen(a, k, i)], dtype=f32) for k, a in enumerate((P, M, V)))
        oracle.adam_tensor(p, m, v, g[i:i + 1].copy(), None, hp, 12)
        for k, x in enumerate((p, m, v)):
            want[k][i] = narrow(k, x[0])
        want[3][i] = narrow(3, widen(want[0], 0, i))
    oracle.adam_tensor_lp(P, M, V, g, Cw, hp, 12, fmts, scales)
    for k, got in enumerate((P, M, V, Cw)):
        assert got.tobytes() == want[k].tobytes(), (regime, k)


def test_binary16_step_against_numpy_arithmetic():
    """Regime with FP16 everywhere, scale 1: numpy's own float16 <-> float32 casts and float32
    elementwise arithmetic (IEEE, one rounding per operation) give the same bits."""
    rng = np.random.default_rng(9)
    n = 20000
    P = rng.normal(0, 0.02, n).astype(np.float16)
    M = rng.normal(0, 1e-3, n).astype(np.float16)
    V = (rng.normal(0, 3e-2, n) ** 2).astype(np.float16)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    hp = oracle.AdamHP(lr=1e-3)
    step = 12
    bc1, bc2 = (np.float32(x) for x in oracle.bias_corrections(hp, step))
    f = np.float32
    p, m, v = P.astype(f), M.astype(f), V.astype(f)
    m = f(hp.beta1) * m + (f(1) - f(hp.beta1)) * g
    v = f(hp.beta2) * v + (f(1) - f(hp.beta2)) * (g * g)
    p = p - f(hp.lr) * ((m / bc1) / (np.sqrt(v / bc2) + f(hp.eps)))
    want = [p.astype(np.float16), m.astype(np.float16), v.astype(np.float16)]
    want.append(want[0].copy())  # compute = FP16 of the stored FP16 master
    Pb, Mb, Vb = (a.view(np.uint16).copy() for a in (P, M, V))
    Cb = np.zeros(n, np.uint16)
    oracle.adam_tensor_lp(Pb, Mb, Vb, g, Cb, hp, step, (F16, F16, F16, F16))
    for got, w in zip((Pb, Mb, Vb, Cb), want):
        assert np.array_equal(got, w.view(np.uint16))


def test_zero_gradient_and_zero_momentum_leave_weights_alone():
    """g = 0 and m = 0: the update is lr * (0 / (sqrt(v_hat) + eps)) = 0, so the stored master weights keep
    their bits (power-of-two scale: widening and narrowing are exact), m stays 0, v decays by beta2."""
    fmts = REGIMES["fp8_fp8_fp8+fp16"]
    rng = np.random.default_rng(2)
    n = 4000
    P = rng.integers(0, 256, n).astype(np.uint8)
    P[(P & 0x7F) == 0x7F] = 0x10  # no NaN
    M = np.zeros(n, np.uint8)
    V = rng.integers(0x0400, 0x7000, n).astype(np.uint16)  # positive normal FP16 values
    g = np.zeros(n, np.float32)
    Cw = np.zeros(n, np.uint8)
    before, v_before = P.copy(), V.copy()
    hp = oracle.AdamHP(beta2=0.5)
    oracle.adam_tensor_lp(P, M, V, g, Cw, hp, 3, fmts, (1024.0, 4096.0, 65536.0, 1024.0))
    zero_codes = np.isin(before, (0x00, 0x80))
    assert np.array_equal(P[~zero_codes], before[~zero_codes]) and not M.any()
    assert np.array_equal(Cw[~zero_codes], before[~zero_codes])  # same format and scale as the master weights
    halved = (v_before.view(np.float16).astype(np.float32) * np.float32(0.5)).astype(np.float16)
    assert np.array_equal(V, halved.view(np.uint16))


@pytest.mark.parametrize("regime", list(REGIMES))
def test_conversion_equals_dense_run_in_every_regime(regime):
    """Sec. 3.3: loading SS_t, SS_t+1, ... and replaying the iterations in between on the active operators
    reproduces the dense state bit for bit -- also when the state is stored in low precision."""
    dtypes = wk.LOW_PRECISION_REGIMES[regime]
    fmts = REGIMES[regime]
    wl = wk.tiny_moe(n_experts=6, d_in=24, d_hidden=37, window=3, n_active=2)
    scales = wk.default_scales(dtypes)
    table = np.array([[s] * wl.n_tensors for s in scales], dtype=np.float32)
    table[0, 1] *= 2.0  # per-tensor scales: not all equal
    table[2, 3] *= 0.5
    st = wk.make_low_precision_state(wl, dtypes, [list(r) for r in table.tolist()], seed=4)
    model = model_of(wl, formats=fmts)
    hp = hp_of(wl)
    state = state_of(st)
    grads = lambda t: [g.numpy() for g in wk.make_grads(wl, t, seed=4)]
    everyone = np.ones(wl.n_ops, np.uint8)
    snaps = []
    for k in range(wl.window):
        snaps.append(oracle.pack(model, k, wl.t0 + k, state))
        oracle.replay_step(model, hp, wl.t0 + k + 1, everyone, grads(wl.t0 + k + 1), state, table)
    rebuilt = oracle.poisoned_like(state)
    mask = np.zeros(wl.n_ops, np.uint8)
    for i in range(wl.window):
        it = oracle.unpack(model, i, snaps[i], rebuilt, mask)
        oracle.replay_step(model, hp, it + 1, mask, grads(it + 1), rebuilt, table)
    assert mask.all() and states_equal(rebuilt, state) == []
    # and the state did move: three steps change most stored values of the 2-byte kinds
    start = state_of(st)
    assert states_equal(start, state) != []
