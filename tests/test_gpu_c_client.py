"""The C ABI used from plain C: tests/c_client/moev_c_client.c (hipMalloc, hipHostMalloc, the calls of moev.h; no
Python, no PyTorch in the process) runs a dense run with a sparse snapshot per iteration and the sparse-to-dense
conversion on inputs this test writes to a file; what it writes back is compared with the oracle."""
import importlib.util
import os
import struct
import subprocess

import numpy as np
import pytest
import torch

from paper_2412_15411_amd import workloads as W
from helpers import hp_of, model_of, np_of, state_of, max_rel_err

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "c_client", "moev_c_client")
KINDS = ("master", "m", "v", "compute")
MAGIC = 0x4d4f4556


def _built_client():
    if not os.path.exists(EXE):
        spec = importlib.util.spec_from_file_location("moev_c_client_build", os.path.join(HERE, "c_client", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build()
    return EXE


def test_c_client_builds_and_states_its_usage():
    """No GPU needed: the client compiles as C99 against moev.h and links libmoev.so; without arguments it prints its
    usage and touches no device."""
    res = subprocess.run([_built_client()], capture_output=True, text=True, timeout=60)
    assert res.returncode == 1 and "usage:" in res.stderr


def _workload():
    # ragged lengths (tails of 1-3 elements, one empty tensor, several tiles), three slots, a non-trivial order
    tensors = [(0, 70001), (0, 5), (1, 4096), (2, 0), (2, 33333), (3, 257), (3, 12288), (4, 65536), (4, 3)]
    return W.Workload("c_client", tensors, [1, 0, 2, 0, 1], 3, order=[3, 1, 4, 0, 2], weight_decay=0.01)


@pytest.mark.gpu
def test_c_client_dense_run_and_conversion_match_the_oracle(orc, tmp_path):
    assert torch.cuda.is_available(), "GPU tests need a GPU (no CPU fallback exists)"
    wl = _workload()
    st_cpu = W.make_state(wl, seed=17)
    grads_cpu = {t: W.make_grads(wl, t, seed=17) for t in range(wl.t0 + 1, wl.t0 + wl.window + 1)}
    src = tmp_path / "in.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("<IIIIQfffff", MAGIC, wl.n_ops, wl.n_tensors, wl.window, wl.t0, wl.lr, wl.beta1, wl.beta2,
                            wl.eps, wl.weight_decay))
        for op, n in wl.tensors:
            f.write(struct.pack("<IQ", op, n))
        f.write(np.asarray(wl.slot_of_op, dtype="<u4").tobytes())
        f.write(np.asarray(wl.order, dtype="<u4").tobytes())
        for t in range(wl.n_tensors):
            for k in KINDS:
                f.write(np_of(st_cpu[k][t]).tobytes())
        for step in range(wl.t0 + 1, wl.t0 + wl.window + 1):
            for g in grads_cpu[step]:
                f.write(np_of(g).tobytes())
    dst = tmp_path / "out.bin"
    res = subprocess.run([_built_client(), str(src), str(dst)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    assert "dense run and conversion written" in res.stdout

    # the oracle on the same inputs: brute-force dense run with a snapshot per iteration
    model, hp = model_of(wl), hp_of(wl)
    dense = state_of(st_cpu)
    snaps = orc.dense_run(model, dense, hp, lambda t: [np_of(g) for g in grads_cpu[t]], wl.t0, wl.window, snapshots=True)

    raw = dst.read_bytes()
    assert struct.unpack_from("<I", raw, 0)[0] == MAGIC
    pos = 4
    for k in range(wl.window):
        (n,) = struct.unpack_from("<Q", raw, pos)
        pos += 8
        assert raw[pos:pos + n] == snaps[k].tobytes(), f"drained snapshot {k} differs from the oracle"
        pos += n
    states = []
    for _ in range(2):     # the dense run's final state, then the converted state
        st = {k: [] for k in KINDS}
        for _, n in wl.tensors:
            for k in KINDS:
                width, dtype = (2, np.uint16) if k == "compute" else (4, np.float32)
                st[k].append(np.frombuffer(raw, dtype=dtype, count=n, offset=pos).copy())
                pos += n * width
        states.append(st)
    mask = np.frombuffer(raw, dtype=np.uint8, count=wl.n_ops, offset=pos)
    assert pos + wl.n_ops == len(raw) and mask.all()
    live, rebuilt = states
    worst = 0.0
    for k in KINDS:
        for t in range(wl.n_tensors):
            assert rebuilt[k][t].tobytes() == live[k][t].tobytes(), f"conversion differs from the dense run: {k}[{t}]"
    for k in ("master", "m", "v"):
        for t in range(wl.n_tensors):
            worst = max(worst, max_rel_err(rebuilt[k][t], dense.kinds()[k][t]))
    assert worst <= 1e-6, f"relative error {worst} against the oracle"
    for t in range(wl.n_tensors):
        same = rebuilt["master"][t].view(np.uint32) == dense.master[t].view(np.uint32)
        assert np.array_equal(rebuilt["compute"][t][same], dense.compute[t][same])
