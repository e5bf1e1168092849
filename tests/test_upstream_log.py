"""Upstream logging ring (Sec. 3.4).  CPU: the ring's bookkeeping against the oracle's plain
keyed store (what is kept, what is dropped) plus the ring's own invariants (live entries disjoint,
inside the buffer).  GPU: logged bytes come back exactly, through the host and through replay."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2412_15411_amd import binding as B


def _ring(nbytes):
    buf = torch.zeros(nbytes + 64, dtype=torch.uint8)
    off = (-buf.data_ptr()) % 16
    return buf[off:off + nbytes]


def test_ring_bookkeeping_matches_keyed_store(orc):
    rng = np.random.default_rng(0)
    for trial in range(30):
        cap = int(rng.integers(8, 200)) * 256
        log = B.uplog_create(_ring(cap), max_entries=64)
        model = orc.UpstreamLog()
        live = {}                      # tag -> (offset, nbytes)
        it, mb = 10, 0
        for _ in range(400):
            action = rng.random()
            if action < 0.75:
                if rng.random() < 0.3:
                    it, mb = it + 1, 0
                kind = int(rng.integers(0, 2))
                tag = (it, mb, kind)
                if tag in live:
                    mb += 1
                    tag = (it, mb, kind)
                n = int(rng.integers(0, cap // 3))
                try:
                    off = B.uplog_reserve(log, it, mb, kind, n)
                except B.MoevError as e:
                    assert e.code == B.E_NOMEM
                    # a full ring: dropping everything makes room again
                    if rng.random() < 0.5:
                        dropped = B.uplog_gc(log, it + 1)
                        assert dropped == model.gc(it + 1) == len(live)
                        live.clear()
                        it += 1
                        mb = 0
                    continue
                model.append(it, mb, kind, b"\0" * n)
                assert off % 256 == 0 and off + n <= cap
                for o2, n2 in live.values():   # disjoint from every live entry (slots are 256-byte granular)
                    a0, a1 = off, off + max(-(-n // 256) * 256, 256)
                    b0, b1 = o2, o2 + max(-(-n2 // 256) * 256, 256)
                    assert a1 <= b0 or b1 <= a0, (trial, off, n, o2, n2)
                live[tag] = (off, n)
            else:
                keep_from = it - int(rng.integers(0, 4))
                dropped = B.uplog_gc(log, keep_from)
                assert dropped == model.gc(keep_from)
                live = {t: v for t, v in live.items() if t[0] >= keep_from}
            assert B.uplog_stats(log)[0] == len(live) == len(model.store)
            base = log.ring.data_ptr()
            for tag, (off, n) in list(live.items())[:5]:
                addr, size = B.uplog_find(log, *tag)
                assert (addr - base, size) == (off, n) and model.find(*tag) is not None
        with pytest.raises(B.MoevError) as e:
            B.uplog_find(log, 10 ** 9, 0, 0)
        assert e.value.code == B.E_RANGE


def test_ring_argument_checks():
    log = B.uplog_create(_ring(4096))
    B.uplog_reserve(log, 5, 0, B.ACTIVATION, 100)
    with pytest.raises(B.MoevError):
        B.uplog_reserve(log, 5, 0, B.ACTIVATION, 100)      # duplicate tag
    with pytest.raises(B.MoevError):
        B.uplog_reserve(log, 4, 0, B.GRADIENT, 100)        # iterations go backwards
    with pytest.raises(B.MoevError):
        B.uplog_reserve(log, 5, 1, 2, 100)                 # unknown kind
    with pytest.raises(B.MoevError) as e:
        B.uplog_reserve(log, 5, 1, B.GRADIENT, 8192)       # larger than the ring
    assert e.value.code == B.E_NOMEM
    with pytest.raises(B.MoevError):
        B.uplog_create(_ring(128))


@pytest.mark.gpu
def test_logged_tensors_come_back_exactly(orc):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    side, main = torch.cuda.Stream(), torch.cuda.Stream()
    ring = torch.empty(24 << 20, dtype=torch.uint8).pin_memory()
    log = B.uplog_create(ring, max_entries=256)
    model = orc.UpstreamLog()
    g = torch.Generator(device=dev).manual_seed(5)
    live = []
    for it in range(10, 30):
        for mb in range(3):
            for kind in (B.ACTIVATION, B.GRADIENT):
                n = int(torch.randint(1, 400000, (1,)).item())
                with torch.cuda.stream(main):
                    t = torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=g)
                    ready = torch.cuda.Event()
                    ready.record(main)
                B.uplog_append(log, it, mb, kind, t, side_stream=side, ready=ready)
                side.synchronize()
                model.append(it, mb, kind, t.cpu().numpy().tobytes())
                live.append((it, mb, kind))
        # the sparse checkpoint of the window before last has persisted: its logs are stale
        dropped = B.uplog_gc(log, it - 2)
        assert dropped == model.gc(it - 2)
        live = [t for t in live if t[0] >= it - 2]
        for tag in live[-8:] + live[:4]:
            addr, n = B.uplog_find(log, *tag)
            host = (ctypes.c_uint8 * n).from_address(addr)
            assert bytes(host) == model.find(*tag)
            back = torch.empty(n, dtype=torch.uint8, device=dev)
            B.uplog_replay(log, *tag, back, stream=main)
            main.synchronize()
            assert back.cpu().numpy().tobytes() == model.find(*tag)
    entries, used, cap = B.uplog_stats(log)
    assert entries == len(live) == len(model.store) and used <= cap
