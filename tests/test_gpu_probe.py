"""The stream probe (bench_probe/, a measurement aid for bench.py outside the product library: a handoff's memory traffic without its arithmetic) moves exactly the bytes
it says: every written word against the exclusive-or definition in numpy, ragged buffer sizes, nothing written
past the last whole unit, host-side refusals."""
import ctypes

import numpy as np
import pytest
import torch

import bench_probe

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def expected(src, units, reads, writes):
    s = src[:units * reads * 1024].view(np.uint32).reshape(units, reads, 64, 4)
    x = np.bitwise_xor.reduce(s, axis=1)                                  # [units, 64 lanes, 4 words]
    k = np.arange(writes, dtype=np.uint32).reshape(1, writes, 1, 1)
    return (x[:, None] + k).astype(np.uint32).reshape(-1).view(np.uint8)


@pytest.mark.parametrize("reads,writes", [(8, 2), (2, 8), (8, 8)])
@pytest.mark.parametrize("nontemporal", [0, 1, 2, 3])
def test_probe_moves_what_it_says(reads, writes, nontemporal):
    print("[case] probe %d:%d nt=%d" % (reads, writes, nontemporal), flush=True)
    rng = np.random.default_rng(reads * 10 + writes + nontemporal)
    units = 1237                                                           # several workgroups and a ragged last one
    src = rng.integers(0, 256, size=units * reads * 1024 + 1000, dtype=np.uint8)     # a partial unit at the end
    dst_bytes = units * writes * 1024 + writes * 1024 + 112              # room for one more unit than the source has
    canary = 0xA5
    dst = torch.full((dst_bytes,), canary, dtype=torch.uint8, device=DEV)
    got_units = bench_probe.stream_probe(torch.from_numpy(src).to(DEV), dst, reads, writes, nontemporal)
    torch.cuda.synchronize()
    assert got_units == units
    out = dst.cpu().numpy()
    assert np.array_equal(out[:units * writes * 1024], expected(src, units, reads, writes))
    assert np.all(out[units * writes * 1024:] == canary)


def test_probe_limited_by_the_destination_and_empty():
    src = torch.zeros(64 * 8 * 1024, dtype=torch.uint8, device=DEV)
    dst = torch.full((5 * 2 * 1024 + 100,), 7, dtype=torch.uint8, device=DEV)
    assert bench_probe.stream_probe(src, dst, 8, 2) == 5
    torch.cuda.synchronize()
    out = dst.cpu().numpy()
    assert np.array_equal(out[:5 * 2048], expected(np.zeros(5 * 8192, dtype=np.uint8), 5, 8, 2)) and np.all(out[5 * 2048:] == 7)
    assert bench_probe.stream_probe(src[:100], dst, 8, 2) == 0                     # not one whole unit: nothing launched


def test_probe_host_errors():
    L = bench_probe.lib()
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    other = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    n = ctypes.c_uint64(0)
    call = lambda s, sb, d, db, r, w, nt: L.qkv_stream_probe(s, sb, d, db, r, w, nt, ctypes.byref(n), None)
    assert call(buf.data_ptr(), buf.numel(), other.data_ptr(), other.numel(), 8, 2, 0) == 0
    assert call(None, buf.numel(), other.data_ptr(), other.numel(), 8, 2, 0) == -1
    assert call(buf.data_ptr(), buf.numel(), other.data_ptr(), other.numel(), 4, 4, 0) == -2
    assert call(buf.data_ptr(), buf.numel(), other.data_ptr(), other.numel(), 8, 2, 4) == -2
    assert call(buf.data_ptr() + 8, buf.numel() - 8, other.data_ptr(), other.numel(), 8, 2, 0) == -6
    assert call(buf.data_ptr(), buf.numel(), buf.data_ptr() + 4096, buf.numel() - 4096, 8, 2, 0) == -10
    torch.cuda.synchronize()
