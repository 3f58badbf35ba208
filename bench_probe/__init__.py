"""Loader and builder of the stream probe, a measurement aid for bench.py (not part of the CacheCard library):
bench_probe/stream_probe.hip -> bench_probe/libqkvprobe.so, one extern "C" entry point, qkv_stream_probe."""
import ctypes
import os
import subprocess

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "stream_probe.hip")
LIB = os.path.join(HERE, "libqkvprobe.so")
_lib = None


def build(verbose=False):
    """Always recompiles; returns the library path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = ctypes.CDLL(LIB)
        vp = ctypes.c_void_p
        L.qkv_stream_probe.restype = ctypes.c_int
        L.qkv_stream_probe.argtypes = [vp, ctypes.c_uint64, vp, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.POINTER(ctypes.c_uint64), vp]
        _lib = L
    return _lib


def stream_probe(src, dst, reads_kib, writes_kib, nontemporal=0, stream=None):
    """src, dst: device uint8 tensors.  Returns the number of units moved (reads_kib KiB read and writes_kib KiB
    written each) on torch's current stream."""
    if stream is None:
        stream = torch.cuda.current_stream()
    units = ctypes.c_uint64(0)
    rc = lib().qkv_stream_probe(ctypes.c_void_p(src.data_ptr()), src.numel(), ctypes.c_void_p(dst.data_ptr()), dst.numel(),
                                int(reads_kib), int(writes_kib), int(nontemporal), ctypes.byref(units),
                                ctypes.c_void_p(stream.cuda_stream))
    if rc != 0:
        raise RuntimeError("qkv_stream_probe returned %d" % rc)
    return units.value
