"""Seeded synthetic alloc/free traces (inputs only; no allocator logic).

The streams stand in for the paper's fine-tuning workloads (Sec. 2.3, Sec. 5.1,
Table 2): recomputation, offloading and LoRA.  Every replay implementation is
fed the same bytes produced here.

Event word (u64): bits 0-30 size in 512-byte units (ALLOC), bit 31 kind
(0 ALLOC, 1 FREE), bits 32-63 slot.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tracegen.c")
_LIB = os.path.join(_HERE, "libvmstracegen.so")

UNIT = 512
KIND_FREE = 1 << 31

# (n_traces, n_events, seed) of the five workloads
CONFIGS = {
    1: dict(n_traces=1, n_events=2_000, seed=0, capacity_bytes=0),
    2: dict(n_traces=1_024, n_events=20_000, seed=2, capacity_bytes=0),
    3: dict(n_traces=4_096, n_events=50_000, seed=3, capacity_bytes=0),
    4: dict(n_traces=4_096, n_events=50_000, seed=4, capacity_bytes=0),
    5: dict(n_traces=16_384, n_events=100_000, seed=5, capacity_bytes=288 << 30),
    # one rank of ZeRO-3 + LoRA + recomputation over 2^(trace mod 5) devices (Sec. 2.4, Sec. 5.3.2)
    6: dict(n_traces=1_280, n_events=20_000, seed=6, capacity_bytes=0),
    # strictly periodic variants of 2, 3, 4 (every step has sequence length 2048): convergence studies
    12: dict(n_traces=1_024, n_events=20_000, seed=2, capacity_bytes=0),
    13: dict(n_traces=4_096, n_events=50_000, seed=3, capacity_bytes=0),
    14: dict(n_traces=4_096, n_events=50_000, seed=4, capacity_bytes=0),
}


def build(force=False):
    """Compile the generator with gcc (host code only)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-pthread",
           "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.tracegen_fill.restype = ctypes.c_uint32
        _lib.tracegen_fill.argtypes = [ctypes.c_int, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                       ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                       ctypes.c_int]
    return _lib


def generate(config, n_traces=None, n_events=None, seed=None, first_trace=0, trace_stride=1, threads=8,
             out=None):
    """Return (events[n_traces, n_events] uint64, max_slots) for traces first_trace,
    first_trace + trace_stride, ... of the configuration."""
    base = CONFIGS[config]
    n_traces = base["n_traces"] if n_traces is None else n_traces
    n_events = base["n_events"] if n_events is None else n_events
    seed = base["seed"] if seed is None else seed
    if out is None:
        out = np.empty((n_traces, n_events), dtype=np.uint64)
    assert out.dtype == np.uint64 and out.shape == (n_traces, n_events) and out.flags.c_contiguous
    if n_traces == 0:
        return out, 1
    m = _load().tracegen_fill(config, seed, first_trace, trace_stride, n_traces, n_events,
                              out.ctypes.data, threads)
    if m == 0:
        raise ValueError("tracegen_fill: bad argument")
    return out, int(m)


def make_events(ops):
    """Hand-written trace: ops is a list of ("A", slot, bytes) / ("F", slot)."""
    ev = []
    for op in ops:
        if op[0] == "A":
            ev.append((op[1] << 32) | ((op[2] + UNIT - 1) // UNIT))
        else:
            ev.append((op[1] << 32) | KIND_FREE)
    return np.array(ev, dtype=np.uint64)


def decode(events):
    """Split event words into (is_free bool[], size_bytes int64[], slot int64[])."""
    e = np.asarray(events, dtype=np.uint64)
    is_free = (e & np.uint64(KIND_FREE)) != 0
    size = (e & np.uint64(0x7FFFFFFF)).astype(np.int64) * UNIT
    slot = (e >> np.uint64(32)).astype(np.int64)
    return is_free, size, slot
