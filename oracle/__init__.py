"""TEST INFRASTRUCTURE ONLY: ctypes loader for the CPU oracle (oracle.cpp).

Used by tests/, the smoke check and the CPU-baseline leg of bench.py; the
product path never imports this package.  It imports nothing from the GPU
package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

MiB = 1 << 20


class Params(ctypes.Structure):
    _fields_ = [("chunk_bytes", ctypes.c_uint64),
                ("small_limit_bytes", ctypes.c_uint64),
                ("frag_limit_bytes", ctypes.c_uint64),
                ("capacity_bytes", ctypes.c_uint64),
                ("spool_threshold", ctypes.c_uint32),
                ("max_slots", ctypes.c_uint32)]


class Stats(ctypes.Structure):
    _fields_ = [("peak_requested", ctypes.c_uint64), ("peak_active", ctypes.c_uint64),
                ("peak_reserved", ctypes.c_uint64), ("final_requested", ctypes.c_uint64),
                ("final_active", ctypes.c_uint64), ("final_reserved", ctypes.c_uint64),
                ("digest", ctypes.c_uint64), ("n_code", ctypes.c_uint32 * 8),
                ("n_split", ctypes.c_uint32), ("n_merge", ctypes.c_uint32),
                ("n_sblock_created", ctypes.c_uint32), ("n_sblock_evicted", ctypes.c_uint32),
                ("first_oom_event", ctypes.c_uint32), ("status", ctypes.c_uint32),
                ("max_pblocks", ctypes.c_uint32), ("max_sblocks", ctypes.c_uint32),
                ("max_free_blocks", ctypes.c_uint32), ("max_members", ctypes.c_uint32),
                ("max_total_members", ctypes.c_uint32), ("reserved0", ctypes.c_uint32),
                ("fragmentation", ctypes.c_double)]


STATS_DTYPE = np.dtype([("peak_requested", "<u8"), ("peak_active", "<u8"), ("peak_reserved", "<u8"),
                        ("final_requested", "<u8"), ("final_active", "<u8"), ("final_reserved", "<u8"),
                        ("digest", "<u8"), ("n_code", "<u4", (8,)),
                        ("n_split", "<u4"), ("n_merge", "<u4"),
                        ("n_sblock_created", "<u4"), ("n_sblock_evicted", "<u4"),
                        ("first_oom_event", "<u4"), ("status", "<u4"),
                        ("max_pblocks", "<u4"), ("max_sblocks", "<u4"),
                        ("max_free_blocks", "<u4"), ("max_members", "<u4"),
                        ("max_total_members", "<u4"), ("reserved0", "<u4"),
                        ("fragmentation", "<f8")])


def build(force=False, sanitize=False):
    """Compile oracle.cpp with g++."""
    lib = _LIB if not sanitize else os.path.join(_HERE, "liboracle_san.so")
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(_SRC):
        return lib
    cmd = ["g++", "-O2", "-std=c++17", "-Wall", "-Wextra", "-shared", "-fPIC", "-pthread"]
    if sanitize:
        cmd += ["-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
    subprocess.run(cmd + ["-o", lib, _SRC], check=True)
    return lib


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        vp = ctypes.c_void_p
        _lib.oracle_replay.restype = ctypes.c_int
        _lib.oracle_replay.argtypes = [vp, ctypes.c_uint32, ctypes.c_uint32, vp,
                                       ctypes.POINTER(Params), ctypes.c_int, vp, vp, ctypes.c_int]
        _lib.oracle_replay_verbose.restype = ctypes.c_int
        _lib.oracle_replay_verbose.argtypes = [vp, ctypes.c_uint32, ctypes.POINTER(Params), ctypes.c_int,
                                               vp, vp, vp, vp, ctypes.c_uint64, vp]
        _lib.oracle_bestfit.restype = ctypes.c_int
        _lib.oracle_bestfit.argtypes = [ctypes.c_uint32, vp, ctypes.c_uint32, vp, ctypes.c_uint32,
                                        ctypes.c_uint32, vp, vp]
        _lib.oracle_stats_size.restype = ctypes.c_uint32
        assert _lib.oracle_stats_size() == ctypes.sizeof(Stats) == STATS_DTYPE.itemsize
    return _lib


def make_params(max_slots, chunk_bytes=2 * MiB, small_limit_bytes=None, frag_limit_bytes=None,
                capacity_bytes=0, spool_threshold=512):
    return Params(chunk_bytes,
                  chunk_bytes if small_limit_bytes is None else small_limit_bytes,
                  chunk_bytes if frag_limit_bytes is None else frag_limit_bytes,
                  capacity_bytes, spool_threshold, max_slots)


SPLIT, VMS = 0, 1


def replay(events, params, policy, n_events=None, want_decisions=True, threads=1):
    """events: uint64[n_traces, max_events].  Returns (decisions or None, stats[n_traces])."""
    ev = np.ascontiguousarray(events, dtype=np.uint64)
    if ev.ndim == 1:
        ev = ev[None, :]
    n_traces, max_events = ev.shape
    dec = np.zeros_like(ev) if want_decisions else None
    st = np.zeros(n_traces, dtype=STATS_DTYPE)
    ne = None
    if n_events is not None:
        ne = np.ascontiguousarray(n_events, dtype=np.uint32)
        assert ne.shape == (n_traces,)
    rc = _load().oracle_replay(ev.ctypes.data, n_traces, max_events,
                               ne.ctypes.data if ne is not None else None, ctypes.byref(params), policy,
                               dec.ctypes.data if dec is not None else None, st.ctypes.data, threads)
    if rc != 0:
        raise ValueError("oracle_replay: bad parameters")
    return dec, st


def replay_verbose(events, params, policy):
    """One trace.  Returns (decisions, stats, series[n,2], handout[m,3])."""
    ev = np.ascontiguousarray(events, dtype=np.uint64).reshape(-1)
    n = ev.shape[0]
    dec = np.zeros(n, dtype=np.uint64)
    st = np.zeros(1, dtype=STATS_DTYPE)
    series = np.zeros((n, 2), dtype=np.uint64)
    cap = 1 << 16
    while True:
        hand = np.zeros((cap, 3), dtype=np.uint64)
        n_hand = ctypes.c_uint64(0)
        rc = _load().oracle_replay_verbose(ev.ctypes.data, n, ctypes.byref(params), policy, dec.ctypes.data,
                                           st.ctypes.data, series.ctypes.data, hand.ctypes.data, cap,
                                           ctypes.byref(n_hand))
        if rc != 0:
            raise ValueError("oracle_replay_verbose: bad parameters")
        if n_hand.value <= cap:
            return dec, st[0], series, hand[:n_hand.value]
        cap = int(n_hand.value)


def bestfit(bsize, sblock_sizes, pblock_sizes, frag_limit=1):
    """Algorithm 1 on bare lists of inactive block sizes (chunks).
    Returns (state, candidates): candidates index pblock_sizes; a stitched
    exact match is reported as -(index+1)."""
    s = np.ascontiguousarray(sblock_sizes, dtype=np.uint32)
    p = np.ascontiguousarray(pblock_sizes, dtype=np.uint32)
    cb = np.zeros(max(1, len(p) + 1), dtype=np.int32)
    n = ctypes.c_uint32(0)
    state = _load().oracle_bestfit(bsize, s.ctypes.data, len(s), p.ctypes.data, len(p), frag_limit,
                                   cb.ctypes.data, ctypes.byref(n))
    return state, cb[:n.value].tolist()
