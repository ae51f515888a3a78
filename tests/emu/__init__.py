"""TEST INFRASTRUCTURE ONLY: the replay kernels compiled for the host (64 lanes as cooperative
fibers, guard bands around every buffer) and a ctypes loader for that build.  Used by the CPU
tests to check the kernels' indexing and decisions without a GPU; never by the product."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "emu_replay.cpp")
_LIB = os.path.join(_HERE, "libemu.so")
_CSRC = os.path.join(_HERE, "..", "..", "paper_2401_08156_amd", "csrc")
_DEPS = [_SRC, os.path.join(_HERE, "wave_hw_emu.hpp")] + [
    os.path.join(_CSRC, f) for f in ("wave_ops.hpp", "replay_plan.hpp", "replay_kernels.hpp", "replay_fine.hpp", "selftest.hpp")]


def build(force=False):
    if not force and os.path.exists(_LIB) and all(os.path.getmtime(_LIB) >= os.path.getmtime(d) for d in _DEPS):
        return _LIB
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-shared", "-fPIC", "-Wall", "-Wno-unused", "-Wno-unknown-pragmas",
                    "-o", _LIB, _SRC], check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        vp = ctypes.c_void_p
        _lib.emu_replay.restype = ctypes.c_int
        _lib.emu_replay.argtypes = [vp, vp, vp, vp, vp, vp]
        _lib.emu_selftest.restype = ctypes.c_uint
    return _lib


def replay(events, cfg, stats_dtype, n_events=None):
    """events: uint64[n_traces, max_events]; cfg: the binding's vms_config.
    Returns (dec_split, dec_vms, stats[2, n_traces])."""
    ev = np.ascontiguousarray(events, dtype=np.uint64)
    assert ev.shape == (cfg.n_traces, cfg.max_events)
    ds, dv = np.zeros_like(ev), np.zeros_like(ev)
    st = np.zeros((2, cfg.n_traces), dtype=stats_dtype)
    ne = None if n_events is None else np.ascontiguousarray(n_events, dtype=np.uint32)
    rc = lib().emu_replay(ctypes.byref(cfg), ev.ctypes.data, None if ne is None else ne.ctypes.data,
                          ds.ctypes.data, dv.ctypes.data, st.ctypes.data)
    if rc != 0:
        raise RuntimeError("emu_replay: %d" % rc)
    return ds, dv, st
