"""ctypes binding of include/vms_replay.h and include/vms_live.h: same names, argument marshalling only.

Every step of the replay runs in the HIP kernels of libvmsreplay.so; PyTorch is
used for device memory and the stream.  There is no CPU fallback: a missing or
unloadable library raises.
"""
import ctypes
import os

import numpy as np

from . import build as _build

VMS_OK = 0
VMS_POLICY_SPLIT, VMS_POLICY_VMS = 1, 2
VMS_VARIANT_AUTO, VMS_VARIANT_FLAT, VMS_VARIANT_FINE = 0, 1, 2
VMS_TABLES_AUTO, VMS_TABLES_LDS, VMS_TABLES_WORKSPACE, VMS_TABLES_WORKSPACE_ALL = 0, 1, 2, 3
VMS_ST_INVALID_EVENT, VMS_ST_TABLE_OVERFLOW = 1, 2
VMS_ST_OVF_FREE_BLOCKS, VMS_ST_OVF_PBLOCKS, VMS_ST_OVF_SBLOCKS, VMS_ST_OVF_RUNS, VMS_ST_OVF_CHUNKS = 4, 8, 16, 32, 64


class vms_config(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("n_traces", ctypes.c_uint32),
                ("max_events", ctypes.c_uint32), ("policy_mask", ctypes.c_uint32),
                ("chunk_bytes", ctypes.c_uint64), ("small_limit_bytes", ctypes.c_uint64),
                ("frag_limit_bytes", ctypes.c_uint64), ("capacity_bytes", ctypes.c_uint64),
                ("spool_threshold", ctypes.c_uint32), ("max_slots", ctypes.c_uint32),
                ("max_free_blocks", ctypes.c_uint32), ("max_pblocks", ctypes.c_uint32),
                ("max_sblocks", ctypes.c_uint32), ("max_runs", ctypes.c_uint32),
                ("max_chunks", ctypes.c_uint32), ("max_small_blocks", ctypes.c_uint32),
                ("max_multi_pblocks", ctypes.c_uint32), ("variant", ctypes.c_uint32),
                ("retry_traces", ctypes.c_uint32), ("table_place", ctypes.c_uint32)]


class vms_summary(ctypes.Structure):
    _fields_ = [("sum_peak_reserved", ctypes.c_uint64 * 2), ("sum_peak_active", ctypes.c_uint64 * 2),
                ("n_flagged", ctypes.c_uint64 * 2), ("max_fragmentation", ctypes.c_double * 2),
                ("mean_fragmentation", ctypes.c_double * 2), ("mem_reduction_ratio", ctypes.c_double)]


class vms_demo_report(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("events_replayed", ctypes.c_uint32),
                ("failed_event", ctypes.c_uint32), ("hip_error", ctypes.c_int32),
                ("granularity_bytes", ctypes.c_uint64), ("chunks_created", ctypes.c_uint64),
                ("n_pblocks_created", ctypes.c_uint32), ("n_splits", ctypes.c_uint32),
                ("n_stitches", ctypes.c_uint32), ("n_sblocks_released", ctypes.c_uint32),
                ("sblocks_cached", ctypes.c_uint32), ("alias_checks", ctypes.c_uint32),
                ("alias_failures", ctypes.c_uint32), ("failed_api", ctypes.c_uint32),
                ("n_reserve", ctypes.c_uint64), ("n_create", ctypes.c_uint64), ("n_map", ctypes.c_uint64),
                ("n_set_access", ctypes.c_uint64), ("n_unmap", ctypes.c_uint64), ("n_release", ctypes.c_uint64),
                ("n_address_free", ctypes.c_uint64),
                ("ms_reserve", ctypes.c_double), ("ms_create", ctypes.c_double), ("ms_map", ctypes.c_double),
                ("ms_set_access", ctypes.c_double), ("ms_unmap", ctypes.c_double), ("ms_release", ctypes.c_double),
                ("ms_address_free", ctypes.c_double),
                ("table1_bytes", ctypes.c_uint64), ("table1_hipmalloc_ms", ctypes.c_double),
                ("table1_reserve_ms", ctypes.c_double), ("table1_create_ms", ctypes.c_double),
                ("table1_map_ms", ctypes.c_double), ("table1_set_access_ms", ctypes.c_double),
                ("peak_mapped_chunks", ctypes.c_uint64)]


class vms_vmm_latency_report(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("hip_error", ctypes.c_int32),
                ("block_bytes", ctypes.c_uint64), ("chunk_bytes", ctypes.c_uint64), ("n_chunks", ctypes.c_uint64),
                ("granularity_bytes", ctypes.c_uint64),
                ("hipmalloc_ms", ctypes.c_double), ("hipfree_ms", ctypes.c_double),
                ("reserve_ms", ctypes.c_double), ("create_ms", ctypes.c_double), ("map_ms", ctypes.c_double),
                ("set_access_ms", ctypes.c_double), ("unmap_ms", ctypes.c_double), ("release_ms", ctypes.c_double)]


class vms_peaks_report(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("hip_error", ctypes.c_int32),
                ("compute_units", ctypes.c_uint32), ("clock_mhz", ctypes.c_uint32),
                ("copy_bytes", ctypes.c_uint64), ("copy_ms", ctypes.c_double), ("hbm_copy_gbs", ctypes.c_double),
                ("lds_bytes", ctypes.c_uint64), ("lds_ms", ctypes.c_double), ("lds_read_gbs", ctypes.c_double),
                ("read_bytes", ctypes.c_uint64), ("read_ms", ctypes.c_double), ("hbm_read_gbs", ctypes.c_double)]


class vms_live_config(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("spool_threshold", ctypes.c_uint32),
                ("chunk_bytes", ctypes.c_uint64), ("small_limit_bytes", ctypes.c_uint64),
                ("frag_limit_bytes", ctypes.c_uint64), ("capacity_bytes", ctypes.c_uint64),
                ("sync_before_unmap", ctypes.c_uint32), ("reserved0", ctypes.c_uint32)]


class vms_live_api_report(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("hip_error", ctypes.c_int32),
                ("n_reserve", ctypes.c_uint64), ("n_create", ctypes.c_uint64), ("n_map", ctypes.c_uint64),
                ("n_set_access", ctypes.c_uint64), ("n_unmap", ctypes.c_uint64), ("n_release", ctypes.c_uint64),
                ("n_address_free", ctypes.c_uint64),
                ("ms_reserve", ctypes.c_double), ("ms_create", ctypes.c_double), ("ms_map", ctypes.c_double),
                ("ms_set_access", ctypes.c_double), ("ms_unmap", ctypes.c_double), ("ms_release", ctypes.c_double),
                ("ms_address_free", ctypes.c_double),
                ("n_malloc", ctypes.c_uint64), ("n_free", ctypes.c_uint64),
                ("ms_malloc", ctypes.c_double), ("ms_free", ctypes.c_double)]


# vms_trace_stats as a numpy record (same layout as the C struct)
STATS_DTYPE = np.dtype([("peak_requested", "<u8"), ("peak_active", "<u8"), ("peak_reserved", "<u8"),
                        ("final_requested", "<u8"), ("final_active", "<u8"), ("final_reserved", "<u8"),
                        ("digest", "<u8"), ("n_code", "<u4", (8,)),
                        ("n_split", "<u4"), ("n_merge", "<u4"),
                        ("n_sblock_created", "<u4"), ("n_sblock_evicted", "<u4"),
                        ("first_oom_event", "<u4"), ("status", "<u4"),
                        ("max_pblocks", "<u4"), ("max_sblocks", "<u4"),
                        ("max_free_blocks", "<u4"), ("max_members", "<u4"),
                        ("max_runs", "<u4"), ("overflow_event", "<u4"),
                        ("max_multi_pblocks", "<u4"), ("reserved1", "<u4"),
                        ("fragmentation", "<f8")])

EXPORTS = ["vms_config_default", "vms_replay_create", "vms_replay_workspace_bytes", "vms_replay_lds_bytes",
           "vms_replay_run", "vms_replay_run_static", "vms_replay_static_workspace_bytes", "vms_replay_stats", "vms_replay_summary", "vms_replay_last_kernel_ms", "vms_demo_plan",
           "vms_replay_destroy", "vms_replay_last_hip_error", "vms_strerror", "vms_selftest",
           "vms_demo_run", "vms_vmm_latency", "vms_measure_peaks",
           "vms_live_config_default", "vms_live_create", "vms_live_malloc", "vms_live_free", "vms_live_run_trace",
           "vms_live_slot", "vms_live_stats", "vms_live_destroy", "vms_torch_malloc", "vms_torch_free",
           "vms_torch_allocator"]

_lib = None


def lib():
    """Load libvmsreplay.so (built in-tree; built now only if it is missing)."""
    global _lib
    if _lib is None:
        # PyTorch ships its own HIP runtime (same soname as the system one).  Import it first so
        # that this library binds to the runtime torch already loaded: one runtime per process.
        import torch  # noqa: F401
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = ctypes.CDLL(path)
        vp, u32, u64, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t
        L.vms_config_default.restype = None
        L.vms_config_default.argtypes = [ctypes.POINTER(vms_config), u32, u32, u32]
        L.vms_replay_create.restype = ctypes.c_int
        L.vms_replay_create.argtypes = [ctypes.POINTER(vms_config), ctypes.POINTER(vp)]
        L.vms_replay_workspace_bytes.restype = sz
        L.vms_replay_workspace_bytes.argtypes = [vp]
        L.vms_replay_lds_bytes.restype = ctypes.c_int
        L.vms_replay_lds_bytes.argtypes = [vp, ctypes.POINTER(u32 * 2)]
        L.vms_replay_run.restype = ctypes.c_int
        L.vms_replay_run.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.vms_replay_run_static.restype = ctypes.c_int
        L.vms_replay_run_static.argtypes = [vp, vp, vp, vp, vp, vp]
        L.vms_replay_static_workspace_bytes.restype = sz
        L.vms_replay_static_workspace_bytes.argtypes = []
        L.vms_replay_stats.restype = ctypes.c_int
        L.vms_replay_stats.argtypes = [vp, vp, sz]
        L.vms_replay_summary.restype = ctypes.c_int
        L.vms_replay_summary.argtypes = [vp, ctypes.POINTER(vms_summary)]
        L.vms_replay_last_kernel_ms.restype = ctypes.c_int
        L.vms_replay_last_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float * 3)]
        L.vms_replay_destroy.restype = None
        L.vms_replay_destroy.argtypes = [vp]
        L.vms_replay_last_hip_error.restype = ctypes.c_int
        L.vms_replay_last_hip_error.argtypes = [vp]
        L.vms_strerror.restype = ctypes.c_char_p
        L.vms_strerror.argtypes = [ctypes.c_int]
        L.vms_selftest.restype = ctypes.c_int
        L.vms_selftest.argtypes = []
        L.vms_demo_run.restype = ctypes.c_int
        L.vms_demo_run.argtypes = [ctypes.POINTER(vms_config), vp, vp, u32, ctypes.POINTER(vms_demo_report)]
        L.vms_demo_plan.restype = ctypes.c_int
        L.vms_demo_plan.argtypes = [ctypes.POINTER(vms_config), vp, vp, u32, ctypes.POINTER(vms_demo_report)]
        L.vms_vmm_latency.restype = ctypes.c_int
        L.vms_vmm_latency.argtypes = [u64, u64, u32, ctypes.POINTER(vms_vmm_latency_report)]
        L.vms_measure_peaks.restype = ctypes.c_int
        L.vms_measure_peaks.argtypes = [ctypes.POINTER(vms_peaks_report)]
        L.vms_live_config_default.restype = None
        L.vms_live_config_default.argtypes = [ctypes.POINTER(vms_live_config)]
        L.vms_live_create.restype = ctypes.c_int
        L.vms_live_create.argtypes = [ctypes.POINTER(vms_live_config), ctypes.POINTER(vp)]
        L.vms_live_malloc.restype = ctypes.c_int
        L.vms_live_malloc.argtypes = [vp, u64, ctypes.POINTER(vp), ctypes.POINTER(u64)]
        L.vms_live_free.restype = ctypes.c_int
        L.vms_live_free.argtypes = [vp, vp, ctypes.POINTER(u64)]
        L.vms_live_run_trace.restype = ctypes.c_int
        L.vms_live_run_trace.argtypes = [vp, vp, u32, u32, vp]
        L.vms_live_slot.restype = ctypes.c_int
        L.vms_live_slot.argtypes = [vp, u32, ctypes.POINTER(vp), ctypes.POINTER(u64)]
        L.vms_live_stats.restype = ctypes.c_int
        L.vms_live_stats.argtypes = [vp, vp, ctypes.POINTER(vms_live_api_report)]
        L.vms_live_destroy.restype = None
        L.vms_live_destroy.argtypes = [vp]
        L.vms_torch_malloc.restype = vp
        L.vms_torch_malloc.argtypes = [ctypes.c_ssize_t, ctypes.c_int, vp]
        L.vms_torch_free.restype = None
        L.vms_torch_free.argtypes = [vp, ctypes.c_ssize_t, ctypes.c_int, vp]
        L.vms_torch_allocator.restype = vp
        L.vms_torch_allocator.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


class VmsError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s: %s (%d)" % (what, lib().vms_strerror(code).decode(), code))
        self.code = code


def vms_config_default(n_traces, max_events, max_slots):
    cfg = vms_config()
    lib().vms_config_default(ctypes.byref(cfg), n_traces, max_events, max_slots)
    return cfg


def vms_strerror(code):
    return lib().vms_strerror(code).decode()


def vms_selftest():
    return lib().vms_selftest()


def vms_demo_run(cfg, h_events, h_dec_vms, n_events=None):
    """Execute one trace's stitching decisions with real HIP virtual-memory mappings.
    h_events / h_dec_vms: 1-D uint64 numpy arrays (host).  Returns (rc, vms_demo_report)."""
    ev = np.ascontiguousarray(h_events, dtype=np.uint64)
    dec = np.ascontiguousarray(h_dec_vms, dtype=np.uint64)
    assert ev.ndim == 1 and ev.shape == dec.shape
    n = ev.shape[0] if n_events is None else min(int(n_events), ev.shape[0])
    rep = vms_demo_report()
    rep.struct_size = ctypes.sizeof(vms_demo_report)
    rc = lib().vms_demo_run(ctypes.byref(cfg), ev.ctypes.data, dec.ctypes.data, n, ctypes.byref(rep))
    return rc, rep


def vms_demo_plan(cfg, h_events, h_dec_vms, n_events=None):
    """The driver calls vms_demo_run would make for this trace, counted on the host.  Returns (rc, report)."""
    ev = np.ascontiguousarray(h_events, dtype=np.uint64)
    dec = np.ascontiguousarray(h_dec_vms, dtype=np.uint64)
    assert ev.ndim == 1 and ev.shape == dec.shape
    n = ev.shape[0] if n_events is None else min(int(n_events), ev.shape[0])
    rep = vms_demo_report()
    rep.struct_size = ctypes.sizeof(vms_demo_report)
    rc = lib().vms_demo_plan(ctypes.byref(cfg), ev.ctypes.data, dec.ctypes.data, n, ctypes.byref(rep))
    return rc, rep


def vms_vmm_latency(block_bytes, chunk_bytes, repeats=3):
    """Time the HIP virtual-memory calls for one block built from chunks.  Returns (rc, report)."""
    rep = vms_vmm_latency_report()
    rep.struct_size = ctypes.sizeof(vms_vmm_latency_report)
    rc = lib().vms_vmm_latency(int(block_bytes), int(chunk_bytes), int(repeats), ctypes.byref(rep))
    return rc, rep


def vms_measure_peaks():
    """HBM copy and LDS read bandwidth reachable on the current device.  Returns (rc, report)."""
    rep = vms_peaks_report()
    rep.struct_size = ctypes.sizeof(vms_peaks_report)
    rc = lib().vms_measure_peaks(ctypes.byref(rep))
    return rc, rep


class Replay:
    """One vms_replay handle.  Tensors are torch CUDA tensors; only their pointers cross the ABI."""

    def __init__(self, cfg):
        self.cfg = cfg
        self._h = ctypes.c_void_p()
        rc = lib().vms_replay_create(ctypes.byref(cfg), ctypes.byref(self._h))
        if rc != VMS_OK:
            self._h = None
            raise VmsError(rc, "vms_replay_create")
        self._ws = None

    def workspace_bytes(self):
        return int(lib().vms_replay_workspace_bytes(self._h))

    def lds_bytes(self):
        out = (ctypes.c_uint32 * 2)()
        lib().vms_replay_lds_bytes(self._h, ctypes.byref(out))
        return [int(out[0]), int(out[1])]

    def run(self, d_events, d_n_events=None, d_dec_split=None, d_dec_vms=None, stream=None):
        """Enqueue one replay of d_events (int64/uint64 CUDA tensor [n_traces, max_events])."""
        import torch
        assert d_events.is_cuda and d_events.is_contiguous() and d_events.element_size() == 8
        assert tuple(d_events.shape) == (self.cfg.n_traces, self.cfg.max_events)
        for d in (d_dec_split, d_dec_vms):
            assert d is None or (d.is_cuda and d.is_contiguous() and d.shape == d_events.shape
                                 and d.element_size() == 8)
        if d_n_events is not None:
            assert d_n_events.is_cuda and d_n_events.is_contiguous() and d_n_events.element_size() == 4
            assert d_n_events.numel() == self.cfg.n_traces
        need = self.workspace_bytes()
        if need and (self._ws is None or self._ws.numel() < need + 256):
            self._ws = torch.empty(need + 256, dtype=torch.uint8, device=d_events.device)
        ws_ptr = 0
        if need:
            ws_ptr = (self._ws.data_ptr() + 255) & ~255
        s = torch.cuda.current_stream(d_events.device) if stream is None else stream
        ptr = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
        rc = lib().vms_replay_run(self._h, ptr(d_events), ptr(d_n_events), ptr(d_dec_split), ptr(d_dec_vms),
                                  ctypes.c_void_p(ws_ptr) if ws_ptr else None, ctypes.c_void_p(s.cuda_stream))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_replay_run (hip error %d)" % lib().vms_replay_last_hip_error(self._h))

    def run_static(self, d_events, d_n_events=None, d_dec_split=None, d_dec_vms=None, stream=None):
        """vms_replay_run_static: the same replay with the library's built-in workspace (nothing is allocated)."""
        import torch
        assert d_events.is_cuda and d_events.is_contiguous() and d_events.element_size() == 8
        assert tuple(d_events.shape) == (self.cfg.n_traces, self.cfg.max_events)
        s = torch.cuda.current_stream(d_events.device) if stream is None else stream
        ptr = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
        rc = lib().vms_replay_run_static(self._h, ptr(d_events), ptr(d_n_events), ptr(d_dec_split), ptr(d_dec_vms),
                                         ctypes.c_void_p(s.cuda_stream))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_replay_run_static (hip error %d)" % lib().vms_replay_last_hip_error(self._h))

    def stats(self):
        """Statistics of the last run: numpy record array [2, n_traces] ([0] splitting, [1] VMS)."""
        out = np.zeros((2, self.cfg.n_traces), dtype=STATS_DTYPE)
        rc = lib().vms_replay_stats(self._h, out.ctypes.data, out.size)
        if rc != VMS_OK:
            raise VmsError(rc, "vms_replay_stats")
        return out

    def summary(self):
        out = vms_summary()
        rc = lib().vms_replay_summary(self._h, ctypes.byref(out))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_replay_summary")
        return out

    def last_kernel_ms(self):
        out = (ctypes.c_float * 3)()
        rc = lib().vms_replay_last_kernel_ms(self._h, ctypes.byref(out))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_replay_last_kernel_ms")
        return dict(split=float(out[0]), vms=float(out[1]), total=float(out[2]))

    def close(self):
        if self._h:
            lib().vms_replay_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def vms_live_config_default():
    cfg = vms_live_config()
    lib().vms_live_config_default(ctypes.byref(cfg))
    return cfg


def _live_stats(handle):
    out = np.zeros(1, dtype=STATS_DTYPE)
    api = vms_live_api_report()
    api.struct_size = ctypes.sizeof(vms_live_api_report)
    rc = lib().vms_live_stats(handle, out.ctypes.data, ctypes.byref(api))
    if rc != VMS_OK:
        raise VmsError(rc, "vms_live_stats")
    return out[0], api


class LiveAllocator:
    """One vms_live handle: the stitching allocator serving real device memory on the current device."""

    def __init__(self, cfg=None):
        self.cfg = cfg if cfg is not None else vms_live_config_default()
        self._h = ctypes.c_void_p()
        rc = lib().vms_live_create(ctypes.byref(self.cfg), ctypes.byref(self._h))
        if rc != VMS_OK:
            self._h = None
            raise VmsError(rc, "vms_live_create")

    def malloc(self, nbytes):
        """Returns (device address or None, decision word)."""
        ptr, dec = ctypes.c_void_p(), ctypes.c_uint64()
        rc = lib().vms_live_malloc(self._h, int(nbytes), ctypes.byref(ptr), ctypes.byref(dec))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_live_malloc")
        return ptr.value, int(dec.value)

    def free(self, ptr):
        dec = ctypes.c_uint64()
        rc = lib().vms_live_free(self._h, ctypes.c_void_p(ptr), ctypes.byref(dec))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_live_free")
        return int(dec.value)

    def run_trace(self, h_events, max_slots):
        """Serve a whole trace of event words (1-D uint64 numpy array); returns the decision words."""
        ev = np.ascontiguousarray(h_events, dtype=np.uint64)
        assert ev.ndim == 1
        dec = np.zeros_like(ev)
        rc = lib().vms_live_run_trace(self._h, ev.ctypes.data, ev.shape[0], int(max_slots), dec.ctypes.data)
        if rc != VMS_OK:
            raise VmsError(rc, "vms_live_run_trace")
        return dec

    def slot(self, slot):
        ptr, nbytes = ctypes.c_void_p(), ctypes.c_uint64()
        rc = lib().vms_live_slot(self._h, int(slot), ctypes.byref(ptr), ctypes.byref(nbytes))
        if rc != VMS_OK:
            raise VmsError(rc, "vms_live_slot")
        return ptr.value, int(nbytes.value)

    def stats(self):
        """(vms_trace_stats record, vms_live_api_report)."""
        return _live_stats(self._h)

    def close(self):
        if self._h:
            lib().vms_live_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def torch_allocator_stats(device=0):
    """Statistics of the allocator behind vms_torch_malloc for a device (None before its first request)."""
    h = lib().vms_torch_allocator(int(device))
    return _live_stats(ctypes.c_void_p(h)) if h else None


def torch_pluggable_allocator():
    """torch.cuda.memory.CUDAPluggableAllocator over vms_torch_malloc / vms_torch_free; install it with
    torch.cuda.memory.change_current_allocator() before the process touches device memory."""
    import torch
    lib()
    return torch.cuda.memory.CUDAPluggableAllocator(_build.LIB, "vms_torch_malloc", "vms_torch_free")
