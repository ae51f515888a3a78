"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

from paper_2401_08156_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in ("vms_replay.h", "vms_live.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(vms_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert "vms_replay_create" in names and "vms_replay_run" in names and "vms_replay_stats" in names
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), "libvmsreplay.so does not export %s" % n
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(binding.vms_config) == 80
    assert binding.STATS_DTYPE.itemsize == 144
    assert ctypes.sizeof(binding.vms_summary) == 88
    assert ctypes.sizeof(binding.vms_demo_report) == 224
    assert ctypes.sizeof(binding.vms_vmm_latency_report) == 104
    assert ctypes.sizeof(binding.vms_peaks_report) == 64
    assert ctypes.sizeof(binding.vms_live_config) == 48
    assert ctypes.sizeof(binding.vms_live_api_report) == 152


def test_config_default_and_argument_errors_need_no_gpu():
    cfg = binding.vms_config_default(7, 100, 9)
    assert (cfg.struct_size, cfg.n_traces, cfg.max_events, cfg.max_slots) == (80, 7, 100, 9)
    assert cfg.chunk_bytes == 2 << 20 and cfg.policy_mask == 3 and cfg.spool_threshold == 512
    L = binding.lib()
    h = ctypes.c_void_p()
    assert L.vms_replay_create(None, ctypes.byref(h)) == -1
    cfg.struct_size = 12
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -2
    cfg = binding.vms_config_default(7, 100, 9)
    cfg.chunk_bytes = 3 << 20
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -1
    assert binding.vms_strerror(-6).startswith("per-trace tables")
    assert L.vms_replay_workspace_bytes(None) == 0


def test_tables_that_exceed_the_lds_are_refused_before_any_device_call():
    L = binding.lib()
    h = ctypes.c_void_p()
    # lists in LDS (at most 16,384 run entries): 4,000 pBlocks + 4,000 sBlocks + 16,000 entries do not fit 160 KB
    cfg = binding.vms_config_default(4, 100, 9)
    cfg.max_pblocks, cfg.max_sblocks, cfg.max_runs = 4000, 4000, 16000
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -6 and not h.value
    # the splitting policy alone needs none of these tables
    cfg.policy_mask = 1
    rc = L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h))
    assert rc in (0, -5)                        # -5: no device here; the layout itself was accepted
    if rc == 0:
        L.vms_replay_destroy(h)
    # lists in the workspace: the tables of the largest offloading traces fit once the last-use stamps
    # go to the workspace too ...
    cfg = binding.vms_config_default(4, 100, 9)
    cfg.max_free_blocks, cfg.max_pblocks, cfg.max_sblocks, cfg.max_runs, cfg.max_chunks = 64, 8192, 4352, 1 << 21, 16384
    rc = L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h))
    assert rc in (0, -5)
    if rc == 0:
        L.vms_replay_destroy(h)
    # ... and beyond that nothing helps
    cfg.max_sblocks = 6000
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -6
