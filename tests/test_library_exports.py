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
    assert ctypes.sizeof(binding.vms_config) == 96
    assert binding.STATS_DTYPE.itemsize == 152
    assert ctypes.sizeof(binding.vms_summary) == 88
    assert ctypes.sizeof(binding.vms_demo_report) == 232
    assert ctypes.sizeof(binding.vms_vmm_latency_report) == 104
    assert ctypes.sizeof(binding.vms_peaks_report) == 88
    assert ctypes.sizeof(binding.vms_live_config) == 48
    assert ctypes.sizeof(binding.vms_live_api_report) == 152


def test_config_default_and_argument_errors_need_no_gpu():
    cfg = binding.vms_config_default(7, 100, 9)
    assert (cfg.struct_size, cfg.n_traces, cfg.max_events, cfg.max_slots) == (96, 7, 100, 9)
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
    # tables beyond those go to the fine-grained variant (lists in the workspace, 6 bytes of LDS per
    # sBlock, single-chunk pBlocks in bitmaps): the largest offloading traces take about 50 KB there ...
    cfg = binding.vms_config_default(4, 100, 9)
    cfg.max_free_blocks, cfg.max_pblocks, cfg.max_sblocks, cfg.max_runs, cfg.max_chunks = 64, 8192, 4352, 1 << 21, 16384
    rc = L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h))
    assert rc in (0, -5)
    if rc == 0:
        L.vms_replay_destroy(h)
    # ... its rank search covers 8,000 sBlocks and 4,096 multi-chunk pBlocks, not more
    cfg.max_sblocks = 9000
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -6
    cfg.max_sblocks, cfg.max_multi_pblocks = 4352, 5000
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -6
    # a chunk bitmap that alone exceeds the LDS
    cfg = binding.vms_config_default(4, 100, 9)
    cfg.chunk_bytes, cfg.small_limit_bytes, cfg.frag_limit_bytes, cfg.max_chunks = 1 << 15, 1 << 15, 1 << 15, 1 << 22
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -6


def test_table_place_is_validated_without_a_device():
    L = binding.lib()
    h = ctypes.c_void_p()
    cfg = binding.vms_config_default(4, 100, 9)
    cfg.variant, cfg.table_place = binding.VMS_VARIANT_FINE, 4                 # no such place
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -1
    cfg.table_place, cfg.max_chunks = binding.VMS_TABLES_WORKSPACE_ALL, 70000   # 32-bit chunk numbers keep their tables in LDS
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -1
    for place in (binding.VMS_TABLES_LDS, binding.VMS_TABLES_WORKSPACE, binding.VMS_TABLES_WORKSPACE_ALL):
        cfg = binding.vms_config_default(4, 100, 9)
        cfg.variant, cfg.table_place = binding.VMS_VARIANT_FINE, place
        rc = L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h))
        assert rc in (0, -5)                    # -5: no device here; the plan itself was accepted
        if rc == 0:
            L.vms_replay_destroy(h)
    # the flat variant has no such tables: the field is ignored there
    cfg = binding.vms_config_default(4, 100, 9)
    cfg.variant, cfg.table_place = binding.VMS_VARIANT_FLAT, binding.VMS_TABLES_WORKSPACE_ALL
    assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) in (0, -5)


def test_table_sizes_that_would_wrap_a_32_bit_layout_are_refused():
    # the LDS layout is computed in 64 bits and every table size is bounded: a huge value must end as
    # "too big" (or invalid), never as a small layout that a kernel would then overrun
    L = binding.lib()
    h = ctypes.c_void_p()
    for field, value in (("max_slots", 0x40000010), ("max_pblocks", 0x20000000), ("max_sblocks", 0x20000000),
                         ("max_free_blocks", 0x20000000), ("max_multi_pblocks", 0x20000000),
                         ("max_slots", 100000), ("max_free_blocks", 30000), ("max_slots", 0xFFFFFFFF)):
        cfg = binding.vms_config_default(4, 100, 9)
        setattr(cfg, field, value)
        assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -6, (field, value)
        assert not h.value
    for field, value in (("max_runs", 0x40000000), ("max_chunks", 0x08000000), ("max_small_blocks", 193)):
        cfg = binding.vms_config_default(4, 100, 9)
        setattr(cfg, field, value)
        assert L.vms_replay_create(ctypes.byref(cfg), ctypes.byref(h)) == -1, (field, value)
