"""Functional stitching demo: one trace's decisions executed with real HIP virtual-memory mappings."""
import numpy as np
import pytest

import gpu_util
from paper_2401_08156_amd import binding, workloads
from paper_2401_08156_amd import tracegen as tg

pytestmark = pytest.mark.gpu
MiB = 1 << 20


def replay_one(config, n_events, **kw):
    ev, ms = tg.generate(config, n_traces=1, n_events=n_events, **kw)
    cfg = workloads.make_config(binding, config, 1, n_events, ms, kind=3 if config == 5 else None)
    _, dv, st = gpu_util.gpu_replay(ev, cfg)
    return cfg, ev[0], dv[0], st


def test_demo_worked_example_maps_without_new_memory():
    # 4 MiB + 2 MiB freed blocks serve 6 MiB by stitching: three chunks in total, one stitched range
    ev = tg.make_events([("A", 0, 4 * MiB), ("A", 1, 2 * MiB), ("F", 0), ("F", 1), ("A", 2, 6 * MiB)])
    cfg = gpu_util.make_cfg(1, 5, 4)
    _, dv, _ = gpu_util.gpu_replay(ev[None, :], cfg)
    rc, rep = binding.vms_demo_run(cfg, ev, dv[0])
    assert rc == 0, (rc, rep.failed_event, rep.hip_error, rep.failed_api, rep.chunks_created, rep.n_map)
    assert rep.chunks_created == 3 and rep.n_stitches == 1 and rep.n_splits == 0
    assert rep.alias_checks == 1 and rep.alias_failures == 0
    assert rep.n_create == 3 and rep.n_release == 3
    assert rep.n_map == 3 + 3            # each chunk under its pBlock and again under the stitched range
    assert rep.table1_bytes == 2 << 30 and rep.table1_hipmalloc_ms > 0


def test_demo_config1_trace():
    cfg, ev, dv, st = replay_one(1, 2000)
    rc, rep = binding.vms_demo_run(cfg, ev, dv)
    assert rc == 0, (rc, rep.failed_event, rep.hip_error, rep.failed_api, rep.chunks_created, rep.n_map)
    assert rep.events_replayed == 2000 and rep.alias_failures == 0 and rep.alias_checks > 0
    assert rep.chunks_created * cfg.chunk_bytes <= st["final_reserved"][1, 0]
    assert rep.n_stitches == st["n_sblock_created"][1, 0]
    assert rep.n_sblocks_released == st["n_sblock_evicted"][1, 0]
    assert rep.n_release == rep.n_create == rep.chunks_created


def test_demo_offload_trace_prefix():
    # an offloading trace of the config-5 mixture (kind 3): gigabyte-sized staging buffers.  Only a
    # prefix: with one mapping per 2 MiB chunk the runtime refuses further hipMemSetAccess calls once
    # about 48,000 chunk mappings are live, which this trace reaches near event 650.
    # The trace: the lowest-index offloading trace whose stitched peak fits half of the free HBM.
    import torch
    free_bytes, _ = torch.cuda.mem_get_info()
    for first in range(1, 64, 3):
        cfg, ev, dv, st = replay_one(5, 400, first_trace=first)
        if int(st["peak_reserved"][1, 0]) <= free_bytes // 2:
            break
    else:
        pytest.fail("no offloading trace fits half of the free device memory")
    rc, rep = binding.vms_demo_run(cfg, ev, dv)
    assert rc == 0, (rc, rep.failed_event, rep.hip_error, rep.failed_api, rep.chunks_created, rep.n_map)
    assert rep.alias_failures == 0 and rep.n_stitches == st["n_sblock_created"][1, 0]
    assert rep.chunks_created * cfg.chunk_bytes == st["final_reserved"][1, 0]    # no small requests here


def test_demo_whole_config5_trace_chosen_by_plan():
    # a whole trace of the 16,384 x 100,000 mixture with real mappings.  vms_demo_plan (host only)
    # counts what a trace would map: the offloading trace would hold over a million chunk mappings at
    # once (hipMemSetAccess is refused at about 48,000 live mappings), the recomputation trace about 31,000.
    chosen = None
    for first, kind in ((1, 3), (0, 2)):
        ev, ms = tg.generate(5, n_traces=1, n_events=100000, first_trace=first)
        cfg = workloads.make_config(binding, 5, 1, 100000, ms, kind=kind)
        _, dv, st = gpu_util.gpu_replay(ev, cfg)
        rc, plan = binding.vms_demo_plan(cfg, ev[0], dv[0])
        assert rc == 0 and plan.events_replayed == 100000
        assert plan.n_stitches == st["n_sblock_created"][1, 0] and plan.n_sblocks_released == st["n_sblock_evicted"][1, 0]
        if kind == 3:
            assert plan.peak_mapped_chunks > 500000
        else:
            assert plan.peak_mapped_chunks < 40000
            chosen = (cfg, ev[0], dv[0], st, plan)
    cfg, ev, dv, st, plan = chosen
    rc, rep = binding.vms_demo_run(cfg, ev, dv)
    assert rc == 0, (rc, rep.failed_event, rep.hip_error, rep.failed_api, rep.chunks_created, rep.n_map)
    assert rep.events_replayed == 100000 and rep.alias_failures == 0 and rep.alias_checks > 0
    assert rep.chunks_created * cfg.chunk_bytes == st["final_reserved"][1, 0]
    # the plan foresaw every call
    for f in ("n_reserve", "n_create", "n_map", "n_set_access", "n_unmap", "n_release", "n_address_free", "peak_mapped_chunks"):
        assert getattr(rep, f) == getattr(plan, f), f


def test_demo_reports_a_refused_mapping_and_leaves_nothing_behind():
    # The prefix of an offloading trace that wants 150,000 chunk mappings at once.  Where the driver
    # refuses a call on the way (seen: hipMemSetAccess -> hipErrorInvalidValue with about 48,000 live
    # mappings), the demo must say which call and which error, give every range and chunk back, and
    # leave no pending HIP error for the caller's next call; where it does not refuse, the prefix runs.
    import torch
    ev, ms = tg.generate(5, n_traces=1, n_events=100000, first_trace=1)
    cfg = workloads.make_config(binding, 5, 1, 100000, ms, kind=3)
    _, dv, st = gpu_util.gpu_replay(ev, cfg)
    lo, hi = 1, 100000
    while lo < hi:                                # the shortest prefix that reaches 150,000
        mid = (lo + hi) // 2
        _, plan = binding.vms_demo_plan(cfg, ev[0], dv[0], n_events=mid)
        lo, hi = (lo, mid) if plan.peak_mapped_chunks >= 150000 else (mid + 1, hi)
    rc, plan = binding.vms_demo_plan(cfg, ev[0], dv[0], n_events=lo)
    free_before, _ = torch.cuda.mem_get_info()
    assert rc == 0 and plan.chunks_created * cfg.chunk_bytes < free_before // 2
    rc, rep = binding.vms_demo_run(cfg, ev[0], dv[0], n_events=lo)
    if rc != 0:
        assert rc == -5 and rep.hip_error != 0 and 1 <= rep.failed_api <= 8
        assert rep.failed_event == rep.events_replayed < lo
        assert rep.n_release == rep.n_create == rep.chunks_created
        print("refused: api %d, hip error %d, at event %d with %d chunk mappings live (peak)"
              % (rep.failed_api, rep.hip_error, rep.failed_event, rep.peak_mapped_chunks))
    else:
        assert rep.events_replayed == lo and rep.alias_failures == 0
    x = torch.ones(1 << 20, device="cuda")        # the next HIP call of the process works
    assert float(x.sum()) == float(1 << 20)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert abs(free_before - free_after) < (1 << 30)


def test_demo_rejects_inconsistent_decisions():
    cfg, ev, dv, _ = replay_one(1, 600)
    bad = dv.copy()
    i = int(np.flatnonzero((bad & np.uint64(15)) == 3)[0])       # a stitch decision: claim one candidate more
    bad[i] += np.uint64(1 << 8)
    rc, rep = binding.vms_demo_run(cfg, ev, bad)
    assert rc == -1 and rep.failed_event == i


def test_vmm_latency_table_small_block():
    # the analogue of the paper's Table 1 on a small block: 256 MiB from 2 MiB and from 64 MiB chunks
    from paper_2401_08156_amd import vmm_table
    rows = vmm_table.measure(256 * MiB, [2 * MiB, 64 * MiB], repeats=2)
    assert [r["n_chunks"] for r in rows] == [128, 4]
    for r in rows:
        assert r["ms"]["hipmalloc"] > 0 and r["ms"]["total"] > 0
        assert all(v >= 0 for v in r["ms"].values())
    # more calls for the same block cannot be cheaper per block by much: create + map + set access grow with the chunk count
    assert rows[0]["ms"]["total"] > rows[1]["ms"]["total"] * 0.5
    # argument errors come back as codes
    rc, rep = binding.vms_vmm_latency(3 * MiB, 2 * MiB, 1)
    assert rc == -1


def test_measured_peaks_are_plausible():
    rc, rep = binding.vms_measure_peaks()
    assert rc == 0 and rep.hip_error == 0
    assert rep.compute_units >= 64
    # a copy kernel reaches a good part of the published 8 TB/s, LDS several times more
    assert 1000 < rep.hbm_copy_gbs < 8000
    assert rep.lds_read_gbs > rep.hbm_copy_gbs
