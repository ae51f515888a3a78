"""GPU parity: the HIP replay (through the C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import gpu_util
import oracle
from paper_2401_08156_amd import binding
from paper_2401_08156_amd import tracegen as tg

pytestmark = pytest.mark.gpu
MiB = 1 << 20


def test_wave_primitives_selftest():
    assert binding.vms_selftest() == 0


def test_config1_full():
    ev, ms = tg.generate(1)
    cfg = gpu_util.make_cfg(1, ev.shape[1], ms)
    st = gpu_util.assert_parity(ev, cfg, label="config 1")
    assert st["status"].max() == 0


@pytest.mark.parametrize("kw", [dict(), dict(frag_limit_bytes=8 * MiB), dict(spool_threshold=8),
                                dict(capacity_bytes=512 * MiB), dict(small_limit_bytes=0)])
def test_config1_variants_many_seeds(kw):
    ev, ms = tg.generate(1, n_traces=96, n_events=1500, seed=11)
    cfg = gpu_util.make_cfg(96, 1500, ms, **kw)
    gpu_util.assert_parity(ev, cfg, label="config 1 %s" % kw)


def test_splitting_pool_in_registers():
    # pools of at most 192 inactive blocks are held in registers by the splitting kernel: random traces
    # with many merges on both sides, and a table so small that it overflows (reported, not fatal)
    ev, ms = tg.generate(1, n_traces=64, n_events=1500, seed=17)
    cfg = gpu_util.make_cfg(64, 1500, ms, max_free_blocks=192)
    st = gpu_util.assert_parity(ev, cfg, label="config 1, register pool")
    assert st["n_merge"][0].min() > 0 and st["max_free_blocks"][0].max() <= 192
    # up to 320: five registers per lane (slot table in registers, then in LDS)
    cfg = gpu_util.make_cfg(64, 1500, ms, max_free_blocks=320)
    gpu_util.assert_parity(ev, cfg, label="config 1, register pool of 320")
    ev4, ms4 = tg.generate(4, n_traces=48, n_events=6000, seed=5)
    st = gpu_util.assert_parity(ev4, gpu_util.make_cfg(48, 6000, ms4, max_free_blocks=320), label="LoRA traces, register pool of 320")
    assert ms4 > 64 and st["max_free_blocks"][0].max() > 64
    ev3, ms3 = tg.generate(3, n_traces=48, n_events=6000, seed=5)
    assert ms3 <= 64
    gpu_util.assert_parity(ev3, gpu_util.make_cfg(48, 6000, ms3, max_free_blocks=320, policy_mask=1),
                           label="offloading traces, slot table and pool of 320 in registers")
    cfg = gpu_util.make_cfg(64, 1500, ms, max_free_blocks=6)
    _, _, st = gpu_util.gpu_replay(ev, cfg)
    assert (st["status"][0] & binding.VMS_ST_TABLE_OVERFLOW).all()
    # the stitching policy's pool for requests below one chunk may have a size of its own: in registers
    # beside a splitting pool in LDS, and too small (reported for that policy only)
    cfg = gpu_util.make_cfg(64, 1500, ms, max_free_blocks=512, max_small_blocks=192)
    gpu_util.assert_parity(ev, cfg, label="config 1, small pool of the stitching policy in registers")
    cfg = gpu_util.make_cfg(64, 1500, ms, max_free_blocks=512, max_small_blocks=3)
    _, _, st = gpu_util.gpu_replay(ev, cfg)
    assert (st["status"][1] & binding.VMS_ST_OVF_FREE_BLOCKS).all() and (st["status"][0] == 0).all()


def test_worked_examples_on_gpu():
    import glob
    import os
    from test_oracle_examples import load_fixture, GOLDEN
    for path in sorted(glob.glob(os.path.join(GOLDEN, "*.txt"))):
        fx = load_fixture(path)
        ev = fx["events"][None, :]
        kw = dict(spool_threshold=int(fx["spool_threshold"])) if "spool_threshold" in fx else {}
        gpu_util.assert_parity(ev, gpu_util.make_cfg(1, ev.shape[1], 16, **kw), label=os.path.basename(path))
        # and through the fine-grained kernel variant
        gpu_util.assert_parity(ev, gpu_util.make_cfg(1, ev.shape[1], 16, variant=binding.VMS_VARIANT_FINE, **kw),
                               label=os.path.basename(path) + " (fine-grained variant)")


def test_ragged_and_empty_traces():
    ev, ms = tg.generate(1, n_traces=70, n_events=333, seed=5)
    n = (np.arange(70) * 37 % 334).astype(np.uint32)
    n[0], n[1], n[2] = 0, 1, 333
    cfg = gpu_util.make_cfg(70, 333, ms)
    gpu_util.assert_parity(ev, cfg, n_events=n, label="ragged")


def test_invalid_events_and_oom():
    ev = tg.make_events([("A", 0, 4 * MiB), ("A", 0, 2 * MiB), ("F", 3), ("A", 99, 2 * MiB), ("F", 0),
                         ("A", 1, 64 * MiB), ("F", 1), ("A", 2, 1024), ("F", 2)])
    ev = np.concatenate([ev, np.array([(1 << 32) | 0], dtype=np.uint64)])[None, :]
    cfg = gpu_util.make_cfg(1, ev.shape[1], 8, capacity_bytes=16 * MiB)
    st = gpu_util.assert_parity(ev, cfg, label="invalid/oom")
    assert st["status"][0, 0] == 1 and st["n_code"][1, 0, 5] == 1


@pytest.mark.parametrize("cfg_id,nt,ne", [(2, 48, 4000), (4, 24, 6000)])
def test_transformer_slices(cfg_id, nt, ne):
    ev, ms = tg.generate(cfg_id, n_traces=nt, n_events=ne)
    cfg = gpu_util.make_cfg(nt, ne, ms)
    gpu_util.assert_parity(ev, cfg, label="config %d slice" % cfg_id)


def test_runs_in_global_memory_variant():
    # more than 16384 run entries per trace: the fine-grained variant, with its lists in the workspace
    ev, ms = tg.generate(1, n_traces=64, n_events=2000, seed=21)
    cfg = gpu_util.make_cfg(64, 2000, ms, max_runs=20000)
    gpu_util.assert_parity(ev, cfg, label="config 1, runs in HBM")
    # tiny arena in HBM: forces compaction through the second half of the workspace slice
    ev, ms = tg.generate(2, n_traces=16, n_events=5000)
    cfg = gpu_util.make_cfg(16, 5000, ms, max_runs=16500, spool_threshold=64)
    gpu_util.assert_parity(ev, cfg, label="config 2, runs in HBM")


def test_arena_compaction_in_lds():
    ev, ms = tg.generate(2, n_traces=16, n_events=6000)
    cfg = gpu_util.make_cfg(16, 6000, ms, max_runs=1100, spool_threshold=96, max_sblocks=256)
    gpu_util.assert_parity(ev, cfg, label="config 2, small arena")


def test_config3_slice_with_large_tables():
    # offloading traces grind pBlocks down to single chunks: thousands of pBlocks, long stitch lists
    ev, ms = tg.generate(3, n_traces=12, n_events=8000)
    cfg = gpu_util.make_cfg(12, 8000, ms, max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=16384)
    gpu_util.assert_parity(ev, cfg, label="config 3 slice")


def test_largest_offloading_tables_with_low_thresholds():
    # the table sizes of the largest offloading traces; low thresholds make StitchFree choose among many
    # inactive sBlocks by their last-use stamps (read from the list headers in the workspace)
    for seed, threshold in ((5, 128), (6, 32)):
        ev, ms = tg.generate(3, n_traces=8, n_events=8000, seed=seed)
        cfg = gpu_util.make_cfg(8, 8000, ms, max_free_blocks=64, max_pblocks=8192, max_sblocks=4352,
                                max_runs=1 << 18, max_chunks=16384, spool_threshold=threshold)
        gpu_util.assert_parity(ev, cfg, label="config 3 slice, largest tables, threshold %d" % threshold)


def test_table_overflow_is_reported_not_fatal():
    ev, ms = tg.generate(1, n_traces=4, n_events=1000, seed=3)
    cfg = gpu_util.make_cfg(4, 1000, ms, max_free_blocks=4, max_pblocks=8)
    _, _, st = gpu_util.gpu_replay(ev, cfg)
    assert (st["status"] & binding.VMS_ST_TABLE_OVERFLOW).all()
    assert (st["overflow_event"] < 1000).all()


def test_periodic_trace_converges_on_gpu():
    # Sec. 4.2.2 / Sec. 5.5: on a strictly periodic stream the stitching allocator ends up with exact
    # hits only (here within the first few steps) and its reserved memory stops growing
    ev, ms = tg.generate(12, n_traces=16, n_events=5000)
    cfg = gpu_util.make_cfg(16, 5000, ms)
    st = gpu_util.assert_parity(ev, cfg, label="periodic recompute")
    _, dv, _ = gpu_util.gpu_replay(ev, cfg)
    is_alloc = (ev & np.uint64(1 << 31)) == 0
    code = (dv & np.uint64(15)).astype(int)
    late = np.zeros_like(is_alloc)
    late[:, 4 * 448:] = True                     # after four training steps of 448 events
    assert (code[is_alloc & late] == 1).all()
    assert (st["fragmentation"][1] == 0.0).all()


def test_zero3_scaleout_slice():
    # one rank of ZeRO-3 over 1, 2, 4, 8, 16 devices (Sec. 2.4, Sec. 5.3.2): shards shrink with the device
    # count, gathered weights come and go; three traces per device count
    from paper_2401_08156_amd import workloads
    ev, ms = tg.generate(6, n_traces=15, n_events=6000)
    cfg = workloads.make_config(binding, 6, 15, 6000, ms)
    st = gpu_util.assert_parity(ev, cfg, label="config 6 slice")
    assert st["status"].max() == 0


def test_randomised_workloads_and_parameters():
    # a seeded sweep over generator kind, batch shape, chunk size, small-request limit, fragmentation
    # limit, StitchFree threshold, capacity, list placement (LDS / workspace, small arena) and ragged lengths
    import random
    from paper_2401_08156_amd import workloads
    ran = 0
    for it in range(64):
        rng = random.Random(4242 + it)
        kind = rng.choice([1, 1, 2, 3, 4, 6])
        nt = rng.choice([3, 16, 40])
        ne = rng.choice([300, 1500, 3000])
        ev, ms = tg.generate(kind, n_traces=nt, n_events=ne, seed=1000 + it)
        chunk = rng.choice([2, 2, 2, 1, 4, 16]) * MiB
        kw = dict(chunk_bytes=chunk, small_limit_bytes=rng.choice([chunk, chunk, chunk // 2, 0, 512]),
                  frag_limit_bytes=chunk * rng.choice([1, 1, 2, 8, 64]), spool_threshold=rng.choice([512, 2, 8, 32, 100]))
        if rng.random() < 0.3:
            kw["capacity_bytes"] = rng.choice([256, 1024, 4096, 16384]) * MiB
        tables = dict(max_free_blocks=512, max_pblocks=2048, max_sblocks=1024, max_runs=16384, max_chunks=32768)
        if kind == 3:                                     # offloading: thousands of blocks, lists in the workspace
            tables.update(max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18)
        elif rng.random() < 0.25:
            tables["max_runs"] = 1 << 18                  # lists in the workspace
        elif rng.random() < 0.25:
            tables["max_runs"] = 1500                     # small arena: compaction
        n_events = None
        if rng.random() < 0.3:
            n_events = np.array([rng.randrange(0, ne + 1) for _ in range(nt)], dtype=np.uint32)
        cfg = gpu_util.make_cfg(nt, ne, ms, **kw, **tables)
        try:
            gpu_util.assert_parity(ev, cfg, n_events=n_events, label="sweep case %d" % it)
            ran += 1
        except AssertionError as e:
            if "table overflow" not in str(e):
                raise
    assert ran >= 48                                      # a few draws outgrow the small arena: reported, not replayed


def test_run_time_argument_errors_are_codes_and_launch_nothing():
    # every call below is refused on the host, before any kernel could see a bad pointer
    import ctypes
    import torch
    L = binding.lib()
    ev, ms = tg.generate(1, n_traces=4, n_events=200, seed=3)
    d_ev = torch.from_numpy(ev.view(np.int64)).cuda()
    r = binding.Replay(gpu_util.make_cfg(4, 200, ms, max_runs=20000))        # lists in the workspace: one is needed
    stats = np.zeros((2, 4), dtype=binding.STATS_DTYPE)
    assert L.vms_replay_stats(r._h, stats.ctypes.data, stats.size) == -7      # nothing has run yet
    summ = binding.vms_summary()
    assert L.vms_replay_summary(r._h, ctypes.byref(summ)) == -7
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ev_ptr = ctypes.c_void_p(d_ev.data_ptr())
    assert L.vms_replay_run(r._h, None, None, None, None, None, stream) == -1                 # no events
    assert L.vms_replay_run(None, ev_ptr, None, None, None, None, stream) == -1               # no handle
    assert r.workspace_bytes() > 0
    assert L.vms_replay_run(r._h, ev_ptr, None, None, None, None, stream) == -4               # workspace missing
    ws = torch.empty(r.workspace_bytes() + 512, dtype=torch.uint8, device="cuda")
    odd = ((ws.data_ptr() + 255) & ~255) + 8
    assert L.vms_replay_run(r._h, ev_ptr, None, None, None, ctypes.c_void_p(odd), stream) == -4   # misaligned
    r.run(d_ev)                                                                # the binding brings its own
    assert L.vms_replay_stats(r._h, stats.ctypes.data, 3) == -1               # wrong record count
    st = r.stats()
    assert (st["status"] & binding.VMS_ST_TABLE_OVERFLOW).sum() == 0 and (st["peak_reserved"] > 0).all()
    r.close()


def test_largest_requests_and_full_capacity():
    # the engine models at most 512 GiB (2^30 units of 512 B): requests of the largest encodable size
    # fail, two of 256 GiB fill the capacity exactly, nothing more fits, and a cached 256 GiB block is cut
    GiB = 1 << 30
    ev = tg.make_events([("A", 0, ((1 << 31) - 1) * 512), ("F", 0), ("A", 1, 256 * GiB), ("A", 2, 256 * GiB),
                         ("A", 3, 2 * MiB), ("F", 3), ("F", 1), ("A", 3, 128 * GiB), ("A", 4, 128 * GiB),
                         ("A", 5, 512), ("F", 2), ("F", 3), ("F", 4), ("A", 6, 512 * GiB - 2 * MiB), ("A", 7, 2 * MiB)])[None, :]
    for cap in (0, 512 * GiB):
        # (a block of 131,072 chunks may need 12,294 list entries: lists in the workspace)
        cfg = gpu_util.make_cfg(1, ev.shape[1], 8, capacity_bytes=cap, max_chunks=1 << 18, max_runs=1 << 16)
        st = gpu_util.assert_parity(ev, cfg, label="largest requests, capacity %d" % cap)
        assert st["n_code"][:, 0, 5].min() >= 2                     # the 1 TiB request and the 2 MiB one fail under both policies
        assert (st["peak_reserved"] == 512 * GiB).all()


def test_batch_summary_matches_the_oracle():
    # Sec. 5.1 "Metric": sums of the peaks, mean and maximum fragmentation over the batch, and the
    # memory reduction ratio (sum reserved splitting - sum reserved stitching) / sum reserved splitting,
    # reduced on the device; here against the same reductions over the oracle's per-trace statistics
    import torch
    ev, ms = tg.generate(4, n_traces=70, n_events=3000, seed=9)
    ev[3] = tg.make_events([("F", 0)] + [("A", 1, 2 * MiB)] * 2999)      # a trace with invalid events: flagged
    for mask in (3, 1, 2):
        cfg = gpu_util.make_cfg(70, 3000, ms, policy_mask=mask)
        r = binding.Replay(cfg)
        r.run(torch.from_numpy(ev.view(np.int64)).cuda())
        got = r.summary()
        gst = r.stats()
        r.close()
        P = gpu_util.oracle_params(cfg)
        ost = [oracle.replay(ev, P, pol, want_decisions=False, threads=8)[1] if mask & (1 << pol) else None for pol in (0, 1)]
        for pol in (0, 1):
            if ost[pol] is None:
                assert got.sum_peak_reserved[pol] == 0 and got.sum_peak_active[pol] == 0 and got.n_flagged[pol] == 0
                assert got.max_fragmentation[pol] == 0.0 and got.mean_fragmentation[pol] == 0.0
                continue
            o = ost[pol]
            assert got.sum_peak_reserved[pol] == int(o["peak_reserved"].sum(dtype=np.uint64))
            assert got.sum_peak_active[pol] == int(o["peak_active"].sum(dtype=np.uint64))
            assert got.n_flagged[pol] == int((o["status"] != 0).sum()) >= 1
            assert got.max_fragmentation[pol] == float(o["fragmentation"].max())
            mean = 0.0
            for f in o["fragmentation"]:                 # summed in trace order, as the device does
                mean += float(f)
            assert got.mean_fragmentation[pol] == mean / 70
            assert np.array_equal(gst[pol]["fragmentation"], o["fragmentation"])
        if mask == 3:
            a, b = int(ost[0]["peak_reserved"].sum(dtype=np.uint64)), int(ost[1]["peak_reserved"].sum(dtype=np.uint64))
            assert got.mem_reduction_ratio == float(a - b) / float(a) and got.mem_reduction_ratio > 0
        else:
            assert got.mem_reduction_ratio == 0.0


def test_kernel_variant_choice():
    # the same traces through the flat and the fine-grained stitching kernels, chosen by hand; what the
    # library chooses by itself; and 32-bit chunk numbers in the fine-grained one
    ev, ms = tg.generate(2, n_traces=24, n_events=4000, seed=31)
    for variant in (binding.VMS_VARIANT_FLAT, binding.VMS_VARIANT_FINE):
        cfg = gpu_util.make_cfg(24, 4000, ms, variant=variant, max_chunks=4096)
        r = binding.Replay(cfg)
        lds = r.lds_bytes()[1]
        r.close()
        assert (lds < 20000) == (variant == binding.VMS_VARIANT_FINE)
        gpu_util.assert_parity(ev, cfg, label="variant %d" % variant)
    # few traces: the flat variant (lower latency per trace); a batch that does not fit the compute
    # units at once, with tables that are small in the fine-grained layout: that one
    few = binding.Replay(gpu_util.make_cfg(24, 4000, ms, max_chunks=4096))
    many = binding.Replay(gpu_util.make_cfg(6000, 4000, ms, max_chunks=4096))
    assert few.lds_bytes()[1] > 30000 > 20000 > many.lds_bytes()[1]
    few.close()
    many.close()
    # tables too large for the flat variant cannot be forced into it
    with pytest.raises(binding.VmsError):
        binding.Replay(gpu_util.make_cfg(24, 4000, ms, variant=binding.VMS_VARIANT_FLAT, max_runs=1 << 18))
    ev, ms = tg.generate(3, n_traces=6, n_events=5000, seed=32)
    cfg = gpu_util.make_cfg(6, 5000, ms, max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=70000)
    gpu_util.assert_parity(ev, cfg, label="fine-grained variant, 32-bit chunk numbers")


@pytest.mark.parametrize("place", [binding.VMS_TABLES_WORKSPACE, binding.VMS_TABLES_WORKSPACE_ALL])
def test_sblock_tables_in_the_workspace(place):
    # the fine-grained kernel with the witnesses and list places of its sBlocks (and, second case, their sizes
    # too) in the workspace instead of LDS: offloading traces with thousands of sBlocks, low thresholds (many
    # releases: the tables move all the time), a tiny arena (compaction rewrites the list places), a slot
    # table in LDS, ragged traces
    W = dict(variant=binding.VMS_VARIANT_FINE, table_place=place)
    ev, ms = tg.generate(3, n_traces=12, n_events=8000)
    big = dict(max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=16384)
    lds = []
    for pl in (binding.VMS_TABLES_LDS, place):
        r = binding.Replay(gpu_util.make_cfg(12, 8000, ms, variant=binding.VMS_VARIANT_FINE, table_place=pl, **big))
        lds.append(r.lds_bytes()[1])
        r.close()
    assert lds[0] - lds[1] == place * (2048 + 80) * 2
    gpu_util.assert_parity(ev, gpu_util.make_cfg(12, 8000, ms, **dict(W, **big)), label="config 3 slice, tables in the workspace")
    for seed, threshold in ((5, 128), (6, 32)):
        ev, ms = tg.generate(3, n_traces=8, n_events=8000, seed=seed)
        cfg = gpu_util.make_cfg(8, 8000, ms, max_free_blocks=64, max_pblocks=8192, max_sblocks=4352, max_runs=1 << 18,
                                max_chunks=16384, spool_threshold=threshold, **W)
        gpu_util.assert_parity(ev, cfg, label="largest tables in the workspace, threshold %d" % threshold)
    ev, ms = tg.generate(2, n_traces=16, n_events=5000)
    gpu_util.assert_parity(ev, gpu_util.make_cfg(16, 5000, ms, max_runs=600, spool_threshold=40, max_sblocks=128, **W),
                           label="tables in the workspace, small arena")
    ev, ms = tg.generate(4, n_traces=6, n_events=4000)
    gpu_util.assert_parity(ev, gpu_util.make_cfg(6, 4000, ms, max_runs=20000, max_chunks=32768, **W),
                           label="tables in the workspace, slot table in LDS")
    ev, ms = tg.generate(1, n_traces=5, n_events=900, seed=44)
    gpu_util.assert_parity(ev, gpu_util.make_cfg(5, 900, ms, **W), n_events=np.array([0, 1, 63, 500, 900], dtype=np.uint32),
                           label="tables in the workspace, ragged")
    # 32-bit chunk numbers keep their tables in LDS: asking for the workspace is refused
    with pytest.raises(binding.VmsError):
        binding.Replay(gpu_util.make_cfg(5, 900, ms, max_chunks=70000, **W))


def test_lists_are_compacted_under_a_slot_table_in_lds():
    # LoRA-type traces (650 slots: the slot table lives in LDS and keeps list places in halfwords), a
    # StitchFree threshold of 16 and a small arena: each trace stitches 220 to 550 sBlocks, more granules
    # one after the other than the arena has, so the lists are squeezed together several times and the
    # slots learn the new places; a trace that outgrows the arena all the same goes to the second pass
    ev, ms = tg.generate(4, n_traces=24, n_events=14000, seed=3)
    assert ms > 64
    for place in (binding.VMS_TABLES_LDS, binding.VMS_TABLES_WORKSPACE_ALL):
        cfg = gpu_util.make_cfg(24, 14000, ms, policy_mask=2, variant=binding.VMS_VARIANT_FINE, table_place=place, spool_threshold=16,
                                max_pblocks=1024, max_sblocks=128, max_runs=700, max_chunks=20480, retry_traces=24)
        st = gpu_util.assert_parity(ev, cfg, label="compaction, slot table in LDS, tables %d" % place)
        assert st["n_sblock_created"][1].min() > 200 and st["n_sblock_evicted"][1].min() > 100


def test_second_pass_replays_traces_that_outgrow_the_tables():
    # 40 transformer traces, three of them replaced by random traces whose many requests below one
    # chunk outgrow the table of the stitching policy's small-request pool: without a second pass those
    # three are flagged; with one they are replayed in full with doubled tables inside the same
    # vms_replay_run, and everything matches the oracle
    ev, ms = tg.generate(2, n_traces=40, n_events=2000, seed=17)
    rnd, ms1 = tg.generate(1, n_traces=3, n_events=2000, seed=18)
    slots = max(ms, ms1)
    for i, t in enumerate((5, 22, 39)):
        ev[t] = rnd[i]
    for variant in (binding.VMS_VARIANT_FLAT, binding.VMS_VARIANT_FINE):
        small = dict(variant=variant, max_free_blocks=128, max_small_blocks=32, max_pblocks=256, max_sblocks=560,
                     max_runs=1200, max_chunks=4096)
        _, _, st = gpu_util.gpu_replay(ev, gpu_util.make_cfg(40, 2000, slots, **small))
        bad = np.flatnonzero((st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any(axis=0))
        assert bad.tolist() == [5, 22, 39] and not (st["status"][0] & binding.VMS_ST_TABLE_OVERFLOW).any()
        gpu_util.assert_parity(ev, gpu_util.make_cfg(40, 2000, slots, retry_traces=4, **small), label="second pass, variant %d" % variant)
        # fewer wavefronts in the second pass than flagged traces: they share the three out
        for waves in (1, 2):
            gpu_util.assert_parity(ev, gpu_util.make_cfg(40, 2000, slots, retry_traces=waves, **small),
                                   label="second pass of %d wavefronts, variant %d" % (waves, variant))
    # the splitting policy's pool too small for most traces (in LDS, then in registers): all replayed again
    for free in (100, 300):
        cfg = gpu_util.make_cfg(40, 2000, slots, max_free_blocks=free // 3 if free == 300 else free, retry_traces=40, policy_mask=1)
        gpu_util.assert_parity(ev, cfg, label="second pass, splitting pool of %d" % cfg.max_free_blocks)
