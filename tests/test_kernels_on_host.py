"""The replay kernels compiled for the host (tests/emu: 64 lanes as cooperative fibers, guard bands
around the LDS and every buffer) against the oracle: finds wrong indexing and wrong decisions
without a GPU.  The lanes run one after another between wave-wide operations, so what this checks
is the kernels' logic and memory accesses, not their timing; the GPU parity tests remain the
proof for the device."""
import glob
import os

import numpy as np
import pytest

import emu
import gpu_util
import oracle
from paper_2401_08156_amd import binding
from paper_2401_08156_amd import tracegen as tg
from test_oracle_examples import GOLDEN, load_fixture

MiB = 1 << 20


def check(ev, cfg, n_events=None, label=""):
    ds, dv, st = emu.replay(ev, cfg, binding.STATS_DTYPE, n_events)
    P = gpu_util.oracle_params(cfg)
    for pol, gdec in ((0, ds), (1, dv)):
        if not (cfg.policy_mask & (1 << pol)):
            continue
        odec, ost = oracle.replay(ev, P, pol, n_events=n_events, threads=8)
        gst = st[pol]
        assert not (gst["status"] & binding.VMS_ST_TABLE_OVERFLOW).any(), (label, pol, gst["status"], gst["overflow_event"])
        valid = np.ones(ev.shape, dtype=bool) if n_events is None else np.arange(ev.shape[1])[None, :] < np.asarray(n_events)[:, None]
        same = (gdec == odec) | ~valid
        if not same.all():
            t, i = np.argwhere(~same)[0]
            raise AssertionError("%s policy %d trace %d event %d: kernel %#x oracle %#x" % (label, pol, t, i, int(gdec[t, i]), int(odec[t, i])))
        assert np.all(gdec[~valid] == np.uint64(0xFFFFFFFFFFFFFFFF)), "wrote past the end of a trace"
        for f in gpu_util.COMPARED_FIELDS:
            assert np.array_equal(gst[f], ost[f]), (label, pol, f, gst[f], ost[f])
    return st


def test_wave_primitives_on_host_lanes():
    assert emu.lib().emu_selftest() == 0


def test_worked_examples_fine_grained_variant():
    for path in sorted(glob.glob(os.path.join(GOLDEN, "*.txt"))):
        fx = load_fixture(path)
        ev = fx["events"][None, :]
        kw = dict(spool_threshold=int(fx["spool_threshold"])) if "spool_threshold" in fx else {}
        for place in (binding.VMS_TABLES_LDS, binding.VMS_TABLES_WORKSPACE, binding.VMS_TABLES_WORKSPACE_ALL):
            cfg = gpu_util.make_cfg(1, ev.shape[1], 16, variant=binding.VMS_VARIANT_FINE, table_place=place, policy_mask=2, **kw)
            check(ev, cfg, label=os.path.basename(path))


def test_splitting_kernels():
    ev, ms = tg.generate(1, n_traces=2, n_events=1500)
    check(ev, gpu_util.make_cfg(2, 1500, ms, policy_mask=1), label="pool in LDS")
    check(ev, gpu_util.make_cfg(2, 1500, ms, policy_mask=1, max_free_blocks=150), label="pool in registers")
    check(ev, gpu_util.make_cfg(2, 1500, ms, policy_mask=1, max_free_blocks=300), label="pool in five registers per lane")
    ev, ms = tg.generate(4, n_traces=1, n_events=2000)
    check(ev, gpu_util.make_cfg(1, 2000, ms, policy_mask=1), label="slot table in LDS")
    check(ev, gpu_util.make_cfg(1, 2000, ms, policy_mask=1, max_free_blocks=320), label="slot table in LDS, pool in five registers per lane")
    ev, ms = tg.generate(3, n_traces=1, n_events=2000)
    assert ms <= 64
    check(ev, gpu_util.make_cfg(1, 2000, ms, policy_mask=1, max_free_blocks=320), label="slot table and pool (five per lane) in registers")


@pytest.mark.parametrize("kind,nt,ne,tables", [
    (1, 2, 2000, dict(max_runs=20000)),
    (2, 2, 3000, dict(max_runs=20000)),
    (3, 2, 4000, dict(max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=16384)),
    (3, 2, 3000, dict(max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=16384, spool_threshold=32)),
    (4, 1, 3000, dict(max_runs=20000, max_chunks=32768)),                       # slot table in LDS
    (1, 1, 1500, dict(max_runs=20000, max_chunks=70000)),                       # 32-bit chunk numbers
    (2, 1, 3000, dict(variant=2, max_runs=600, spool_threshold=40, max_sblocks=128)),   # small arena: lists are squeezed
    (1, 2, 1200, dict(variant=2, frag_limit_bytes=8 * MiB, small_limit_bytes=512)),
    (1, 2, 1200, dict(variant=2, capacity_bytes=256 * MiB)),
])
def test_fine_grained_variant(kind, nt, ne, tables):
    # the witness and list-place tables of the sBlocks in LDS, then in the workspace (16-bit chunk numbers only)
    ev, ms = tg.generate(kind, n_traces=nt, n_events=ne, seed=7 + kind)
    for place in (binding.VMS_TABLES_LDS, binding.VMS_TABLES_WORKSPACE, binding.VMS_TABLES_WORKSPACE_ALL):
        if place != binding.VMS_TABLES_LDS and tables.get("max_chunks", 0) > 63000:
            continue
        cfg = gpu_util.make_cfg(nt, ne, ms, policy_mask=2, **dict(dict(variant=2), table_place=place, **tables))
        check(ev, cfg, label="generator %d %s tables %d" % (kind, tables, place))


def test_ragged_traces_and_nothing_written_past_the_end():
    ev, ms = tg.generate(1, n_traces=3, n_events=700, seed=11)
    check(ev, gpu_util.make_cfg(3, 700, ms, max_runs=20000), n_events=np.array([0, 333, 700], dtype=np.uint32), label="ragged")


def test_second_pass_replays_traces_that_outgrow_the_tables():
    # tables far too small for the first trace's pools (the other two fit): flagged without a second
    # pass, replayed in full with doubled tables with one.  (The flat stitching kernel as first pass is
    # covered on the GPU: its sources carry no lane-switch marks for this host build.)
    ev, ms = tg.generate(1, n_traces=3, n_events=900, seed=13)
    ev[1:, 60:] = ev[1:, :1] * 0 + tg.make_events([("A", 0, 2 * MiB), ("F", 0)] * 420)[None, :]
    for variant in (binding.VMS_VARIANT_FINE,):
        small = dict(variant=variant, max_free_blocks=24, max_pblocks=40, max_sblocks=560, max_runs=900, max_chunks=8192)
        _, _, st = emu.replay(ev, gpu_util.make_cfg(3, 900, ms, **small), binding.STATS_DTYPE)
        assert (st["status"][:, 0] & binding.VMS_ST_TABLE_OVERFLOW).all() and not (st["status"][:, 1:] & binding.VMS_ST_TABLE_OVERFLOW).any()
        check(ev, gpu_util.make_cfg(3, 900, ms, retry_traces=2, **small), label="second pass, first pass variant %d" % variant)
        # both passes with the sBlock tables in the workspace
        check(ev, gpu_util.make_cfg(3, 900, ms, retry_traces=2, table_place=binding.VMS_TABLES_WORKSPACE_ALL, **small),
              label="second pass, tables in the workspace")
    # more such traces than the second pass has wavefronts: one wavefront replays all three in turn
    ev, ms = tg.generate(1, n_traces=3, n_events=900, seed=13)
    cfg = gpu_util.make_cfg(3, 900, ms, policy_mask=2, variant=2, max_pblocks=40, max_sblocks=560)
    _, _, st = emu.replay(ev, cfg, binding.STATS_DTYPE)
    assert ((st["status"][1] & binding.VMS_ST_TABLE_OVERFLOW) != 0).sum() == 3
    check(ev, gpu_util.make_cfg(3, 900, ms, retry_traces=1, variant=2, max_pblocks=40, max_sblocks=560), label="second pass of one wavefront")
    # 70 traces, every third flagged: the wavefronts take their trace numbers 64 at a time
    ev, ms = tg.generate(1, n_traces=70, n_events=300, seed=21)
    ev[np.arange(70) % 3 != 0, 10:] = tg.make_events([("A", 0, 2 * MiB), ("F", 0)] * 145)[None, :]
    small = dict(variant=2, max_free_blocks=24, max_pblocks=24, max_sblocks=560, max_runs=900, max_chunks=8192)
    _, _, st = emu.replay(ev, gpu_util.make_cfg(70, 300, ms, **small), binding.STATS_DTYPE)
    assert 10 < (st["status"] & binding.VMS_ST_TABLE_OVERFLOW != 0).any(axis=0).sum() <= 24
    check(ev, gpu_util.make_cfg(70, 300, ms, retry_traces=3, **small), label="second pass over 70 traces")


def test_lists_are_compacted_under_a_slot_table_in_lds():
    # 650 slots (in LDS: list places are halfwords there), a StitchFree threshold of 16 and an arena
    # of 290 granules: the 408 sBlocks this trace stitches take more granules than that one after the
    # other, so their lists are squeezed together several times and the slots that hold one learn
    # its new place; every later FREE of such a slot must still find the right list
    ev, ms = tg.generate(4, n_traces=1, n_events=14000, seed=3)
    assert ms > 64
    for place in (binding.VMS_TABLES_LDS, binding.VMS_TABLES_WORKSPACE_ALL):
        cfg = gpu_util.make_cfg(1, 14000, ms, policy_mask=2, variant=binding.VMS_VARIANT_FINE, table_place=place, spool_threshold=16,
                                max_pblocks=1024, max_sblocks=92, max_runs=700, max_chunks=20480)
        st = check(ev, cfg, label="compaction, slot table in LDS, tables %d" % place)
        assert st["n_sblock_created"][1, 0] > 400 and st["n_sblock_evicted"][1, 0] > 300


def test_table_overflow_is_flagged_not_fatal():
    ev, ms = tg.generate(3, n_traces=1, n_events=2500, seed=5)
    cfg = gpu_util.make_cfg(1, 2500, ms, policy_mask=2, variant=2, max_pblocks=64, max_sblocks=520, max_chunks=4096)
    _, _, st = emu.replay(ev, cfg, binding.STATS_DTYPE)
    assert st["status"][1, 0] & binding.VMS_ST_TABLE_OVERFLOW and st["overflow_event"][1, 0] < 2500
