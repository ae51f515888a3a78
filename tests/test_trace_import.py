"""Recorded allocation streams -> event words (host logic only; the replay itself is covered elsewhere)."""
import numpy as np

import oracle
from paper_2401_08156_amd import trace_import as ti
from paper_2401_08156_amd import tracegen as tg

MiB = 1 << 20


def test_records_become_the_same_events_as_a_hand_written_trace():
    recs = [("alloc", "a", 4 * MiB), ("alloc", "b", 2 * MiB), ("free", "a"), ("free", "b"), ("alloc", "c", 6 * MiB)]
    ev, max_slots, dropped = ti.events_from_records(recs)
    want = tg.make_events([("A", 0, 4 * MiB), ("A", 1, 2 * MiB), ("F", 0), ("F", 1), ("A", 0, 6 * MiB)])
    assert np.array_equal(ev, want) and max_slots == 2 and not any(dropped.values())
    # Fig. 1 of the paper: the splitting allocator has to reserve 12 MiB, stitching serves it from 6 MiB
    P = oracle.make_params(max_slots)
    _, st = oracle.replay(ev[None, :], P, oracle.SPLIT)
    assert st["peak_reserved"][0] == 12 * MiB
    _, st = oracle.replay(ev[None, :], P, oracle.VMS)
    assert st["peak_reserved"][0] == 6 * MiB and st["fragmentation"][0] == 0.0


def test_lowest_free_slot_and_rounding():
    recs = [("alloc", 10, 1), ("alloc", 11, 513), ("alloc", 12, 512), ("free", 10), ("free", 11),
            ("alloc", 13, 100), ("alloc", 14, 100), ("alloc", 15, 100)]
    ev, max_slots, _ = ti.events_from_records(recs)
    slots = (ev >> np.uint64(32)).tolist()
    assert slots == [0, 1, 2, 0, 1, 0, 1, 3] and max_slots == 4
    sizes = (ev & np.uint64(0x7FFFFFFF)).tolist()
    assert sizes[:3] == [1, 2, 1]                       # 512-byte units, rounded up
    assert [int(e >> np.uint64(31)) & 1 for e in ev] == [0, 0, 0, 1, 1, 0, 0, 0]


def test_unreplayable_records_are_counted_not_emitted():
    recs = [("free", "ghost"), ("alloc", "x", 0), ("alloc", "x", 1024), ("alloc", "x", 2048), ("free", "x"),
            ("free", "x"), ("alloc", "big", 1 << 41)]
    ev, max_slots, dropped = ti.events_from_records(recs)
    assert len(ev) == 2 and max_slots == 1
    assert dropped == dict(free_unknown=2, alloc_live_key=1, alloc_empty=1, alloc_too_large=1)
    # what is emitted is always a well-formed trace: the oracle sees no invalid event
    _, st = oracle.replay(ev[None, :], oracle.make_params(max_slots), oracle.VMS)
    assert st["status"][0] == 0


def test_text_round_trip(tmp_path):
    recs = [("alloc", "0x7f00", 4096), ("alloc", "0x7f10", 3 * MiB), ("free", "0x7f00"), ("free", "0x7f10")]
    p = tmp_path / "trace.txt"
    ti.records_to_text(recs, str(p))
    p.write_text("# a comment\n" + p.read_text() + "\n   \nalloc t 7 # trailing\n")
    back = ti.records_from_text(str(p))
    assert back == recs + [("alloc", "t", 7)]


def test_torch_snapshot_layouts():
    new = {"device_traces": [[
        {"action": "segment_alloc", "addr": 4096, "size": 2 * MiB, "stream": 0},
        {"action": "alloc", "addr": 4096, "size": 1024, "stream": 0},
        {"action": "alloc", "addr": 8192, "size": 512, "stream": 0},
        {"action": "free_requested", "addr": 4096, "size": 1024, "stream": 0},
        {"action": "free_completed", "addr": 4096, "size": 1024, "stream": 0},
        {"action": "alloc", "addr": 4096, "size": 2048, "stream": 0},
    ], []]}
    recs = ti.records_from_torch_snapshot(new, 0)
    assert recs == [("alloc", 4096, 1024), ("alloc", 8192, 512), ("free", 4096), ("alloc", 4096, 2048)]
    assert ti.records_from_torch_snapshot(new, 1) == []
    old = {"device_traces": [[
        {"action": "alloc", "addr": 1, "size": 600},
        {"action": "free", "addr": 1, "size": 600},
    ]]}
    assert ti.records_from_torch_snapshot(old) == [("alloc", 1, 600), ("free", 1)]
    ev, max_slots, dropped = ti.events_from_records(recs)
    assert len(ev) == 4 and max_slots == 2 and not any(dropped.values())
