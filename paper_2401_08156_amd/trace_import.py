"""Recorded allocation streams as replay input (Sec. 2.4 and Sec. 5 of the paper work from the
alloc / free streams of real fine-tuning runs; this turns such a recording into the engine's event
words).

A recording is a sequence of records ("alloc", key, bytes) / ("free", key), where `key` is anything
hashable that names a live allocation (an address, a tensor id).  Sources:

* `records_from_torch_snapshot(torch.cuda.memory._snapshot())` - the allocator history PyTorch keeps
  after `torch.cuda.memory._record_memory_history()`; no files are read;
* `records_from_text(path)` - one record per line: `alloc <key> <bytes>` or `free <key>`
  (`#` starts a comment);
* `record_torch_loop(fn)` - runs `fn()` on the GPU with PyTorch's history recording switched on.

`events_from_records` binds every allocation to the lowest free slot, as the synthetic generators
do, and returns the event array and the number of slots.  Frees of unknown keys and a second alloc
of a live key cannot be replayed and are counted, not emitted.

    python -m paper_2401_08156_amd.trace_import --text trace.txt     # replay a text recording
    python -m paper_2401_08156_amd.trace_import --record             # record a small PyTorch loop, replay it
"""
import argparse
import heapq
import json

import numpy as np

UNIT = 512
KIND_FREE = 1 << 31
MAX_UNITS = (1 << 31) - 1


def events_from_records(records):
    """-> (events uint64[n], max_slots, dropped) for an iterable of ("alloc", key, bytes) / ("free", key)."""
    slot_of = {}
    free_slots = []            # heap of released slot numbers
    next_slot = 0
    ev = []
    dropped = dict(free_unknown=0, alloc_live_key=0, alloc_empty=0, alloc_too_large=0)
    for rec in records:
        kind, key = rec[0], rec[1]
        if kind == "alloc":
            units = (int(rec[2]) + UNIT - 1) // UNIT
            if units == 0:
                dropped["alloc_empty"] += 1
            elif units > MAX_UNITS:
                dropped["alloc_too_large"] += 1
            elif key in slot_of:
                dropped["alloc_live_key"] += 1
            else:
                if free_slots:
                    slot = heapq.heappop(free_slots)
                else:
                    slot = next_slot
                    next_slot += 1
                slot_of[key] = slot
                ev.append((slot << 32) | units)
        elif kind == "free":
            slot = slot_of.pop(key, None)
            if slot is None:
                dropped["free_unknown"] += 1
            else:
                heapq.heappush(free_slots, slot)
                ev.append((slot << 32) | KIND_FREE)
        else:
            raise ValueError("unknown record kind %r" % (kind,))
    return np.array(ev, dtype=np.uint64), max(next_slot, 1), dropped


def records_from_torch_snapshot(snapshot, device=0):
    """Records of one device from the dictionary `torch.cuda.memory._snapshot()` returns.

    Its `device_traces[device]` lists allocator actions in time order; a block is named by its
    address.  `alloc` hands a block out, `free_requested` is the moment the program released it
    (`free_completed` follows once no stream uses it any longer; older versions only have `free`).
    Segment-level actions (the caching allocator's own traffic with the driver) are not requests
    of the program and are skipped."""
    trace = snapshot["device_traces"][device]
    has_requested = any(t["action"] == "free_requested" for t in trace)
    release = "free_requested" if has_requested else "free"
    out = []
    for t in trace:
        a = t["action"]
        if a == "alloc":
            out.append(("alloc", int(t["addr"]), int(t["size"])))
        elif a == release:
            out.append(("free", int(t["addr"])))
    return out


def records_from_text(path):
    out = []
    with open(path) as f:
        for n, line in enumerate(f, 1):
            line = line.split("#", 1)[0].split()
            if not line:
                continue
            if line[0] == "alloc" and len(line) == 3:
                out.append(("alloc", line[1], int(line[2])))
            elif line[0] == "free" and len(line) == 2:
                out.append(("free", line[1]))
            else:
                raise ValueError("%s:%d: expected 'alloc <key> <bytes>' or 'free <key>'" % (path, n))
    return out


def records_to_text(records, path):
    with open(path, "w") as f:
        for r in records:
            f.write("alloc %s %d\n" % (r[1], r[2]) if r[0] == "alloc" else "free %s\n" % (r[1],))


def record_torch_loop(fn, device=0, max_entries=1 << 22):
    """Run fn() with PyTorch's allocator history on; -> (records, PyTorch's own peaks during fn)."""
    import torch
    torch.cuda.synchronize(device)
    torch.cuda.reset_peak_memory_stats(device)
    base_alloc, base_res = torch.cuda.memory_allocated(device), torch.cuda.memory_reserved(device)
    torch.cuda.memory._record_memory_history(enabled="all", context=None, stacks="python", max_entries=max_entries)
    try:
        fn()
        torch.cuda.synchronize(device)
        snap = torch.cuda.memory._snapshot()
    finally:
        torch.cuda.memory._record_memory_history(enabled=None)
    peaks = dict(allocated_before=base_alloc, reserved_before=base_res,
                 peak_allocated=torch.cuda.max_memory_allocated(device),
                 peak_reserved=torch.cuda.max_memory_reserved(device))
    return records_from_torch_snapshot(snap, device), peaks


def replay(events, max_slots, **overrides):
    """One trace through the replay engine under both policies -> dict of its results."""
    import torch
    from . import binding
    n = int(events.shape[0])
    cfg = binding.vms_config_default(1, max(n, 1), max_slots)
    tables = dict(max_free_blocks=2048, max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=65536)
    for k, v in dict(tables, **overrides).items():
        setattr(cfg, k, v)
    d = torch.from_numpy(np.ascontiguousarray(events).view(np.int64).reshape(1, -1)).cuda()
    r = binding.Replay(cfg)
    r.run(d, None, None, None)
    st = r.stats()
    r.close()
    if (st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any():
        raise RuntimeError("engine tables too small for this recording")
    out = dict(n_events=n, max_slots=max_slots)
    for p, name in ((0, "split"), (1, "vms")):
        s = st[p][0]
        out[name] = dict(peak_requested=int(s["peak_requested"]), peak_active=int(s["peak_active"]),
                         peak_reserved=int(s["peak_reserved"]), fragmentation=float(s["fragmentation"]),
                         n_code=[int(x) for x in s["n_code"]])
    return out


def _demo_loop(steps=12, hidden=1024, layers=6):
    from .torch_plugin import train
    train(steps, hidden, layers)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--text", help="replay a text recording (alloc <key> <bytes> / free <key> per line)")
    ap.add_argument("--record", action="store_true", help="record a small PyTorch training loop on the GPU and replay it")
    ap.add_argument("--save", help="with --record: also write the recording as text")
    args = ap.parse_args()
    if args.record:
        records, peaks = record_torch_loop(_demo_loop)
        if args.save:
            records_to_text(records, args.save)
    elif args.text:
        records, peaks = records_from_text(args.text), None
    else:
        ap.error("one of --text, --record")
    events, max_slots, dropped = events_from_records(records)
    out = replay(events, max_slots)
    out["dropped"] = dropped
    if peaks:
        out["pytorch"] = peaks
    print(json.dumps(out))


if __name__ == "__main__":
    main()
