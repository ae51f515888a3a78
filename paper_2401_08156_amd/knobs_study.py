"""The robustness knobs of the stitching allocator (Sec. 4.2.3) and its convergence (Sec. 4.2.2,
Sec. 5.5) on the synthetic workloads, replayed on the GPU:

  * fragmentation limit: blocks below it are neither split nor stitched;
  * StitchFree threshold: how many stitched blocks stay cached;
  * convergence: on a strictly periodic trace, the event after which every request is an exact
    hit (state S1), in training steps.

    python -m paper_2401_08156_amd.knobs_study [--traces 64] [--json]
"""
import argparse
import json

import numpy as np

from . import binding, workloads
from . import tracegen as tg

MiB = 1 << 20
EVENTS_PER_STEP = {2: 448, 3: 560, 4: 1472}        # base events of one training step of each recipe


def replay(config, n_traces, n_events=None, **overrides):
    import torch
    base = config % 10
    n_events = n_events or tg.CONFIGS[config]["n_events"]
    ev, max_slots = tg.generate(config, n_traces=n_traces, n_events=n_events, threads=16)
    # roomy engine tables: the knobs change how many blocks and chunks a trace needs
    roomy = dict(max_pblocks=2048, max_sblocks=1024, max_runs=16000, max_chunks=32768, max_free_blocks=1024)
    cfg = workloads.make_config(binding, config, n_traces, n_events, max_slots, **dict(roomy, **overrides))
    d = torch.from_numpy(ev.view(np.int64)).cuda()
    ds, dv = torch.empty_like(d), torch.empty_like(d)
    r = binding.Replay(cfg)
    r.run(d, None, ds, dv)
    st = r.stats()
    dec = dv.cpu().numpy().view(np.uint64)
    r.close()
    if (st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any():
        raise RuntimeError("engine tables too small for config %d with %s" % (config, overrides))
    code = (dec & np.uint64(15)).astype(np.int64)
    is_alloc = (ev & np.uint64(1 << 31)) == 0
    n_alloc = is_alloc.sum()
    out = dict(config=config, base=base, n_traces=n_traces, n_events=n_events, **{k: int(v) for k, v in overrides.items()})
    out["frag_split"] = float(st["fragmentation"][0].mean())
    out["frag_vms"] = float(st["fragmentation"][1].mean())
    res = st["peak_reserved"].sum(axis=1).astype(float)
    out["mem_reduction_ratio"] = float((res[0] - res[1]) / res[0])
    out["s1_share"] = float((is_alloc & (code == 1)).sum() / n_alloc)
    out["stitch_share"] = float((is_alloc & (code == 3)).sum() / n_alloc)
    out["evicted_per_trace"] = float(st["n_sblock_evicted"][1].mean())
    # convergence: the last request that was not an exact hit, in steps
    not_s1 = is_alloc & (code != 1)
    last = np.array([np.flatnonzero(row).max() if row.any() else -1 for row in not_s1])
    out["last_non_s1_event_max"] = int(last.max())
    out["steps_to_converge_max"] = float((last.max() + 1) / EVENTS_PER_STEP.get(base, 1))
    return out


def study(n_traces=64):
    rows = []
    for config in (2, 4):
        n_events = 20000
        for limit in (2, 8, 32, 128):
            rows.append(dict(knob="frag_limit", **replay(config, n_traces, n_events, frag_limit_bytes=limit * MiB)))
        for thr in (64, 128, 256, 512):
            rows.append(dict(knob="spool_threshold", **replay(config, n_traces, n_events, spool_threshold=thr)))
    for config in (12, 14):
        rows.append(dict(knob="periodic", **replay(config, n_traces, 20000)))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--traces", type=int, default=64)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    rows = study(args.traces)
    if args.json:
        print(json.dumps(rows))
        return
    print("%-16s %4s %10s %10s %10s %8s %8s %9s %9s %10s" % ("knob", "cfg", "value", "frag split", "frag vms", "MRR", "S1", "stitch", "evicted", "conv steps"))
    for r in rows:
        val = r.get("frag_limit_bytes", 0) // MiB if r["knob"] == "frag_limit" else r.get("spool_threshold", "")
        print("%-16s %4d %10s %10.4f %10.4f %8.4f %8.4f %9.4f %9.1f %10.1f" % (
            r["knob"], r["config"], val, r["frag_split"], r["frag_vms"], r["mem_reduction_ratio"], r["s1_share"],
            r["stitch_share"], r["evicted_per_trace"], r["steps_to_converge_max"]))


if __name__ == "__main__":
    main()
