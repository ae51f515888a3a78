"""Fragmentation against the number of data-parallel devices (Sec. 2.4 Observation 2, Sec. 5.3.2):
one rank of ZeRO-3 + LoRA + recomputation over 1, 2, 4, 8, 16 devices, replayed on the GPU under
both allocators.  Parameter, gradient and optimizer-state shards shrink with the device count while
full-size gathered weights come and go between the activations.

    python -m paper_2401_08156_amd.scaleout_study [--traces 64] [--json]
"""
import argparse
import json

import numpy as np

from . import binding, workloads
from . import tracegen as tg

WORLD_SIZES = (1, 2, 4, 8, 16)          # generator: trace t is a rank of a job on 2^(t mod 5) devices
GiB = float(1 << 30)


def replay(world_index, n_traces, n_events):
    import torch
    ev, max_slots = tg.generate(6, n_traces=n_traces, n_events=n_events, first_trace=world_index,
                                trace_stride=len(WORLD_SIZES), threads=16)
    cfg = workloads.make_config(binding, 6, n_traces, n_events, max_slots)
    d = torch.from_numpy(ev.view(np.int64)).cuda()
    r = binding.Replay(cfg)
    r.run(d, None, None, None)
    st = r.stats()
    r.close()
    if (st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any():
        raise RuntimeError("engine tables too small")
    res = st["peak_reserved"].sum(axis=1).astype(float)
    return dict(devices=WORLD_SIZES[world_index], n_traces=n_traces, n_events=n_events,
                frag_split=float(st["fragmentation"][0].mean()), frag_vms=float(st["fragmentation"][1].mean()),
                util_split=float(1 - st["fragmentation"][0].mean()), util_vms=float(1 - st["fragmentation"][1].mean()),
                reserved_split_gib=float(st["peak_reserved"][0].mean() / GiB),
                reserved_vms_gib=float(st["peak_reserved"][1].mean() / GiB),
                active_gib=float(st["peak_active"][1].mean() / GiB),
                mem_reduction_ratio=float((res[0] - res[1]) / res[0]))


def study(n_traces=64, n_events=20000):
    return [replay(k, n_traces, n_events) for k in range(len(WORLD_SIZES))]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--traces", type=int, default=64, help="traces per device count")
    ap.add_argument("--events", type=int, default=20000)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    rows = study(args.traces, args.events)
    if args.json:
        print(json.dumps(rows))
        return
    print("%8s %11s %11s %14s %14s %8s" % ("devices", "util split", "util vms", "reserved split", "reserved vms", "MRR"))
    for r in rows:
        print("%8d %11.4f %11.4f %10.2f GiB %10.2f GiB %8.4f" % (
            r["devices"], r["util_split"], r["util_vms"], r["reserved_split_gib"], r["reserved_vms_gib"],
            r["mem_reduction_ratio"]))


if __name__ == "__main__":
    main()
