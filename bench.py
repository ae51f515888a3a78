#!/usr/bin/env python3
"""Benchmark: allocator events replayed per second (splitting + stitching policies) on one MI355X.

A step is one vms_replay_run over the whole workload: every trace replayed under both
policies, events resident in HBM, decision words and statistics written to HBM.
Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
BYTES_PER_EVENT_PER_KERNEL = 16       # 8 B event word read + 8 B decision word written


def recorded_traffic(config):
    """HBM bytes per launch of the stitching kernel from the committed rocprofv3 counter summary,
    or None when there is none for this workload or the kernel sources changed since it was taken."""
    import hashlib
    if config != 2:
        return None
    path = os.path.join(ROOT, "profiles", "replay_kernels_config2_hbm_traffic.txt")
    csrc = os.path.join(ROOT, "paper_2401_08156_amd", "csrc")
    try:
        h = hashlib.sha256()
        for f in ("replay_kernels.hpp", "vms_replay.hip", "wave_ops.hpp"):      # the replay kernels and their launches
            h.update(open(os.path.join(csrc, f), "rb").read())
        fields = dict(l.split(":", 1) for l in open(path).read().splitlines() if l.startswith("traffic_"))
        if fields["traffic_source_hash"].strip() != h.hexdigest()[:16]:
            return None
        return int(fields["traffic_bytes_stitching_kernel"])
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(events, cfg_kw, max_slots, sample_traces):
    """The oracle, as it stands, on a bounded sample of the same workload, all host cores."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    ev = events[:sample_traces]
    P = oracle.make_params(max_slots, **cfg_kw)
    t0 = time.perf_counter()
    for pol in (oracle.SPLIT, oracle.VMS):
        oracle.replay(ev, P, pol, want_decisions=True, threads=cores)
    dt = time.perf_counter() - t0
    # the same on one core, over a share of the sample that takes about as long
    one = ev[:max(1, ev.shape[0] // max(cores, 1))]
    t0 = time.perf_counter()
    for pol in (oracle.SPLIT, oracle.VMS):
        oracle.replay(one, P, pol, want_decisions=True, threads=1)
    dt_one = time.perf_counter() - t0
    return dict(value=ev.size / dt, unit="events/s", cores=min(cores, sample_traces), kind="oracle",
                sample="%d of %d traces x %d events, both policies, decisions written" % (
                    ev.shape[0], events.shape[0], ev.shape[1]),
                one_core_value=one.size / dt_one, one_core_sample="%d traces" % one.shape[0])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload (default: config 2, the transformer step with recomputation)")
    ap.add_argument("--traces", type=int, default=None)
    ap.add_argument("--events", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=1024, help="traces the oracle is timed on (the default workload has 1,024: all of it)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the replay engine runs on one GPU only (traces are independent and would shard "
              "by trace index); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2401_08156_amd import binding, workloads
    from paper_2401_08156_amd import tracegen as tg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")

    base = tg.CONFIGS[args.config]
    n_traces = args.traces or base["n_traces"]
    n_events = args.events or base["n_events"]
    # config 5 is replayed as three batches (one per generator kind, each with its own table sizes);
    # every other config is one batch
    kinds = [2, 3, 4] if args.config == 5 else [None]
    batches = []
    for b, kind in enumerate(kinds):
        nt = len(range(b, n_traces, len(kinds)))
        events, max_slots = tg.generate(args.config, n_traces=nt, n_events=n_events, first_trace=b,
                                        trace_stride=len(kinds), threads=16)
        cfg = workloads.make_config(binding, args.config, nt, n_events, max_slots, kind=kind)
        d_events = torch.from_numpy(events.view(np.int64)).to(dev)
        batches.append(dict(events=events, max_slots=max_slots, cfg=cfg, d_events=d_events,
                            d_split=torch.empty_like(d_events), d_vms=torch.empty_like(d_events),
                            rep=binding.Replay(cfg)))
    stream = torch.cuda.current_stream(dev)

    def step(acc=None):
        for bt in batches:
            bt["rep"].run(bt["d_events"], None, bt["d_split"], bt["d_vms"], stream)
            if acc is not None:
                # HIP events recorded by the library on this stream around each kernel; reading them
                # waits for the batch, which is also what serialises runs on one handle
                ms = bt["rep"].last_kernel_ms()
                for k in acc:
                    acc[k] += ms[k]

    # one plain device-to-device copy of known size (the event array): the reference the HBM
    # traffic counters of a profiled run are scaled by
    batches[0]["d_split"].copy_(batches[0]["d_events"])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms = dict(split=0.0, vms=0.0, total=0.0)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(kernel_ms)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    for k in kernel_ms:
        kernel_ms[k] /= max(args.steps, 1)

    rep, cfg, events, max_slots = batches[0]["rep"], batches[0]["cfg"], batches[0]["events"], batches[0]["max_slots"]
    st = np.concatenate([bt["rep"].stats() for bt in batches], axis=1)
    summ = rep.summary()
    flagged = int((st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any(axis=0).sum())
    if flagged:
        names = dict(free_blocks=binding.VMS_ST_OVF_FREE_BLOCKS, pblocks=binding.VMS_ST_OVF_PBLOCKS,
                     sblocks=binding.VMS_ST_OVF_SBLOCKS, runs=binding.VMS_ST_OVF_RUNS,
                     chunks=binding.VMS_ST_OVF_CHUNKS)
        for bt, kind in zip(batches, kinds):
            s = bt["rep"].stats()["status"]
            which = {k: int(((s & v) != 0).any(axis=0).sum()) for k, v in names.items()}
            high = {k: int(bt["rep"].stats()["max_" + k].max()) for k in names if k != "chunks"}
            print("bench.py: batch %s: traces over a table: %s; high-water marks reached: %s" % (kind, which, high),
                  file=sys.stderr)
        print("bench.py: engine tables overflowed; the measurement is invalid", file=sys.stderr)
        sys.exit(1)

    total_events = n_traces * n_events
    ms_per_step = dt / args.steps * 1e3
    dom = "vms" if kernel_ms["vms"] >= kernel_ms["split"] else "split"
    algo_bytes = BYTES_PER_EVENT_PER_KERNEL * total_events
    achieved = algo_bytes / (kernel_ms[dom] * 1e-3) / 1e9
    lds = rep.lds_bytes()
    out = {
        "metric": "allocator events replayed/sec (split + VMS) on 1 MI355X; bit-exact peaks vs oracle",
        "value": total_events / (dt / args.steps),
        "unit": "events/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": workloads.NAMES[args.config], "n_traces": n_traces, "n_events": n_events,
                   "policies": "split+vms", "chunk_bytes": int(cfg.chunk_bytes),
                   "spool_threshold": int(cfg.spool_threshold), "frag_limit_bytes": int(cfg.frag_limit_bytes),
                   "batches": len(batches), "lds_bytes_per_wave": {"split": lds[0], "vms": lds[1]}},
        "policy_events_per_s": 2 * total_events / (dt / args.steps),     # every event is decided under both policies
        "kernel_ms": kernel_ms,
        # one wavefront per (trace, policy); how many fit a compute unit at once is set by their LDS (160 KB per CU)
        "resident_waves_per_cu": {k: min(-(-n_traces // 256), (160 * 1024) // max(b, 1) if b else 32)
                                  for k, b in (("split", lds[0]), ("vms", lds[1]))},
        # a single trace is a single wavefront per policy: a latency figure, not a throughput
        "ns_per_event": ms_per_step * 1e6 / n_events if n_traces == 1 else None,
        "roofline": {"bound": "hbm", "kernel": "replay_vms_kernel (stitching policy)" if dom == "vms" else "replay_split_kernel (splitting policy)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": recorded_traffic(args.config) if dom == "vms" and n_traces == base["n_traces"]
                     and n_events == base["n_events"] else None,
                     "note": "latency/issue-bound serial state machine per trace; algorithmic bytes = 16 B per event "
                             "(8 B event read + 8 B decision written) x events per launch"},
        "table_high_water": {k: int(st[k].max()) for k in ("max_free_blocks", "max_pblocks", "max_sblocks", "max_runs",
                                                            "max_members")},
        "results": {"mean_fragmentation_split": float(st["fragmentation"][0].mean()),
                    "mean_fragmentation_vms": float(st["fragmentation"][1].mean()),
                    "mem_reduction_ratio_first_batch": summ.mem_reduction_ratio},
    }
    if not args.no_cpu_baseline:
        kw = dict(capacity_bytes=int(cfg.capacity_bytes), spool_threshold=int(cfg.spool_threshold),
                  frag_limit_bytes=int(cfg.frag_limit_bytes), small_limit_bytes=int(cfg.small_limit_bytes),
                  chunk_bytes=int(cfg.chunk_bytes))
        out["cpu_baseline"] = cpu_baseline(events, kw, max_slots, min(args.cpu_sample, n_traces))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
