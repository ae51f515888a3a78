#!/usr/bin/env python3
"""Benchmark: allocator events replayed per second (splitting + stitching policies) on one MI355X.

The workload is the largest one, the mixture of 16,384 traces x 100,000 events with a 288 GiB cap:
trace i comes from generator 2 + i mod 3 (recomputation, offloading, LoRA).  A step is one pass of
the whole hot path over it: every trace replayed under both policies, events resident in HBM,
decision words and statistics written to HBM.  The traces are handed over as three batches, one per
generator kind (each batch has table sizes of its own); a step launches the three batches side by
side on three streams.  After the timed steps one trace's stitching decisions are executed with real HIP
virtual-memory mappings and the call latencies are reported.  Prints one JSON line.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
# A step of the mixture launches on six streams (three batches, two policies each).  The HIP runtime's
# default of four hardware queues makes pairs of streams share a queue, and a kernel then waits behind
# another batch's kernels for no reason of its own (measured: 1,510 ms per step against 1,448 ms).
# Read by the runtime when it starts, so it is set before torch is imported.
if int(os.environ.get("GPU_MAX_HW_QUEUES", "4") or 4) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

HBM_PEAK_GBS = 8000.0
BYTES_PER_EVENT_PER_KERNEL = 16       # 8 B event word read + 8 B decision word written
KERNEL_SOURCES = ("replay_kernels.hpp", "replay_fine.hpp", "replay_plan.hpp", "vms_replay.hip", "wave_ops.hpp", "wave_hw.hpp")
MAPPING_LIMIT = 40000                 # chunk mappings the demo may hold at once (hipMemSetAccess was refused at about 48,000)


def source_hash():
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2401_08156_amd", "csrc")
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def recorded_counters(config):
    """Figures taken from the committed rocprofv3 counter summary of this workload (HBM bytes, LDS
    bytes, instructions and wave occupancy per launch of each kernel), or {} when there is none or
    the kernel sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "replay_kernels_config%d_counters.txt" % config)
    try:
        lines = open(path).read().splitlines()
        fields = dict(l.split(":", 1) for l in lines if l.startswith("counters_"))
        if fields["counters_source_hash"].strip() != source_hash():
            return {}
        return json.loads(fields["counters_json"])
    except (OSError, KeyError, ValueError):
        return {}


VALU_PEAK_GIPS = 256 * 4 * 2.4 / 4        # G wave64 VALU instructions per second: 614.4


def alu_view(c, ms):
    if "valu_instructions" not in c or not ms:
        return None
    a = c["valu_instructions"] / (ms * 1e-3) / 1e9
    return {"achieved": a, "peak": VALU_PEAK_GIPS, "unit": "G wave64 VALU instructions/s", "frac": a / VALU_PEAK_GIPS,
            "all_instructions_per_simd_cycle": c["instructions"] / (ms * 1e-3 * 2.4e9 * 1024)}


def step_alu_view(counters, ms):
    if not counters or not all("valu_instructions" in c for c in counters.values()):
        return None
    valu = sum(c["valu_instructions"] for c in counters.values())
    every = sum(c["instructions"] for c in counters.values())
    a = valu / (ms * 1e-3) / 1e9
    return {"achieved": a, "peak": VALU_PEAK_GIPS, "unit": "G wave64 VALU instructions/s", "frac": a / VALU_PEAK_GIPS,
            "all_instructions_per_simd_cycle": every / (ms * 1e-3 * 2.4e9 * 1024)}


def cpu_baseline(batches, per_kind, max_seconds=40.0):
    """The oracle, as it stands, on a bounded sample of the same workload (the first traces of every
    batch), all host cores, both policies, decisions written."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    events = 0
    t0 = time.perf_counter()
    used = []
    for bt in batches:
        ev = bt["events"][:per_kind]
        cfg = bt["cfg"]
        P = oracle.make_params(bt["max_slots"], capacity_bytes=int(cfg.capacity_bytes), spool_threshold=int(cfg.spool_threshold),
                               frag_limit_bytes=int(cfg.frag_limit_bytes), small_limit_bytes=int(cfg.small_limit_bytes),
                               chunk_bytes=int(cfg.chunk_bytes))
        for pol in (oracle.SPLIT, oracle.VMS):
            oracle.replay(ev, P, pol, want_decisions=True, threads=cores)
        events += ev.size
        used.append(ev.shape[0])
        if time.perf_counter() - t0 > max_seconds:
            break
    dt = time.perf_counter() - t0
    return dict(value=events / dt, unit="events/s", cores=min(cores, max(used)), kind="oracle",
                sample="the first %s traces of the %d batches (of %s), %d events each, both policies, decisions written; %.1f s" % (
                    "/".join(map(str, used)), len(batches), "/".join(str(bt["events"].shape[0]) for bt in batches),
                    batches[0]["events"].shape[1], dt))


def demo_tail(batches, kinds, binding):
    """One trace's stitching decisions executed with real device mappings (hipMemCreate / hipMemMap / ...).
    The trace: the first one, in trace order, that the device can hold: at most MAPPING_LIMIT chunk
    mappings alive at once and at most half of the free HBM."""
    import torch
    free_bytes, _ = torch.cuda.mem_get_info()
    n = len(batches)
    skipped = []
    for i in range(3 * n):                      # trace i of the workload = trace i // n of batch i % n
        bt = batches[i % n]
        t = i // n
        if t >= bt["events"].shape[0]:
            continue
        ev = bt["events"][t]
        dec = bt["d_vms"][t].cpu().numpy().view(np.uint64)
        rc, plan = binding.vms_demo_plan(bt["cfg"], ev, dec)
        if rc != 0:
            return dict(error="decisions of trace %d inconsistent at event %d" % (i, plan.failed_event))
        if plan.peak_mapped_chunks > MAPPING_LIMIT or plan.chunks_created * int(bt["cfg"].chunk_bytes) > free_bytes // 2:
            skipped.append(dict(trace=i, generator=kinds[i % n], peak_mapped_chunks=int(plan.peak_mapped_chunks),
                                chunks=int(plan.chunks_created)))
            continue
        t0 = time.perf_counter()
        rc, rep = binding.vms_demo_run(bt["cfg"], ev, dec)
        wall = time.perf_counter() - t0
        out = dict(trace=i, generator=kinds[i % n], rc=rc, events_replayed=int(rep.events_replayed), wall_s=wall,
                   chunks_created=int(rep.chunks_created), peak_mapped_chunks=int(rep.peak_mapped_chunks),
                   stitches=int(rep.n_stitches), splits=int(rep.n_splits), sblocks_released=int(rep.n_sblocks_released),
                   alias_checks=int(rep.alias_checks), alias_failures=int(rep.alias_failures),
                   traces_passed_over=skipped)
        if rc != 0:
            out.update(failed_event=int(rep.failed_event), hip_error=int(rep.hip_error), failed_api=int(rep.failed_api))
            return out
        calls = {}
        for name in ("reserve", "create", "map", "set_access", "unmap", "release", "address_free"):
            cnt, ms = int(getattr(rep, "n_" + name)), float(getattr(rep, "ms_" + name))
            calls[name] = dict(calls=cnt, ms=ms, us_per_call=1e3 * ms / cnt if cnt else None)
        out["calls"] = calls
        # one 2 GiB block from 2 MiB chunks against hipMalloc(2 GiB): the paper's Table 1, on this device
        mall = rep.table1_hipmalloc_ms
        if rep.table1_bytes and mall > 0:
            out["table1_2GiB_over_hipmalloc"] = dict(
                hipmalloc_ms=mall, reserve=rep.table1_reserve_ms / mall, create=rep.table1_create_ms / mall,
                map=rep.table1_map_ms / mall, set_access=rep.table1_set_access_ms / mall,
                total=(rep.table1_reserve_ms + rep.table1_create_ms + rep.table1_map_ms + rep.table1_set_access_ms) / mall,
                paper_a100_2MB_chunks=dict(reserve=0.003, create=18.1, map=0.70, set_access=96.8, total=115.4))
        return out
    return dict(error="no trace among the first %d fits the device" % (3 * n), traces_passed_over=skipped)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5, help="workload (default: config 5, the mixture of 16,384 x 100,000 events)")
    ap.add_argument("--traces", type=int, default=None)
    ap.add_argument("--events", type=int, default=None)
    ap.add_argument("--launch", choices=("overlap", "serial"), default="overlap")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-demo", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=64, help="traces per batch the oracle is timed on")
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
    # Every batch is launched on a stream of its own (--launch overlap), the long-running offloading
    # batch first, or all on one stream one after the other (--launch serial).
    main_stream = torch.cuda.current_stream(dev)
    streams = [torch.cuda.Stream(device=dev) if args.launch == "overlap" else main_stream for _ in batches]
    order = sorted(range(len(batches)), key=lambda i: 0 if kinds[i] == 3 else 1)

    def step(acc=None):
        for i in order:
            if streams[i] is not main_stream:
                streams[i].wait_stream(main_stream)
            batches[i]["rep"].run(batches[i]["d_events"], None, batches[i]["d_split"], batches[i]["d_vms"], streams[i])
        for i in order:
            if streams[i] is not main_stream:
                main_stream.wait_stream(streams[i])
        if acc is not None:
            # HIP events recorded by the library on each batch's stream around its kernels; reading
            # them waits for the batch, which is also what serialises runs on one handle
            for i, bt in enumerate(batches):
                ms = bt["rep"].last_kernel_ms()
                for k in ms:
                    acc[i][k] += ms[k]

    # one plain device-to-device copy of known size (the first batch's event array): the reference the
    # HBM traffic counters of a profiled run are scaled by
    batches[0]["d_split"].copy_(batches[0]["d_events"])
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    per_batch = [dict(split=0.0, vms=0.0, total=0.0) for _ in batches]
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(per_batch)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    for acc in per_batch:
        for k in acc:
            acc[k] /= max(args.steps, 1)

    stats = [bt["rep"].stats() for bt in batches]
    st = np.concatenate(stats, axis=1)
    flagged = int((st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any(axis=0).sum())
    if flagged:
        names = dict(free_blocks=binding.VMS_ST_OVF_FREE_BLOCKS, pblocks=binding.VMS_ST_OVF_PBLOCKS,
                     sblocks=binding.VMS_ST_OVF_SBLOCKS, runs=binding.VMS_ST_OVF_RUNS,
                     chunks=binding.VMS_ST_OVF_CHUNKS)
        for s, kind in zip(stats, kinds):
            which = {k: int(((s["status"] & v) != 0).any(axis=0).sum()) for k, v in names.items()}
            high = {k: int(s["max_" + k].max()) for k in names if k != "chunks"}
            print("bench.py: batch %s: traces over a table: %s; high-water marks reached: %s" % (kind, which, high),
                  file=sys.stderr)
        print("bench.py: engine tables overflowed; the measurement is invalid", file=sys.stderr)
        sys.exit(1)

    total_events = n_traces * n_events
    ms_per_step = dt / args.steps * 1e3
    counters = recorded_counters(args.config) if n_traces == base["n_traces"] and n_events == base["n_events"] else {}
    # The dominant kernel: the launch (batch, policy) with the most work.  Side by side every launch
    # lasts about as long as the step, so where the profiled figures exist the launch that takes
    # longest ALONE is named; its duration here is still the one measured in this run.
    launches = [(i, p) for i in range(len(batches)) for p in ("vms", "split")]
    if all("ms_alone" in counters.get("batch%d_%s" % bp, {}) for bp in launches):
        dom_b, dom_p = max(launches, key=lambda bp: counters["batch%d_%s" % bp]["ms_alone"])
    else:
        dom_b, dom_p = max(launches, key=lambda bp: per_batch[bp[0]][bp[1]])
    dom_events = batches[dom_b]["events"].size
    algo_bytes = BYTES_PER_EVENT_PER_KERNEL * dom_events
    achieved = algo_bytes / (per_batch[dom_b][dom_p] * 1e-3) / 1e9
    dom_name = "%s policy, batch %d%s" % ("stitching" if dom_p == "vms" else "splitting", dom_b,
                                          " (generator %d)" % kinds[dom_b] if kinds[dom_b] else "")
    dom_counters = counters.get("batch%d_%s" % (dom_b, dom_p), {})
    lds = [bt["rep"].lds_bytes() for bt in batches]
    summaries = [bt["rep"].summary() for bt in batches]
    sum_res = [sum(int(s.sum_peak_reserved[p]) for s in summaries) for p in (0, 1)]
    out = {
        "metric": "allocator events replayed/sec (split + VMS) on 1 MI355X; bit-exact peaks vs oracle",
        "value": total_events / (dt / args.steps),
        "unit": "events/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": workloads.NAMES[args.config], "n_traces": n_traces, "n_events": n_events,
                   "policies": "split+vms", "chunk_bytes": int(batches[0]["cfg"].chunk_bytes),
                   "capacity_bytes": int(batches[0]["cfg"].capacity_bytes),
                   "spool_threshold": int(batches[0]["cfg"].spool_threshold),
                   "frag_limit_bytes": int(batches[0]["cfg"].frag_limit_bytes),
                   "batches": [dict(generator=kinds[i], n_traces=int(bt["events"].shape[0]),
                                    lds_bytes_per_wave={"split": lds[i][0], "vms": lds[i][1]},
                                    kernel_ms=per_batch[i]) for i, bt in enumerate(batches)]},
        "policy_events_per_s": 2 * total_events / (dt / args.steps),     # every event is decided under both policies
        # a single trace is a single wavefront per policy: a latency figure, not a throughput
        "ns_per_event": ms_per_step * 1e6 / n_events if n_traces == 1 else None,
        "roofline": {"bound": "hbm", "kernel": dom_name,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": dom_counters.get("hbm_bytes"),
                     "kernel_ms": per_batch[dom_b][dom_p],                    # in this run, beside the other launches
                     "kernel_ms_alone": dom_counters.get("ms_alone"),        # profiled (--pmc runs the launches one by one)
                     "note": "algorithmic bytes = 16 B per event (8 B event read + 8 B decision written) x the events of "
                             "that launch; the path is a serial state machine per trace, bound by instruction issue and "
                             "LDS / list latency, not by bandwidth: see issue_rate and lds below",
                     # from the committed counter summary of this workload (null once the kernels have changed)
                     "issue_rate": dom_counters.get("issue_rate"),           # wave instructions per SIMD cycle
                     "lds": dom_counters.get("lds"),                         # bytes, GB/s and fraction of the measured peak
                     "waves_per_cu_observed": dom_counters.get("waves_per_cu"),
                     # What bounds the path is the rate at which the SIMDs issue: the launch's vector ALU
                     # instructions (counted by the profiler; the same for every run of the same kernel on
                     # the same input) over its duration in this run, against one wave64 instruction per
                     # 4 cycles on each of 256 x 4 SIMDs at 2.4 GHz.
                     "alu": alu_view(dom_counters, per_batch[dom_b][dom_p])},
        # the same over the whole step: all launches' instructions over the step time
        "step_alu": step_alu_view(counters, ms_per_step),
        "kernels": counters or None,
        "table_high_water": {k: int(st[k].max()) for k in ("max_free_blocks", "max_pblocks", "max_multi_pblocks", "max_sblocks",
                                                            "max_runs", "max_members")},
        "results": {"mean_fragmentation_split": float(st["fragmentation"][0].mean()),
                    "mean_fragmentation_vms": float(st["fragmentation"][1].mean()),
                    # Sec. 5.1: (sum of reserved under splitting - sum under stitching) / sum under splitting
                    "mem_reduction_ratio": (sum_res[0] - sum_res[1]) / sum_res[0] if sum_res[0] else 0.0},
    }
    if not args.no_demo:
        out["vmm_demo"] = demo_tail(batches, kinds, binding)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(batches, min(args.cpu_sample, min(bt["events"].shape[0] for bt in batches)))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
