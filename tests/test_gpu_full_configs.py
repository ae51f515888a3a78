"""The workloads at their full sizes, in the launch configuration bench.py times.

Configs 1, 2, 4 and 6 are compared with the oracle on every trace, every event.  Configs 3 and 5
are launched whole, exactly as bench.py launches them; their offloading traces (which take the
oracle seconds each) are compared on 256 traces drawn from inside each launch, every other trace
of config 5 through its digest and statistics, and all traces through properties that hold at any
size (Sec. 4.2.1: the stitching allocator's reserved peak equals its active peak
when every request is at least one chunk; the splitting allocator's active bytes are the requested
bytes; reserved >= active).
"""
import numpy as np
import pytest

import gpu_util
import oracle
from paper_2401_08156_amd import binding, workloads
from paper_2401_08156_amd import tracegen as tg

pytestmark = pytest.mark.gpu


def check_properties(st, all_requests_large):
    assert ((st["status"] & binding.VMS_ST_TABLE_OVERFLOW) == 0).all()
    assert (st["peak_reserved"] >= st["peak_active"]).all()
    assert (st["peak_active"] >= st["peak_requested"]).all()
    assert np.array_equal(st["peak_requested"][0], st["peak_requested"][1])     # policy independent
    no_oom = st["n_code"][:, :, 5] == 0
    assert np.array_equal(st["peak_active"][0][no_oom[0]], st["peak_requested"][0][no_oom[0]])
    if all_requests_large:
        assert np.array_equal(st["peak_reserved"][1], st["peak_active"][1])
        assert (st["fragmentation"][1] == 0.0).all()


@pytest.mark.parametrize("config", [1, 2, 4, 6])
def test_full_config_every_trace(config):
    n_traces, n_events = workloads.shape(config)
    ev, ms = tg.generate(config, threads=16)
    cfg = workloads.make_config(binding, config, n_traces, n_events, ms)
    st = gpu_util.assert_parity(ev, cfg, threads=16, label="config %d full" % config)
    check_properties(st, all_requests_large=(config == 2))


@pytest.mark.parametrize("config,seed", [(2, 20240817), (4, 77), (6, 5)])
def test_presets_and_second_pass_serve_other_seeds(config, seed):
    # the table presets were sized on the default seeds; traces of another seed go through the same
    # call with no preset of their own: whatever outgrows a table is replayed by the second pass, and
    # everything matches the oracle with no trace left flagged
    n_traces, n_events = 512, workloads.shape(config)[1]
    ev, ms = tg.generate(config, n_traces=n_traces, seed=seed, threads=16)
    cfg = workloads.make_config(binding, config, n_traces, n_events, ms)
    assert cfg.retry_traces > 0
    st = gpu_util.assert_parity(ev, cfg, threads=16, label="config %d, seed %d" % (config, seed))
    check_properties(st, all_requests_large=(config == 2))


def sample_rows(n, count, seed):
    """`count` distinct rows of 0..n-1, spread over the whole range (seeded)."""
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(n, size=min(count, n), replace=False))


def compare_rows(ev, cfg, rows, dec, st, label):
    """Decisions and every statistic of the given rows of a launch against the oracle."""
    P = gpu_util.oracle_params(cfg)
    for pol in (0, 1):
        odec, ost = oracle.replay(ev[rows], P, pol, threads=16)
        assert np.array_equal(dec[pol], odec), "%s policy %d: decisions differ" % (label, pol)
        for f in gpu_util.COMPARED_FIELDS:
            assert np.array_equal(st[pol][rows][f], ost[f]), (label, pol, f)


def test_full_config3_one_launch_256_traces_sampled():
    # all 4,096 offloading traces in ONE launch (four rounds of the fine-grained kernel at four
    # wavefronts per compute unit), as bench.py --config 3 launches them; 256 traces drawn from
    # inside that launch are compared event by event, all of them through properties
    import torch
    n_traces, n_events = workloads.shape(3)
    ev, ms = tg.generate(3, threads=16)
    cfg = workloads.make_config(binding, 3, n_traces, n_events, ms)
    d_ev = torch.from_numpy(ev.view(np.int64)).cuda()
    ds, dv = torch.full_like(d_ev, -1), torch.full_like(d_ev, -1)
    r = binding.Replay(cfg)
    r.run(d_ev, None, ds, dv)
    st = r.stats()
    rows = sample_rows(n_traces, 256, 3)
    idx = torch.from_numpy(rows).cuda()
    dec = [d[idx].cpu().numpy().view(np.uint64) for d in (ds, dv)]
    r.close()
    compare_rows(ev, cfg, rows, dec, st, "config 3")
    check_properties(st, all_requests_large=True)


def test_config5_full_batches_every_recompute_and_lora_trace_256_offloading_traces():
    # 16,384 traces x 100,000 events with a 288 GiB cap, launched as bench.py launches them: one
    # batch per generator kind (5,462 / 5,461 / 5,461 traces), the three batches side by side on
    # three streams.  Every recomputation and LoRA trace is compared through its digest (a checksum
    # over every decision word and the byte totals after every event) and all statistics; 256
    # offloading traces drawn from inside their launch are compared decision by decision as well.
    import torch
    n_traces, n_events = workloads.shape(5)
    kinds = (2, 3, 4)
    batches = []
    for b, kind in enumerate(kinds):
        nt = len(range(b, n_traces, 3))
        ev, ms = tg.generate(5, n_traces=nt, n_events=n_events, first_trace=b, trace_stride=3, threads=16)
        ref, _ = tg.generate(kind, n_traces=1, n_events=200, seed=tg.CONFIGS[5]["seed"], first_trace=b)
        assert np.array_equal(ev[0, :200], ref[0])           # the mixture really uses that generator
        cfg = workloads.make_config(binding, 5, nt, n_events, ms, kind=kind)
        assert cfg.capacity_bytes == 288 << 30
        d_ev = torch.from_numpy(ev.view(np.int64)).cuda()
        batches.append(dict(ev=ev, cfg=cfg, d_ev=d_ev, ds=torch.full_like(d_ev, -1), dv=torch.full_like(d_ev, -1),
                            rep=binding.Replay(cfg), stream=torch.cuda.Stream()))
    main = torch.cuda.current_stream()
    for i in (1, 0, 2):                                      # the long-running offloading batch first
        bt = batches[i]
        bt["stream"].wait_stream(main)
        bt["rep"].run(bt["d_ev"], None, bt["ds"], bt["dv"], bt["stream"])
    for bt in batches:
        main.wait_stream(bt["stream"])
    torch.cuda.synchronize()
    print("config 5: replayed", flush=True)
    for kind, bt in zip(kinds, batches):
        st = bt["rep"].stats()
        check_properties(st, all_requests_large=(kind != 4))
        P = gpu_util.oracle_params(bt["cfg"])
        if kind == 3:
            rows = sample_rows(bt["ev"].shape[0], 256, 5)
            idx = torch.from_numpy(rows).cuda()
            dec = [d[idx].cpu().numpy().view(np.uint64) for d in (bt["ds"], bt["dv"])]
            compare_rows(bt["ev"], bt["cfg"], rows, dec, st, "config 5 offloading")
        else:
            for pol in (0, 1):
                _, ost = oracle.replay(bt["ev"], P, pol, want_decisions=False, threads=16)
                for f in gpu_util.COMPARED_FIELDS:
                    assert np.array_equal(st[pol][f], ost[f]), ("config 5 kind %d" % kind, pol, f)
            # and a few of them decision by decision
            rows = sample_rows(bt["ev"].shape[0], 32, 50 + kind)
            idx = torch.from_numpy(rows).cuda()
            dec = [d[idx].cpu().numpy().view(np.uint64) for d in (bt["ds"], bt["dv"])]
            compare_rows(bt["ev"], bt["cfg"], rows, dec, st, "config 5 kind %d" % kind)
        bt["rep"].close()
        print("config 5: kind %d compared" % kind, flush=True)
