"""The workloads at their full sizes, in the launch configuration bench.py times.

Configs 1, 2, 4 and 6 are compared with the oracle on every trace, every event.  Configs 3 and 5
(whose offloading traces take the oracle seconds each) run on the GPU at full trace length, are
compared with the oracle on a sample of traces, and are checked on all traces through properties
that hold at any size (Sec. 4.2.1: the stitching allocator's reserved peak equals its active peak
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


def test_full_config3_sampled():
    n_traces, n_events = workloads.shape(3)
    sample = np.arange(0, n_traces, 64)[:48]                # traces compared event by event
    batch = 1024                                            # a few seconds of GPU time per launch
    stats = []
    for first in range(0, n_traces, batch):
        ev, ms = tg.generate(3, n_traces=batch, first_trace=first, threads=16)
        cfg = workloads.make_config(binding, 3, batch, n_events, ms)
        ds, dv, st = gpu_util.gpu_replay(ev, cfg)
        stats.append(st)
        pick = sample[(sample >= first) & (sample < first + batch)] - first
        P = gpu_util.oracle_params(cfg)
        for pol, gdec in ((0, ds), (1, dv)):
            odec, ost = oracle.replay(ev[pick], P, pol, threads=16)
            assert np.array_equal(gdec[pick], odec), "config 3 policy %d batch at %d" % (pol, first)
            for f in gpu_util.COMPARED_FIELDS:
                assert np.array_equal(st[pol][pick][f], ost[f]), (f, pol, first)
        print("config 3: traces %d-%d done" % (first, first + batch - 1), flush=True)
    check_properties(np.concatenate(stats, axis=1), all_requests_large=True)


def test_config5_sampled_full_length():
    # 16,384 traces x 100,000 events with a 288 GiB cap; trace i uses generator 2 + i mod 3.
    # Replayed as one batch per generator kind; 32 traces of each kind, full length.
    n_traces, n_events = workloads.shape(5)
    per_kind = 32
    for b, kind in enumerate((2, 3, 4)):
        first = b + 3 * 171 * b                              # spread over the index range, same kind
        ev, ms = tg.generate(5, n_traces=per_kind, n_events=n_events, first_trace=first, trace_stride=3 * 151,
                             threads=16)
        ref, _ = tg.generate(kind, n_traces=1, n_events=200, seed=tg.CONFIGS[5]["seed"], first_trace=first)
        assert np.array_equal(ev[0, :200], ref[0])           # the mixture really uses that generator
        cfg = workloads.make_config(binding, 5, per_kind, n_events, ms, kind=kind)
        assert cfg.capacity_bytes == 288 << 30
        st = gpu_util.assert_parity(ev, cfg, threads=16, label="config 5 kind %d" % kind)
        check_properties(st, all_requests_large=(kind != 4))
        print("config 5: kind %d done" % kind, flush=True)
