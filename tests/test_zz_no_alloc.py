"""vms_replay_run_static (the entry point that allocates nothing: its workspace is an array inside the
library's device code) against vms_replay_run, through the C ABI."""
import ctypes

import numpy as np
import pytest

import gpu_util
from paper_2401_08156_amd import binding
from paper_2401_08156_amd import tracegen as tg

pytestmark = pytest.mark.gpu


def both_ways(ev, cfg):
    import torch
    d_ev = torch.from_numpy(ev.view(np.int64)).cuda()
    out = []
    for static in (False, True):
        r = binding.Replay(cfg)
        ds, dv = torch.full_like(d_ev, -1), torch.full_like(d_ev, -1)
        if static:
            assert 0 < r.workspace_bytes() <= binding.lib().vms_replay_static_workspace_bytes()
            r.run_static(d_ev, None, ds, dv)
        else:
            r.run(d_ev, None, ds, dv)
        st = r.stats()
        out.append((ds.cpu().numpy().view(np.uint64), dv.cpu().numpy().view(np.uint64), st))
        r.close()
    return out


def test_static_workspace_two_calls_in_a_row_the_second_smaller():
    # offloading traces in the fine-grained kernel (lists in the workspace, squeezed when the arena is
    # full), then a smaller batch of shorter transformer traces in the flat kernel (the workspace is
    # where its lists are squeezed): the second call finds the first call's lists in the array
    ev1, ms1 = tg.generate(3, n_traces=24, n_events=6000, seed=41)
    cfg1 = gpu_util.make_cfg(24, 6000, ms1, max_pblocks=4096, max_sblocks=2048, max_runs=1 << 16, max_chunks=16384, spool_threshold=128)
    ev2, ms2 = tg.generate(2, n_traces=9, n_events=2500, seed=42)
    cfg2 = gpu_util.make_cfg(9, 2500, ms2, max_runs=1100, spool_threshold=96, max_sblocks=256)
    for ev, cfg in ((ev1, cfg1), (ev2, cfg2)):
        (ds, dv, st), (ds_s, dv_s, st_s) = both_ways(ev, cfg)
        assert not (st["status"] & binding.VMS_ST_TABLE_OVERFLOW).any()
        assert np.array_equal(ds, ds_s) and np.array_equal(dv, dv_s)
        for f in st.dtype.names:
            assert np.array_equal(st[f], st_s[f]), f
    # and both agree with the oracle
    gpu_util.assert_parity(ev2, cfg2, label="small batch")


def test_static_workspace_refuses_what_does_not_fit():
    import torch
    ev, ms = tg.generate(3, n_traces=64, n_events=500, seed=43)
    cfg = gpu_util.make_cfg(64, 500, ms, max_pblocks=4096, max_sblocks=2048, max_runs=1 << 18, max_chunks=16384)
    r = binding.Replay(cfg)
    assert r.workspace_bytes() > binding.lib().vms_replay_static_workspace_bytes()
    d_ev = torch.from_numpy(ev.view(np.int64)).cuda()
    rc = binding.lib().vms_replay_run_static(r._h, ctypes.c_void_p(d_ev.data_ptr()), None, None, None,
                                             ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == -4
    r.close()
