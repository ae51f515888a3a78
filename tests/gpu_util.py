"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI and the
oracle on the same events, compare bit for bit."""
import numpy as np

import oracle
from paper_2401_08156_amd import binding

COMPARED_FIELDS = ["peak_requested", "peak_active", "peak_reserved", "final_requested", "final_active",
                   "final_reserved", "digest", "n_code", "n_split", "n_merge", "n_sblock_created",
                   "n_sblock_evicted", "first_oom_event", "status", "max_pblocks", "max_sblocks",
                   "max_free_blocks", "max_members", "fragmentation"]


def make_cfg(n_traces, max_events, max_slots, **kw):
    cfg = binding.vms_config_default(n_traces, max_events, max_slots)
    for k, v in kw.items():
        assert hasattr(cfg, k), k
        setattr(cfg, k, v)
    return cfg


def oracle_params(cfg):
    return oracle.Params(cfg.chunk_bytes, cfg.small_limit_bytes, cfg.frag_limit_bytes, cfg.capacity_bytes,
                         cfg.spool_threshold, cfg.max_slots)


def gpu_replay(events, cfg, n_events=None, want_decisions=True):
    """Returns (dec_split, dec_vms, stats[2, n_traces]) as numpy arrays."""
    import torch
    dev = torch.device("cuda:0")
    ev = torch.from_numpy(np.ascontiguousarray(events).view(np.int64)).to(dev)
    ne = None if n_events is None else torch.from_numpy(np.ascontiguousarray(n_events, dtype=np.uint32).view(np.int32)).to(dev)
    r = binding.Replay(cfg)
    ds = dv = None
    if want_decisions:
        # poison so that entries the kernel must write are distinguishable from untouched ones
        if cfg.policy_mask & 1:
            ds = torch.full_like(ev, -1)
        if cfg.policy_mask & 2:
            dv = torch.full_like(ev, -1)
    r.run(ev, ne, ds, dv)
    st = r.stats()
    out = [None if d is None else d.cpu().numpy().view(np.uint64) for d in (ds, dv)]
    r.close()
    return out[0], out[1], st


def assert_parity(events, cfg, n_events=None, threads=8, label=""):
    """Bit-exact comparison of decisions and statistics of both policies with the oracle."""
    ds, dv, st = gpu_replay(events, cfg, n_events)
    P = oracle_params(cfg)
    for pol, gdec in ((0, ds), (1, dv)):
        if not (cfg.policy_mask & (1 << pol)):
            continue
        odec, ost = oracle.replay(events, P, pol, n_events=n_events, threads=threads)
        gst = st[pol]
        bad = np.flatnonzero(gst["status"] & binding.VMS_ST_TABLE_OVERFLOW)
        assert bad.size == 0, "%s policy %d: table overflow in traces %s at events %s, status %s" % (
            label, pol, bad[:8].tolist(), gst["overflow_event"][bad[:8]].tolist(), gst["status"][bad[:8]].tolist())
        if n_events is None:
            same = gdec == odec
        else:
            valid = np.arange(events.shape[1])[None, :] < np.asarray(n_events)[:, None]
            same = (gdec == odec) | ~valid
            assert np.all(gdec[~valid] == np.uint64(0xFFFFFFFFFFFFFFFF)), "wrote past the end of a trace"
        if not same.all():
            t, i = np.argwhere(~same)[0]
            raise AssertionError("%s policy %d trace %d event %d: gpu %#x oracle %#x (event word %#x)" % (
                label, pol, t, i, int(gdec[t, i]), int(odec[t, i]), int(events[t, i])))
        for f in COMPARED_FIELDS:
            if not np.array_equal(gst[f], ost[f]):
                t = np.flatnonzero((gst[f] != ost[f]).reshape(len(gst), -1).any(axis=1))[0]
                raise AssertionError("%s policy %d trace %d field %s: gpu %s oracle %s" % (
                    label, pol, t, f, gst[f][t], ost[f][t]))
    return st
