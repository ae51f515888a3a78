"""A recorded PyTorch allocation stream through the replay engine."""
import gc

import pytest

import gpu_util
from paper_2401_08156_amd import trace_import as ti

pytestmark = pytest.mark.gpu


def test_recorded_torch_loop_replays_bit_exactly_and_matches_pytorch_peaks():
    import torch
    from paper_2401_08156_amd.torch_plugin import train
    gc.collect()
    torch.cuda.empty_cache()
    records, peaks = ti.record_torch_loop(lambda: train(6, 512, 4))
    ev, max_slots, dropped = ti.events_from_records(records)
    assert len(ev) > 500 and dropped["alloc_live_key"] == 0 and dropped["alloc_empty"] == 0
    cfg = gpu_util.make_cfg(1, len(ev), max_slots, max_free_blocks=2048, max_pblocks=4096, max_sblocks=2048,
                            max_runs=1 << 18, max_chunks=65536)
    st = gpu_util.assert_parity(ev[None, :], cfg, label="recorded PyTorch loop")
    assert st["status"].max() == 0
    if dropped["free_unknown"] == 0:
        # what the program asked for, at its peak, is what PyTorch counted as allocated, up to the
        # remainders below 1 MiB that PyTorch leaves attached to a large block instead of splitting them off
        slack = peaks["peak_allocated"] - peaks["allocated_before"] - int(st["peak_requested"][0, 0])
        assert 0 <= slack <= 0.02 * peaks["peak_allocated"], slack
    assert st["peak_reserved"][1, 0] <= st["peak_reserved"][0, 0]
    assert st["fragmentation"][1, 0] < 0.05
    if peaks["reserved_before"] == 0:
        # the splitting model is the caching allocator PyTorch runs: its reserved peak lands close to the real one
        assert abs(int(st["peak_reserved"][0, 0]) - peaks["peak_reserved"]) <= 0.1 * peaks["peak_reserved"]
