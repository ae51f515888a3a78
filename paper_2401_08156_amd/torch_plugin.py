"""The live stitching allocator as PyTorch's device allocator for a whole process (the paper's
artefact is such a plug-in, Sec. 4.3), on a small training loop whose tensor sizes change every step.

    python -m paper_2401_08156_amd.torch_plugin            # every device allocation goes through vms_live
    python -m paper_2401_08156_amd.torch_plugin --native   # PyTorch's own caching allocator, for comparison

The allocator has to be installed before the process touches device memory, hence one process per
mode.  Prints one JSON line: step time, loss of the last step, reserved / active peaks and, for the
plug-in, its decision counts and the time spent in the driver's virtual-memory calls.
"""
import argparse
import json
import time


def install():
    import torch
    from . import binding
    alloc = binding.torch_pluggable_allocator()
    torch.cuda.memory.change_current_allocator(alloc)
    return alloc


def train(steps, hidden, layers, seed=0, on_step=None):
    """An MLP stack with recomputation-like reuse: the batch x sequence extent changes every step."""
    import torch
    torch.manual_seed(seed)
    dev = torch.device("cuda:0")
    ws = [(torch.randn(hidden, 4 * hidden, device=dev) * 0.02).requires_grad_(True) for _ in range(layers)]
    vs = [(torch.randn(4 * hidden, hidden, device=dev) * 0.02).requires_grad_(True) for _ in range(layers)]
    times, loss = [], None
    for i in range(steps):
        tokens = 1024 + 256 * ((i * 7) % 13)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        x = torch.randn(tokens, hidden, device=dev)
        for w, v in zip(ws, vs):
            x = torch.nn.functional.layer_norm(x + torch.nn.functional.gelu(x @ w) @ v, (hidden,))
        loss = (x[:, :8] ** 2).mean()
        loss.backward()
        with torch.no_grad():
            for p in ws + vs:
                p -= 1e-3 * p.grad
                p.grad = None
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        if on_step:
            on_step(i)
    return times, float(loss.detach())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--native", action="store_true")
    ap.add_argument("--steps", type=int, default=78)
    ap.add_argument("--hidden", type=int, default=2048)
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--threshold", type=int, default=None, help="StitchFree threshold (cached sBlocks)")
    args = ap.parse_args()
    new_blocks = []                 # sBlocks created so far, after every step
    on_step = None
    if not args.native:
        import os
        if args.threshold is not None:
            os.environ["VMS_LIVE_SPOOL_THRESHOLD"] = str(args.threshold)
        install()
        from . import binding
        on_step = lambda i: new_blocks.append(int(binding.torch_allocator_stats(0)[0]["n_sblock_created"]))
    import torch
    times, loss = train(args.steps, args.hidden, args.layers, on_step=on_step)
    half = len(times) // 2
    out = dict(mode="native" if args.native else "vms_live", steps=args.steps, loss=loss,
               ms_per_step_first_half=1e3 * sum(times[:half]) / half,
               ms_per_step_second_half=1e3 * sum(times[half:]) / (len(times) - half))
    if args.native:
        out["peak_reserved_mib"] = torch.cuda.max_memory_reserved() / 2 ** 20
        out["peak_active_mib"] = torch.cuda.max_memory_allocated() / 2 ** 20
    else:
        from . import binding
        st, api = binding.torch_allocator_stats(0)
        out["peak_reserved_mib"] = int(st["peak_reserved"]) / 2 ** 20
        out["peak_active_mib"] = int(st["peak_active"]) / 2 ** 20
        out["fragmentation"] = float(st["fragmentation"])
        out["decisions"] = dict(exact=int(st["n_code"][1]), split=int(st["n_code"][2]), stitch=int(st["n_code"][3]),
                                grow=int(st["n_code"][4]), oom=int(st["n_code"][5]), free=int(st["n_code"][0]))
        out["sblocks_created"] = int(st["n_sblock_created"])
        period = 13                 # the token counts repeat every 13 steps
        out["sblocks_created_per_period"] = [new_blocks[min(k + period, len(new_blocks)) - 1] - (new_blocks[k - 1] if k else 0)
                                             for k in range(0, len(new_blocks), period)]
        out["sblocks_released"] = int(st["n_sblock_evicted"])
        out["driver_ms"] = dict(create=api.ms_create, map=api.ms_map, set_access=api.ms_set_access,
                                reserve=api.ms_reserve, unmap=api.ms_unmap)
        out["malloc_calls"] = int(api.n_malloc)
        out["ms_in_malloc"] = api.ms_malloc
    print(json.dumps(out))


if __name__ == "__main__":
    main()
