"""Latency of the HIP virtual-memory calls on this device, laid out like Table 1 of the paper
(Sec. 2.5): for each chunk size a block is built from chunks (reserve, create, map, set access)
and every call class is normalised by hipMalloc of the same block.

    python -m paper_2401_08156_amd.vmm_table [--block-mib 2048] [--chunks-mib 2 128 1024] [--repeats 3]

The paper's numbers (A100, 2 GB block; chunk 2 MB / 128 MB / 1024 MB): Reserve 0.003 / 0.003 / 0.002,
Create 18.1 / 0.89 / 0.79, Map 0.70 / 0.01 / 0.002, SetAccess 96.8 / 8.2 / 0.7, Total 115.4 / 9.1 / 1.5.
"""
import argparse
import json

from . import binding

MiB = 1 << 20


def measure(block_bytes, chunk_sizes, repeats=3):
    """One row per chunk size: dict with the raw milliseconds and the ratios to hipMalloc."""
    rows = []
    for chunk in chunk_sizes:
        if chunk > block_bytes or block_bytes % chunk:
            continue
        rc, r = binding.vms_vmm_latency(block_bytes, chunk, repeats)
        if rc != binding.VMS_OK:
            raise binding.VmsError(rc, "vms_vmm_latency(block %d, chunk %d, hip error %d)" % (block_bytes, chunk, r.hip_error))
        total = r.reserve_ms + r.create_ms + r.map_ms + r.set_access_ms
        norm = r.hipmalloc_ms
        rows.append(dict(block_bytes=block_bytes, chunk_bytes=chunk, n_chunks=int(r.n_chunks),
                         granularity_bytes=int(r.granularity_bytes),
                         ms=dict(hipmalloc=r.hipmalloc_ms, hipfree=r.hipfree_ms, reserve=r.reserve_ms, create=r.create_ms,
                                 map=r.map_ms, set_access=r.set_access_ms, unmap=r.unmap_ms, release=r.release_ms, total=total),
                         ratio=dict(reserve=r.reserve_ms / norm, create=r.create_ms / norm, map=r.map_ms / norm,
                                    set_access=r.set_access_ms / norm, total=total / norm)))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--block-mib", type=int, nargs="+", default=[2048])
    ap.add_argument("--chunks-mib", type=int, nargs="+", default=[2, 128, 1024])
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    out = []
    for b in args.block_mib:
        rows = measure(b * MiB, [c * MiB for c in args.chunks_mib], args.repeats)
        out += rows
        if args.json:
            continue
        print("block %d MiB, normalised by hipMalloc (%.3f ms)" % (b, rows[0]["ms"]["hipmalloc"] if rows else 0.0))
        print("%-12s %10s %10s %10s %10s %10s %12s" % ("chunk", "Reserve", "Create", "Map", "SetAccess", "Total", "total ms"))
        for r in rows:
            q = r["ratio"]
            print("%-12s %10.3f %10.3f %10.3f %10.3f %10.3f %12.3f" % ("%d MiB" % (r["chunk_bytes"] // MiB), q["reserve"], q["create"],
                                                                    q["map"], q["set_access"], q["total"], r["ms"]["total"]))
    if args.json:
        print(json.dumps(out))


if __name__ == "__main__":
    main()
