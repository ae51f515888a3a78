"""The synthetic workloads and the engine table sizes that fit them.

Table sizes (per trace) are capacity settings of the replay engine, not parameters of the
allocators: a trace that outgrows them is replayed a second time with doubled tables (up to
retry_traces traces per run), and flagged VMS_ST_TABLE_OVERFLOW, never replayed wrongly, if that
does not suffice.  The values below hold the high-water marks measured on the full workloads with headroom;
smaller tables mean less LDS per wavefront and therefore more resident wavefronts per compute unit.
"""
from . import tracegen

NAMES = {1: "config1-random", 2: "config2-recompute", 3: "config3-offload", 4: "config4-lora",
         5: "config5-mixture", 6: "config6-zero3-scaleout"}

TABLES = {
    # config: splitting free list (max_small_blocks: the stitching policy's own, smaller one), pBlocks, sBlocks,
    # chunk-run list entries, chunks (x 2 MiB)
    1: dict(max_free_blocks=512, max_pblocks=1024, max_sblocks=640, max_runs=4096, max_chunks=8192),
    2: dict(max_free_blocks=192, max_pblocks=544, max_sblocks=576, max_runs=3840, max_chunks=4096),
    # offloading grinds pBlocks down to single chunks: thousands of pBlocks and sBlocks (the fine-grained kernel
    # variant: single chunks in bitmaps, a table for the pBlocks of two or more chunks, lists in the workspace)
    # (31,680 B of LDS per wavefront: LDS is handed out in 1,280-byte granules, 128 per compute unit, so five
    # wavefronts per compute unit need at most 32,000 B each; with 2,816 places for multi-chunk pBlocks it was four)
    3: dict(max_free_blocks=64, max_pblocks=8192, max_multi_pblocks=2592, max_sblocks=2560, max_runs=1 << 18, max_chunks=10240),
    # (the fine-grained kernel with its sBlock tables in the workspace, chunk tables for the 17,699 chunks the
    # largest trace reserves: 19.5 KB of LDS per wavefront, eight per compute unit instead of the flat kernel's
    # three, 153 against 179 ms per step)
    4: dict(max_free_blocks=320, max_small_blocks=192, max_pblocks=640, max_sblocks=576, max_runs=3840, max_chunks=18432,
            variant=2, table_place=3),
    # (the same for the 1,280 traces of the scale-out regime, 9,408 chunks at most: 22.9 KB, all traces resident
    # at once, 20.0 against 25.8 ms)
    6: dict(max_free_blocks=192, max_pblocks=512, max_sblocks=576, max_runs=3072, max_chunks=9728, variant=2, table_place=3),
}
# config 5 mixes the generators of configs 2, 3 and 4 (trace i uses kind 2 + i mod 3) with twice the
# events; replayed as three batches, one per kind, each with tables of its own
TABLES_5 = {
    2: dict(max_free_blocks=192, max_pblocks=640, max_sblocks=640, max_runs=5120, max_chunks=4096),
    # (the margins over the high-water marks are one to two per cent; a trace that outgrows a table is replayed
    # again by the second pass.  40,208 B of LDS per wavefront with every table in LDS, four wavefronts per compute
    # unit; the library moves the sBlock tables to the workspace: 14,960 B, ten)
    3: dict(max_free_blocks=64, max_pblocks=8192, max_multi_pblocks=2720, max_sblocks=4128, max_runs=1 << 18, max_chunks=8480),
    # (beside the other two batches the fine-grained kernel with its sBlock tables in the workspace, 19.9 KB of LDS
    # per wavefront, finishes the step sooner than the flat one with 50.8 KB: 1,339 against 1,456 ms; 18,055
    # chunks is the most a trace of this kind reserves)
    4: dict(max_free_blocks=320, max_small_blocks=192, max_pblocks=736, max_sblocks=576, max_runs=4224, max_chunks=18432,
            variant=2, table_place=3),
}


def shape(config):
    c = tracegen.CONFIGS[config]
    return c["n_traces"], c["n_events"]


def make_config(binding, config, n_traces, n_events, max_slots, kind=None, **overrides):
    """vms_config for a workload (kind: the generator of a config-5 batch)."""
    cfg = binding.vms_config_default(n_traces, n_events, max_slots)
    cfg.capacity_bytes = tracegen.CONFIGS[config]["capacity_bytes"]
    tables = TABLES_5[kind] if config == 5 else TABLES[config % 10]
    for k, v in tables.items():
        setattr(cfg, k, v)
    # the tables hold the high-water marks of the seeded workloads with little headroom; a trace of
    # another seed that outgrows one is replayed a second time with doubled tables
    cfg.retry_traces = min(32, n_traces)
    for k, v in overrides.items():
        assert hasattr(cfg, k), k
        setattr(cfg, k, v)
    return cfg
