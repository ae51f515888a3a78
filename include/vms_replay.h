/*
 * vms_replay: batched allocator trace replay on one AMD MI355X (gfx950).
 *
 * Thousands of independent alloc/free traces are replayed on the GPU, one
 * wavefront per (trace, policy), under two allocator policies from the GMLake
 * paper (arXiv 2401.08156):
 *   VMS_POLICY_SPLIT  the splitting caching allocator: best fit, split, lazy
 *                     free, merge with inactive neighbours (Sec. 2.2,
 *                     "Caching Allocator");
 *   VMS_POLICY_VMS    the virtual-memory-stitching allocator: pBlock / sBlock
 *                     pools (Sec. 3.2), Alloc / Split / Stitch (Sec. 3.3.1),
 *                     BestFit (Algorithm 1), Update / StitchFree (Sec. 3.3.2),
 *                     the four allocation states S1-S5 (Sec. 4.1, Fig. 9), the
 *                     fragmentation limit (Sec. 4.2.3) and the splitting path
 *                     for requests below one chunk (Sec. 3.1).
 * Per event it emits one decision word per policy; per trace it emits peak
 * requested / active / reserved bytes and fragmentation = 1 - peak active /
 * peak reserved (Sec. 5.1, "Metric").
 *
 * Plain C ABI: no C++ or framework types.  Pointers named d_* are DEVICE
 * pointers owned by the caller; h_* and unprefixed pointers are HOST pointers.
 * Every function returns VMS_OK (0) or a negative VMS_E* code and never
 * throws or aborts.  Conditions inside a trace (out of memory, malformed
 * events) are results, reported in the decision stream and the status word,
 * not errors of the call.
 *
 * Event word (u64), the input format:
 *   bits  0-30  request size in 512-byte units (ALLOC only, must be >= 1)
 *   bit   31    kind: 0 = ALLOC, 1 = FREE
 *   bits 32-63  slot: handle chosen by the trace; ALLOC binds an unbound slot,
 *               FREE releases a bound one; slot < max_slots
 *
 * Decision word (u64), one per event and policy:
 *   bits  0-3   code: 0 FREE, 1 EXACT (S1), 2 SPLIT (S2), 3 STITCH (S3),
 *               4 GROW (S4, or a new segment of a splitting pool), 5 OOM (S5),
 *               6 FREE_NOOP (free of a slot whose ALLOC hit OOM), 15 INVALID
 *   bit   4     served by the small-request splitting pool of the VMS policy
 *   bit   5     the block is a stitched block (sBlock)
 *   bit   6     ALLOC: a block was cut (Split);  FREE in a splitting pool:
 *               merged with the left neighbour
 *   bit   7     ALLOC: StitchFree released at least one sBlock;  FREE in a
 *               splitting pool: merged with the right neighbour
 *   bits  8-31  number of candidate blocks taken from the pool (|CB| of
 *               Algorithm 1; 1 for a hit in a splitting pool, 0 for pure growth)
 *   bits 32-63  where: splitting pools: block address in 512-byte units in
 *               that pool's address space; VMS pBlock: its first physical
 *               chunk number; VMS sBlock: its creation number
 *   OOM, FREE_NOOP and INVALID words carry the code only.
 */
#ifndef VMS_REPLAY_H
#define VMS_REPLAY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VMS_OK          0
#define VMS_EINVAL     (-1)   /* bad argument or inconsistent configuration            */
#define VMS_ESTRUCT    (-2)   /* struct_size does not match this library               */
#define VMS_ENOMEM     (-3)   /* host or device allocation failed                      */
#define VMS_EWORKSPACE (-4)   /* workspace missing or misaligned                       */
#define VMS_EHIP       (-5)   /* a HIP call failed; see vms_replay_last_hip_error      */
#define VMS_ETOOBIG    (-6)   /* per-trace tables do not fit the 160 KB of LDS per CU  */
#define VMS_ESTATE     (-7)   /* call out of order (stats before run, ...)             */

#define VMS_VARIANT_AUTO 0u
#define VMS_VARIANT_FLAT 1u
#define VMS_VARIANT_FINE 2u

#define VMS_TABLES_AUTO      0u
#define VMS_TABLES_LDS       1u
#define VMS_TABLES_WORKSPACE 2u       /* witnesses and list places */
#define VMS_TABLES_WORKSPACE_ALL 3u   /* and the sizes */

#define VMS_POLICY_SPLIT 1u
#define VMS_POLICY_VMS   2u

/* status bits of vms_trace_stats.status */
#define VMS_ST_INVALID_EVENT   1u   /* at least one INVALID decision (a result, not a failure) */
#define VMS_ST_TABLE_OVERFLOW  2u   /* an engine table (below) was too small: replay of this
                                       trace stopped early, its results are not valid; one
                                       of the following bits names the table                */
#define VMS_ST_OVF_FREE_BLOCKS 4u
#define VMS_ST_OVF_PBLOCKS     8u
#define VMS_ST_OVF_SBLOCKS     16u
#define VMS_ST_OVF_RUNS        32u
#define VMS_ST_OVF_CHUNKS      64u

typedef struct vms_config {
    uint32_t struct_size;        /* sizeof(vms_config)                                      */
    uint32_t n_traces;
    uint32_t max_events;         /* row length of the event / decision arrays               */
    uint32_t policy_mask;        /* VMS_POLICY_SPLIT | VMS_POLICY_VMS                        */
    uint64_t chunk_bytes;        /* physical chunk, 2 MiB in the paper (Sec. 3.1); a power
                                    of two >= 512; also the growth granularity of the
                                    splitting pools                                          */
    uint64_t small_limit_bytes;  /* VMS: requests below this use the splitting pool
                                    (Sec. 3.1); <= chunk_bytes                               */
    uint64_t frag_limit_bytes;   /* VMS: blocks below this are neither split nor stitched
                                    (Sec. 4.2.3); a multiple of chunk_bytes; chunk_bytes
                                    or 0 disables it                                         */
    uint64_t capacity_bytes;     /* reserved-memory limit per trace (state S5); 0 selects
                                    the engine maximum of 512 GiB                            */
    uint32_t spool_threshold;    /* StitchFree releases least-recently-used inactive sBlocks
                                    while more than this many are cached (Sec. 4.2.3)        */
    uint32_t max_slots;          /* slots are 0 .. max_slots-1                               */
    /* engine table sizes per trace; a trace that needs more gets VMS_ST_TABLE_OVERFLOW     */
    uint32_t max_free_blocks;    /* inactive blocks of a splitting pool (up to 320: registers) */
    uint32_t max_pblocks;        /* pBlocks (active and inactive)                            */
    uint32_t max_sblocks;        /* cached sBlocks; must exceed spool_threshold + 2          */
    uint32_t max_runs;           /* chunk runs summed over all cached sBlocks                */
    uint32_t max_chunks;         /* physical chunks of the VMS large path                    */
    uint32_t max_small_blocks;   /* VMS: inactive blocks of its pool for requests below
                                    small_limit_bytes; 0 = max_free_blocks.  At most 192:
                                    that pool is held in registers                           */
    uint32_t max_multi_pblocks;  /* VMS, tables of the fine-grained variant (more than 16384
                                    runs, or more than 4096 pBlocks or sBlocks): pBlocks of
                                    two or more chunks, at most 4096; 0 = min(max_pblocks,
                                    4096).  pBlocks of one chunk take no table space there   */
    uint32_t variant;            /* VMS kernel: 0 = chosen by the library (VMS_VARIANT_AUTO),
                                    VMS_VARIANT_FLAT = flat sorted tables and lists in LDS
                                    (lowest latency per trace; up to 16384 runs and 4096
                                    pBlocks / sBlocks), VMS_VARIANT_FINE = the fine-grained
                                    variant (a fraction of the LDS, lists in the workspace:
                                    more traces resident per compute unit)                   */
    uint32_t retry_traces;       /* wavefronts of the second pass (0: no second pass; traces
                                    that outgrow one of the tables above stay flagged
                                    VMS_ST_TABLE_OVERFLOW).  The second pass runs right
                                    behind the first inside vms_replay_run: retry_traces
                                    wavefronts with every table doubled (as far as a compute
                                    unit's LDS goes) share out the flagged traces and replay
                                    each of them from its first event; it needs workspace
                                    for retry_traces traces of that size                     */
    uint32_t table_place;        /* fine-grained variant: where the tables of the sBlocks
                                    live.  VMS_TABLES_LDS; VMS_TABLES_WORKSPACE (witnesses
                                    and list places in the workspace: 4 bytes of LDS less
                                    per sBlock) or VMS_TABLES_WORKSPACE_ALL (sizes too: 6
                                    bytes less): more wavefronts per compute unit, each of
                                    them slower; at most 63000 chunks.  0: the library
                                    chooses by the rounds of wavefronts the batch takes      */
} vms_config;

typedef struct vms_trace_stats {        /* one per (policy, trace) */
    uint64_t peak_requested;     /* bytes: running maximum of live request sizes            */
    uint64_t peak_active;        /* bytes held by live blocks (Sec. 5.1 "active memory")    */
    uint64_t peak_reserved;      /* bytes obtained from the device (Sec. 5.1 "reserved")    */
    uint64_t final_requested, final_active, final_reserved;
    uint64_t digest;             /* checksum of the decision stream: the sum over events i
                                    (from 0) of (decision_i * 0x9E3779B97F4A7C15 +
                                    (active_i / 512 << 32 | reserved_i / 512)) *
                                    ((2 i + 1) * 0xD6E8FEB86659FD93)  mod 2^64, with the
                                    totals taken after event i                               */
    uint32_t n_code[8];          /* events per decision code 0..6; [7] counts INVALID       */
    uint32_t n_split;            /* blocks cut (both kinds of pool)                          */
    uint32_t n_merge;            /* neighbour merges in splitting pools                      */
    uint32_t n_sblock_created, n_sblock_evicted;
    uint32_t first_oom_event;    /* 0xFFFFFFFF if none                                       */
    uint32_t status;             /* VMS_ST_* bits                                            */
    uint32_t max_pblocks, max_sblocks, max_free_blocks, max_members;  /* high-water marks;
                                    max_members = most blocks stitched into one sBlock       */
    uint32_t max_runs;           /* high-water mark of chunk runs held by cached sBlocks     */
    uint32_t overflow_event;     /* event at which a table overflowed, else 0xFFFFFFFF       */
    uint32_t max_multi_pblocks;  /* fine-grained variant: high-water mark of its table of
                                    pBlocks of two or more chunks; 0 from the other kernels  */
    uint32_t reserved1;          /* 0                                                        */
    double   fragmentation;      /* 1.0 - (double)peak_active / (double)peak_reserved;
                                    0.0 when nothing was reserved                            */
} vms_trace_stats;

typedef struct vms_summary {            /* over all traces of one run (Sec. 5.1) */
    uint64_t sum_peak_reserved[2];   /* [0] splitting, [1] VMS                               */
    uint64_t sum_peak_active[2];
    uint64_t n_flagged[2];           /* traces with a non-zero status                        */
    double   max_fragmentation[2];
    double   mean_fragmentation[2];
    double   mem_reduction_ratio;    /* (sum reserved split - sum reserved VMS) / sum reserved
                                        split; 0 unless both policies ran                    */
} vms_summary;

typedef struct vms_replay vms_replay;   /* opaque handle */

/* Fill *cfg with the defaults (2 MiB chunks, limits disabled, threshold 512,
 * table sizes for transformer-like traces) for the given shape.               */
void vms_config_default(vms_config *cfg, uint32_t n_traces, uint32_t max_events, uint32_t max_slots);

/* Validate cfg, choose the LDS layout and allocate the device statistics
 * buffer (n_traces * 2 records) on the current HIP device.  *out is owned by
 * the caller until vms_replay_destroy.                                         */
int vms_replay_create(const vms_config *cfg, vms_replay **out);

/* Bytes of device scratch memory vms_replay_run needs (may be 0); the caller
 * allocates it, 256-byte aligned, and may reuse it between runs.              */
size_t vms_replay_workspace_bytes(const vms_replay *h);

/* LDS bytes per wavefront for each policy's kernel ([0] splitting, [1] VMS). */
int vms_replay_lds_bytes(const vms_replay *h, uint32_t out[2]);

/* Replay.  d_events[n_traces][max_events] holds the event words; d_n_events
 * (nullable) the number of valid events per trace (default: max_events).
 * d_dec_split / d_dec_vms (nullable each) receive the decision words in the
 * same shape; entries past a trace's length are not written.  d_workspace as
 * sized above.  Work is enqueued on hip_stream (a hipStream_t, NULL = default
 * stream) and the call returns without waiting; buffers must stay alive until
 * the stream has drained.  Runs on one handle must not overlap.               */
int vms_replay_run(vms_replay *h, const uint64_t *d_events, const uint32_t *d_n_events,
                   uint64_t *d_dec_split, uint64_t *d_dec_vms, void *d_workspace, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): vms_replay_run with the workspace taken from an array
 * that is part of the library's device code (vms_replay_static_workspace_bytes() = 32 MiB per
 * device, held from the first use on that device until the process ends) instead of from the
 * caller.  Allocates nothing and calls no allocating routine.  VMS_EWORKSPACE if the handle needs
 * more workspace than the array holds (vms_replay_workspace_bytes), VMS_EINVAL if the current
 * device is not the one the handle was created on.  All calls on one device share the one array:
 * runs that overlap on a device race (also across handles); the array keeps the last run's lists,
 * which the next run overwrites before reading.  Everything else as vms_replay_run.            */
int vms_replay_run_static(vms_replay *h, const uint64_t *d_events, const uint32_t *d_n_events,
                          uint64_t *d_dec_split, uint64_t *d_dec_vms, void *hip_stream);
size_t vms_replay_static_workspace_bytes(void);

/* Wait for the last run and copy statistics to the host: h_out[p * n_traces + t]
 * with p = 0 splitting, 1 VMS; n must be 2 * n_traces.  Records of a policy
 * that did not run are zero.                                                  */
int vms_replay_stats(vms_replay *h, vms_trace_stats *h_out, size_t n);

/* Wait for the last run and reduce the per-trace statistics on the device.   */
int vms_replay_summary(vms_replay *h, vms_summary *h_out);

/* Milliseconds the kernels of the last run took on their stream (HIP events
 * recorded around them inside vms_replay_run); waits for the run.
 * out_ms[0] splitting kernel, [1] VMS kernel (both: the first pass alone),
 * [2] whole run, second pass included.                                        */
int vms_replay_last_kernel_ms(vms_replay *h, float out_ms[3]);

void vms_replay_destroy(vms_replay *h);

int vms_replay_last_hip_error(const vms_replay *h);   /* hipError_t of the last VMS_EHIP */
const char *vms_strerror(int code);

/* What vms_demo_run measured.  Times are host wall-clock milliseconds summed over the calls.   */
typedef struct vms_demo_report {
    uint32_t struct_size;        /* sizeof(vms_demo_report), set by the caller               */
    uint32_t events_replayed;
    uint32_t failed_event;       /* event at which replay stopped, if the call failed        */
    int32_t  hip_error;          /* hipError_t of the first failing HIP call, else 0         */
    uint64_t granularity_bytes;  /* hipMemGetAllocationGranularity (minimum) of the device   */
    uint64_t chunks_created;     /* physical chunks obtained with hipMemCreate               */
    uint32_t n_pblocks_created, n_splits, n_stitches, n_sblocks_released;
    uint32_t sblocks_cached;     /* stitched ranges still mapped at the end                  */
    uint32_t alias_checks;       /* stitched ranges verified to alias their members' memory  */
    uint32_t alias_failures;     /* ... and how many did not (must be 0)                     */
    uint32_t failed_api;         /* which call gave hip_error: 1 reserve, 2 create, 3 map, 4 set
                                    access, 5 unmap, 6 release, 7 address free, 8 memcpy     */
    uint64_t n_reserve, n_create, n_map, n_set_access, n_unmap, n_release, n_address_free;
    double   ms_reserve, ms_create, ms_map, ms_set_access, ms_unmap, ms_release, ms_address_free;
    /* one 2 GiB block built from chunk_bytes chunks, against hipMalloc(2 GiB): Table 1      */
    uint64_t table1_bytes;
    double   table1_hipmalloc_ms, table1_reserve_ms, table1_create_ms, table1_map_ms, table1_set_access_ms;
    uint64_t peak_mapped_chunks; /* most chunk mappings alive at once, over all virtual ranges  */
} vms_demo_report;

/* Functional demonstration (Sec. 3.3.1, Sec. 2.5): execute the first n_events decisions of ONE
 * trace of the stitching policy with real device mappings on the current HIP device
 * (hipMemAddressReserve / hipMemCreate / hipMemMap / hipMemSetAccess / hipMemUnmap /
 * hipMemRelease / hipMemAddressFree), one physical allocation per chunk.  h_events and
 * h_dec_vms are HOST arrays: the trace's event words and the decision words vms_replay_run
 * wrote for it under the same cfg.  Requests served by the small-request pool are skipped.
 * The decisions are cross-checked against books kept by the demo: VMS_EINVAL (with
 * failed_event) if they are inconsistent, VMS_EHIP if a HIP call fails (e.g. out of device
 * memory: the trace's reserved bytes are really allocated).  Everything is unmapped and
 * released before returning.  Synchronous; host code only, no kernel is launched.              */
int vms_demo_run(const vms_config *cfg, const uint64_t *h_events, const uint64_t *h_dec_vms, uint32_t n_events,
                 vms_demo_report *out);

/* The same walk over the decisions with every driver call counted instead of made (host only, no
 * device needed): out receives the call counts, chunks_created and peak_mapped_chunks that
 * vms_demo_run would reach, so that a caller can pick a trace the device can hold (the driver
 * refuses further mappings beyond some tens of thousands).  VMS_EINVAL (with failed_event) if the
 * decisions contradict the books.                                                              */
int vms_demo_plan(const vms_config *cfg, const uint64_t *h_events, const uint64_t *h_dec_vms, uint32_t n_events,
                  vms_demo_report *out);

/* What vms_vmm_latency measured: host wall-clock milliseconds, the best of the rounds, summed over
 * the calls of one kind (n_chunks calls for create / map / set access / unmap / release).        */
typedef struct vms_vmm_latency_report {
    uint32_t struct_size;        /* sizeof(vms_vmm_latency_report), set by the caller              */
    int32_t  hip_error;          /* hipError_t of the first failing HIP call, else 0               */
    uint64_t block_bytes, chunk_bytes, n_chunks, granularity_bytes;
    double   hipmalloc_ms, hipfree_ms;                       /* the native allocator, same size     */
    double   reserve_ms, create_ms, map_ms, set_access_ms;   /* the four columns of Table 1         */
    double   unmap_ms, release_ms;
} vms_vmm_latency_report;

/* Latency of the virtual memory management calls on the current HIP device (Sec. 2.5, Fig. 6 and
 * Table 1 of the paper): a block of block_bytes is built from physical chunks of chunk_bytes
 * (hipMemAddressReserve once; hipMemCreate, hipMemMap and hipMemSetAccess once per chunk), taken
 * apart again, and compared with hipMalloc + hipFree of block_bytes; `repeats` rounds, the best
 * time of each call class is reported.  chunk_bytes must be a multiple of the device's
 * allocation granularity and divide block_bytes; at most 2^20 chunks.  The block is really
 * allocated: VMS_EHIP (with hip_error) if the device cannot provide it.  Everything is released
 * before returning.  Synchronous; host code only, no kernel is launched.                          */
int vms_vmm_latency(uint64_t block_bytes, uint64_t chunk_bytes, uint32_t repeats, vms_vmm_latency_report *out);

/* What vms_measure_peaks measured on the current device.                                            */
typedef struct vms_peaks_report {
    uint32_t struct_size;        /* sizeof(vms_peaks_report), set by the caller                    */
    int32_t  hip_error;          /* hipError_t of the first failing HIP call, else 0               */
    uint32_t compute_units, clock_mhz;
    uint64_t copy_bytes;         /* bytes read + written by the copy kernel per launch             */
    double   copy_ms, hbm_copy_gbs;
    uint64_t lds_bytes;          /* bytes read from LDS by the read loop per launch                */
    double   lds_ms, lds_read_gbs;
    uint64_t read_bytes;         /* bytes read by the read-only kernel per launch                  */
    double   read_ms, hbm_read_gbs;
} vms_peaks_report;

/* Two micro-benchmarks for the proportions of Sec. 5.1-style reports on the device at hand: a
 * plain 1 GiB device-to-device copy kernel and the same kernel without its stores (HBM bandwidth
 * actually reachable: read + write, and read alone; four 16-byte loads in flight per lane), and a
 * conflict-free 16-byte-per-lane LDS read loop on every compute unit (LDS bandwidth actually
 * reachable).  Allocates 2 GiB of device memory for the duration of the call; best of three timed
 * rounds each.  Synchronous, on the default stream.                                                */
int vms_measure_peaks(vms_peaks_report *out);

/* In-wavefront primitives self-test (reductions, scans, sorted insert): runs a
 * small kernel on the current device and returns VMS_OK if every lane layout
 * matches its definition.  Diagnostic; not part of a replay.                  */
int vms_selftest(void);

#ifdef __cplusplus
}
#endif
#endif
