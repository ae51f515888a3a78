// Host-side planning of a replay: checks a vms_config, chooses the kernel variants and lays out
// the per-wavefront LDS arrays and the per-trace workspace slice.  Plain C++ with no device or
// runtime calls, so that the same code serves the library and host-only checks of the kernels.
#ifndef VMS_REPLAY_PLAN_HPP
#define VMS_REPLAY_PLAN_HPP
#include <stdint.h>
#include <string.h>

#include "../../include/vms_replay.h"

// Launch-constant parameters (passed by value as a kernel argument).
struct KParams {
    uint32_t n_traces, max_events;
    uint32_t chunk_shift;            // log2(chunk in 512-byte units)
    uint32_t small_limit_units;
    uint32_t frag_limit_chunks;
    uint32_t spool_threshold;
    uint32_t capacity_units;         // at most 2^30 (512 GiB)
    uint32_t max_slots;
    uint32_t cap_free, cap_pblocks, cap_sblocks, cap_runs, cap_chunks;
    // byte offsets of the per-wave arrays inside dynamic LDS
    uint32_t off_slot_req, off_slot_a, off_slot_b, off_slot_c, off_fl, off_pool, off_bmp, off_skey, off_smeta,
        off_sstamp, off_swit, off_tmp, off_arena;
    uint32_t lds_bytes;
    uint32_t small_regs;             // stitching kernel: its pool for small requests is held in registers (cap_free <= 192)
    uint64_t ws_stride;              // workspace bytes per trace
    // fine-grained variant only (see replay_fine.hpp)
    uint32_t off_bnd, off_soff;      // block-start bitmap; list places of the sBlocks
    uint32_t bmp_words;              // words per bitmap that scans may read (a multiple of 4: they are read 16 bytes at a time)
    uint32_t gran_shift;             // a list starts on a multiple of 2^gran_shift 8-byte words of the arena
    uint32_t cap_grans;              // granules per arena half
    uint64_t ws_half;                // bytes of one arena half; the second starts there
    uint32_t ws_tbl_bytes;           // tables in the workspace: bytes of each (witnesses, list places), behind the halves; else 0
    uint32_t reserved_pad;
    // second pass over the traces whose tables overflowed (see ReplayPlan::retry)
    uint32_t retry;                  // this launch is that pass: traces without an overflow flag are left alone
    uint32_t retry_slots;            // traces it has workspace for
    uint64_t retry_ws_off;           // where that workspace starts (bytes from the start of the caller's workspace)
};

struct ReplayPlan {
    KParams kp[2];                   // [0] splitting kernel, [1] stitching kernel
    bool fine;                       // stitching kernel: the fine-grained variant (lists in the workspace)
    bool wide;                       // fine-grained variant with 32-bit chunk numbers (more than 65,000 chunks)
    int tbl_ws;                      // fine-grained variant: 0 the sBlock tables in LDS; 2 witnesses and list places in the workspace; 3 sizes too
    bool slot_regs;                  // slot table in registers (at most 64 slots)
    bool fl_regs;                    // splitting policy: inactive blocks in registers (at most 320)
    uint32_t fl_tiles;               // ... in that many registers per lane: 3 (at most 192 blocks) or 5; 0: in LDS
    size_t ws_bytes;
    bool has_retry;                  // a second pass with the plan below follows the first
};

namespace plan_detail {

const uint64_t UNIT = 512;
const uint64_t ENGINE_MAX_BYTES = 1ull << 39;       // 30-bit block addresses in 512-byte units
const uint64_t LDS_PER_CU = 160 * 1024;
const uint32_t TABLE_MAX = 1u << 24;                // upper bound of every per-trace table size

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }
inline bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }

// Per-wave LDS layout, in 64-bit arithmetic (a table size that would wrap a 32-bit offset must end
// as "too big", not as a small layout).  Returns the bytes needed.
inline uint64_t layout(KParams &k, int policy, const vms_config &c, const ReplayPlan &p)
{
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) {
        uint64_t at = off;
        off = align_up(off + bytes, 16);
        return (uint32_t)(at <= 0xFFFFFFFFu ? at : 0xFFFFFFFFu);
    };
    k.off_slot_req = k.off_slot_a = k.off_slot_b = k.off_slot_c = 0;
    k.off_pool = k.off_bmp = k.off_skey = k.off_smeta = k.off_sstamp = k.off_swit = k.off_tmp = k.off_arena = 0;
    k.off_bnd = k.off_soff = 0;
    if (policy) take(256);      // scalars of the trace (see replay_kernels.hpp)
    if (!p.slot_regs) {
        k.off_slot_req = take((uint64_t)c.max_slots * 4);
        k.off_slot_a = take((uint64_t)c.max_slots * 4);
        k.off_slot_b = policy ? take((uint64_t)c.max_slots * 4) : 0;
        k.off_slot_c = policy && p.fine ? take((uint64_t)c.max_slots * 2) : 0;   // 16-bit list places
    }
    // the splitting policy keeps small pools in registers: no LDS array then
    // (up to 320 blocks; the stitching policy's pool for small requests: up to 192)
    k.off_fl = k.cap_free <= (policy ? 192u : 320u) ? 0 : take(((uint64_t)k.cap_free + 128) * 8);   // 128 spare places: scans read whole tiles
    if (policy && p.fine) {
        const uint64_t idx = p.wide ? 4 : 2;                    // bytes of a chunk number
        k.off_pool = take(((uint64_t)k.cap_pblocks + 80) * 2 * idx);      // 64 spare places, and moves of whole 16-byte blocks
        k.off_bmp = take(((uint64_t)k.bmp_words + 1) * 4);      // and one spare word
        k.off_bnd = take(((uint64_t)k.bmp_words + 1) * 4);      // scans read one word ahead
        k.off_tmp = take(((uint64_t)k.bmp_words + 64) * 4);     // and 64 spare words
        if (p.tbl_ws != 3) k.off_skey = take(((uint64_t)c.max_sblocks + 80) * idx);    // 64 spare places, and shifts move whole 16-byte blocks
        if (!p.tbl_ws) {
            k.off_swit = take(((uint64_t)c.max_sblocks + 80) * idx);
            k.off_soff = take(((uint64_t)c.max_sblocks + 80) * 2);
        }
    } else if (policy) {
        // 64 spare places behind each searched array: reads there need no bounds check
        k.off_pool = take(((uint64_t)c.max_pblocks + 64) * 8);
        k.off_bmp = take(((uint64_t)c.max_chunks + 31) / 32 * 4 + 4);     // and one spare bitmap word
        k.off_skey = take(((uint64_t)c.max_sblocks + 64) * 8);
        k.off_smeta = take(((uint64_t)c.max_sblocks + 64) * 4);
        k.off_sstamp = take(((uint64_t)c.max_sblocks + 64) * 4);
        k.off_swit = take(((uint64_t)c.max_sblocks + 64) * 4);
        k.off_tmp = take(((uint64_t)c.max_chunks + 31) / 32 * 4 + 256);   // and 64 spare words
        k.off_arena = take(((uint64_t)c.max_runs + 64) * 4);
    }
    k.lds_bytes = (uint32_t)(off <= 0xFFFFFFFFu ? off : 0xFFFFFFFFu);
    return off;
}

}  // namespace plan_detail

// The plan for cfg with the variant it names (0: flat unless the tables are too large for it).
// VMS_OK, VMS_EINVAL / VMS_ESTRUCT for a configuration that makes no sense, VMS_ETOOBIG for tables
// that do not fit a compute unit's LDS.  Touches no device.
inline int replay_plan_for(const vms_config *cfg, ReplayPlan &p)
{
    using namespace plan_detail;
    if (!cfg) return VMS_EINVAL;
    if (cfg->struct_size != sizeof(vms_config)) return VMS_ESTRUCT;
    const vms_config &c = *cfg;
    if (c.n_traces == 0 || c.max_events == 0 || c.max_slots == 0) return VMS_EINVAL;
    if ((c.policy_mask & ~3u) || c.policy_mask == 0) return VMS_EINVAL;
    if (!is_pow2(c.chunk_bytes) || c.chunk_bytes < UNIT || c.chunk_bytes > (1ull << 30)) return VMS_EINVAL;
    if (c.small_limit_bytes > c.chunk_bytes || c.small_limit_bytes % UNIT) return VMS_EINVAL;
    if (c.frag_limit_bytes % c.chunk_bytes) return VMS_EINVAL;
    if (c.max_free_blocks == 0 || c.max_pblocks < 4 || c.max_runs < 4 || c.max_runs > TABLE_MAX || c.max_chunks == 0)
        return VMS_EINVAL;
    if (c.max_chunks > TABLE_MAX) return VMS_EINVAL;
    if (c.max_sblocks < c.spool_threshold + 3) return VMS_EINVAL;
    if ((uint64_t)c.max_chunks * c.chunk_bytes > ENGINE_MAX_BYTES) return VMS_EINVAL;
    if ((uint64_t)c.n_traces * c.max_events > (1ull << 40)) return VMS_EINVAL;
    if (c.max_small_blocks > 192) return VMS_EINVAL;            // that pool is held in registers
    // table sizes no LDS could hold: too big, whatever a 32-bit layout would make of them
    if (c.max_slots > TABLE_MAX || c.max_free_blocks > TABLE_MAX || c.max_pblocks > TABLE_MAX || c.max_sblocks > TABLE_MAX ||
        c.max_multi_pblocks > TABLE_MAX)
        return VMS_ETOOBIG;

    memset(&p, 0, sizeof p);
    if (c.variant > VMS_VARIANT_FINE || c.table_place > VMS_TABLES_WORKSPACE_ALL) return VMS_EINVAL;
    // tables beyond what flat sorted LDS arrays serve (lists of more than 64 KB, thousands of blocks)
    // need the fine-grained variant with its lists in the workspace
    const bool big = c.max_runs > 16384 || c.max_pblocks > 4096 || c.max_sblocks > 4096;
    if (big && c.variant == VMS_VARIANT_FLAT) return VMS_ETOOBIG;
    p.fine = big || c.variant == VMS_VARIANT_FINE;
    p.wide = c.max_chunks > 63000;
    p.tbl_ws = p.fine && !p.wide && c.table_place >= VMS_TABLES_WORKSPACE ? (int)c.table_place : 0;
    if (c.table_place >= VMS_TABLES_WORKSPACE && p.fine && p.wide) return VMS_EINVAL;
    p.slot_regs = c.max_slots <= 64;
    p.fl_tiles = c.max_free_blocks <= 192 ? 3u : c.max_free_blocks <= 320 ? 5u : 0u;
    p.fl_regs = p.fl_tiles != 0;
    uint32_t shift = 0;
    while ((UNIT << shift) < c.chunk_bytes) shift++;
    const uint64_t cap = c.capacity_bytes ? (c.capacity_bytes < ENGINE_MAX_BYTES ? c.capacity_bytes : ENGINE_MAX_BYTES)
                                          : ENGINE_MAX_BYTES;
    for (int pol = 0; pol < 2; pol++) {
        KParams &k = p.kp[pol];
        k.n_traces = c.n_traces;
        k.max_events = c.max_events;
        k.chunk_shift = shift;
        k.small_limit_units = (uint32_t)(c.small_limit_bytes / UNIT);
        k.frag_limit_chunks = (uint32_t)(c.frag_limit_bytes / c.chunk_bytes);
        k.spool_threshold = c.spool_threshold;
        k.capacity_units = (uint32_t)(cap / UNIT);
        k.max_slots = c.max_slots;
        // the stitching policy's pool for small requests may be given a size of its own
        k.cap_free = pol && c.max_small_blocks ? c.max_small_blocks : c.max_free_blocks;
        k.small_regs = pol && k.cap_free <= 192;
        k.cap_pblocks = c.max_pblocks;
        k.cap_sblocks = c.max_sblocks;
        k.cap_runs = c.max_runs;
        k.cap_chunks = c.max_chunks;
        k.ws_stride = 0;
        if (pol && p.fine) {
            // pool[] holds the pBlocks of two or more chunks only; its rank search covers 4096 keys,
            // the one over the sBlocks 8064
            k.cap_pblocks = c.max_multi_pblocks ? c.max_multi_pblocks : (c.max_pblocks < 4096 ? c.max_pblocks : 4096);
            if (k.cap_pblocks > 4096 || c.max_sblocks > 8000) return VMS_ETOOBIG;
            k.bmp_words = (uint32_t)align_up((uint64_t)c.max_chunks / 32 + 1, 4);
            // The arena holds 8-byte words: per sBlock two header words and at most one word per
            // run, rounded up to whole granules of 2^gran_shift words.  List places are 16-bit
            // granule numbers; a slot table in LDS keeps them in 15 bits beside a mark.
            const uint64_t words = (uint64_t)c.max_runs + 5ull * c.max_sblocks;
            k.gran_shift = 2;
            while ((words >> k.gran_shift) > (p.slot_regs ? 65535u : 32767u)) k.gran_shift++;
            k.cap_grans = (uint32_t)(words >> k.gran_shift);
            if (k.cap_grans < 4) return VMS_EINVAL;
            // two halves (the lists, and where compaction copies them), each followed by 64 spare words;
            // behind them the two 16-bit tables, if they are kept here
            k.ws_half = align_up((((uint64_t)k.cap_grans << k.gran_shift) + 64) * 8, 256);
            k.ws_tbl_bytes = p.tbl_ws ? (uint32_t)align_up(((uint64_t)c.max_sblocks + 80) * 2, 256) : 0u;
            k.ws_stride = 2 * k.ws_half + (uint64_t)p.tbl_ws * k.ws_tbl_bytes;          // (2 or 3 tables)
        } else if (pol) {
            k.ws_stride = align_up(((uint64_t)c.max_runs + 64) * 4, 256);     // where compaction copies the lists
        }
        const uint64_t need = layout(k, pol, c, p);
        if ((c.policy_mask & (1u << pol)) && need > LDS_PER_CU) return VMS_ETOOBIG;
    }
    p.ws_bytes = (c.policy_mask & VMS_POLICY_VMS) ? (size_t)p.kp[1].ws_stride * c.n_traces : 0;
    return VMS_OK;
}

// Wavefronts of the stitching kernel that share a compute unit: LDS is handed out in granules of
// 1,280 bytes, 128 of them per compute unit (measured: 31,680 B per wavefront gives five wavefronts
// per compute unit, 32,576 B four).
inline uint32_t plan_waves_per_cu(const ReplayPlan &x)
{
    const uint64_t granules = ((uint64_t)x.kp[1].lds_bytes + 1279) / 1280;
    const uint64_t w = granules ? plan_detail::LDS_PER_CU / 1280 / granules : 32;
    return (uint32_t)(w < 32 ? w : 32);                     // a compute unit holds 32 wavefronts at most
}

// The plan for cfg.  With variant 0 the library chooses: a trace replays about twice as fast on the
// flat variant (its lists are in LDS), but when the batch does not fit the compute units at once and
// the fine-grained variant holds at least 2.5 times as many traces per compute unit, the latter
// finishes the batch sooner.  With table_place 0 it chooses where the fine-grained variant keeps the
// tables of the sBlocks: throughput grows almost in proportion to the wavefronts per compute unit
// (measured from 4 to 9) while a wavefront with tables in the workspace is slower, so the workspace it
// is when the LDS layout leaves fewer than two wavefronts per SIMD and the batch then takes fewer
// rounds of wavefronts by more than the wavefronts lose.
inline int replay_plan_make(const vms_config *cfg, ReplayPlan &p)
{
    int rc = replay_plan_for(cfg, p);
    if (rc != VMS_OK || !cfg || !(cfg->policy_mask & VMS_POLICY_VMS)) return rc;
    const uint32_t CUS = 256;
    if (cfg->variant == VMS_VARIANT_AUTO && !p.fine) {
        vms_config alt = *cfg;
        alt.variant = VMS_VARIANT_FINE;
        ReplayPlan q;
        if (replay_plan_for(&alt, q) == VMS_OK) {
            const uint32_t flat = plan_waves_per_cu(p), fine = plan_waves_per_cu(q);
            if ((uint64_t)cfg->n_traces > (uint64_t)CUS * flat && 2 * fine >= 5 * flat) p = q;
        }
    }
    if (p.fine && !p.wide && cfg->table_place == VMS_TABLES_AUTO) {
        // rounds of wavefronts the batch takes, times what a wavefront pays for tables in the workspace
        // (measured on offloading traces: 1.2 with two tables there, 1.45 with all three)
        auto cost = [&](const ReplayPlan &x, uint32_t tenths) {
            const uint64_t slots = (uint64_t)CUS * plan_waves_per_cu(x);
            return ((cfg->n_traces + slots - 1) / slots) * tenths;
        };
        uint64_t best = cost(p, 100);
        if (plan_waves_per_cu(p) < 8)
            for (uint32_t place = VMS_TABLES_WORKSPACE; place <= VMS_TABLES_WORKSPACE_ALL; place++) {
                vms_config alt = *cfg;
                alt.variant = VMS_VARIANT_FINE;
                alt.table_place = place;
                ReplayPlan q;
                if (replay_plan_for(&alt, q) != VMS_OK) continue;
                const uint64_t c = cost(q, place == VMS_TABLES_WORKSPACE ? 120 : 145);
                if (c < best) {
                    best = c;
                    p = q;
                }
            }
    }
    return VMS_OK;
}

// The plan of the second pass for cfg: every table doubled, as far as the fine-grained variant and a
// compute unit's LDS allow.  VMS_OK and q.has_retry = false if no larger plan exists.
inline int replay_plan_retry(const vms_config *cfg, const ReplayPlan &first, ReplayPlan &q)
{
    memset(&q, 0, sizeof q);
    if (!cfg->retry_traces) return VMS_OK;
    vms_config big = *cfg;
    auto twice = [](uint32_t x, uint32_t cap) -> uint32_t { return (uint64_t)x * 2 > cap ? cap : x * 2; };
    big.variant = VMS_VARIANT_FINE;
    big.max_free_blocks = twice(cfg->max_free_blocks, 1u << 14);
    big.max_small_blocks = 0;
    big.max_pblocks = twice(cfg->max_pblocks, 1u << 20);
    big.max_multi_pblocks = twice(first.fine ? first.kp[1].cap_pblocks : cfg->max_pblocks, 4096);
    big.max_sblocks = twice(cfg->max_sblocks, 8000);
    big.max_runs = twice(cfg->max_runs < (1u << 16) ? (1u << 16) : cfg->max_runs, plan_detail::TABLE_MAX);
    big.max_chunks = twice(cfg->max_chunks, plan_detail::TABLE_MAX);
    while ((uint64_t)big.max_chunks * big.chunk_bytes > plan_detail::ENGINE_MAX_BYTES) big.max_chunks /= 2;
    // shrink towards the first pass's sizes until the tables fit
    for (int tries = 0; tries < 8; tries++) {
        const int rc = replay_plan_for(&big, q);
        if (rc == VMS_OK) {
            q.has_retry = true;
            for (int pol = 0; pol < 2; pol++) {
                q.kp[pol].retry = 1;
                q.kp[pol].retry_slots = cfg->retry_traces;
                q.kp[pol].retry_ws_off = first.ws_bytes;
            }
            q.ws_bytes = (cfg->policy_mask & VMS_POLICY_VMS) ? (size_t)q.kp[1].ws_stride * cfg->retry_traces : 0;
            return VMS_OK;
        }
        if (rc != VMS_ETOOBIG) return rc;
        big.max_chunks = big.max_chunks / 2 > cfg->max_chunks ? big.max_chunks / 2 : cfg->max_chunks;
        big.max_sblocks = big.max_sblocks * 3 / 4 > cfg->max_sblocks ? big.max_sblocks * 3 / 4 : cfg->max_sblocks;
        big.max_free_blocks = big.max_free_blocks / 2 > cfg->max_free_blocks ? big.max_free_blocks / 2 : cfg->max_free_blocks;
    }
    memset(&q, 0, sizeof q);
    return VMS_OK;
}

#endif
