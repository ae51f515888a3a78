// Host side of the C ABI declared in include/vms_replay.h: validates the
// configuration, lays out the per-wavefront LDS arrays, launches the replay
// kernels and copies statistics back.  No allocator logic lives here.
#include <hip/hip_runtime.h>
#include <new>
#include <string.h>

#include "replay_kernels.hpp"
#include "selftest.hpp"

namespace {

const uint64_t UNIT = 512;
const uint64_t ENGINE_MAX_BYTES = 1ull << 39;       // 30-bit block addresses in 512-byte units
const uint32_t LDS_PER_CU = 160 * 1024;

uint32_t align_up(uint32_t x, uint32_t a) { return (x + a - 1) / a * a; }

bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }

}  // namespace

struct vms_replay {
    vms_config cfg;
    KParams kp[2];              // [0] splitting kernel, [1] stitching kernel
    bool big;                   // sBlock chunk runs in global memory (see VmsT)
    bool slot_regs;             // slot table in registers (see SlotsT)
    bool fl_regs;               // splitting policy: inactive blocks in registers (see SplitRegs)
    vms_trace_stats *d_stats;
    vms_summary *d_summary;
    hipEvent_t ev[5];           // run start, VMS kernel end, split kernel start / end, run end
    hipStream_t side;           // the splitting kernel runs here, beside the stitching kernel
    hipStream_t last_stream;
    int device;
    int last_hip;
    bool ran;
    size_t ws_bytes;
};

namespace {

int hip_fail(vms_replay *h, hipError_t e)
{
    if (h) h->last_hip = (int)e;
    return VMS_EHIP;
}

#define HIP_TRY(h, call)                              \
    do {                                              \
        hipError_t e_ = (call);                       \
        if (e_ != hipSuccess) return hip_fail(h, e_); \
    } while (0)

// Per-wave LDS layout.  The splitting kernel only needs the slot table and its free list; with at
// most 64 slots the slot table lives in registers and takes no LDS at all.
// stamps_ws: the last-use stamps of the sBlocks move to the trace's slice of the global workspace
// (tables that would not fit the LDS otherwise; the hot path only ever stores to them).
void layout(KParams &k, int policy, const vms_config &c, bool big, bool slot_regs, bool stamps_ws)
{
    uint32_t off = 0;
    auto take = [&](uint32_t bytes) {
        uint32_t at = off;
        off = align_up(off + bytes, 16);
        return at;
    };
    k.off_slot_req = k.off_slot_a = k.off_slot_b = k.off_slot_c = 0;
    if (policy) take(256);      // scalars of the trace (see replay_kernels.hpp)
    if (!slot_regs) {
        k.off_slot_req = take(c.max_slots * 4);
        k.off_slot_a = take(c.max_slots * 4);
        k.off_slot_b = policy ? take(c.max_slots * 4) : 0;
    }
    // the splitting policy keeps small pools in registers: no LDS array then
    k.off_fl = k.cap_free <= 192 ? 0 : take((k.cap_free + 128) * 8);   // 128 spare places: scans read whole tiles
    if (policy) {
        // 64 spare places behind each searched array: reads there need no bounds check
        k.off_pool = take((c.max_pblocks + 64) * 8);
        k.off_bmp = take((c.max_chunks + 31) / 32 * 4 + 4);     // and one spare bitmap word
        k.off_skey = take((c.max_sblocks + 64) * 8);
        k.off_smeta = take((c.max_sblocks + 64) * (big ? 8 : 4));
        k.off_sstamp = stamps_ws ? 0 : take((c.max_sblocks + 64) * 4);
        k.off_swit = take((c.max_sblocks + 64) * 4);
        k.off_tmp = take((c.max_chunks + 31) / 32 * 4 + 256);   // and 64 spare words
        k.off_arena = big ? 0 : take((c.max_runs + 64) * 4);
    } else {
        k.off_pool = k.off_bmp = k.off_skey = k.off_smeta = k.off_sstamp = k.off_swit = k.off_tmp = k.off_arena = 0;
    }
    k.lds_bytes = off;
}

typedef void (*vms_fn)(KParams, const u64 *, const u32 *, u64 *, vms_trace_stats *, char *);
typedef void (*split_fn)(KParams, const u64 *, const u32 *, u64 *, vms_trace_stats *);

// the kernel variants: chunk-run lists in HBM or LDS, slot table in LDS or registers
vms_fn pick_vms(bool big, bool slot_regs)
{
    if (big) return slot_regs ? replay_vms_kernel<true, true> : replay_vms_kernel<true, false>;
    return slot_regs ? replay_vms_kernel<false, true> : replay_vms_kernel<false, false>;
}
// fl_regs: the splitting pool's inactive blocks fit three registers per lane (at most 192 blocks)
split_fn pick_split(bool slot_regs, bool fl_regs)
{
    if (fl_regs) return slot_regs ? replay_split_kernel<true, 3> : replay_split_kernel<false, 3>;
    return slot_regs ? replay_split_kernel<true, 0> : replay_split_kernel<false, 0>;
}

}  // namespace

extern "C" {

void vms_config_default(vms_config *cfg, uint32_t n_traces, uint32_t max_events, uint32_t max_slots)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->struct_size = (uint32_t)sizeof(vms_config);
    cfg->n_traces = n_traces;
    cfg->max_events = max_events;
    cfg->policy_mask = VMS_POLICY_SPLIT | VMS_POLICY_VMS;
    cfg->chunk_bytes = 2u << 20;
    cfg->small_limit_bytes = cfg->chunk_bytes;
    cfg->frag_limit_bytes = cfg->chunk_bytes;
    cfg->capacity_bytes = 0;
    cfg->spool_threshold = 512;
    cfg->max_slots = max_slots ? max_slots : 1;
    cfg->max_free_blocks = 512;
    cfg->max_pblocks = 1024;
    cfg->max_sblocks = 640;
    cfg->max_runs = 4096;
    cfg->max_chunks = 32768;    // 64 GiB of 2 MiB chunks
}

int vms_replay_create(const vms_config *cfg, vms_replay **out)
{
    if (!cfg || !out) return VMS_EINVAL;
    *out = nullptr;
    if (cfg->struct_size != sizeof(vms_config)) return VMS_ESTRUCT;
    const vms_config &c = *cfg;
    if (c.n_traces == 0 || c.max_events == 0 || c.max_slots == 0) return VMS_EINVAL;
    if ((c.policy_mask & ~3u) || c.policy_mask == 0) return VMS_EINVAL;
    if (!is_pow2(c.chunk_bytes) || c.chunk_bytes < UNIT || c.chunk_bytes > (1ull << 30)) return VMS_EINVAL;
    if (c.small_limit_bytes > c.chunk_bytes || c.small_limit_bytes % UNIT) return VMS_EINVAL;
    if (c.frag_limit_bytes % c.chunk_bytes) return VMS_EINVAL;
    if (c.max_free_blocks == 0 || c.max_pblocks < 4 || c.max_runs < 4 || c.max_runs > (1u << 24) || c.max_chunks == 0)
        return VMS_EINVAL;
    if (c.max_chunks > (1u << 24)) return VMS_EINVAL;
    if (c.max_sblocks < c.spool_threshold + 3) return VMS_EINVAL;
    if ((uint64_t)c.max_chunks * c.chunk_bytes > ENGINE_MAX_BYTES) return VMS_EINVAL;
    if ((uint64_t)c.n_traces * c.max_events > (1ull << 40)) return VMS_EINVAL;

    vms_replay *h = new (std::nothrow) vms_replay;
    if (!h) return VMS_ENOMEM;
    memset(h, 0, sizeof *h);
    h->cfg = c;
    // more than 64 KB of chunk-run lists per trace: keep them in HBM; that kernel variant is also
    // the one whose rank searches cope with pools beyond 4096 blocks
    h->big = c.max_runs > 16384 || c.max_pblocks > 4096 || c.max_sblocks > 4096;
    h->slot_regs = c.max_slots <= 64;
    h->fl_regs = c.max_free_blocks <= 192;
    uint32_t shift = 0;
    while ((UNIT << shift) < c.chunk_bytes) shift++;
    const uint64_t cap = c.capacity_bytes ? (c.capacity_bytes < ENGINE_MAX_BYTES ? c.capacity_bytes : ENGINE_MAX_BYTES)
                                          : ENGINE_MAX_BYTES;
    for (int p = 0; p < 2; p++) {
        KParams &k = h->kp[p];
        memset(&k, 0, sizeof k);
        k.n_traces = c.n_traces;
        k.max_events = c.max_events;
        k.chunk_shift = shift;
        k.small_limit_units = (uint32_t)(c.small_limit_bytes / UNIT);
        k.frag_limit_chunks = (uint32_t)(c.frag_limit_bytes / c.chunk_bytes);
        k.spool_threshold = c.spool_threshold;
        k.capacity_units = (uint32_t)(cap / UNIT);
        k.max_slots = c.max_slots;
        // the stitching policy's pool for small requests may be given a size of its own
        k.cap_free = p && c.max_small_blocks ? c.max_small_blocks : c.max_free_blocks;
        k.small_regs = p && k.cap_free <= 192;
        k.cap_pblocks = c.max_pblocks;
        k.cap_sblocks = c.max_sblocks;
        k.cap_runs = c.max_runs;
        k.cap_chunks = c.max_chunks;
        layout(k, p, c, h->big, h->slot_regs, false);
        // compaction buffer, and for the big variant the lists themselves (each with 64 spare entries)
        k.ws_stride = p ? (uint64_t)align_up((c.max_runs + 64) * 4 * (h->big ? 2 : 1), 256) : 0;
        k.ws_stamp_off = 0;
        if (p && h->big && k.lds_bytes > LDS_PER_CU) {
            layout(k, p, c, h->big, h->slot_regs, true);
            k.ws_stamp_off = (uint32_t)k.ws_stride;     // behind the lists: never 0
            k.ws_stride += align_up((c.max_sblocks + 64) * 4, 256);
        }
        if ((c.policy_mask & (1u << p)) && k.lds_bytes > LDS_PER_CU) {
            delete h;
            return VMS_ETOOBIG;
        }
    }
    h->ws_bytes = (c.policy_mask & VMS_POLICY_VMS) ? (size_t)h->kp[1].ws_stride * c.n_traces : 0;

    if (hipGetDevice(&h->device) != hipSuccess) {
        delete h;
        return VMS_EHIP;
    }
    hipError_t e = hipMalloc((void **)&h->d_stats, sizeof(vms_trace_stats) * 2 * (size_t)c.n_traces);
    // records of a policy that never runs stay zero; a run rewrites every record of its policies
    if (e == hipSuccess) e = hipMemset(h->d_stats, 0, sizeof(vms_trace_stats) * 2 * (size_t)c.n_traces);
    if (e == hipSuccess) e = hipMalloc((void **)&h->d_summary, sizeof(vms_summary));
    for (int i = 0; i < 5 && e == hipSuccess; i++) e = hipEventCreate(&h->ev[i]);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking);
    // LDS above 64 KB per workgroup has to be requested explicitly
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)pick_split(h->slot_regs, h->fl_regs), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)LDS_PER_CU);
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)pick_vms(h->big, h->slot_regs), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)LDS_PER_CU);
    if (e != hipSuccess) {
        int rc = e == hipErrorOutOfMemory ? VMS_ENOMEM : VMS_EHIP;
        vms_replay_destroy(h);
        return rc;
    }
    *out = h;
    return VMS_OK;
}

size_t vms_replay_workspace_bytes(const vms_replay *h) { return h ? h->ws_bytes : 0; }

int vms_replay_lds_bytes(const vms_replay *h, uint32_t out[2])
{
    if (!h || !out) return VMS_EINVAL;
    out[0] = h->kp[0].lds_bytes;
    out[1] = h->kp[1].lds_bytes;
    return VMS_OK;
}

int vms_replay_run(vms_replay *h, const uint64_t *d_events, const uint32_t *d_n_events, uint64_t *d_dec_split,
                   uint64_t *d_dec_vms, void *d_workspace, void *hip_stream)
{
    if (!h || !d_events) return VMS_EINVAL;
    const vms_config &c = h->cfg;
    if ((c.policy_mask & VMS_POLICY_VMS) && h->ws_bytes && (!d_workspace || ((uintptr_t)d_workspace & 255)))
        return VMS_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    // Fork: the two policies are independent, so the short splitting kernel runs on a second
    // stream beside the long stitching kernel and the caller's stream joins it at the end.
    HIP_TRY(h, hipEventRecord(h->ev[0], st));
    const bool both = c.policy_mask == (VMS_POLICY_SPLIT | VMS_POLICY_VMS);
    hipStream_t sst = both ? h->side : st;
    if (both) HIP_TRY(h, hipStreamWaitEvent(sst, h->ev[0], 0));
    if (c.policy_mask & VMS_POLICY_VMS) {
        hipLaunchKernelGGL(pick_vms(h->big, h->slot_regs), dim3(c.n_traces), dim3(64), h->kp[1].lds_bytes, st, h->kp[1],
                           d_events, d_n_events, d_dec_vms, h->d_stats, (char *)d_workspace);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->ev[1], st));
    HIP_TRY(h, hipEventRecord(h->ev[2], sst));
    if (c.policy_mask & VMS_POLICY_SPLIT) {
        hipLaunchKernelGGL(pick_split(h->slot_regs, h->fl_regs), dim3(c.n_traces), dim3(64), h->kp[0].lds_bytes, sst, h->kp[0],
                           d_events, d_n_events, d_dec_split, h->d_stats);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->ev[3], sst));
    if (both) HIP_TRY(h, hipStreamWaitEvent(st, h->ev[3], 0));
    HIP_TRY(h, hipEventRecord(h->ev[4], st));
    h->last_stream = st;
    h->ran = true;
    return VMS_OK;
}

int vms_replay_stats(vms_replay *h, vms_trace_stats *h_out, size_t n)
{
    if (!h || !h_out || n != 2 * (size_t)h->cfg.n_traces) return VMS_EINVAL;
    if (!h->ran) return VMS_ESTATE;
    HIP_TRY(h, hipStreamSynchronize(h->last_stream));
    HIP_TRY(h, hipMemcpy(h_out, h->d_stats, sizeof(vms_trace_stats) * n, hipMemcpyDeviceToHost));
    return VMS_OK;
}

int vms_replay_summary(vms_replay *h, vms_summary *h_out)
{
    if (!h || !h_out) return VMS_EINVAL;
    if (!h->ran) return VMS_ESTATE;
    hipLaunchKernelGGL(summary_kernel, dim3(1), dim3(64), 0, h->last_stream, h->d_stats, h->cfg.n_traces,
                       h->cfg.policy_mask, h->d_summary);
    HIP_TRY(h, hipGetLastError());
    HIP_TRY(h, hipStreamSynchronize(h->last_stream));
    HIP_TRY(h, hipMemcpy(h_out, h->d_summary, sizeof(vms_summary), hipMemcpyDeviceToHost));
    return VMS_OK;
}

int vms_replay_last_kernel_ms(vms_replay *h, float out_ms[3])
{
    if (!h || !out_ms) return VMS_EINVAL;
    if (!h->ran) return VMS_ESTATE;
    HIP_TRY(h, hipEventSynchronize(h->ev[4]));
    HIP_TRY(h, hipEventElapsedTime(&out_ms[1], h->ev[0], h->ev[1]));
    HIP_TRY(h, hipEventElapsedTime(&out_ms[0], h->ev[2], h->ev[3]));
    HIP_TRY(h, hipEventElapsedTime(&out_ms[2], h->ev[0], h->ev[4]));
    return VMS_OK;
}

void vms_replay_destroy(vms_replay *h)
{
    if (!h) return;
    if (h->d_stats) (void)hipFree(h->d_stats);
    if (h->d_summary) (void)hipFree(h->d_summary);
    for (int i = 0; i < 5; i++)
        if (h->ev[i]) (void)hipEventDestroy(h->ev[i]);
    if (h->side) (void)hipStreamDestroy(h->side);
    delete h;
}

int vms_replay_last_hip_error(const vms_replay *h) { return h ? h->last_hip : 0; }

const char *vms_strerror(int code)
{
    switch (code) {
    case VMS_OK: return "ok";
    case VMS_EINVAL: return "invalid argument or inconsistent configuration";
    case VMS_ESTRUCT: return "vms_config.struct_size does not match this library";
    case VMS_ENOMEM: return "out of host or device memory";
    case VMS_EWORKSPACE: return "workspace missing or not 256-byte aligned";
    case VMS_EHIP: return "a HIP call failed (see vms_replay_last_hip_error)";
    case VMS_ETOOBIG: return "per-trace tables exceed the 160 KB of LDS of a compute unit";
    case VMS_ESTATE: return "call out of order";
    default: return "unknown error";
    }
}

int vms_selftest(void) { return selftest_run(); }

}  // extern "C"
