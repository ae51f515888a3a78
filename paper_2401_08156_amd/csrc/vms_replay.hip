// Host side of the C ABI declared in include/vms_replay.h: validates the
// configuration, lays out the per-wavefront LDS arrays, launches the replay
// kernels and copies statistics back.  No allocator logic lives here.
#include <hip/hip_runtime.h>
#include <new>
#include <string.h>

#include "replay_kernels.hpp"
#include "replay_fine.hpp"
#include "selftest.hpp"

namespace {

const uint32_t LDS_PER_CU = 160 * 1024;

// Workspace for callers that cannot allocate (vms_replay_run_static): one array per device, part of
// the loaded code object, held until the process ends.  In host code the name below is only a
// handle for hipGetSymbolAddress; the device address it yields is what the kernels are given.
const size_t STATIC_WS_BYTES = (size_t)32 << 20;
const int STATIC_WS_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_WS_BYTES];
void *g_scratch_ptr[STATIC_WS_DEVICES];     // per device: address of its copy of scratch[]

}  // namespace

struct vms_replay {
    vms_config cfg;
    ReplayPlan plan;            // kernel variants, LDS layouts, workspace slice (replay_plan.hpp)
    ReplayPlan retry;           // the same for the second pass over traces that outgrew the tables (has_retry)
    vms_trace_stats *d_stats;
    vms_summary *d_summary;
    hipEvent_t ev[6];           // run start, stitching kernel end, splitting kernel start / end, run end, side stream done
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

// Batch summary (Sec. 5.1, memory reduction ratio): one wavefront reduces the statistics.
__global__ __launch_bounds__(64) void summary_kernel(const vms_trace_stats *__restrict__ stats, u32 n_traces,
                                                     u32 policy_mask, vms_summary *__restrict__ out)
{
    __shared__ u64 acc[64 * 3];
    __shared__ double facc[64 * 2];
    const u32 lane = lane_id();
    vms_summary r;
    for (int p = 0; p < 2; p++) {
        u64 res = 0, act = 0, flagged = 0;
        double fmax = 0.0, fsum = 0.0;
        if (policy_mask & (1u << p)) {
            for (u32 t = lane; t < n_traces; t += 64) {
                const vms_trace_stats &s = stats[(size_t)p * n_traces + t];
                res += s.peak_reserved;
                act += s.peak_active;
                flagged += s.status != 0;
                fmax = fmax > s.fragmentation ? fmax : s.fragmentation;
            }
        }
        acc[lane] = res;
        acc[64 + lane] = act;
        acc[128 + lane] = flagged;
        facc[lane] = fmax;
        __syncthreads();
        if (lane == 0) {
            res = act = flagged = 0;
            fmax = 0.0;
            for (int i = 0; i < 64; i++) {
                res += acc[i];
                act += acc[64 + i];
                flagged += acc[128 + i];
                fmax = fmax > facc[i] ? fmax : facc[i];
            }
            // the mean is summed in trace order so that it does not depend on the lane split
            if (policy_mask & (1u << p))
                for (u32 t = 0; t < n_traces; t++) fsum += stats[(size_t)p * n_traces + t].fragmentation;
            r.sum_peak_reserved[p] = res;
            r.sum_peak_active[p] = act;
            r.n_flagged[p] = flagged;
            r.max_fragmentation[p] = fmax;
            r.mean_fragmentation[p] = n_traces ? fsum / (double)n_traces : 0.0;
        }
        __syncthreads();
    }
    if (lane == 0) {
        r.mem_reduction_ratio = 0.0;
        if (policy_mask == 3u && r.sum_peak_reserved[0])
            r.mem_reduction_ratio = (double)((long long)r.sum_peak_reserved[0] - (long long)r.sum_peak_reserved[1]) /
                                    (double)r.sum_peak_reserved[0];
        *out = r;
    }
}

static int selftest_run()
{
    u32 *d = nullptr, h = 0xFFFFFFFFu;
    if (hipMalloc((void **)&d, sizeof(u32)) != hipSuccess) return VMS_EHIP;
    hipLaunchKernelGGL(selftest_kernel, dim3(1), dim3(64), 0, 0, d);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpy(&h, d, sizeof h, hipMemcpyDeviceToHost);
    (void)hipFree(d);
    if (e != hipSuccess) return VMS_EHIP;
    return h == 0 ? VMS_OK : -(int)(1000 + (h & 0xFFFF));
}

typedef void (*vms_fn)(KParams, const u64 *, const u32 *, u64 *, vms_trace_stats *, char *);
typedef void (*split_fn)(KParams, const u64 *, const u32 *, u64 *, vms_trace_stats *);

// the kernel variants: flat sorted tables in LDS or the fine-grained layout (16- or 32-bit chunk
// numbers; witness and list-place tables in LDS or in the workspace), slot table in LDS or registers
vms_fn pick_vms(const ReplayPlan &p)
{
    if (p.fine) {
        if (p.wide) return p.slot_regs ? replay_vms_fine_kernel<true, u32, 0> : replay_vms_fine_kernel<false, u32, 0>;
        if (p.tbl_ws == 3) return p.slot_regs ? replay_vms_fine_kernel<true, u16, 3> : replay_vms_fine_kernel<false, u16, 3>;
        if (p.tbl_ws) return p.slot_regs ? replay_vms_fine_kernel<true, u16, 2> : replay_vms_fine_kernel<false, u16, 2>;
        return p.slot_regs ? replay_vms_fine_kernel<true, u16, 0> : replay_vms_fine_kernel<false, u16, 0>;
    }
    return p.slot_regs ? replay_vms_kernel<true> : replay_vms_kernel<false>;
}
// fl_tiles: the splitting pool's inactive blocks fit three or five registers per lane (at most 192 / 320 blocks)
split_fn pick_split(bool slot_regs, uint32_t fl_tiles)
{
    if (fl_tiles == 3) return slot_regs ? replay_split_kernel<true, 3> : replay_split_kernel<false, 3>;
    if (fl_tiles == 5) return slot_regs ? replay_split_kernel<true, 5> : replay_split_kernel<false, 5>;
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
    ReplayPlan plan;
    const int prc = replay_plan_make(cfg, plan);      // refuses bad or oversized tables before any device call
    if (prc != VMS_OK) return prc;
    const vms_config &c = *cfg;

    vms_replay *h = new (std::nothrow) vms_replay;
    if (!h) return VMS_ENOMEM;
    memset(h, 0, sizeof *h);
    h->cfg = c;
    h->plan = plan;
    const int rrc = replay_plan_retry(cfg, plan, h->retry);
    if (rrc != VMS_OK) {
        delete h;
        return rrc;
    }
    if (h->retry.has_retry)
        for (int pol = 0; pol < 2; pol++) h->plan.kp[pol].retry_slots = c.retry_traces;    // the first pass resets the count
    h->ws_bytes = plan.ws_bytes + h->retry.ws_bytes;

    if (hipGetDevice(&h->device) != hipSuccess) {
        delete h;
        return VMS_EHIP;
    }
    // one record more than the traces need: its first word counts the traces the second pass takes on
    hipError_t e = hipMalloc((void **)&h->d_stats, sizeof(vms_trace_stats) * (2 * (size_t)c.n_traces + 1));
    // records of a policy that never runs stay zero; a run rewrites every record of its policies
    if (e == hipSuccess) e = hipMemset(h->d_stats, 0, sizeof(vms_trace_stats) * (2 * (size_t)c.n_traces + 1));
    if (e == hipSuccess) e = hipMalloc((void **)&h->d_summary, sizeof(vms_summary));
    for (int i = 0; i < 6 && e == hipSuccess; i++) e = hipEventCreate(&h->ev[i]);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking);
    // LDS above 64 KB per workgroup has to be requested explicitly
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)pick_split(h->plan.slot_regs, h->plan.fl_tiles), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)LDS_PER_CU);
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)pick_vms(h->plan), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)LDS_PER_CU);
    if (e == hipSuccess && h->retry.has_retry)
        e = hipFuncSetAttribute((const void *)pick_split(h->retry.slot_regs, h->retry.fl_tiles),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_PER_CU);
    if (e == hipSuccess && h->retry.has_retry)
        e = hipFuncSetAttribute((const void *)pick_vms(h->retry), hipFuncAttributeMaxDynamicSharedMemorySize,
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
    out[0] = h->plan.kp[0].lds_bytes;
    out[1] = h->plan.kp[1].lds_bytes;
    return VMS_OK;
}

static inline uint32_t second_pass_waves(const vms_config &c) { return c.retry_traces < c.n_traces ? c.retry_traces : c.n_traces; }

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
        hipLaunchKernelGGL(pick_vms(h->plan), dim3(c.n_traces), dim3(64), h->plan.kp[1].lds_bytes, st, h->plan.kp[1],
                           d_events, d_n_events, d_dec_vms, h->d_stats, (char *)d_workspace);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->ev[1], st));       // the kernel times are those of the first pass
    if ((c.policy_mask & VMS_POLICY_VMS) && h->retry.has_retry) {
        // second pass: retry_traces wavefronts with larger tables replay the traces whose tables overflowed
        hipLaunchKernelGGL(pick_vms(h->retry), dim3(second_pass_waves(c)), dim3(64), h->retry.kp[1].lds_bytes, st, h->retry.kp[1],
                           d_events, d_n_events, d_dec_vms, h->d_stats, (char *)d_workspace);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->ev[2], sst));
    if (c.policy_mask & VMS_POLICY_SPLIT) {
        hipLaunchKernelGGL(pick_split(h->plan.slot_regs, h->plan.fl_tiles), dim3(c.n_traces), dim3(64), h->plan.kp[0].lds_bytes, sst, h->plan.kp[0],
                           d_events, d_n_events, d_dec_split, h->d_stats);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->ev[3], sst));
    if ((c.policy_mask & VMS_POLICY_SPLIT) && h->retry.has_retry) {
        hipLaunchKernelGGL(pick_split(h->retry.slot_regs, h->retry.fl_tiles), dim3(second_pass_waves(c)), dim3(64),
                           h->retry.kp[0].lds_bytes, sst, h->retry.kp[0], d_events, d_n_events, d_dec_split, h->d_stats);
        HIP_TRY(h, hipGetLastError());
    }
    HIP_TRY(h, hipEventRecord(h->ev[5], sst));
    if (both) HIP_TRY(h, hipStreamWaitEvent(st, h->ev[5], 0));
    HIP_TRY(h, hipEventRecord(h->ev[4], st));
    h->last_stream = st;
    h->ran = true;
    return VMS_OK;
}

size_t vms_replay_static_workspace_bytes(void) { return STATIC_WS_BYTES; }

int vms_replay_run_static(vms_replay *h, const uint64_t *d_events, const uint32_t *d_n_events, uint64_t *d_dec_split,
                          uint64_t *d_dec_vms, void *hip_stream)
{
    if (!h || !d_events) return VMS_EINVAL;
    if (h->ws_bytes > STATIC_WS_BYTES) return VMS_EWORKSPACE;   // this handle needs more than the built-in array holds
    int dev = -1;
    HIP_TRY(h, hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_WS_DEVICES || dev != h->device) return VMS_EINVAL;
    if (!g_scratch_ptr[dev]) {
        // once per device, with that device current: every device holds its own copy of the array
        void *p = nullptr;
        HIP_TRY(h, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255)) return VMS_EWORKSPACE;
        g_scratch_ptr[dev] = p;
    }
    // Nothing in the array has to start at zero: the kernels write every word of a trace's slice
    // before they read it.  Calls that overlap on one device share the array and race.
    return vms_replay_run(h, d_events, d_n_events, d_dec_split, d_dec_vms, h->ws_bytes ? g_scratch_ptr[dev] : nullptr,
                          hip_stream);
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
    for (int i = 0; i < 6; i++)
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
