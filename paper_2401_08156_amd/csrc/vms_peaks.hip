// Two micro-benchmarks that put the replay's figures into proportion on the device at hand: what a
// plain copy kernel reaches in HBM bandwidth and what a wavefront-wide 16-byte LDS read loop reaches
// in LDS bandwidth.  Diagnostics; not part of a replay.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/vms_replay.h"

namespace {

typedef uint32_t u32;
typedef uint64_t u64;
typedef unsigned int v4u __attribute__((ext_vector_type(4)));     // 16 bytes, a type the nontemporal builtins take

// grid-stride copy: every lane has four 16-byte loads in flight before its first store (64 KB per
// workgroup and trip); n16 is a multiple of 4 * 256
__global__ __launch_bounds__(256) void peaks_copy_kernel(const v4u *__restrict__ src, v4u *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 1024;
    for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
        v4u v[4];
#pragma unroll
        for (int q = 0; q < 4; q++) v[q] = __builtin_nontemporal_load(src + i + q * 256);
#pragma unroll
        for (int q = 0; q < 4; q++) __builtin_nontemporal_store(v[q], dst + i + q * 256);
    }
}

// the same loads without the stores: what reading alone reaches; the xor of what was read is stored once
__global__ __launch_bounds__(256) void peaks_read_kernel(const v4u *__restrict__ src, u32 *out, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 1024;
    v4u acc = { 0, 0, 0, 0 };
    for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
        v4u v[4];
#pragma unroll
        for (int q = 0; q < 4; q++) v[q] = __builtin_nontemporal_load(src + i + q * 256);
#pragma unroll
        for (int q = 0; q < 4; q++) acc ^= v[q];
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

// every lane reads 16 bytes of the workgroup's 32 KB of LDS per trip, `iters` trips, conflict-free
// (consecutive lanes, consecutive 16-byte words); the xor of what was read is stored once
__global__ __launch_bounds__(256) void peaks_lds_kernel(u32 *out, u32 iters)
{
    __shared__ uint4 buf[2048];
    for (u32 i = threadIdx.x; i < 2048; i += 256) buf[i] = make_uint4(i, i * 3u, i * 5u, i * 7u);
    __syncthreads();
    uint4 acc = make_uint4(0, 0, 0, 0);
    u32 at = threadIdx.x;
    for (u32 it = 0; it < iters; it++) {
#pragma unroll
        for (u32 q = 0; q < 8; q++) {
            const uint4 v = buf[(at + q * 256) & 2047];
            acc.x ^= v.x;
            acc.y ^= v.y;
            acc.z ^= v.z;
            acc.w ^= v.w;
        }
        at += acc.x & 1u;           // keeps the loop's reads from being hoisted
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

}  // namespace

extern "C" int vms_measure_peaks(vms_peaks_report *out)
{
    if (!out) return VMS_EINVAL;
    if (out->struct_size != sizeof(vms_peaks_report)) return VMS_ESTRUCT;
    memset((char *)out + sizeof(uint32_t), 0, sizeof *out - sizeof(uint32_t));
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return VMS_EHIP;
    out->compute_units = (uint32_t)prop.multiProcessorCount;
    out->clock_mhz = (uint32_t)(prop.clockRate / 1000);

    hipEvent_t e0 = nullptr, e1 = nullptr;
    void *a = nullptr, *b = nullptr;
    u32 *o = nullptr;
    const size_t bytes = (size_t)1 << 30;           // 1 GiB each way
    const u32 groups = (u32)prop.multiProcessorCount * 8, iters = 4096;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = hipMalloc(&a, bytes);
    if (e == hipSuccess) e = hipMalloc(&b, bytes);
    if (e == hipSuccess) e = hipMalloc((void **)&o, (size_t)groups * 256 * sizeof(u32));
    if (e == hipSuccess) e = hipMemset(a, 1, bytes);
    float best_copy = 1e30f, best_lds = 1e30f, best_read = 1e30f;
    for (int round = 0; round < 4 && e == hipSuccess; round++) {
        (void)hipEventRecord(e0, nullptr);
        hipLaunchKernelGGL(peaks_copy_kernel, dim3((u32)prop.multiProcessorCount * 8), dim3(256), 0, nullptr,
                           (const v4u *)a, (v4u *)b, bytes / 16);
        (void)hipEventRecord(e1, nullptr);
        e = hipEventSynchronize(e1);
        float ms = 0;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (round && ms < best_copy) best_copy = ms;  // the first round warms up
        (void)hipEventRecord(e0, nullptr);
        hipLaunchKernelGGL(peaks_read_kernel, dim3(groups), dim3(256), 0, nullptr, (const v4u *)a, o, bytes / 16);
        (void)hipEventRecord(e1, nullptr);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (round && ms < best_read) best_read = ms;
        (void)hipEventRecord(e0, nullptr);
        hipLaunchKernelGGL(peaks_lds_kernel, dim3(groups), dim3(256), 0, nullptr, o, iters);
        (void)hipEventRecord(e1, nullptr);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (round && ms < best_lds) best_lds = ms;
    }
    if (e == hipSuccess) e = hipGetLastError();
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
    if (o) (void)hipFree(o);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) {
        out->hip_error = (int32_t)e;
        return VMS_EHIP;
    }
    out->copy_bytes = 2 * (uint64_t)bytes;          // read + written
    out->copy_ms = best_copy;
    out->hbm_copy_gbs = (double)out->copy_bytes / (best_copy * 1e-3) / 1e9;
    out->read_bytes = (uint64_t)bytes;
    out->read_ms = best_read;
    out->hbm_read_gbs = (double)out->read_bytes / (best_read * 1e-3) / 1e9;
    out->lds_bytes = (uint64_t)groups * 256 * 16 * 8 * iters;
    out->lds_ms = best_lds;
    out->lds_read_gbs = (double)out->lds_bytes / (best_lds * 1e-3) / 1e9;
    return VMS_OK;
}
