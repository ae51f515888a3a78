/*
 * vms_live: the virtual-memory-stitching allocator of the GMLake paper
 * (arXiv 2401.08156) as a live device allocator on one AMD GPU, backed by HIP's
 * virtual memory management API (hipMemCreate / hipMemAddressReserve /
 * hipMemMap / hipMemSetAccess / hipMemUnmap / hipMemRelease).
 *
 * It takes the same decisions as the VMS policy of vms_replay_run (pBlock /
 * sBlock pools of Sec. 3.2, BestFit of Algorithm 1, the states S1-S5 of
 * Sec. 4.1, Update / StitchFree of Sec. 3.3.2, the fragmentation limit of
 * Sec. 4.2.3, a splitting pool for requests below one chunk, Sec. 3.1) and
 * reports each one in the decision-word format of vms_replay.h, so a trace can
 * be served live and compared word for word with its replay.  Host code only:
 * no kernel is launched by this library part.
 *
 * How the paper's three primitives are realised here:
 *   Alloc   one hipMemCreate per physical chunk, one virtual range for the new
 *           pBlock, one hipMemMap per chunk, one hipMemSetAccess for the range;
 *   Split   book-keeping only: the two halves keep their places inside the
 *           range their chunks were first mapped to (no driver call);
 *   Stitch  one new virtual range, one hipMemMap per chunk of the member blocks,
 *           whose own mappings stay in place, one hipMemSetAccess.
 * StitchFree unmaps and frees the range of the released sBlock.
 *
 * Pointers named d_* are DEVICE pointers handed out by the allocator; all
 * other pointers are HOST pointers.  Functions return VMS_OK or a negative
 * VMS_E* code of vms_replay.h and never throw.  A request that cannot be
 * served (state S5: the capacity is reached or the device has no memory left)
 * is a result, not an error of the call: *d_ptr is NULL and the decision word
 * carries code 5.  One handle serves one device; calls on one handle are
 * serialised by a lock inside.  Memory is reused as soon as it is freed, as in
 * any caching allocator: the caller orders work on different streams itself.
 */
#ifndef VMS_LIVE_H
#define VMS_LIVE_H

#include <stddef.h>
#include <stdint.h>

#include "vms_replay.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vms_live_config {
    uint32_t struct_size;        /* sizeof(vms_live_config)                                   */
    uint32_t spool_threshold;    /* StitchFree: cached sBlocks above this are released, least
                                    recently used inactive first (Sec. 4.2.3); default 512     */
    uint64_t chunk_bytes;        /* physical chunk (Sec. 3.1), default 2 MiB; a power of two
                                    and a multiple of the device's allocation granularity      */
    uint64_t small_limit_bytes;  /* requests below this use the splitting pool; <= chunk_bytes */
    uint64_t frag_limit_bytes;   /* blocks below this are neither split nor stitched
                                    (Sec. 4.2.3); multiple of chunk_bytes; chunk_bytes or 0
                                    disables it                                                */
    uint64_t capacity_bytes;     /* limit on reserved memory (state S5); 0 = 512 GiB, i.e. the
                                    device decides                                             */
    uint32_t sync_before_unmap;  /* 1 (default): hipDeviceSynchronize before StitchFree unmaps
                                    a range, so that no kernel still running on a block freed
                                    a moment ago loses its mapping                             */
    uint32_t reserved0;
} vms_live_config;

/* Driver calls made so far and the host wall-clock milliseconds spent in them. */
typedef struct vms_live_api_report {
    uint32_t struct_size;        /* sizeof(vms_live_api_report), set by the caller            */
    int32_t  hip_error;          /* hipError_t of the last failing HIP call, else 0           */
    uint64_t n_reserve, n_create, n_map, n_set_access, n_unmap, n_release, n_address_free;
    double   ms_reserve, ms_create, ms_map, ms_set_access, ms_unmap, ms_release, ms_address_free;
    uint64_t n_malloc, n_free;   /* requests served                                           */
    double   ms_malloc, ms_free; /* whole calls, driver time included                         */
} vms_live_api_report;

typedef struct vms_live vms_live;       /* opaque handle */

void vms_live_config_default(vms_live_config *cfg);

/* Create an allocator on the current HIP device.  Nothing is reserved yet.
 * VMS_EINVAL if chunk_bytes does not fit the device's granularity.            */
int vms_live_create(const vms_live_config *cfg, vms_live **out);

/* Serve a request of `bytes` (> 0; rounded up to 512).  *d_ptr receives the
 * block's device address (NULL in state S5); *decision (nullable) the decision
 * word.  The memory is readable and writable from the handle's device.        */
int vms_live_malloc(vms_live *h, uint64_t bytes, void **d_ptr, uint64_t *decision);

/* Update (Sec. 3.3.2): the block becomes inactive and stays cached.  d_ptr must
 * be an address vms_live_malloc returned and not freed since: VMS_EINVAL
 * otherwise (nothing changes).                                                */
int vms_live_free(vms_live *h, void *d_ptr, uint64_t *decision);

/* Serve a whole trace of event words (vms_replay.h): ALLOC binds the slot to a
 * new block, FREE releases it; h_decisions[n_events] receives the decision
 * words, malformed events get code 15 as in the replay.  Slots still bound at
 * the end stay allocated and are owned by the handle (released by destroy).
 * May be called once per handle, before any other request.                    */
int vms_live_run_trace(vms_live *h, const uint64_t *h_events, uint32_t n_events, uint32_t max_slots,
                       uint64_t *h_decisions);

/* Address currently bound to a slot of the trace served by vms_live_run_trace
 * (NULL if unbound), and the bytes requested for it.                          */
int vms_live_slot(vms_live *h, uint32_t slot, void **d_ptr, uint64_t *bytes);

/* The same statistics record as the replay's (vms_replay.h), over all requests
 * served so far, numbered in order of arrival; max_runs and overflow_event
 * are not used (0 and 0xFFFFFFFF).  api (nullable) receives the driver-call
 * counts and times.                                                            */
int vms_live_stats(vms_live *h, vms_trace_stats *out, vms_live_api_report *api);

/* Unmap everything, release every physical chunk and free the handle.  Blocks
 * still allocated become invalid.  Waits for the device first.                */
void vms_live_destroy(vms_live *h);

/* Entry points with the signature PyTorch's pluggable device allocator loads
 * by name (torch.cuda.memory.CUDAPluggableAllocator): one allocator per device,
 * created on first use with the defaults above, overridable through the
 * environment variables VMS_LIVE_CHUNK_MB, VMS_LIVE_FRAG_LIMIT_MB,
 * VMS_LIVE_SPOOL_THRESHOLD and VMS_LIVE_CAPACITY_MB.  vms_torch_malloc returns
 * NULL when the request cannot be served.  `stream` is not used: memory freed
 * on one stream may be handed to another at once.                             */
void *vms_torch_malloc(ptrdiff_t size, int device, void *stream);
void vms_torch_free(void *d_ptr, ptrdiff_t size, int device, void *stream);

/* The allocator vms_torch_malloc uses for `device` (NULL before its first
 * request): for reading its statistics.  Owned by the library.                */
vms_live *vms_torch_allocator(int device);

#ifdef __cplusplus
}
#endif
#endif
