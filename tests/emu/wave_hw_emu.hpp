// TEST INFRASTRUCTURE ONLY.  A host stand-in for csrc/wave_hw.hpp: the 64 lanes of a wavefront
// run as 64 cooperative fibers of one thread, switched round-robin at every wavefront-wide
// operation (ballot, lane read, reduction, wave_sync, wave_lockstep).  The kernel sources are
// compiled unchanged on top of it, so their indexing can be checked on the CPU with bounds
// checks (guard bands around LDS and every device buffer).  Control flow must be wave-uniform at
// every such operation, as on the GPU.  Nothing in the product path includes this file.
#ifndef VMS_WAVE_HW_HPP
#define VMS_WAVE_HW_HPP
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <ucontext.h>
#include <algorithm>

typedef uint32_t u32;
typedef uint64_t u64;

#define DI inline
#define __global__
#define __device__
#define __shared__ static
#define WAVE_DYNAMIC_LDS(name) extern char name[]
#define __forceinline__ inline
#define __launch_bounds__(x)

using std::max;
using std::min;

namespace emu {
struct Dim { u32 x; };
const int LANES = 64;
extern int cur;                     // the lane that is running
extern ucontext_t ctx[LANES], back;
extern u64 xchg[2][LANES];
extern u64 n_coll;                  // collectives passed so far (the same in every lane when it matters)
extern u64 coll_of[LANES];
extern bool trace_on;               // debugging aid: remember where each lane's wave-wide operations were called from
void note(void *site);
void launch(void (*body)(void *), void *arg, u32 block);
// hand over to the next lane; returns when every other lane has reached its next switch
inline void switch_lane()
{
    if (trace_on) note(__builtin_return_address(0));
    const int me = cur, next = (me + 1) % LANES;
    cur = next;
    swapcontext(&ctx[me], &ctx[next]);
}
// every lane contributes v and receives all 64 values
inline const u64 *all(u64 v)
{
    const u64 k = coll_of[cur]++;
    u64 *buf = xchg[k & 1];
    buf[cur] = v;
    switch_lane();
    return buf;
}
}  // namespace emu

extern emu::Dim blockIdx;
extern char lds[];

DI u32 lane_id() { return (u32)emu::cur; }
DI void wave_sync() { emu::coll_of[emu::cur]++; emu::switch_lane(); }
DI void wave_lockstep() { emu::coll_of[emu::cur]++; emu::switch_lane(); }
#define __builtin_amdgcn_fence(order, scope) wave_sync()

DI u64 ld_list(const u64 *p) { return *p; }
DI u32 ld_tab(const uint16_t *p) { return *p; }
template <int PRIO>
DI void wave_priority() {}
DI u32 dec_sat(u32 c) { return c - min(c, 1u); }

DI u64 ballot(bool p)
{
    const u64 *v = emu::all(p ? 1 : 0);
    u64 m = 0;
    for (int l = 0; l < emu::LANES; l++) m |= (v[l] & 1) << l;
    return m;
}
DI u32 first_lane(u64 mask) { return (u32)__builtin_ctzll(mask); }
DI u32 popc64(u64 m) { return (u32)__builtin_popcountll(m); }
DI u32 rank_in(u64 mask) { return popc64(mask & ((1ull << lane_id()) - 1)); }

DI u64 from_lane64(u64 v, u32 lane)
{
    if (lane >= 64) { fprintf(stderr, "emu: lane read of lane %u\n", lane); abort(); }
    return emu::all(v)[lane];
}
DI u32 from_lane(u32 v, u32 lane) { return (u32)from_lane64(v, lane); }
DI u32 uni(u32 v) { return (u32)emu::all(v)[0]; }
DI u64 uni64(u64 v) { return emu::all(v)[0]; }

DI u32 wave_min_u32(u32 v)
{
    const u64 *a = emu::all(v);
    u32 m = 0xFFFFFFFFu;
    for (int l = 0; l < emu::LANES; l++) m = min(m, (u32)a[l]);
    return m;
}
DI u32 wave_scan_add(u32 v, u32 *total)
{
    const u64 *a = emu::all(v);
    u32 run = 0, mine = 0;
    for (int l = 0; l < emu::LANES; l++) {
        run += (u32)a[l];
        if (l == emu::cur) mine = run;
    }
    *total = run;
    return mine;
}
DI u32 write_lane(u32 vec, u32 val, u32 lane) { return lane_id() == lane ? val : vec; }
DI void write_lane4(u32 &a, u32 &b, u32 &c, u32 &d, u32 va, u32 vb, u32 vc, u32 vd, u32 lane)
{
    if (lane_id() == lane) { a = va; b = vb; c = vc; d = vd; }
}

#define LIKELY(x) __builtin_expect(!!(x), 1)
#define UNLIKELY(x) __builtin_expect(!!(x), 0)
DI u32 pin(u32 x) { return x; }
DI u64 pin64(u64 x) { return x; }

// LDS atomics: the lanes run one after another, so plain updates are atomic
template <class T> DI T atomicOr(T *p, T v) { T o = *p; *p = o | v; return o; }
template <class T> DI T atomicXor(T *p, T v) { T o = *p; *p = o ^ v; return o; }
template <class T> DI T atomicAnd(T *p, T v) { T o = *p; *p = o & v; return o; }
template <class T> DI T atomicAdd(T *p, T v) { T o = *p; *p = o + v; return o; }
template <class T> DI T atomicMax(T *p, T v) { T o = *p; *p = max(o, v); return o; }
template <class T> DI T atomicMin(T *p, T v) { T o = *p; *p = min(o, v); return o; }

#endif
