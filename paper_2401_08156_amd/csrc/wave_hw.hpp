// Wavefront-wide primitives for gfx950 (wave64): the ones that name the hardware (lane
// numbers, ballots, lane reads and writes, DPP reductions, fences).  Every workgroup of the
// replay kernels is exactly one wavefront, so "the wave" and "the workgroup" coincide and all
// of these must be called from wave-uniform control flow (EXEC full).
#ifndef VMS_WAVE_HW_HPP
#define VMS_WAVE_HW_HPP
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;

#define DI __device__ __forceinline__

DI u32 lane_id() { return threadIdx.x; }

// the wavefront's dynamically sized LDS (a kernel declares it once, at function scope)
#define WAVE_DYNAMIC_LDS(name) extern __shared__ __attribute__((aligned(16))) char name[]

// Other lanes' LDS/global writes become visible to this lane's later reads.
// LDS operations of one wavefront execute in order, so no hardware wait is
// needed; the fence only stops the compiler from caching values across it.
DI void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Marks a place where the 64 lanes must have finished the memory accesses before it (a load of
// places that other lanes store to right after, or the other way round).  The hardware runs the
// lanes of a wavefront in lockstep, instruction by instruction, so nothing is emitted; a host
// build that runs the lanes one after another switches lanes here.
DI void wave_lockstep() {}

// a 64-bit word of a list in global memory: read at device scope, past the compute unit's
// vector cache (lists are written and read by the same wavefront, and read once)
DI u64 ld_list(const u64 *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// the same for one 16-bit element of a table kept in global memory
DI u32 ld_tab(const uint16_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// The wavefront's priority at instruction issue (0, the default, to 3) from here on.  The stitching
// kernels hold LDS for as long as they run and the splitting kernels beside them hold none, so the
// former go first where both wait at one SIMD.
template <int PRIO>
DI void wave_priority() { __builtin_amdgcn_s_setprio(PRIO); }

// c - 1, or 0 for 0, on a wave-uniform count: two scalar instructions (the conditional form is
// compiled into a clamped vector subtract and a v_readfirstlane)
DI u32 dec_sat(u32 c) { return c - min(c, 1u); }

DI u64 ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
DI u32 first_lane(u64 mask) { return (u32)__builtin_ctzll(mask); }
DI u32 popc64(u64 m) { return (u32)__builtin_popcountll(m); }

// number of set bits of mask below this lane
DI u32 rank_in(u64 mask)
{
    return __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
}

DI u32 uni(u32 v) { return __builtin_amdgcn_readfirstlane(v); }
DI u64 uni64(u64 v)
{
    u32 lo = __builtin_amdgcn_readfirstlane((u32)v);
    u32 hi = __builtin_amdgcn_readfirstlane((u32)(v >> 32));
    return ((u64)hi << 32) | lo;
}
DI u32 from_lane(u32 v, u32 lane) { return __builtin_amdgcn_readlane(v, lane); }
DI u64 from_lane64(u64 v, u32 lane)
{
    u32 lo = __builtin_amdgcn_readlane((u32)v, lane);
    u32 hi = __builtin_amdgcn_readlane((u32)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// DPP lane permutations (all rows / banks enabled, out-of-range source reads 0)
template <int CTRL>
DI u32 dpp_zero(u32 v)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
DI u32 dpp_perm(u32 v)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

enum {
    DPP_QUAD_XOR1 = 0xB1,       // quad_perm [1,0,3,2]
    DPP_QUAD_XOR2 = 0x4E,       // quad_perm [2,3,0,1]
    DPP_ROW_HALF_MIRROR = 0x141,
    DPP_ROW_MIRROR = 0x140,
    DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118
};

// minimum over the 64 lanes, returned wave-uniform
DI u32 wave_min_u32(u32 v)
{
    v = min(v, dpp_perm<DPP_QUAD_XOR1>(v));
    v = min(v, dpp_perm<DPP_QUAD_XOR2>(v));
    v = min(v, dpp_perm<DPP_ROW_HALF_MIRROR>(v));
    v = min(v, dpp_perm<DPP_ROW_MIRROR>(v));          // every lane: minimum of its row of 16
    u32 a = from_lane(v, 0), b = from_lane(v, 16), c = from_lane(v, 32), d = from_lane(v, 48);
    return min(min(a, b), min(c, d));
}

// inclusive prefix sum over the 64 lanes; *total receives the wave sum (uniform)
DI u32 wave_scan_add(u32 v, u32 *total)
{
    v += dpp_zero<DPP_ROW_SHR1>(v);
    v += dpp_zero<DPP_ROW_SHR2>(v);
    v += dpp_zero<DPP_ROW_SHR4>(v);
    v += dpp_zero<DPP_ROW_SHR8>(v);                    // inclusive scan inside each row of 16
    u32 t0 = from_lane(v, 15), t1 = from_lane(v, 31), t2 = from_lane(v, 47), t3 = from_lane(v, 63);
    u32 row = lane_id() >> 4;
    u32 add = (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);     // three selects, no branch
    *total = t0 + t1 + t2 + t3;
    return v + add;
}

// vec with lane `lane` replaced by val (both wave-uniform): one v_writelane instead of a compare and a
// select.  On this target the lane select of v_writelane travels in m0 when the value is in a scalar
// register too (one scalar register operand per vector instruction).
DI u32 write_lane(u32 vec, u32 val, u32 lane)
{
    // (uni(): a value the compiler cannot prove wave-uniform would arrive in a vector register)
    asm("s_mov_b32 m0, %2\n\ts_nop 0\n\tv_writelane_b32 %0, %1, m0" : "+v"(vec) : "s"(uni(val)), "s"(uni(lane)) : "m0");
    return vec;
}
// four vectors, the same lane
DI void write_lane4(u32 &a, u32 &b, u32 &c, u32 &d, u32 va, u32 vb, u32 vc, u32 vd, u32 lane)
{
    asm("s_mov_b32 m0, %8\n\ts_nop 0\n\tv_writelane_b32 %0, %4, m0\n\tv_writelane_b32 %1, %5, m0\n\t"
        "v_writelane_b32 %2, %6, m0\n\tv_writelane_b32 %3, %7, m0"
        : "+v"(a), "+v"(b), "+v"(c), "+v"(d)
        : "s"(uni(va)), "s"(uni(vb)), "s"(uni(vc)), "s"(uni(vd)), "s"(uni(lane))
        : "m0");
}

// which way a wave-uniform branch usually goes: the usual way becomes the fall-through
#define LIKELY(x) __builtin_expect(!!(x), 1)
#define UNLIKELY(x) __builtin_expect(!!(x), 0)

// keeps a loaded value where it is: the compiler may not sink the load into a later branch
DI u32 pin(u32 x)
{
    asm volatile("" : "+v"(x));
    return x;
}
DI u64 pin64(u64 x)
{
    asm volatile("" : "+v"(x));
    return x;
}

#endif
