// Wavefront-wide primitives for gfx950 (wave64).  Every workgroup of the replay
// kernels is exactly one wavefront, so "the wave" and "the workgroup" coincide
// and all of these must be called from wave-uniform control flow (EXEC full).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;

#define DI __device__ __forceinline__

DI u32 lane_id() { return threadIdx.x; }

// Other lanes' LDS/global writes become visible to this lane's later reads.
// LDS operations of one wavefront execute in order, so no hardware wait is
// needed; the fence only stops the compiler from caching values across it.
DI void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

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

// ---- arrays of one trace, shared by the 64 lanes ---------------------------

// read one element at a wave-uniform index; result is wave-uniform
DI u32 ld_uni(const u32 *a, u32 i) { return uni(a[i]); }
DI u64 ld_uni(const u64 *a, u32 i) { return uni64(a[i]); }

// store of a wave-uniform value at a wave-uniform place: every lane writes it (one address, one
// value: no bank conflict, measured cheaper than a store under a one-lane mask, and no
// divergent branch)
template <class T>
DI void st_one(T *a, u32 i, T v)
{
    a[i] = v;
}

// The searches and shifts below work on arrays that are followed by 64 spare places holding zero
// keys (live keys are never zero): whole tiles are read without clamping, a key past the end
// compares as "not greater", and no lane is ever switched off.

// number of elements of a[0..n) that are greater than key
DI u32 count_gt(const u64 *a, u32 n, u64 key)
{
    u32 c = 0;
    for (u32 base = 0; base < n; base += 64) c += popc64(ballot(a[base + lane_id()] > key));
    return c;
}

// same for two keys in one pass (k1 >= k2, hence c1 <= c2)
DI void count_gt2(const u64 *a, u32 n, u64 k1, u64 k2, u32 *c1, u32 *c2)
{
    u32 x = 0, y = 0;
    for (u32 base = 0; base < n; base += 64) {
        const u64 v = a[base + lane_id()];
        x += popc64(ballot(v > k1));
        y += popc64(ballot(v > k2));
    }
    *c1 = x;
    *c2 = y;
}

// Rank of key in a[0..n) sorted in DESCENDING order: the number of elements greater than key.
// 64-ary search: the lanes first probe every stride-th element, then the one block of
// `stride` elements that contains the boundary (two dependent LDS reads for n <= 4096).
DI u32 rank_desc(const u64 *a, u32 n, u64 key)
{
    const u32 lane = lane_id();
    if (n <= 64) return popc64(ballot(a[lane] > key));
    if (n > 4096) return count_gt(a, n, key);
    const u32 stride = (n + 63) >> 6;
    const u32 c = popc64(ballot(a[lane * stride] > key));    // probes above key form a prefix
    const u32 b0 = dec_sat(c) * stride;                // a[b0] > key >= a[b0 + stride] (if c)
    return b0 + popc64(ballot(a[b0 + lane] > key));          // keys from b0 + stride on are not greater
}

// ranks of two keys (k1 >= k2, hence r1 <= r2) sharing the probe pass
DI void rank_desc2(const u64 *a, u32 n, u64 k1, u64 k2, u32 *r1, u32 *r2)
{
    const u32 lane = lane_id();
    if (n <= 64) {
        const u64 v = a[lane];
        *r1 = popc64(ballot(v > k1));
        *r2 = popc64(ballot(v > k2));
        return;
    }
    if (n > 4096) {
        count_gt2(a, n, k1, k2, r1, r2);
        return;
    }
    const u32 stride = (n + 63) >> 6;
    const u64 pv = a[lane * stride];
    const u32 c1 = popc64(ballot(pv > k1)), c2 = popc64(ballot(pv > k2));
    const u32 b1 = dec_sat(c1) * stride, b2 = dec_sat(c2) * stride;
    const u64 v1 = a[b1 + lane], v2 = a[b2 + lane];
    *r1 = b1 + popc64(ballot(v1 > k1));
    *r2 = b2 + popc64(ballot(v2 > k2));
}

// a[pos..n) -> a[pos+1..n+1), highest tile first.  Lanes above the part that moves rewrite
// the place above their own with what it holds (places that are final already).
template <class T>
DI void shift_up(T *a, u32 pos, u32 n)
{
    for (u32 hi = n; hi > pos;) {
        const u32 lo = hi - pos > 64 ? hi - 64 : pos;
        const u32 i = lo + lane_id();
        const T x = a[i < hi ? i : i + 1];
        a[i + 1] = x;
        hi = lo;
    }
    wave_sync();
}

// a[pos+1..n) -> a[pos..n-1), lowest tile first.  Lanes past the end rewrite their own
// (spare, zero) place.
template <class T>
DI void shift_down(T *a, u32 pos, u32 n)
{
    for (u32 lo = pos + 1; lo < n; lo += 64) {
        const u32 i = lo + lane_id();
        const T x = a[i];
        a[i < n ? i - 1 : i] = x;
    }
    wave_sync();
}

// maximum over the 64 lanes, returned wave-uniform
DI u32 wave_max_u32(u32 v) { return ~wave_min_u32(~v); }

// sum of a 64-bit value over the 64 lanes (mod 2^64), returned wave-uniform
DI u64 wave_sum_u64(u64 v)
{
    u64 s = 0;
    for (u32 l = 0; l < 64; l++) s += from_lane64(v, l);
    return s;
}

// ---- rank search with the first level held in registers ---------------------
// Probe caches every stride-th key of a descending array (lane l holds
// a[l * stride], or 0 past the end: keys are never 0).  A rank query then costs
// one LDS round trip (the block of `stride` keys around the boundary) and
// none at all for arrays of at most 64 keys.  The cache must be refreshed
// after the array changes.
struct Probe {
    u64 v;          // per lane
    u32 stride;     // wave-uniform
};

DI void probe_refresh(Probe &p, const u64 *a, u32 n)
{
    p.stride = n > 64 ? (n + 63) >> 6 : 1;
    const u32 pi = lane_id() * p.stride;
    const u64 x = a[pi < n ? pi : 0];
    p.v = pi < n ? x : 0;
}

struct RankReq {
    u32 b0;         // block start; the rank itself if !need
    u64 v;          // this lane's key of the block (0: none)
    bool need;      // second level pending
};

// first half: probe ballot and the block load (no wait for the load here)
DI RankReq rank_begin(const Probe &p, const u64 *a, u32 n, u64 key)
{
    RankReq r;
    const u32 c = popc64(ballot(p.v > key));
    r.need = p.stride > 1 && c > 0;
    r.b0 = c;
    r.v = 0;
    if (r.need) {
        r.b0 = (c - 1) * p.stride;
        if (p.stride <= 64) {
            const u32 i = r.b0 + lane_id();
            const u64 x = a[i < n ? i : n - 1];
            r.v = (lane_id() < p.stride && i < n) ? x : 0;
        } else {
            // arrays beyond 4096 keys: count the block in tiles right away
            u32 cnt = 0;
            for (u32 o = 0; o < p.stride; o += 64) {
                const u32 i = r.b0 + o + lane_id();
                const u64 x = a[i < n ? i : n - 1];
                cnt += popc64(ballot(o + lane_id() < p.stride && i < n && x > key));
            }
            r.b0 += cnt;
            r.need = false;
        }
    }
    return r;
}

// second half: a[0..n) sorted descending, returns the number of keys greater than key
DI u32 rank_end(const RankReq &r, u64 key) { return r.need ? r.b0 + popc64(ballot(r.v > key)) : r.b0; }

DI u32 rank_probe(const Probe &p, const u64 *a, u32 n, u64 key)
{
    RankReq r = rank_begin(p, a, n, key);
    return rank_end(r, key);
}

// The rank with one block load and no branch on the way.  The array must be followed by at
// least 64 zero keys (a[n .. n + 64) == 0), so that no index needs clamping: every key from the
// block start on that is greater than key lies in the block.  WIDE: the array may hold more than
// 4096 keys (then the general route is taken when it does).
template <bool WIDE>
DI u32 rank_fast(const Probe &p, const u64 *a, u32 n, u64 key)
{
    if (WIDE && p.stride > 64) return rank_probe(p, a, n, key);
    const u32 c = popc64(ballot(p.v > key));
    const u32 b0 = dec_sat(c) * p.stride;
    return b0 + popc64(ballot(a[b0 + lane_id()] > key));
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
