// Wavefront-wide searches, shifts and reductions over the arrays of one trace, built on the
// hardware primitives of wave_hw.hpp.
#ifndef VMS_WAVE_OPS_HPP
#define VMS_WAVE_OPS_HPP
#include "wave_hw.hpp"

// ---- arrays of one trace, shared by the 64 lanes ---------------------------

// read one element at a wave-uniform index; result is wave-uniform
DI u32 ld_uni(const u32 *a, u32 i) { return uni(a[i]); }
DI u64 ld_uni(const u64 *a, u32 i) { return uni64(a[i]); }
DI u32 ld_uni(const uint16_t *a, u32 i) { return uni(a[i]); }

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
        wave_lockstep();
        a[i + 1] = x;
        wave_lockstep();
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
        wave_lockstep();
        a[i < n ? i - 1 : i] = x;
        wave_lockstep();
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

// ---- sorted arrays of narrow keys (K = uint16_t, u32 or u64) ------------------------------------
// Same conventions: descending order, at least 64 zero keys behind the live ones, live keys never 0.

// number of elements of a[0..n) that are greater than key, by a two-level search whose first level
// is read on the spot (two dependent LDS reads; every n up to 64 * 64)
template <class K>
DI u32 rank_desc_k(const K *a, u32 n, K key)
{
    const u32 lane = lane_id();
    if (n <= 64) return popc64(ballot(a[lane] > key));
    const u32 stride = (n + 63) >> 6;               // at most 64 for n <= 4096
    const u32 pi = lane * stride;
    const K pv = a[pi < n ? pi : n];                // a[n] is a spare zero key
    const u32 c = popc64(ballot(pv > key));
    const u32 b0 = dec_sat(c) * stride;             // a[b0] > key >= a[b0 + stride] (if c)
    return b0 + popc64(ballot(a[b0 + lane] > key));
}

// the same for two keys (k1 >= k2, hence r1 <= r2) sharing the probe pass
template <class K>
DI void rank_desc2_k(const K *a, u32 n, K k1, K k2, u32 *r1, u32 *r2)
{
    const u32 lane = lane_id();
    if (n <= 64) {
        const K v = a[lane];
        *r1 = popc64(ballot(v > k1));
        *r2 = popc64(ballot(v > k2));
        return;
    }
    const u32 stride = (n + 63) >> 6;
    const u32 pi = lane * stride;
    const K pv = a[pi < n ? pi : n];
    const u32 c1 = popc64(ballot(pv > k1)), c2 = popc64(ballot(pv > k2));
    const u32 b1 = dec_sat(c1) * stride, b2 = dec_sat(c2) * stride;
    const K v1 = a[b1 + lane], v2 = a[b2 + lane];
    *r1 = b1 + popc64(ballot(v1 > k1));
    *r2 = b2 + popc64(ballot(v2 > k2));
}

// 128 probes held in registers: lane l holds a[l * stride] and a[(64 + l) * stride] (0 past the
// end).  With stride < 64 (n <= 8064) the block of 64 keys from block() on holds every key greater
// than `key` that lies behind its start, and the first key not greater than `key`.
template <class K>
struct Probe2 {
    K v0, v1;       // per lane
    u32 stride;     // wave-uniform
    // G: the array is a table in global memory (16-bit keys, read past the vector cache)
    template <bool G = false>
    DI K at(const K *a, u32 i) const
    {
        if constexpr (G) return (K)ld_tab(a + i);
        else return a[i];
    }
    template <bool G = false>
    DI void refresh(const K *a, u32 n)
    {
        stride = n > 128 ? (n + 127) >> 7 : 1;
        const u32 p0 = lane_id() * stride, p1 = (64 + lane_id()) * stride;
        const K x0 = at<G>(a, p0 < n ? p0 : n), x1 = at<G>(a, p1 < n ? p1 : n);     // a[n] is a spare zero key
        v0 = x0;
        v1 = x1;
    }
    DI u32 block(K key) const
    {
        const u32 c = popc64(ballot(v0 > key)) + popc64(ballot(v1 > key));
        return dec_sat(c) * stride;
    }
    template <bool G = false>
    DI u32 rank(const K *a, K key) const
    {
        const u32 b0 = block(key);
        return b0 + popc64(ballot(at<G>(a, b0 + lane_id()) > key));
    }
};

// Moves of arrays of 2- or 4-byte elements, sixteen bytes (one block of E elements) per lane and
// step.  The array starts on a 16-byte boundary, every place behind the n live ones is zero, and the
// array is allocated two blocks beyond the one that holds place n.  A block is four 32-bit words;
// moving it by one element is a funnel shift through the neighbouring block's edge element.
struct Blk16 {
    u32 w[4];
};

// the words of `moved` where the element index (block * E + j) is at least `from`, else of `old`
template <class T>
DI Blk16 blk_select(const Blk16 &old, const Blk16 &moved, u32 first_elem, u32 from)
{
    Blk16 out;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (u32 k = 0; k < 4; k++) {
            const u32 m = (first_elem + 2 * k >= from ? 0x0000FFFFu : 0u) | (first_elem + 2 * k + 1 >= from ? 0xFFFF0000u : 0u);
            out.w[k] = (moved.w[k] & m) | (old.w[k] & ~m);
        }
    } else {
#pragma unroll
        for (u32 k = 0; k < 4; k++) out.w[k] = first_elem + k >= from ? moved.w[k] : old.w[k];
    }
    return out;
}

// a[pos..n) -> a[pos+1..n+1) in each of the N arrays a[0..N) of equal element size (they hold the
// fields of the same records), highest blocks first.  The loads of all arrays are on their way before
// the first store: one LDS round trip per step, whatever N is.  a[pos] keeps its old value (the
// caller overwrites it).
template <class T, int N>
DI void blk_shift_up(T *const (&a)[N], u32 pos, u32 n)
{
    constexpr u32 E = 16 / sizeof(T);
    const u32 bf = (pos + 1) / E, bl = n / E;       // first and last block that receive an element
    for (u32 hi = bl + 1; hi > bf;) {
        const u32 lo = hi - bf > 64 ? hi - 64 : bf;
        const u32 B = lo + lane_id();
        const bool mine = B < hi;
        Blk16 old[N];
        u32 prev[N];
#pragma unroll
        for (int f = 0; f < N; f++) {
            old[f] = ((const Blk16 *)a[f])[mine ? B : lo];
            prev[f] = a[f][(mine && B ? B : 1u) * E - 1];       // last element of the block below
        }
        wave_lockstep();
#pragma unroll
        for (int f = 0; f < N; f++) {
            Blk16 mv;
            if constexpr (sizeof(T) == 2) {
                mv.w[0] = (old[f].w[0] << 16) | prev[f];
#pragma unroll
                for (u32 k = 1; k < 4; k++) mv.w[k] = (old[f].w[k] << 16) | (old[f].w[k - 1] >> 16);
            } else {
                mv.w[0] = prev[f];
#pragma unroll
                for (u32 k = 1; k < 4; k++) mv.w[k] = old[f].w[k - 1];
            }
            const Blk16 out = blk_select<T>(old[f], mv, B * E, pos + 1);
            if (mine) ((Blk16 *)a[f])[B] = out;
        }
        wave_lockstep();
        hi = lo;
    }
    wave_sync();
}

// a[pos+1..n) -> a[pos..n-1) in each array, lowest blocks first; a[n-1] becomes 0 (the zero behind it moves in)
template <class T, int N>
DI void blk_shift_down(T *const (&a)[N], u32 pos, u32 n)
{
    constexpr u32 E = 16 / sizeof(T);
    const u32 bf = pos / E, bl = (n - 1) / E;
    for (u32 lo = bf; lo <= bl; lo += 64) {
        const u32 B = lo + lane_id();
        const bool mine = B <= bl;
        Blk16 old[N];
        u32 next[N];
#pragma unroll
        for (int f = 0; f < N; f++) {
            old[f] = ((const Blk16 *)a[f])[mine ? B : bl];
            next[f] = a[f][(mine ? B : bl) * E + E];            // first element of the block above
        }
        wave_lockstep();
#pragma unroll
        for (int f = 0; f < N; f++) {
            Blk16 mv;
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (u32 k = 0; k < 3; k++) mv.w[k] = (old[f].w[k] >> 16) | (old[f].w[k + 1] << 16);
                mv.w[3] = (old[f].w[3] >> 16) | (next[f] << 16);
            } else {
#pragma unroll
                for (u32 k = 0; k < 3; k++) mv.w[k] = old[f].w[k + 1];
                mv.w[3] = next[f];
            }
            const Blk16 out = blk_select<T>(old[f], mv, B * E, pos);
            if (mine) ((Blk16 *)a[f])[B] = out;
        }
        wave_lockstep();
    }
    wave_sync();
}

template <class T>
DI void blk_shift_up(T *a, u32 pos, u32 n)
{
    T *const one[1] = { a };
    blk_shift_up<T, 1>(one, pos, n);
}
template <class T>
DI void blk_shift_down(T *a, u32 pos, u32 n)
{
    T *const one[1] = { a };
    blk_shift_down<T, 1>(one, pos, n);
}

// The same moves for N arrays of 16-bit elements kept in GLOBAL memory (tables of the fine-grained
// stitching kernel that do not fit the LDS budget).  Blocks are read with device-scope loads (other
// lanes of this wavefront wrote them; tbl_fence() first, so that their stores have arrived), G steps of
// 64 blocks are on their way before the first store.  A step never reads a block that an earlier step
// of the same call has written.
DI void tbl_fence() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); }
DI Blk16 gblk_load(const uint16_t *a, u32 B)
{
    const u64 *p = (const u64 *)a + 2 * (size_t)B;
    const u64 lo = ld_list(p), hi = ld_list(p + 1);
    return Blk16{ { (u32)lo, (u32)(lo >> 32), (u32)hi, (u32)(hi >> 32) } };
}
DI void gblk_store(uint16_t *a, u32 B, const Blk16 &v)
{
    u64 *p = (u64 *)a + 2 * (size_t)B;
    p[0] = v.w[0] | ((u64)v.w[1] << 32);
    p[1] = v.w[2] | ((u64)v.w[3] << 32);
}

template <int N>
DI void gblk_shift_up(uint16_t *const (&a)[N], u32 pos, u32 n)
{
    constexpr u32 E = 8, G = 2;
    const u32 bf = (pos + 1) / E, bl = n / E;       // first and last block that receive an element
    tbl_fence();
    for (u32 hi = bl + 1; hi > bf;) {
        Blk16 old[G][N];
        u32 prev[G][N], B[G];
        bool mine[G];
        u32 h = hi;
#pragma unroll
        for (u32 g = 0; g < G; g++) {
            const u32 lo = h - bf > 64 ? h - 64 : bf;
            B[g] = lo + lane_id();
            mine[g] = B[g] < h;                     // (a group past the first block: h == lo == bf, no lane takes part)
#pragma unroll
            for (int f = 0; f < N; f++) {
                old[g][f] = gblk_load(a[f], mine[g] ? B[g] : bf);
                prev[g][f] = ld_tab(a[f] + (size_t)(mine[g] && B[g] ? B[g] : 1u) * E - 1);    // last element of the block below
            }
            h = lo;
        }
        wave_lockstep();
#pragma unroll
        for (u32 g = 0; g < G; g++)
#pragma unroll
            for (int f = 0; f < N; f++) {
                Blk16 mv;
                mv.w[0] = (old[g][f].w[0] << 16) | prev[g][f];
#pragma unroll
                for (u32 k = 1; k < 4; k++) mv.w[k] = (old[g][f].w[k] << 16) | (old[g][f].w[k - 1] >> 16);
                const Blk16 out = blk_select<uint16_t>(old[g][f], mv, B[g] * E, pos + 1);
                if (mine[g]) gblk_store(a[f], B[g], out);
            }
        wave_lockstep();
        hi = h;
    }
    wave_sync();
}

template <int N>
DI void gblk_shift_down(uint16_t *const (&a)[N], u32 pos, u32 n)
{
    constexpr u32 E = 8, G = 2;
    const u32 bf = pos / E, bl = (n - 1) / E;
    tbl_fence();
    for (u32 lo = bf; lo <= bl; lo += 64 * G) {
        Blk16 old[G][N];
        u32 next[G][N], B[G];
        bool mine[G];
#pragma unroll
        for (u32 g = 0; g < G; g++) {
            B[g] = lo + 64 * g + lane_id();
            mine[g] = B[g] <= bl;
#pragma unroll
            for (int f = 0; f < N; f++) {
                old[g][f] = gblk_load(a[f], mine[g] ? B[g] : bl);
                next[g][f] = ld_tab(a[f] + (size_t)(mine[g] ? B[g] : bl) * E + E);            // first element of the block above
            }
        }
        wave_lockstep();
#pragma unroll
        for (u32 g = 0; g < G; g++)
#pragma unroll
            for (int f = 0; f < N; f++) {
                Blk16 mv;
#pragma unroll
                for (u32 k = 0; k < 3; k++) mv.w[k] = (old[g][f].w[k] >> 16) | (old[g][f].w[k + 1] << 16);
                mv.w[3] = (old[g][f].w[3] >> 16) | (next[g][f] << 16);
                const Blk16 out = blk_select<uint16_t>(old[g][f], mv, B[g] * E, pos);
                if (mine[g]) gblk_store(a[f], B[g], out);
            }
        wave_lockstep();
    }
    wave_sync();
}

#endif
