// Replay kernels: one wavefront (= one workgroup of 64 lanes) replays one trace
// under one policy.  All allocator state of the trace lives in that wave's LDS;
// scalar state (counters, byte totals, digest) stays wave-uniform so the
// compiler keeps it in SGPRs.  Control flow is wave-uniform throughout: the 64
// lanes only ever split up to scan / shift / mark the pool arrays in parallel.
//
// Policies (GMLake, arXiv 2401.08156): the splitting caching allocator of
// Sec. 2.2 and the stitching allocator of Sec. 3 and Sec. 4.1 (Algorithm 1).
#pragma once
#include <type_traits>
#include "wave_ops.hpp"
#include "../../include/vms_replay.h"

enum { C_FREE = 0, C_EXACT = 1, C_SPLIT = 2, C_STITCH = 3, C_GROW = 4, C_OOM = 5, C_FREE_NOOP = 6, C_INVALID = 15 };
enum : u64 { B_SMALL = 1u << 4, B_SBLOCK = 1u << 5, B_6 = 1u << 6, B_7 = 1u << 7 };
enum { SLOT_UNBOUND = 0u, SLOT_OOM = 0xFFFFFFFFu };
enum { KIND_SMALL = 0u, KIND_PBLOCK = 1u, KIND_SBLOCK = 2u };
#define NONE32 0xFFFFFFFFu

// Launch-constant parameters (passed by value as a kernel argument).
struct KParams {
    u32 n_traces, max_events;
    u32 chunk_shift;            // log2(chunk in 512-byte units)
    u32 small_limit_units;
    u32 frag_limit_chunks;
    u32 spool_threshold;
    u64 capacity_units;
    u32 max_slots;
    u32 cap_free, cap_pblocks, cap_sblocks, cap_runs, cap_chunks;
    // byte offsets of the per-wave arrays inside dynamic LDS
    u32 off_slot_req, off_slot_a, off_slot_b, off_fl, off_pool, off_bmp, off_skey, off_smeta, off_sstamp,
        off_arena;
    u32 lds_bytes;
    u32 run_len_bits;           // see VmsD::arena
    u64 ws_stride;              // workspace bytes per trace (sBlock run compaction buffer)
};

// Running totals of one (trace, policy).
struct Acct {
    u64 requested, active;      // 512-byte units
    u64 peak_requested, peak_active, peak_reserved;
    u64 digest;
    u32 n_split, n_merge, n_created, n_evicted, first_oom, status, overflow_event;
    u32 hw_pblocks, hw_sblocks, hw_free, hw_members, hw_runs;
    bool stop;
};

DI void acct_init(Acct &A)
{
    A.requested = A.active = A.peak_requested = A.peak_active = A.peak_reserved = 0;
    A.digest = 0xCBF29CE484222325ull;
    A.n_split = A.n_merge = A.n_created = A.n_evicted = A.status = 0;
    A.first_oom = A.overflow_event = NONE32;
    A.hw_pblocks = A.hw_sblocks = A.hw_free = A.hw_members = A.hw_runs = 0;
    A.stop = false;
}

// An engine table is too small for this trace: stop replaying it.
DI void table_overflow(Acct &A, u32 ev, u32 which)
{
    A.status |= VMS_ST_TABLE_OVERFLOW | which;
    if (A.overflow_event == NONE32) A.overflow_event = ev;
    A.stop = true;
}

// ---------------------------------------------------------------------------
// Splitting pool (Sec. 2.2): the inactive blocks of the pool as an unordered
// LDS array of 64-bit keys
//     bits 32-62 size (units) | bits 2-31 address (units) | bit 1 first-in-segment | bit 0 last-in-segment
// so that the minimum key >= (request << 32) is the best fit with the lowest
// address.  Active blocks are not stored: a block's address, size and segment
// flags travel with the slot that holds it.  The two flags replace neighbour
// links: a block may merge to the right iff it is not last in its segment and
// the block starting where it ends is in the array (inactive); same to the left.
// ---------------------------------------------------------------------------
struct SplitPoolD {
    u64 *fl;
    u32 n, cap;
    u64 reserved;               // units obtained so far = next segment address
};

struct SplitRes {
    u32 code, addr, flags;
    bool split;
};

DI SplitRes sp_alloc(SplitPoolD &sp, u32 size, u32 seg, bool may_grow, Acct &A, u32 ev)
{
    const u32 lane = lane_id();
    SplitRes r;
    r.split = false;
    // step 1: best fit = smallest key not below (size, address 0)
    const u64 thresh = (u64)size << 32;
    u64 best = ~0ull;
    u32 besti = 0;
    for (u32 base = 0; base < sp.n; base += 64) {
        u32 i = base + lane;
        u64 k = i < sp.n ? sp.fl[i] : ~0ull;
        if (k >= thresh && k < best) {
            best = k;
            besti = i;
        }
    }
    u32 hi = (u32)(best >> 32);
    u32 mhi = sp.n ? wave_min_u32(hi) : NONE32;
    u32 bsize;
    if (mhi != NONE32) {
        u32 lo = hi == mhi ? (u32)best : NONE32;
        u32 mlo = wave_min_u32(lo);
        u32 owner = first_lane(ballot(hi == mhi && lo == mlo));
        u32 idx = from_lane(besti, owner);
        bsize = mhi;
        r.addr = mlo >> 2;
        r.flags = mlo & 3;
        r.code = C_EXACT;
        u32 last = sp.n - 1;                    // unordered array: fill the hole with the last key
        if (lane == 0 && idx != last) sp.fl[idx] = sp.fl[last];
        sp.n = last;
        wave_sync();
    } else {
        if (!may_grow) {
            r.code = C_OOM;
            r.addr = r.flags = 0;
            return r;
        }
        r.addr = (u32)sp.reserved;              // "native allocation": a fresh segment
        sp.reserved += seg;
        bsize = seg;
        r.flags = 3;
        r.code = C_GROW;
    }
    // step 2: cut off what is not needed; it stays cached as the right neighbour
    if (bsize > size) {
        if (sp.n == sp.cap) {
            table_overflow(A, ev, VMS_ST_OVF_FREE_BLOCKS);
            return r;
        }
        u64 rest = ((u64)(bsize - size) << 32) | ((u64)(r.addr + size) << 2) | (r.flags & 1);
        st_one(sp.fl, sp.n, rest);
        sp.n++;
        A.hw_free = max(A.hw_free, sp.n);
        wave_sync();
        r.flags &= 2;
        r.split = true;
        if (r.code == C_EXACT) r.code = C_SPLIT;
        A.n_split++;
    }
    return r;
}

// steps 3 and 4: the block becomes inactive and absorbs inactive neighbours of its segment
DI void sp_free(SplitPoolD &sp, u32 addr, u32 size, u32 flags, bool *ml, bool *mr, Acct &A, u32 ev)
{
    const u32 lane = lane_id();
    const bool can_l = !(flags & 2), can_r = !(flags & 1);
    u32 lidx = NONE32, ridx = NONE32;
    u64 lkey = 0, rkey = 0;
    if (can_l || can_r) {
        for (u32 base = 0; base < sp.n; base += 64) {
            u32 i = base + lane;
            u64 k = i < sp.n ? sp.fl[i] : 0;
            u32 ka = (u32)k >> 2, ks = (u32)(k >> 32);
            u64 mL = ballot(can_l && i < sp.n && ka + ks == addr);
            u64 mR = ballot(can_r && i < sp.n && ka == addr + size);
            if (mL) {
                lidx = base + first_lane(mL);
                lkey = from_lane64(k, first_lane(mL));
            }
            if (mR) {
                ridx = base + first_lane(mR);
                rkey = from_lane64(k, first_lane(mR));
            }
        }
    }
    *ml = lidx != NONE32;
    *mr = ridx != NONE32;
    if (*mr) {
        size += (u32)(rkey >> 32);
        flags = (flags & 2) | ((u32)rkey & 1);
    }
    if (*ml) {
        addr = (u32)lkey >> 2;
        size += (u32)(lkey >> 32);
        flags = ((u32)lkey & 2) | (flags & 1);
    }
    A.n_merge += (*ml ? 1u : 0u) + (*mr ? 1u : 0u);
    u64 key = ((u64)size << 32) | ((u64)addr << 2) | flags;
    if (*ml) {
        st_one(sp.fl, lidx, key);               // merged block takes the left neighbour's place
        wave_sync();
        if (*mr) {
            u32 last = sp.n - 1;
            if (lane == 0 && ridx != last) sp.fl[ridx] = sp.fl[last];
            sp.n = last;
        }
    } else if (*mr) {
        st_one(sp.fl, ridx, key);
    } else {
        if (sp.n == sp.cap) {
            table_overflow(A, ev, VMS_ST_OVF_FREE_BLOCKS);
            return;
        }
        st_one(sp.fl, sp.n, key);
        sp.n++;
        A.hw_free = max(A.hw_free, sp.n);
    }
    wave_sync();
}

// ---------------------------------------------------------------------------
// Virtual memory pool (Sec. 3.2) in LDS.
//   pool[]   every pBlock (active or not) as key  size << 32 | ~first_chunk, sorted descending:
//            pool order = size descending, then first chunk ascending.  It changes only when
//            Alloc creates or Split cuts a pBlock.
//   bmp[]    one bit per physical chunk: set while the pBlock owning it is active.  A pBlock is
//            inactive iff the bit of its first chunk is clear; an sBlock is inactive iff all bits
//            of all its chunk runs are clear (Sec. 3.2: one active pBlock makes the sBlock active).
//            Handing out / releasing any block is therefore only bit-range work.
//   skey[]   sBlocks as key  size << 32 | ~creation_number, sorted descending (size descending,
//            then older first), with smeta[] = arena offset << 16 | run count, sstamp[] = last use.
//   arena[]  chunk runs of all cached sBlocks, bump-allocated, 32 bits each:
//            first_chunk << len_bits | (chunks - 1); a longer run takes several entries.
//            Compacted through a global-memory buffer when full.
// ---------------------------------------------------------------------------
// BIG: for traces whose sBlocks hold more chunk runs than LDS can take, the arena lives in the
// trace's slice of the global workspace (the other arrays stay in LDS) and smeta[] widens to
// arena offset << 32 | run count.
template <bool BIG>
struct VmsT {
    typedef typename std::conditional<BIG, u64, u32>::type meta_t;
    u64 *pool;
    u32 *bmp;
    u64 *skey;
    meta_t *smeta;
    u32 *sstamp;
    u32 *arena, *bounce;
    u32 np, ns, n_chunks, top, live_runs, next_sid, clock;
    u32 len_bits;               // low bits of a run entry holding chunks - 1
    static DI meta_t pack(u32 off, u32 cnt) { return BIG ? (meta_t)(((u64)off << 32) | cnt) : (meta_t)((off << 16) | cnt); }
    static DI u32 off(meta_t m) { return BIG ? (u32)((u64)m >> 32) : (u32)m >> 16; }
    static DI u32 cnt(meta_t m) { return BIG ? (u32)m : (u32)m & 0xFFFFu; }
};

template <bool BIG>
DI u32 run_start(const VmsT<BIG> &V, u32 run) { return run >> V.len_bits; }
template <bool BIG>
DI u32 run_end(const VmsT<BIG> &V, u32 run) { return (run >> V.len_bits) + (run & ((1u << V.len_bits) - 1u)) + 1u; }
template <bool BIG>
DI u32 run_entries(const VmsT<BIG> &V, u32 len) { return (len + (1u << V.len_bits) - 1u) >> V.len_bits; }

// write the entries of one run (wave-uniform arguments) at arena[at..]; returns how many
template <bool BIG>
DI u32 arena_put(VmsT<BIG> &V, u32 at, u32 start, u32 len)
{
    const u32 n = run_entries(V, len), q = lane_id(), maxlen = 1u << V.len_bits;
    if (q < n) {
        u32 l = min(maxlen, len - q * maxlen);
        V.arena[at + q] = ((start + q * maxlen) << V.len_bits) | (l - 1u);
    }
    wave_sync();
    return n;
}

DI bool bmp_test(const u32 *bmp, u32 c) { return (bmp[c >> 5] >> (c & 31)) & 1u; }

DI u32 word_mask(u32 w, u32 start, u32 end)    // bits of word w inside [start, end)
{
    u32 b0 = (w == (start >> 5)) ? (start & 31) : 0u;
    u32 b1 = (w == ((end - 1) >> 5)) ? ((end - 1) & 31) + 1u : 32u;
    u32 n = b1 - b0;
    return (n == 32 ? 0xFFFFFFFFu : ((1u << n) - 1u)) << b0;
}

// one run, the lanes take one bitmap word each
DI void bmp_fill(u32 *bmp, u32 start, u32 len, bool set)
{
    const u32 end = start + len, w0 = start >> 5, w1 = (end - 1) >> 5;
    for (u32 wb = w0; wb <= w1; wb += 64) {
        u32 w = wb + lane_id();
        if (w <= w1) {
            u32 m = word_mask(w, start, end);
            bmp[w] = set ? (bmp[w] | m) : (bmp[w] & ~m);
        }
    }
    wave_sync();
}

// all runs of one sBlock, one lane per run (runs may share a word: atomics)
template <bool BIG>
DI void bmp_fill_runs(const VmsT<BIG> &V, u32 off, u32 cnt, bool set)
{
    for (u32 rb = 0; rb < cnt; rb += 64) {
        u32 r = rb + lane_id();
        if (r < cnt) {
            u32 run = V.arena[off + r];
            u32 start = run_start(V, run), end = run_end(V, run);
            for (u32 w = start >> 5; w <= (end - 1) >> 5; w++) {
                u32 m = word_mask(w, start, end);
                if (set) atomicOr(&V.bmp[w], m);
                else atomicAnd(&V.bmp[w], ~m);
            }
        }
    }
    wave_sync();
}

// Is sBlock i inactive?  Evaluated by ONE lane for its own index i (lanes work on different
// sBlocks side by side): walks the runs and tests the bitmap words they cover.  A run found
// active is moved to the front of the list (the order of the runs carries no meaning here), so
// the next look at a still-active sBlock usually ends at its first run.
template <bool BIG>
DI bool sblock_inactive_lane(const VmsT<BIG> &V, u32 i)
{
    auto meta = V.smeta[i];
    u32 *runs = V.arena + V.off(meta);
    u32 cnt = V.cnt(meta);
    for (u32 r = 0; r < cnt; r++) {
        u32 run = runs[r];
        u32 start = run_start(V, run), end = run_end(V, run);
        for (u32 w = start >> 5; w <= (end - 1) >> 5; w++) {
            if (V.bmp[w] & word_mask(w, start, end)) {
                if (r) {
                    runs[r] = runs[0];
                    runs[0] = run;
                }
                return false;
            }
        }
    }
    return true;
}

// First inactive sBlock among skey[slo, shi) (pool order), or NONE32.  Sixteen candidates are
// tested side by side, four lanes per candidate, each lane taking every fourth chunk run.
template <bool BIG>
DI u32 first_inactive_sblock(const VmsT<BIG> &V, u32 slo, u32 shi)
{
    const u32 lane = lane_id(), sub = lane & 3, grp = lane >> 2;
    for (u32 base = slo; base < shi; base += 16) {
        const u32 i = base + grp;
        const bool valid = i < shi;
        const auto meta = valid ? V.smeta[i] : 0;
        u32 *runs = V.arena + V.off(meta);
        const u32 cnt = V.cnt(meta);
        u32 at = NONE32, busy_run = 0;                  // index and value of the active run this lane met
        for (u32 r = sub; r < cnt && at == NONE32; r += 4) {
            u32 run = runs[r];
            u32 start = run_start(V, run), end = run_end(V, run);
            for (u32 w = start >> 5; w <= (end - 1) >> 5; w++) {
                if (V.bmp[w] & word_mask(w, start, end)) {
                    at = r;
                    busy_run = run;
                    break;
                }
            }
        }
        const u64 found = ballot(at != NONE32);
        // the first lane of a candidate that met an active run moves it to the front of the list
        if (at != NONE32 && at != 0 && ((found >> (grp * 4)) & ((1u << sub) - 1u)) == 0) {
            runs[at] = runs[0];
            runs[0] = busy_run;
        }
        u64 b = found;
        b |= b >> 1;
        b |= b >> 2;                                    // bit 4g: some lane of candidate g saw an active chunk
        const u64 free16 = ballot(valid && sub == 0) & ~b;
        if (free16) return base + (first_lane(free16) >> 2);
    }
    wave_sync();
    return NONE32;
}

template <bool BIG>
DI void pool_insert(VmsT<BIG> &V, u32 size, u32 start, Acct &A)
{
    u64 key = ((u64)size << 32) | (u32)~start;
    u32 pos = rank_desc(V.pool, V.np, key);
    shift_up(V.pool, pos, V.np);
    st_one(V.pool, pos, key);
    V.np++;
    A.hw_pblocks = max(A.hw_pblocks, V.np);
    wave_sync();
}

template <bool BIG>
DI void pool_remove(VmsT<BIG> &V, u32 idx)
{
    shift_down(V.pool, idx, V.np);
    V.np--;
}

// Stitch: the only creator of sBlocks (Sec. 3.3.1).  The runs are already in the arena.
template <bool BIG>
DI void spool_insert(VmsT<BIG> &V, u32 size, u32 off, u32 cnt, Acct &A)
{
    u32 id = V.next_sid++;
    u64 key = ((u64)size << 32) | (u32)~id;
    u32 pos = rank_desc(V.skey, V.ns, key);
    shift_up(V.skey, pos, V.ns);
    shift_up(V.smeta, pos, V.ns);
    shift_up(V.sstamp, pos, V.ns);
    st_one(V.skey, pos, key);
    st_one(V.smeta, pos, V.pack(off, cnt));
    st_one(V.sstamp, pos, ++V.clock);
    V.ns++;
    V.live_runs += cnt;
    A.n_created++;
    wave_sync();
}

template <bool BIG>
DI void spool_remove(VmsT<BIG> &V, u32 idx)
{
    V.live_runs -= V.cnt(ld_uni(V.smeta, idx));
    shift_down(V.skey, idx, V.ns);
    shift_down(V.smeta, idx, V.ns);
    shift_down(V.sstamp, idx, V.ns);
    V.ns--;
}

// Squeeze the runs of evicted sBlocks out of the arena: copy the live lists to the
// global buffer in sPool order, then back.
template <bool BIG>
DI void arena_compact(VmsT<BIG> &V)
{
    u32 top = 0;
    for (u32 s = 0; s < V.ns; s++) {
        auto meta = ld_uni(V.smeta, s);
        u32 off = V.off(meta), cnt = V.cnt(meta);
        for (u32 r = lane_id(); r < cnt; r += 64) V.bounce[top + r] = V.arena[off + r];
        st_one(V.smeta, s, V.pack(top, cnt));
        top += cnt;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");     // later reads are of other lanes' global writes
    wave_sync();
    if (BIG) {
        u32 *t = V.arena;       // both halves are global: the copy becomes the arena
        V.arena = V.bounce;
        V.bounce = t;
    } else {
        for (u32 r = lane_id(); r < top; r += 64) V.arena[r] = V.bounce[r];
    }
    V.top = top;
    wave_sync();
}

template <bool BIG>
DI bool arena_reserve(VmsT<BIG> &V, u32 need, const KParams &P, Acct &A, u32 ev)
{
    if (V.top + need > P.cap_runs && V.live_runs < V.top) arena_compact(V);
    if (V.top + need > P.cap_runs) {
        table_overflow(A, ev, VMS_ST_OVF_RUNS);
        return false;
    }
    return true;
}

// StitchFree (Sec. 3.3.2, Sec. 4.2.3): while more sBlocks than the threshold are cached,
// release the least recently used one that is inactive.
template <bool BIG>
DI bool stitch_free(VmsT<BIG> &V, const KParams &P, Acct &A)
{
    const u32 lane = lane_id();
    bool any = false;
    while (V.ns > P.spool_threshold) {
        // every lane tests its own sBlocks; the oldest stamp among the inactive ones wins
        u32 best = NONE32, besti = 0;
        for (u32 base = 0; base < V.ns; base += 64) {
            u32 i = base + lane;
            if (i < V.ns) {
                u32 st = V.sstamp[i];
                if (st < best && sblock_inactive_lane(V, i)) {
                    best = st;
                    besti = i;
                }
            }
        }
        u32 m = wave_min_u32(best);
        if (m == NONE32) break;                 // everything cached is in use: the threshold stays exceeded
        u32 victim = from_lane(besti, first_lane(ballot(best == m)));
        spool_remove(V, victim);
        A.n_evicted++;
        any = true;
    }
    A.hw_sblocks = max(A.hw_sblocks, V.ns);     // high-water marks as seen between events
    A.hw_runs = max(A.hw_runs, V.live_runs);
    return any;
}

struct VmsRes {
    u64 dec;                    // decision word (code C_OOM alone when the request failed)
    u32 kind, ref, held;        // what the slot now holds: pBlock first chunk / sBlock number, chunks held
};

// One request of bsize chunks on the stitching path: S1 exact match, else BestFit's
// second loop and the post-processing of its state (Sec. 4.1, Fig. 9).
template <bool BIG>
DI VmsRes vms_alloc(VmsT<BIG> &V, u32 bsize, u64 reserved_units, const KParams &P, Acct &A, u32 ev)
{
    const u32 lane = lane_id();
    VmsRes R;
    R.kind = KIND_PBLOCK;
    R.held = bsize;
    R.ref = 0;

    // ---- S1, stitched blocks: the run of equal sizes in skey[], oldest first
    {
        u32 slo, shi;
        rank_desc2(V.skey, V.ns, ((u64)bsize << 32) | 0xFFFFFFFFu, ((u64)bsize << 32) - 1, &slo, &shi);
        const u32 s = first_inactive_sblock(V, slo, shi);
        if (s != NONE32) {
            auto meta = ld_uni(V.smeta, s);
            bmp_fill_runs(V, V.off(meta), V.cnt(meta), true);
            st_one(V.sstamp, s, ++V.clock);
            wave_sync();
            R.kind = KIND_SBLOCK;
            R.ref = ~(u32)ld_uni(V.skey, s);
            R.dec = C_EXACT | B_SBLOCK | (1ull << 8) | ((u64)R.ref << 32);
            return R;
        }
    }
    // ---- S1, primitive blocks: pool[lo_p, hi_p) are the pBlocks of exactly bsize chunks
    u32 lo_p, hi_p;
    rank_desc2(V.pool, V.np, ((u64)bsize << 32) | 0xFFFFFFFFu, ((u64)bsize << 32) - 1, &lo_p, &hi_p);
    for (u32 base = lo_p; base < hi_p; base += 64) {
        u32 i = base + lane;
        u64 key = i < hi_p ? V.pool[i] : 0;
        u64 m = ballot(i < hi_p && !bmp_test(V.bmp, ~(u32)key));
        if (m) {
            u32 start = ~(u32)from_lane64(key, first_lane(m));
            bmp_fill(V.bmp, start, bsize, true);
            R.ref = start;
            R.dec = C_EXACT | (1ull << 8) | ((u64)start << 32);
            return R;
        }
    }

    // worst-case arena entries of the runs created below, beyond one per candidate
    const u32 slack = 2u * ((P.cap_chunks >> V.len_bits) + 1u) + 2u;

    // ---- Algorithm 1, second loop.  Larger blocks are pool[0, lo_p): the last inactive one in
    // pool order is the single-block candidate (state 2).
    for (u32 hi = lo_p; hi > 0;) {
        u32 lo = hi > 64 ? hi - 64 : 0;
        bool v = lane < hi - lo;
        u64 key = v ? V.pool[hi - 1 - lane] : 0;
        u64 m = ballot(v && !bmp_test(V.bmp, ~(u32)key));
        if (m) {
            u32 l = first_lane(m), idx = hi - 1 - l;
            u64 pk = from_lane64(key, l);
            u32 psize = (u32)(pk >> 32), pstart = ~(u32)pk;
            if (psize < P.frag_limit_chunks) {
                // below the fragmentation limit: not worth cutting, hand it out whole (Sec. 4.2.3)
                bmp_fill(V.bmp, pstart, psize, true);
                R.ref = pstart;
                R.held = psize;
                R.dec = C_SPLIT | (1ull << 8) | ((u64)pstart << 32);
                return R;
            }
            if (V.np + 1 > P.cap_pblocks || V.ns + 1 > P.cap_sblocks || !arena_reserve(V, slack, P, A, ev)) {
                table_overflow(A, ev, (V.np + 1 > P.cap_pblocks ? VMS_ST_OVF_PBLOCKS : 0u) | (V.ns + 1 > P.cap_sblocks ? VMS_ST_OVF_SBLOCKS : 0u));
                R.dec = C_INVALID;
                return R;
            }
            // S2: Split into the request and the rest; a stitched block keeps the uncut size on record
            pool_remove(V, idx);
            pool_insert(V, bsize, pstart, A);
            pool_insert(V, psize - bsize, pstart + bsize, A);
            A.n_split++;
            u32 n = arena_put(V, V.top, pstart, psize);
            spool_insert(V, psize, V.top, n, A);
            V.top += n;
            bmp_fill(V.bmp, pstart, bsize, true);
            R.ref = pstart;
            R.dec = C_SPLIT | B_6 | (1ull << 8) | ((u64)pstart << 32);
            if (stitch_free(V, P, A)) R.dec |= B_7;
            return R;
        }
        hi = lo;
    }

    // Smaller blocks, largest first, until the request is covered (states 3 and 4).  Blocks
    // below the fragmentation limit sit at the tail of the pool and are never stitched.
    u32 lim = V.np;
    if (P.frag_limit_chunks > 1) lim = rank_desc(V.pool, V.np, ((u64)P.frag_limit_chunks << 32) - 1);
    u32 sum = 0, k = 0, pos = NONE32;
    for (u32 base = hi_p; base < lim; base += 64) {
        u32 i = base + lane;
        u64 key = i < lim ? V.pool[i] : 0;
        bool inact = i < lim && !bmp_test(V.bmp, ~(u32)key);
        u32 tot, incl = wave_scan_add(inact ? (u32)(key >> 32) : 0u, &tot);
        u64 im = ballot(inact);
        if (sum + tot >= bsize) {
            u32 l = first_lane(ballot(inact && sum + incl >= bsize));
            pos = base + l;
            k += popc64(im & ((2ull << l) - 1));
            sum += from_lane(incl, l);
            break;
        }
        k += popc64(im);
        sum += tot;
    }
    const bool s3 = pos != NONE32;
    const u32 excess = s3 ? sum - bsize : 0, deficit = s3 ? 0 : bsize - sum;
    if (!s3) {
        // S4 needs new physical chunks; S5 if the device cannot provide them
        if (reserved_units + ((u64)deficit << P.chunk_shift) > P.capacity_units) {
            R.dec = C_OOM;
            return R;
        }
        if (V.n_chunks + deficit > P.cap_chunks) {
            table_overflow(A, ev, VMS_ST_OVF_CHUNKS);
            R.dec = C_INVALID;
            return R;
        }
    }
    if (V.np + 2 > P.cap_pblocks || V.ns + 2 > P.cap_sblocks ||
        !arena_reserve(V, k + (bsize >> V.len_bits) + slack, P, A, ev)) {
        table_overflow(A, ev, (V.np + 2 > P.cap_pblocks ? VMS_ST_OVF_PBLOCKS : 0u) | (V.ns + 2 > P.cap_sblocks ? VMS_ST_OVF_SBLOCKS : 0u));
        R.dec = C_INVALID;
        return R;
    }
    if (!s3 && k == 0) {
        // nothing cached is usable: the new pBlock serves the request directly
        u32 start = V.n_chunks;
        pool_insert(V, deficit, start, A);
        V.n_chunks += deficit;
        bmp_fill(V.bmp, start, deficit, true);
        R.ref = start;
        R.dec = C_GROW | ((u64)start << 32);
        return R;
    }
    // second pass: the candidates' chunk runs go to the arena in pool order
    u32 cnt = 0;
    {
        const u32 endi = s3 ? pos + 1 : lim, maxlen = 1u << V.len_bits;
        for (u32 base = hi_p; base < endi; base += 64) {
            u32 i = base + lane;
            u64 key = i < endi ? V.pool[i] : 0;
            bool inact = i < endi && !bmp_test(V.bmp, ~(u32)key);
            u32 len = (u32)(key >> 32), start = ~(u32)key;
            if (i == pos) len -= excess;
            u64 im = ballot(inact);
            if (ballot(inact && len > maxlen) == 0) {
                if (inact) V.arena[V.top + cnt + rank_in(im)] = (start << V.len_bits) | (len - 1u);
                cnt += popc64(im);
            } else {
                // some candidate is longer than one entry can describe
                u32 ne = inact ? run_entries(V, len) : 0u, tot, incl = wave_scan_add(ne, &tot);
                for (u32 q = 0; q < ne; q++) {
                    u32 l = min(maxlen, len - q * maxlen);
                    V.arena[V.top + cnt + incl - ne + q] = ((start + q * maxlen) << V.len_bits) | (l - 1u);
                }
                cnt += tot;
            }
        }
        wave_sync();
    }
    u32 used = cnt;             // arena entries consumed, including a restore block's
    R.dec = 0;
    if (s3) {
        if (excess) {
            // cut the last candidate so the sum is exact; remember its uncut size (Fig. 9, sBlock 2)
            u64 qk = ld_uni(V.pool, pos);
            u32 qsize = (u32)(qk >> 32), qstart = ~(u32)qk;
            pool_remove(V, pos);
            pool_insert(V, qsize - excess, qstart, A);
            pool_insert(V, excess, qstart + qsize - excess, A);
            A.n_split++;
            u32 n = arena_put(V, V.top + cnt, qstart, qsize);
            spool_insert(V, qsize, V.top + cnt, n, A);
            used += n;
            R.dec |= B_6;
        }
        R.dec |= C_STITCH;
    } else {
        u32 start = V.n_chunks;                 // Alloc: exactly the missing chunks
        pool_insert(V, deficit, start, A);
        V.n_chunks += deficit;
        cnt += arena_put(V, V.top + cnt, start, deficit);
        used = cnt;
        R.dec |= C_GROW;
    }
    R.ref = V.next_sid;
    spool_insert(V, bsize, V.top, cnt, A);
    bmp_fill_runs(V, V.top, cnt, true);
    V.top += used;
    A.hw_members = max(A.hw_members, k + (s3 ? 0u : 1u));
    R.kind = KIND_SBLOCK;
    R.dec |= B_SBLOCK | ((u64)k << 8) | ((u64)R.ref << 32);
    if (stitch_free(V, P, A)) R.dec |= B_7;
    return R;
}

// Update (Sec. 3.3.2): only activity flips; memory stays with its pBlocks.
template <bool BIG>
DI void vms_free(VmsT<BIG> &V, u32 kind, u32 ref, u32 held)
{
    if (kind == KIND_PBLOCK) {
        bmp_fill(V.bmp, ref, held, false);
    } else {
        u64 key = ((u64)held << 32) | (u32)~ref;
        u32 idx = rank_desc(V.skey, V.ns, key);
        auto meta = ld_uni(V.smeta, idx);
        bmp_fill_runs(V, V.off(meta), V.cnt(meta), false);
    }
}

// ---------------------------------------------------------------------------
// The replay loop of one wavefront.  POLICY 0: splitting allocator only.
// POLICY 1: stitching allocator with the splitting pool for small requests.
// ---------------------------------------------------------------------------
template <int POLICY, bool BIG>
__global__ __launch_bounds__(64) void replay_kernel(KParams P, const u64 *__restrict__ events,
                                                    const u32 *__restrict__ n_events, u64 *__restrict__ decisions,
                                                    vms_trace_stats *__restrict__ stats, char *__restrict__ workspace)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const u32 lane = lane_id();
    const u32 trace = blockIdx.x;

    u32 *slot_req = (u32 *)(lds + P.off_slot_req);
    u32 *slot_a = (u32 *)(lds + P.off_slot_a);
    u32 *slot_b = (u32 *)(lds + P.off_slot_b);

    SplitPoolD sp;
    sp.fl = (u64 *)(lds + P.off_fl);
    sp.n = 0;
    sp.cap = P.cap_free;
    sp.reserved = 0;

    VmsT<BIG> V;
    V.np = V.ns = V.n_chunks = V.top = V.live_runs = V.next_sid = V.clock = 0;
    if (POLICY == 1) {
        V.pool = (u64 *)(lds + P.off_pool);
        V.bmp = (u32 *)(lds + P.off_bmp);
        V.skey = (u64 *)(lds + P.off_skey);
        V.smeta = (typename VmsT<BIG>::meta_t *)(lds + P.off_smeta);
        V.sstamp = (u32 *)(lds + P.off_sstamp);
        V.bounce = (u32 *)(workspace + (size_t)trace * P.ws_stride);
        V.arena = BIG ? V.bounce + P.cap_runs : (u32 *)(lds + P.off_arena);
        V.len_bits = P.run_len_bits;
        for (u32 i = lane; i < (P.cap_chunks + 31) / 32; i += 64) V.bmp[i] = 0;
    }
    for (u32 i = lane; i < P.max_slots; i += 64) slot_req[i] = SLOT_UNBOUND;
    wave_sync();

    Acct A;
    acct_init(A);
    u32 code_count = 0;
    const u32 chunk_units = 1u << P.chunk_shift;
    const u32 n_ev = n_events ? min(uni(n_events[trace]), P.max_events) : P.max_events;
    const u64 *ev_row = events + (size_t)trace * P.max_events;
    u64 *dec_row = decisions ? decisions + (size_t)trace * P.max_events : nullptr;

    u64 ev_next = lane < n_ev ? ev_row[lane] : 0;
    for (u32 base = 0; base < n_ev && !A.stop; base += 64) {
        const u32 tile = min(64u, n_ev - base);
        const u64 evw = ev_next;
        if (base + 64 < n_ev) ev_next = base + 64 + lane < n_ev ? ev_row[base + 64 + lane] : 0;   // prefetch
        u32 d_lo = 0, d_hi = 0;
        for (u32 j = 0; j < tile && !A.stop; j++) {
            const u32 ev = base + j;
            const u32 w = from_lane((u32)evw, j), slot = from_lane((u32)(evw >> 32), j);
            const u32 size = w & 0x7FFFFFFFu;
            const bool is_free = w >> 31;
            u64 dec = C_INVALID;
            if (slot < P.max_slots) {
                const u32 req = ld_uni(slot_req, slot);
                if (!is_free) {
                    if (size != 0 && req == SLOT_UNBOUND) {
                        const u64 reserved = sp.reserved + ((u64)V.n_chunks << P.chunk_shift);
                        bool oom = false;
                        u32 held_units = size;
                        if (POLICY == 0 || size < P.small_limit_units) {
                            u32 seg = ((size + chunk_units - 1) >> P.chunk_shift) << P.chunk_shift;
                            SplitRes r = sp_alloc(sp, size, seg, reserved + seg <= P.capacity_units, A, ev);
                            if (r.code == C_OOM) {
                                oom = true;
                            } else {
                                st_one(slot_a, slot, (r.addr << 2) | r.flags);
                                if (POLICY == 1) st_one(slot_b, slot, (u32)KIND_SMALL);
                                dec = r.code | (POLICY == 1 ? B_SMALL : 0) | (r.split ? B_6 : 0) |
                                      ((u64)(r.code == C_GROW ? 0 : 1) << 8) | ((u64)r.addr << 32);
                            }
                        } else {
                            u32 bsize = (size + chunk_units - 1) >> P.chunk_shift;
                            VmsRes r = vms_alloc(V, bsize, reserved, P, A, ev);
                            if ((r.dec & 15) == C_OOM) {
                                oom = true;
                            } else {
                                st_one(slot_a, slot, r.ref);
                                st_one(slot_b, slot, r.kind | (r.held << 2));
                                held_units = r.held << P.chunk_shift;
                                dec = r.dec;
                            }
                        }
                        if (oom) {
                            st_one(slot_req, slot, (u32)SLOT_OOM);
                            if (A.first_oom == NONE32) A.first_oom = ev;
                            dec = C_OOM;
                        } else if (!A.stop) {
                            st_one(slot_req, slot, size);
                            A.requested += size;
                            A.active += held_units;
                            // Sec. 5.1: active and reserved memory are recorded at their peaks; all
                            // three totals can only rise on an allocation
                            A.peak_requested = max(A.peak_requested, A.requested);
                            A.peak_active = max(A.peak_active, A.active);
                            A.peak_reserved = max(A.peak_reserved, sp.reserved + ((u64)V.n_chunks << P.chunk_shift));
                        }
                    }
                } else if (req == SLOT_OOM) {
                    st_one(slot_req, slot, (u32)SLOT_UNBOUND);
                    dec = C_FREE_NOOP;
                } else if (req != SLOT_UNBOUND) {
                    const u32 a = ld_uni(slot_a, slot);
                    const u32 b = POLICY == 1 ? ld_uni(slot_b, slot) : (u32)KIND_SMALL;
                    u32 held_units = req;
                    if ((b & 3) == KIND_SMALL) {
                        bool ml, mr;
                        sp_free(sp, a >> 2, req, a & 3, &ml, &mr, A, ev);
                        dec = C_FREE | (POLICY == 1 ? B_SMALL : 0) | (ml ? B_6 : 0) | (mr ? B_7 : 0) | ((u64)(a >> 2) << 32);
                    } else {
                        vms_free(V, b & 3, a, b >> 2);
                        held_units = (b >> 2) << P.chunk_shift;
                        dec = C_FREE | ((b & 3) == KIND_SBLOCK ? B_SBLOCK : 0) | ((u64)a << 32);
                    }
                    st_one(slot_req, slot, (u32)SLOT_UNBOUND);
                    A.requested -= req;
                    A.active -= held_units;
                }
            }
            wave_sync();
            if (A.stop) break;

            // accounting.  Lane c keeps the event count of decision code c (lane 7: invalid).
            const u32 code = (u32)dec & 15;
            if (code == C_INVALID) A.status |= VMS_ST_INVALID_EVENT;
            code_count += lane == (code == C_INVALID ? 7u : code) ? 1u : 0u;
            const u64 reserved = sp.reserved + ((u64)V.n_chunks << P.chunk_shift);
            const u64 K = 0x9E3779B97F4A7C15ull;
            A.digest = (A.digest ^ dec) * K;
            A.digest = (A.digest ^ A.active) * K;
            A.digest = (A.digest ^ reserved) * K;
            if (lane == j) {
                d_lo = (u32)dec;
                d_hi = (u32)(dec >> 32);
            }
        }
        if (dec_row && lane < tile) dec_row[base + lane] = ((u64)d_hi << 32) | d_lo;
    }

    wave_sync();
    if (lane < 8) stats[(size_t)POLICY * P.n_traces + trace].n_code[lane] = code_count;
    if (lane == 0) {
        vms_trace_stats &s = stats[(size_t)POLICY * P.n_traces + trace];
        const u64 reserved = sp.reserved + ((u64)V.n_chunks << P.chunk_shift);
        s.peak_requested = A.peak_requested * 512;
        s.peak_active = A.peak_active * 512;
        s.peak_reserved = A.peak_reserved * 512;
        s.final_requested = A.requested * 512;
        s.final_active = A.active * 512;
        s.final_reserved = reserved * 512;
        s.digest = A.digest;
        s.n_split = A.n_split;
        s.n_merge = A.n_merge;
        s.n_sblock_created = A.n_created;
        s.n_sblock_evicted = A.n_evicted;
        s.first_oom_event = A.first_oom;
        s.status = A.status;
        s.max_pblocks = A.hw_pblocks;
        s.max_sblocks = A.hw_sblocks;
        s.max_free_blocks = A.hw_free;
        s.max_members = A.hw_members;
        s.max_runs = A.hw_runs;
        s.overflow_event = A.overflow_event;
        // Sec. 5.1: fragmentation = 1 - utilisation, utilisation = peak active / peak reserved
        s.fragmentation = A.peak_reserved ? 1.0 - (double)A.peak_active / (double)A.peak_reserved : 0.0;
    }
}

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
