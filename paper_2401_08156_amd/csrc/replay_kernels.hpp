// Replay kernels: one wavefront (= one workgroup of 64 lanes) replays one trace
// under one policy.  All allocator state of the trace lives in that wave's LDS
// and registers; scalar state (counters, byte totals) stays wave-uniform so the
// compiler keeps it in SGPRs.  Control flow is wave-uniform throughout: the 64
// lanes only ever split up to scan / shift / mark the pool arrays in parallel.
//
// A wave replays alone on its SIMD most of the time, so an event costs
//   4 cycles x instructions issued  +  ~130 cycles x dependent LDS round trips.
// The data layout below is chosen to keep both small on the two hot paths
// (an exact hit on a cached block, and a free): first search level in
// registers, slot table in registers, per-event results parked in lane j of
// four registers and digested once per tile of 64 events.
//
// Policies (GMLake, arXiv 2401.08156): the splitting caching allocator of
// Sec. 2.2 and the stitching allocator of Sec. 3 and Sec. 4.1 (Algorithm 1).
#pragma once
#include <type_traits>
#include "wave_ops.hpp"
#include "replay_plan.hpp"

enum { C_FREE = 0, C_EXACT = 1, C_SPLIT = 2, C_STITCH = 3, C_GROW = 4, C_OOM = 5, C_FREE_NOOP = 6, C_INVALID = 15 };
enum : u32 { B_SMALL = 1u << 4, B_SBLOCK = 1u << 5, B_6 = 1u << 6, B_7 = 1u << 7 };
enum { SLOT_UNBOUND = 0u, SLOT_OOM = 0xFFFFFFFFu };
enum { KIND_SMALL = 0u, KIND_PBLOCK = 1u, KIND_SBLOCK = 2u };
#define NONE32 0xFFFFFFFFu
#define WIT_NONE 32u            // a list entry with an empty mask (first bit 1, last bit 0 of word 0): "no witness"
#define ENT_WORD(e) ((e) >> 12)

// Scalars of one trace that live in LDS (stitching kernel): index k is the u32 at lds[4 k].  The
// first SC_STATE_COUNT are state that only the rare paths need (read when they start, written back
// when they end); the counters after them are only ever updated in place.
enum {
    SC_TOP, SC_LIVE, SC_NEXT_SID,                       // arena top, live list entries, next creation number
    SC_SP_N,                                            // blocks in the splitting pool for requests below one chunk
    SC_NP_ALL,                                          // fine-grained variant: pBlocks of any size
    SC_STATE_COUNT,
    SC_N_SPLIT = SC_STATE_COUNT, SC_N_MERGE, SC_N_CREATED, SC_N_EVICTED, SC_FIRST_OOM, SC_STATUS, SC_OVF_EVENT, SC_STOP,
    SC_HW_PBLOCKS, SC_HW_SBLOCKS, SC_HW_FREE, SC_HW_MEMBERS, SC_HW_RUNS, SC_HW_MULTI,
    SC_COUNT
};

// Event counters and high-water marks of one (trace, policy), addressed by the SC_* indices.
// Two holders with the same interface: registers (splitting kernel, everything inline) and the
// LDS scalars (rare paths of the stitching kernel: updated in place, nothing to load or store).
struct AcctRegs {
    u32 f[SC_COUNT];
    bool stop;
    DI void init()
    {
#pragma unroll
        for (u32 k = 0; k < SC_COUNT; k++) f[k] = 0;
        f[SC_FIRST_OOM] = f[SC_OVF_EVENT] = NONE32;
        stop = false;
    }
    DI void add(u32 k, u32 x) { f[k] += x; }
    DI void peak(u32 k, u32 v) { f[k] = max(f[k], v); }
    // An engine table is too small for this trace: stop replaying it.
    DI void overflow(u32 ev, u32 which)
    {
        f[SC_STATUS] |= VMS_ST_TABLE_OVERFLOW | which;
        if (f[SC_OVF_EVENT] == NONE32) f[SC_OVF_EVENT] = ev;
        stop = true;
    }
};

struct AcctLds {
    u32 *sc;
    u32 *idle;                  // 64 spare words: what the lanes other than lane 0 aim at
    // LDS atomics without a result: nothing to wait for.  Lane 0 updates the scalar, the other lanes
    // a spare word each (no lane is switched off, no two lanes meet at one address)
    DI void add(u32 k, u32 x) { atomicAdd(lane_id() == 0 ? &sc[k] : &idle[lane_id()], x); }
    DI void peak(u32 k, u32 v) { atomicMax(lane_id() == 0 ? &sc[k] : &idle[lane_id()], v); }
    DI void overflow(u32 ev, u32 which)
    {
        st_one(sc, (u32)SC_STATUS, ld_uni(sc, (u32)SC_STATUS) | VMS_ST_TABLE_OVERFLOW | which);
        st_one(sc, (u32)SC_OVF_EVENT, min(ld_uni(sc, (u32)SC_OVF_EVENT), ev));
        st_one(sc, (u32)SC_STOP, 1u);
        wave_sync();
    }
};

// ---------------------------------------------------------------------------
// Slot table: what each handle of the trace currently holds.
//   req  request size in units; 0 = unbound; 0xFFFFFFFF = its ALLOC hit OOM
//   a    splitting pools: address << 2 | segment flags; pBlock: first chunk; sBlock: creation number
//   b    kind | chunks held << 2 (stitching policy only)
//   c    sBlock: its chunk-run list in the arena, offset << 16 | entries (see VmsT)
// IN_REGS: the table is four registers, slot s in lane s (traces with at most 64
// slots): a lookup is a v_readlane, an update a compare-and-select, no LDS round trip.
// ---------------------------------------------------------------------------
template <bool IN_REGS>
struct SlotsT;

template <>
struct SlotsT<true> {
    u32 req, a, b, c;
    DI void init(char *, const KParams &) { req = a = b = c = 0; }
    DI u32 get_req(u32 s) const { return from_lane(req, s); }
    DI u32 get_a(u32 s) const { return from_lane(a, s); }
    DI u32 get_b(u32 s) const { return from_lane(b, s); }
    DI u32 get_c(u32 s) const { return from_lane(c, s); }
    DI void set_req(u32 s, u32 v) { req = write_lane(req, v, s); }
    DI void set_a(u32 s, u32 v) { a = write_lane(a, v, s); }
    DI void set_b(u32 s, u32 v) { b = write_lane(b, v, s); }
    DI void set_c(u32 s, u32 v) { c = write_lane(c, v, s); }
    DI void bind(u32 s, u32 vreq, u32 va, u32 vb, u32 vc) { write_lane4(req, a, b, c, vreq, va, vb, vc, s); }
    // the arena was compacted: the list that was at `from` is now at `to`
    // the lists of the sBlocks have moved: look each held sBlock up by its key (creation number a,
    // b >> 2 chunks) in skey[0..ns) (descending) and take its new place from smeta[]
    DI void relist(const u64 *skey, const u32 *smeta, u32 ns)
    {
        // every lane searches (13 halvings cover 4096 sBlocks), lanes without an sBlock for nothing:
        // no lane is switched off, so the caller keeps its wave-uniform control flow
        const bool holds = req + 1u > 1u && (b & 3) == KIND_SBLOCK;
        const u64 key = ((u64)(b >> 2) << 32) | (u32)~a;
        u32 lo = 0, hi = ns;                    // first index whose key is not greater than key
#pragma unroll 1
        for (u32 it = 0; it < 13; it++) {
            const u32 mid = (lo + hi) >> 1;     // < ns while lo < hi; else a place that exists
            const bool open = lo < hi, greater = skey[mid] > key;
            lo = open && greater ? mid + 1 : lo;
            hi = open && !greater ? mid : hi;
        }
        const u32 found = pin(smeta[lo]);
        c = holds ? found : c;
        wave_sync();
    }
    // fine-grained variant: c is the place of the held sBlock's list.  The list at `from` has moved
    // to `to`; bit 31 marks a slot that has its new place already (places are reused as lists move)
    DI void relocate(u32 from, u32 to)
    {
        const bool hit = req + 1u > 1u && (b & 3) == KIND_SBLOCK && c == from;
        c = hit ? (to | 0x80000000u) : c;
    }
    DI void relocate_done() { c &= 0x7FFFFFFFu; }
};

template <>
struct SlotsT<false> {
    u32 *req, *a, *b;
    uint16_t *c;                // fine-grained variant only: a list place (a 15-bit granule number) and the mark of relocate()
    DI void init(char *lds, const KParams &P)
    {
        req = (u32 *)(lds + P.off_slot_req);
        a = (u32 *)(lds + P.off_slot_a);
        b = (u32 *)(lds + P.off_slot_b);
        c = (uint16_t *)(lds + P.off_slot_c);
        n_slots = P.max_slots;
        for (u32 i = lane_id(); i < P.max_slots; i += 64) req[i] = SLOT_UNBOUND;
    }
    DI u32 get_req(u32 s) const { return ld_uni(req, s); }
    DI u32 get_a(u32 s) const { return ld_uni(a, s); }
    DI u32 get_b(u32 s) const { return ld_uni(b, s); }
    DI u32 get_c(u32 s) const { return ld_uni(c, s); }
    DI void set_req(u32 s, u32 v) { st_one(req, s, v); }
    DI void set_a(u32 s, u32 v) { st_one(a, s, v); }
    DI void set_b(u32 s, u32 v) { st_one(b, s, v); }
    DI void set_c(u32 s, u32 v) { st_one(c, s, (uint16_t)v); }
    DI void bind(u32 s, u32 vreq, u32 va, u32 vb, u32)
    {
        st_one(req, s, vreq);
        st_one(a, s, va);
        st_one(b, s, vb);           // c is not used with the table in LDS
    }
    DI void relist(const u64 *, const u32 *, u32) {}  // c is not used with the table in LDS
    // fine-grained variant (c is used): see SlotsT<true>
    u32 n_slots;
    DI void relocate(u32 from, u32 to)
    {
        for (u32 i = lane_id(); i < n_slots; i += 64) {
            const bool hit = req[i] + 1u > 1u && (b[i] & 3) == KIND_SBLOCK && c[i] == from;
            if (hit) c[i] = (uint16_t)(to | 0x8000u);
        }
        wave_sync();
    }
    DI void relocate_done()
    {
        for (u32 i = lane_id(); i < n_slots; i += 64) c[i] &= 0x7FFFu;
        wave_sync();
    }
};

// ---------------------------------------------------------------------------
// Splitting pool (Sec. 2.2): the inactive blocks of the pool as an unordered
// LDS array of 64-bit keys
//     bits 32-62 size (units) | bits 2-31 address (units) | bit 1 first-in-segment | bit 0 last-in-segment
// so that the minimum key >= (request << 32) is the best fit with the lowest
// address.  Active blocks are not stored: a block's address, size and segment
// flags travel with the slot that holds it.  The two flags replace neighbour
// links: a block may merge to the right iff it is not last in its segment and
// the block starting where it ends is in the array (inactive); same to the left.
// The array is scanned four tiles of 64 keys at a time, all loads issued before
// the first is used, so a scan of up to 256 keys costs one LDS round trip.
// ---------------------------------------------------------------------------
struct SplitPoolD {
    u64 *fl;
    u32 n, cap;
    u32 reserved;               // units obtained so far = next segment address
};

struct SplitRes {
    u32 code, addr, flags;
    bool split;
};

// fl[] is followed by zero keys (128 places past cap): a scan reads whole tiles without
// clamping, and a zero key neither fits a request nor neighbours a block.
template <class AcctT>
DI void sp_alloc(SplitPoolD &sp, u32 size, u32 seg, bool may_grow, AcctT &A, u32 ev, SplitRes &r)
{
    const u32 lane = lane_id();
    r.split = false;
    // step 1: best fit = smallest key not below (size, address 0)
    u64 best = ~0ull;
    u32 besti = 0;
    const u32 last = sp.n - 1;
    const u64 lastk = sp.fl[sp.n ? last : 0u];          // every lane reads the last key: it will fill the hole
    for (u32 base = 0; base < sp.n; base += 256) {
        u64 k[4];
        k[0] = sp.fl[base + lane];
        k[1] = sp.fl[base + 64 + lane];
        k[2] = k[3] = 0;
        if (base + 128 < sp.n) {
            k[2] = sp.fl[base + 128 + lane];
            k[3] = sp.fl[base + 192 + lane];
        }
#pragma unroll
        for (u32 t = 0; t < 4; t++) {
            if (t < 2 || base + 128 < sp.n) {
                const bool ok = (u32)(k[t] >> 32) >= size && k[t] < best;
                best = ok ? k[t] : best;
                besti = ok ? base + t * 64 + lane : besti;
            }
        }
    }
    const u32 hi = (u32)(best >> 32);
    const u32 mhi = sp.n ? wave_min_u32(hi) : NONE32;
    u32 bsize;
    if (mhi != NONE32) {
        const u64 m = ballot(hi == mhi);
        u32 owner = first_lane(m);
        if (m & (m - 1)) {                      // several blocks of that size: lowest address
            const u32 lo = hi == mhi ? (u32)best : NONE32;
            const u32 mlo = wave_min_u32(lo);
            owner = first_lane(ballot(lo == mlo));
        }
        const u32 blo = from_lane((u32)best, owner);
        const u32 idx = from_lane(besti, owner);
        bsize = mhi;
        r.addr = blo >> 2;
        r.flags = blo & 3;
        r.code = C_EXACT;
        if (idx != last) st_one(sp.fl, idx, lastk);     // unordered: the last key fills the hole, a zero its place
        st_one(sp.fl, last, (u64)0);
        sp.n = last;
        wave_sync();
    } else {
        if (!may_grow) {
            r.code = C_OOM;
            r.addr = r.flags = 0;
            return;
        }
        r.addr = sp.reserved;                   // "native allocation": a fresh segment
        sp.reserved += seg;
        bsize = seg;
        r.flags = 3;
        r.code = C_GROW;
    }
    // step 2: cut off what is not needed; it stays cached as the right neighbour
    if (bsize > size) {
        if (sp.n == sp.cap) {
            A.overflow(ev, VMS_ST_OVF_FREE_BLOCKS);
            return;
        }
        const u64 rest = ((u64)(bsize - size) << 32) | ((u64)(r.addr + size) << 2) | (r.flags & 1);
        st_one(sp.fl, sp.n, rest);
        sp.n++;
        A.peak(SC_HW_FREE, sp.n);
        wave_sync();
        r.flags &= 2;
        r.split = true;
        if (r.code == C_EXACT) r.code = C_SPLIT;
        A.add(SC_N_SPLIT, 1);
    }
}

// steps 3 and 4: the block becomes inactive and absorbs inactive neighbours of its segment
template <class AcctT>
DI void sp_free(SplitPoolD &sp, u32 addr, u32 size, u32 flags, bool *ml, bool *mr, AcctT &A, u32 ev)
{
    const u32 lane = lane_id();
    const bool can_l = !(flags & 2), can_r = !(flags & 1);
    const u32 end = addr + size;
    u32 lidx = NONE32, ridx = NONE32;
    u64 lkey = 0, rkey = 0;
    if (can_l || can_r) {
        for (u32 base = 0; base < sp.n; base += 256) {
            u64 k[4];
            k[0] = sp.fl[base + lane];
            k[1] = sp.fl[base + 64 + lane];
            k[2] = k[3] = 0;
            if (base + 128 < sp.n) {
                k[2] = sp.fl[base + 128 + lane];
                k[3] = sp.fl[base + 192 + lane];
            }
#pragma unroll
            for (u32 t = 0; t < 4; t++) {
                if (t < 2 || base + 128 < sp.n) {
                    // a zero key matches nothing: no block ends at 0 that could merge, none starts at an end
                    const u32 ka = (u32)k[t] >> 2, ks = (u32)(k[t] >> 32);
                    const u64 mL = ballot(ka + ks == addr), mR = ballot(ka == end);
                    if (can_l && mL) {
                        lidx = base + t * 64 + first_lane(mL);
                        lkey = from_lane64(k[t], first_lane(mL));
                    }
                    if (can_r && mR) {
                        ridx = base + t * 64 + first_lane(mR);
                        rkey = from_lane64(k[t], first_lane(mR));
                    }
                }
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
    A.add(SC_N_MERGE, (*ml ? 1u : 0u) + (*mr ? 1u : 0u));
    const u64 key = ((u64)size << 32) | ((u64)addr << 2) | flags;
    if (*ml) {
        st_one(sp.fl, lidx, key);               // merged block takes the left neighbour's place
        wave_sync();
        if (*mr) {
            const u32 last = sp.n - 1;
            const u64 lastk = ld_uni(sp.fl, last);
            if (ridx != last) st_one(sp.fl, ridx, lastk);
            st_one(sp.fl, last, (u64)0);
            sp.n = last;
        }
    } else if (*mr) {
        st_one(sp.fl, ridx, key);
    } else {
        if (sp.n == sp.cap) {
            A.overflow(ev, VMS_ST_OVF_FREE_BLOCKS);
            return;
        }
        st_one(sp.fl, sp.n, key);
        sp.n++;
        A.peak(SC_HW_FREE, sp.n);
    }
    wave_sync();
}

// The two holders of a splitting pool behind one interface: the LDS array above, and, for pools of
// at most 64 * TILES inactive blocks, registers.
struct SplitLds {
    SplitPoolD sp;
    DI void init(char *lds, const KParams &P)
    {
        sp.fl = (u64 *)(lds + P.off_fl);
        sp.n = 0;
        sp.cap = P.cap_free;
        sp.reserved = 0;
        for (u32 i = lane_id(); i < P.cap_free + 128; i += 64) sp.fl[i] = 0;    // zero keys behind the live ones
        wave_sync();
    }
    DI u32 reserved() const { return sp.reserved; }
    // done(code, addr, flags, split) once the request is decided (code C_OOM: it failed), ovf() if
    // the table is full instead (see SplitRegs)
    template <class AcctT, class Done, class Ovf>
    DI void alloc(u32 size, u32 seg, bool may_grow, AcctT &A, u32 ev, Done done, Ovf ovf)
    {
        SplitRes r;
        sp_alloc(sp, size, seg, may_grow, A, ev, r);
        if (UNLIKELY(A.stop)) ovf();
        else done(r.code, r.addr, r.flags, r.split);
    }
    template <class AcctT, class Done, class Ovf>
    DI void release(u32 addr, u32 size, u32 flags, AcctT &A, u32 ev, Done done, Ovf ovf)
    {
        bool ml, mr;
        sp_free(sp, addr, size, flags, &ml, &mr, A, ev);
        if (UNLIKELY(A.stop)) ovf();
        else done(ml, mr);
    }
};

// The inactive blocks in registers: key t * 64 + l of the array is k[t] of lane l, 0 = empty place.
// The order of the array means nothing (best fit and the neighbour searches look at every key), so a
// block that leaves just zeroes its place and a new one takes the first empty place.  No LDS access
// at all: a request is compares, one or two wave-wide minima and a few lane selects.
template <u32 TILES>
struct SplitRegs {
    u64 k[TILES];
    u32 n, cap, res;
    DI void init(char *, const KParams &P)
    {
#pragma unroll
        for (u32 t = 0; t < TILES; t++) k[t] = 0;
        n = 0;
        cap = P.cap_free;
        res = 0;
    }
    DI u32 reserved() const { return res; }
    // keys are unique (they contain the address): the place that holds `from` (not 0) takes `to`,
    // found by comparing every place with it, with no book-keeping of where a key sits
    DI void swap_key(u64 from, u64 to)
    {
#pragma unroll
        for (u32 q = 0; q < TILES; q++) k[q] = k[q] == from ? to : k[q];
    }
    DI void insert(u64 key)                     // into an empty place (n < cap <= 64 * TILES: there is one)
    {
        bool any = false;
#pragma unroll
        for (u32 q = 0; q < TILES; q++) any = any || k[q] == 0;
        bool todo = lane_id() == first_lane(ballot(any));       // the first lane with room, its first empty place
#pragma unroll
        for (u32 q = 0; q < TILES; q++) {
            const bool here = todo && k[q] == 0;
            k[q] = here ? key : k[q];
            todo = todo && !here;
        }
        n++;
    }
    // Every outcome ends in a call of its own: done(code, addr, flags, split) once the request is
    // decided (code C_OOM: it failed) or ovf() if the table is full.  Results handed back through
    // one return would meet again in flags that the caller has to test, event after event.
    template <class AcctT, class Done, class Ovf>
    DI void alloc(u32 size, u32 seg, bool may_grow, AcctT &A, u32 ev, Done done, Ovf ovf)
    {
        // step 1: best fit = smallest key not below (size, address 0); an empty place never fits
        u64 best = ~0ull;
#pragma unroll
        for (u32 t = 0; t < TILES; t++) {
            const bool ok = (u32)(k[t] >> 32) >= size && k[t] < best;
            best = ok ? k[t] : best;
        }
        const u32 hi = (u32)(best >> 32);
        const u32 mhi = wave_min_u32(hi);
        if (LIKELY(mhi != NONE32)) {
            const u64 m = ballot(hi == mhi);
            u32 owner = first_lane(m);
            if (m & (m - 1)) {                  // several blocks of that size: lowest address
                const u32 lo = hi == mhi ? (u32)best : NONE32;
                const u32 mlo = wave_min_u32(lo);
                owner = first_lane(ballot(lo == mlo));
            }
            const u32 blo = from_lane((u32)best, owner);
            const u64 chosen = ((u64)mhi << 32) | blo;
            const u32 addr = blo >> 2, flags = blo & 3;
            if (LIKELY(mhi > size)) {
                // step 2: cut off what is not needed; it stays cached as the right neighbour, in the
                // place the block had
                swap_key(chosen, ((u64)(mhi - size) << 32) | ((u64)(addr + size) << 2) | (flags & 1));
                A.peak(SC_HW_FREE, n);
                A.add(SC_N_SPLIT, 1);
                done((u32)C_SPLIT, addr, flags & 2, true);
                return;
            }
            swap_key(chosen, 0);
            n--;
            done((u32)C_EXACT, addr, flags, false);
            return;
        }
        if (!may_grow) {
            done((u32)C_OOM, 0u, 0u, false);
            return;
        }
        const u32 addr = res;                   // "native allocation": a fresh segment
        res += seg;
        if (seg > size) {                       // the rest of a fresh segment
            if (n == cap) {
                A.overflow(ev, VMS_ST_OVF_FREE_BLOCKS);
                ovf();
                return;
            }
            insert(((u64)(seg - size) << 32) | ((u64)(addr + size) << 2) | 1u);
            A.peak(SC_HW_FREE, n);
            A.add(SC_N_SPLIT, 1);
            done((u32)C_GROW, addr, 2u, true);
            return;
        }
        done((u32)C_GROW, addr, 3u, false);
    }
    // steps 3 and 4: the block becomes inactive and absorbs inactive neighbours of its segment
    template <class AcctT, class Done, class Ovf>
    DI void release(u32 addr, u32 size, u32 flags, AcctT &A, u32 ev, Done done, Ovf ovf)
    {
        bool ml_, mr_;
        bool *ml = &ml_, *mr = &mr_;
        const bool can_l = !(flags & 2), can_r = !(flags & 1);
        const u32 end = addr + size;
        // at most one block ends where this one starts and at most one starts where it ends: every
        // lane folds its places into one candidate per side, two ballots decide
        u64 lk = 0, rk = 0;
#pragma unroll
        for (u32 t = 0; t < TILES; t++) {
            // an empty place matches nothing: no block ends at 0 that could merge, none starts at an end
            const u32 ka = (u32)k[t] >> 2, ks = (u32)(k[t] >> 32);
            lk = ka + ks == addr ? k[t] : lk;
            rk = ka == end ? k[t] : rk;
        }
        const u64 mL = can_l ? ballot(lk != 0) : 0, mR = can_r ? ballot(rk != 0) : 0;
        const u64 lkey = from_lane64(lk, first_lane(mL | (1ull << 63))), rkey = from_lane64(rk, first_lane(mR | (1ull << 63)));
        *ml = mL != 0;
        *mr = mR != 0;
        if (*mr) {
            size += (u32)(rkey >> 32);
            flags = (flags & 2) | ((u32)rkey & 1);
        }
        if (*ml) {
            addr = (u32)lkey >> 2;
            size += (u32)(lkey >> 32);
            flags = ((u32)lkey & 2) | (flags & 1);
        }
        A.add(SC_N_MERGE, (*ml ? 1u : 0u) + (*mr ? 1u : 0u));
        const u64 key = ((u64)size << 32) | ((u64)addr << 2) | flags;
        if (UNLIKELY(*ml)) {
            swap_key(lkey, key);                // the merged block takes the left neighbour's place
            if (*mr) {
                swap_key(rkey, 0);
                n--;
            }
        } else if (*mr) {
            swap_key(rkey, key);
        } else {
            if (n == cap) {
                A.overflow(ev, VMS_ST_OVF_FREE_BLOCKS);
                ovf();
                return;
            }
            insert(key);
            A.peak(SC_HW_FREE, n);
        }
        done(ml_, mr_);
    }
};

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
//            then older first), with smeta[] = arena offset << 16 | entries, sstamp[] = last use,
//            swit[] = a "witness": the list entry that was seen active last (or WIT_NONE).  While the
//            witness is still active the sBlock is known to be active after one bitmap read.
//   arena[]  chunk runs of all cached sBlocks, bump-allocated, cut at bitmap word boundaries:
//            one 32-bit entry  word << 12 | first bit << 5 | last bit  per range of consecutive
//            chunks inside one bitmap word (bits 10-11 number the ranges of one word; unused).
//            Testing, setting or clearing an sBlock is one step over its entries, one lane per
//            entry: the test reads the words, set and clear are LDS atomics without a result, so
//            several ranges of one word need no ordering and a FREE waits for nothing but its list.
//   tmp[]    scratch bitmap of the same size as bmp[] (+ 64 spare words), zero between uses: a new list is OR-ed
//            together here and read back word by word, which merges touching runs.
//            Compacted through a global-memory buffer when full.
//   pp, sp   first level of the rank searches in pool[] and skey[], held in registers.
// ---------------------------------------------------------------------------
struct VmsT {
    typedef u32 meta_t;
    u64 *pool;
    u32 *bmp;
    u64 *skey;
    meta_t *smeta;
    u32 *sstamp, *swit, *tmp;
    u32 *idle;                  // 64 spare words behind tmp[]: targets of lanes that have nothing to update
    u32 *arena, *bounce;
    u32 np, ns, n_chunks, top, live_ent, next_sid, clock;
    u32 e_skip;                 // a list entry with an empty mask on the spare word behind the bitmap
    Probe pp, sp;
    static DI meta_t pack(u32 off, u32 cnt) { return (off << 16) | cnt; }
    static DI u32 off(meta_t m) { return m >> 16; }
    static DI u32 cnt(meta_t m) { return m & 0xFFFFu; }
    static DI meta_t pinm(meta_t m) { return pin(m); }      // pin() for a list place
};

DI u32 from_lane_any(u32 v, u32 l) { return from_lane(v, l); }
DI u64 from_lane_any(u64 v, u32 l) { return from_lane64(v, l); }

// bits of one list entry inside its bitmap word
DI u32 emask(u32 e) { return (2u << (e & 31)) - (1u << ((e >> 5) & 31)); }

DI u32 run_words(u32 start, u32 len) { return ((start + len - 1) >> 5) - (start >> 5) + 1; }

// entry q of the run [start, start + len)
DI u32 run_entry(u32 start, u32 len, u32 q)
{
    const u32 w0 = start >> 5, endm1 = start + len - 1, w = w0 + q;
    const u32 lo = q == 0 ? (start & 31) : 0u;
    const u32 hi = w == (endm1 >> 5) ? (endm1 & 31) : 31u;
    return (w << 12) | (lo << 5) | hi;
}

// write the entries of one run (wave-uniform arguments) at arena[at..]; returns how many
DI u32 arena_put(VmsT &V, u32 at, u32 start, u32 len)
{
    const u32 n = run_words(start, len);
    for (u32 qb = 0; qb < n; qb += 64) {
        // lanes past the run write its last entry again
        const u32 q = min(qb + lane_id(), n - 1);
        V.arena[at + q] = run_entry(start, len, q);
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

// one run, the lanes take one bitmap word each; lanes past its end rewrite the spare word behind
// the bitmap (no divergent branch)
DI void bmp_fill(u32 *bmp, u32 spare, u32 start, u32 len, bool set)
{
    const u32 end = start + len, w0 = start >> 5, w1 = (end - 1) >> 5;
    for (u32 wb = w0; wb <= w1; wb += 64) {
        const u32 w = wb + lane_id();
        const bool in = w <= w1;
        const u32 mw = pin(word_mask(w, start, end));          // computed by every lane: no branch
        const u32 m = in ? mw : 0u, wi = in ? w : spare;
        const u32 old = pin(bmp[wi]);
        bmp[wi] = set ? (old | m) : (old & ~m);
    }
    wave_sync();
}

// One tile of list entries, one lane per entry (e, if live): their bits are set or cleared with LDS
// atomics that return nothing, so entries that share a bitmap word need no ordering and the wave
// does not wait for the result.  Lanes without an entry OR a zero into a spare word of their own.
DI void entries_apply(const VmsT &V, u32 e, bool live, bool set)
{
    u32 *t = live ? &V.bmp[ENT_WORD(e)] : &V.idle[lane_id()];
    const u32 m = live ? emask(e) : 0u;
    if (set) atomicOr(t, m);
    else atomicAnd(t, ~m);
}

// all entries of one sBlock
DI void bmp_fill_entries(const VmsT &V, u32 off, u32 cnt, bool set)
{
    for (u32 rb = 0; rb < cnt; rb += 64) {
        const u32 r = rb + lane_id();
        const u32 e = V.arena[off + (r < cnt ? r : 0u)];
        entries_apply(V, e, r < cnt, set);
    }
    wave_sync();
}

// A new list is collected in tmp[]: mark one run per lane (lanes with len == 0 mark nothing;
// wmin / wmax: per-lane range of the bitmap words touched so far) ...
DI void list_mark(const VmsT &V, u32 start, u32 len, u32 &wmin, u32 &wmax)
{
    const u32 end = start + len;
    const u32 w0 = len ? start >> 5 : NONE32, w1 = len ? (end - 1) >> 5 : 0u;
    for (u32 q = 0; ballot(len && w0 + q <= w1); q++) {
        // lanes with nothing left OR a zero into a word of their own
        const bool in = len && w0 + q <= w1;
        const u32 mw = pin(word_mask(w0 + q, start, end));
        atomicOr(in ? &V.tmp[w0 + q] : &V.idle[lane_id()], in ? mw : 0u);
    }
    wmin = min(wmin, w0);
    wmax = max(wmax, w1);
}

// ... and read back as entries at arena[at..], one per range of consecutive chunks inside a word
// (touching runs have merged), leaving tmp[] zero.  Returns the number of entries.
DI u32 list_extract(const VmsT &V, u32 wmin, u32 wmax, u32 at, u32 spare)
{
    u32 cnt = 0;
    for (u32 wb = wmin; wb <= wmax; wb += 64) {
        const u32 w = min(wb + lane_id(), wmax);     // lanes past the end: the last word again, taken as empty
        const u32 mw = pin(V.tmp[w]);
        u32 m = wb + lane_id() <= wmax ? mw : 0u;
        wave_sync();
        V.tmp[w] = 0;
        const u32 nr = (u32)__builtin_popcount(m & ~(m << 1));      // ranges start where a set bit follows a clear one
        u32 tot;
        const u32 incl = wave_scan_add(nr, &tot);
        const u32 o = at + cnt + incl - nr;
        for (u32 r = 0; ballot(m != 0); r++) {
            // a lane whose word is used up writes into the spare places behind the arena
            const bool some = m != 0;
            const u32 mm = some ? m : 1u;
            const u32 lo = (u32)__builtin_ctz(mm);
            const u32 rest = ~(mm >> lo);
            const u32 len = rest ? (u32)__builtin_ctz(rest) : 32u;
            const u32 hi = lo + len - 1;
            V.arena[some ? o + r : spare + lane_id()] = (w << 12) | ((r < 3 ? r : 3u) << 10) | (lo << 5) | hi;
            m = some ? m & ~((2u << hi) - (1u << lo)) : 0u;
        }
        cnt += tot;
    }
    wave_sync();
    return cnt;
}

// Is sBlock i inactive?  Evaluated by ONE lane for its own index i (lanes work on different
// sBlocks side by side): the witness first, then the whole list.
DI bool sblock_inactive_lane(const VmsT &V, u32 i)
{
    const u32 wit = V.swit[i];
    if (V.bmp[ENT_WORD(wit)] & emask(wit)) return false;
    const auto meta = V.smeta[i];
    const u32 *list = V.arena + V.off(meta);
    const u32 cnt = V.cnt(meta);
    for (u32 r = 0; r < cnt; r++) {
        const u32 e = list[r];
        if (V.bmp[ENT_WORD(e)] & emask(e)) {
            V.swit[i] = e;
            return false;
        }
    }
    return true;
}

template <class AcctT>
DI void pool_insert(VmsT &V, u32 size, u32 start, AcctT &A)
{
    u64 key = ((u64)size << 32) | (u32)~start;
    u32 pos = rank_desc(V.pool, V.np, key);
    shift_up(V.pool, pos, V.np);
    st_one(V.pool, pos, key);
    V.np++;
    A.peak(SC_HW_PBLOCKS, V.np);
    wave_sync();
}

// Split (Sec. 3.3.1): the pBlock at pool[idx] is replaced by its two pieces, both smaller and
// therefore further down in pool order.  Only the keys between the old place and the new
// places move: down by one up to the larger piece, up by one after the smaller piece.
template <class AcctT>
DI void pool_cut(VmsT &V, u32 idx, u32 size_a, u32 start_a, u32 size_b, u32 start_b, AcctT &A)
{
    u64 k1 = ((u64)size_a << 32) | (u32)~start_a, k2 = ((u64)size_b << 32) | (u32)~start_b;
    if (k1 < k2) {
        const u64 t = k1;
        k1 = k2;
        k2 = t;
    }
    u32 r1, r2;                                 // ranks among the old keys (the cut block counts in both)
    rank_desc2(V.pool, V.np, k1, k2, &r1, &r2);
    shift_down(V.pool, idx, r1);                // pool[idx+1 .. r1) -> pool[idx .. r1-1)
    shift_up(V.pool, r2, V.np);                 // pool[r2 .. np) -> pool[r2+1 .. np+1)
    st_one(V.pool, r1 - 1, k1);
    st_one(V.pool, r2, k2);
    V.np++;
    A.peak(SC_HW_PBLOCKS, V.np);
    wave_sync();
}

// skey[], smeta[], sstamp[] and swit[] move together: entries [pos, n) one place up (highest
// tile first) or entries (pos, n) one place down (lowest tile first), one LDS round trip per tile
DI void spool_shift_up(VmsT &V, u32 pos, u32 n)
{
    for (u32 hi = n; hi > pos;) {
        const u32 lo = hi - pos > 64 ? hi - 64 : pos;
        const u32 i = lo + lane_id(), src = i < hi ? i : i + 1;   // lanes above the part that moves: see shift_up
        const u64 k = V.skey[src];
        const auto m = V.smeta[src];
        const u32 st = V.sstamp[src], w = V.swit[src];
        V.skey[i + 1] = k;
        V.smeta[i + 1] = m;
        V.sstamp[i + 1] = st;
        V.swit[i + 1] = w;
        hi = lo;
    }
    wave_sync();
}

DI void spool_shift_down(VmsT &V, u32 pos, u32 n)
{
    for (u32 lo = pos + 1; lo < n; lo += 64) {
        const u32 i = lo + lane_id(), dst = i < n ? i - 1 : i;   // lanes past the end: see shift_down
        const u64 k = V.skey[i];
        const auto m = V.smeta[i];
        const u32 st = V.sstamp[i], w = V.swit[i];
        V.skey[dst] = k;
        V.smeta[dst] = m;
        V.sstamp[dst] = st;
        V.swit[dst] = w;
    }
    wave_sync();
}

// Stitch: the only creator of sBlocks (Sec. 3.3.1).  The entries are already in the arena.
// Returns the position of the new sBlock in skey[].
template <class AcctT>
DI u32 spool_insert(VmsT &V, u32 size, u32 off, u32 cnt, AcctT &A, bool probe_valid)
{
    u32 id = V.next_sid++;
    u64 key = ((u64)size << 32) | (u32)~id;
    // probe_valid: skey[] has not changed since its first search level was put into registers
    u32 pos = probe_valid ? rank_fast<false>(V.sp, V.skey, V.ns, key) : rank_desc(V.skey, V.ns, key);
    spool_shift_up(V, pos, V.ns);
    st_one(V.skey, pos, key);
    st_one(V.smeta, pos, V.pack(off, cnt));
    st_one(V.sstamp, pos, ++V.clock);
    // every sBlock starts out active (it is handed out, or the first part of the block it records
    // is): its first entry is a valid witness from the end of this event on
    st_one(V.swit, pos, ld_uni(V.arena, off));
    V.ns++;
    V.live_ent += cnt;
    A.add(SC_N_CREATED, 1);
    wave_sync();
    return pos;
}

DI void spool_remove(VmsT &V, u32 idx)
{
    V.live_ent -= V.cnt(ld_uni(V.smeta, idx));
    spool_shift_down(V, idx, V.ns);
    V.ns--;
    st_one(V.skey, V.ns, (u64)0);               // zero keys follow the live ones (see rank_fast)
    wave_sync();
}

// Squeeze the entries of evicted sBlocks out of the arena: copy the live lists to the
// global buffer in sPool order, then back.  Slots holding an sBlock learn its new place.
template <class Slots>
DI void arena_compact(VmsT &V, Slots &S, const KParams &P)
{
    u32 top = 0;
    for (u32 s = 0; s < V.ns; s++) {
        auto meta = ld_uni(V.smeta, s);
        u32 off = V.off(meta), cnt = V.cnt(meta);
        for (u32 rb = 0; rb < cnt; rb += 64) {          // lanes past the end copy the last entry again
            const u32 r = min(rb + lane_id(), cnt - 1);
            V.bounce[top + r] = V.arena[off + r];
        }
        st_one(V.smeta, s, V.pack(top, cnt));
        S.moved((u32)meta, (u32)V.pack(top, cnt), P);
        top += cnt;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");     // later reads are of other lanes' global writes
    wave_sync();
    for (u32 rb = 0; rb < top; rb += 64) {
        const u32 r = min(rb + lane_id(), top - 1);
        V.arena[r] = V.bounce[r];
    }
    V.top = top;
    wave_sync();
}

template <class Slots, class AcctT>
DI bool arena_reserve(VmsT &V, Slots &S, u32 need, const KParams &P, AcctT &A, u32 ev)
{
    if (UNLIKELY(V.top + need > P.cap_runs && V.live_ent < V.top)) arena_compact(V, S, P);
    if (UNLIKELY(V.top + need > P.cap_runs)) {
        A.overflow(ev, VMS_ST_OVF_RUNS);
        return false;
    }
    return true;
}

// Is any chunk of the list arena[off .. off + cnt) active?  All lanes work on the one list; if so,
// *witness receives an entry that was seen active.
DI bool list_busy(const VmsT &V, u32 off, u32 cnt, u32 *witness)
{
    for (u32 eb = 0; eb < cnt; eb += 64) {
        const u32 k = eb + lane_id();
        const u32 ek = pin(V.arena[off + (k < cnt ? k : 0u)]);
        const u32 e = k < cnt ? ek : V.e_skip;
        const u32 wk = pin(V.bmp[ENT_WORD(e)]);
        const u64 bm = ballot((wk & emask(e)) != 0);
        if (bm) {
            *witness = from_lane(e, first_lane(bm));
            return true;
        }
    }
    return false;
}

// StitchFree (Sec. 3.3.2, Sec. 4.2.3): while more sBlocks than the threshold are cached,
// release the least recently used one that is inactive.  One scan rules out, side by side, every
// sBlock whose witness is still active (three tiles at a time: all stamps and witnesses are loaded,
// then all witness words, two LDS round trips per 192 sBlocks) and leaves in every lane the two
// least recently used of the sBlocks it saw.  The oldest of all is tested with all lanes on its
// list; if it is active after all, its lane falls back on its second and the search goes on
// without a new scan (a lane that runs out of its two forces one).
template <class AcctT>
DI bool stitch_free(VmsT &V, const KParams &P, AcctT &A)
{
    const u32 lane = lane_id();
    bool any = false;
    while (V.ns > P.spool_threshold) {
        u32 victim = NONE32;
        bool rescan = true;
        u32 b1 = NONE32, i1 = 0, b2 = NONE32, i2 = 0;
        bool spent = false;                     // this lane has given up its best once since the scan
        for (;;) {
            if (rescan) {
                b1 = b2 = NONE32;
                i1 = i2 = 0;
                spent = false;
                for (u32 g = 0; g < V.ns; g += 192) {
                    u32 st[3], wit[3], ww[3];
#pragma unroll
                    for (u32 t = 0; t < 3; t++) {
                        const u32 i = g + t * 64 + lane, ic = i < V.ns ? i : 0u;
                        st[t] = V.sstamp[ic];
                        wit[t] = V.swit[ic];
                    }
#pragma unroll
                    for (u32 t = 0; t < 3; t++) ww[t] = pin(V.bmp[ENT_WORD(wit[t])]);
#pragma unroll
                    for (u32 t = 0; t < 3; t++) {
                        const u32 i = g + t * 64 + lane;
                        const bool ok = (i < V.ns) & ((ww[t] & emask(wit[t])) == 0);
                        const u32 sv = ok ? st[t] : NONE32;
                        const bool lt1 = sv < b1, lt2 = sv < b2;
                        b2 = lt1 ? b1 : (lt2 ? sv : b2);
                        i2 = lt1 ? i1 : (lt2 ? i : i2);
                        b1 = lt1 ? sv : b1;
                        i1 = lt1 ? i : i1;
                    }
                }
                rescan = false;
            }
            const u32 m = wave_min_u32(b1);
            if (m == NONE32) break;             // everything cached is in use: the threshold stays exceeded
            const u32 owner = first_lane(ballot(b1 == m));
            const u32 c = from_lane(i1, owner);
            const auto meta = ld_uni(V.smeta, c);
            u32 witness;
            if (!list_busy(V, V.off(meta), V.cnt(meta), &witness)) {
                victim = c;
                break;
            }
            st_one(V.swit, c, witness);         // active after all: remember where, look further
            wave_sync();
            rescan = from_lane(spent ? 1u : 0u, owner) != 0;
            const bool mine = lane == owner;
            b1 = mine ? b2 : b1;
            i1 = mine ? i2 : i1;
            b2 = mine ? NONE32 : b2;
            spent = spent || mine;
        }
        if (victim == NONE32) break;
        spool_remove(V, victim);
        A.add(SC_N_EVICTED, 1);
        any = true;
    }
    A.peak(SC_HW_SBLOCKS, V.ns);     // high-water marks as seen between events
    A.peak(SC_HW_RUNS, V.live_ent);
    return any;
}


// ---- S1 (Algorithm 1, first loop; Sec. 4.1 state S1), stitched blocks, oldest first.  The
// sBlocks of exactly bsize chunks start at the rank of (bsize, oldest) in skey[].  One lane per
// candidate reads its witness: a candidate whose witness is still active is out after two LDS
// round trips for the whole tile.  The others are tested in pool order with all lanes over the
// entries of one list; the first inactive one is handed out (ref = creation number, list = where
// its entries are).  This is the general route, from the tile that starts at `base`.
DI bool s1_sblock_from(VmsT &V, u32 bsize, u32 base, u32 &ref, u32 &list)
{
    const u32 lane = lane_id();
    for (;;) {
        // skey[] is followed by zero keys and swit[] by harmless entries: no index is clamped
        const u32 i = base + lane;
        const u64 key = V.skey[i];
        const u32 wit = V.swit[i];
        const auto meta = V.smeta[i];
        const u64 vm = ballot((u32)(key >> 32) == bsize);
        if (!vm) return false;
        const u32 wv = pin(V.bmp[ENT_WORD(wit)]);
        u64 unknown = vm & ~ballot((wv & emask(wit)) != 0);
        while (unknown) {
            const u32 l = first_lane(unknown);
            const auto m = from_lane_any(meta, l);
            const u32 off = V.off(m), cnt = V.cnt(m);
            // lanes past the end of the list hold an entry with an empty mask on the spare word
            const u32 e0 = pin(V.arena[off + lane]);
            u32 e = lane < cnt ? e0 : V.e_skip;
            const u32 word = pin(V.bmp[ENT_WORD(e)]);
            u64 bm = ballot((word & emask(e)) != 0);
            if (cnt > 64) {                     // long list: the rest of it, a tile at a time
                for (u32 eb = 64; eb < cnt && !bm; eb += 64) {
                    const u32 k = eb + lane;
                    const u32 ek = pin(V.arena[off + (k < cnt ? k : 0u)]);
                    e = k < cnt ? ek : V.e_skip;
                    const u32 wk = pin(V.bmp[ENT_WORD(e)]);
                    bm = ballot((wk & emask(e)) != 0);
                }
                if (!bm) {
                    bmp_fill_entries(V, off, cnt, true);
                    st_one(V.sstamp, base + l, ++V.clock);
                    ref = ~from_lane((u32)key, l);
                    list = (u32)m;
                    return true;
                }
            }
            if (!bm) {
                entries_apply(V, e, lane < cnt, true);      // inactive: hand it out
                st_one(V.sstamp, base + l, ++V.clock);
                ref = ~from_lane((u32)key, l);
                list = (u32)m;
                return true;
            }
            st_one(V.swit, base + l, from_lane(e, first_lane(bm)));
            unknown &= unknown - 1;
        }
        if (~vm) return false;                  // the run of equal sizes ended inside this tile
        base += 64;
    }
}

// (The usual route is written out in the replay loop and costs four dependent LDS round trips:
// the block of keys that the rank search reads, first level in registers, is taken as the first
// tile of candidates right away, together with their witnesses and list places; then the
// witnesses' bitmap words; then the list of the first candidate not ruled out; then the bitmap
// words of its entries.  Anything unusual - a long list, a candidate that turns out active, a run
// of equal sizes that leaves the tile - comes here.)

// ---- S1, primitive blocks: the first inactive pBlock of exactly bsize chunks in pool order.  As
// above, the block of the rank search doubles as the first tile of candidates.
DI bool s1_pblock(VmsT &V, u32 bsize, u32 &start)
{
    const u32 lane = lane_id();
    const u64 q = ((u64)bsize << 32) | 0xFFFFFFFFu;
    u32 base;
    if (V.pp.stride >= 64) {
        base = rank_fast<false>(V.pp, V.pool, V.np, q);
    } else {
        const u32 c = popc64(ballot(V.pp.v > q));
        base = dec_sat(c) * V.pp.stride;  // the first pBlock of bsize chunks lies inside this tile
    }
    for (;;) {
        const u32 i = base + lane;
        const u64 key = V.pool[i];                  // zero keys follow the pool
        const bool eq = (u32)(key >> 32) == bsize;
        const u64 vm = ballot(eq);
        if (!vm) return false;
        const u32 st = ~(u32)key;
        const u32 word = pin(V.bmp[eq ? st >> 5 : 0u]);
        const u64 m = ballot(eq && !((word >> (st & 31)) & 1u));
        if (LIKELY(m)) {
            start = from_lane(st, first_lane(m));
            return true;
        }
        if (~vm >> 63) return false;                // the run ended inside the tile
        base += 64;
    }
}

struct VmsRes {
    u32 dec_lo;                 // low decision word (code C_OOM alone when the request failed)
    u32 ref;                    // pBlock first chunk / sBlock creation number (= high decision word)
    u32 kind, held;             // what the slot now holds, chunks held
    u32 list;                   // sBlock: offset << 16 | entries of its list
};

// No block of exactly bsize chunks is free: BestFit's second loop and the post-processing of
// its state (Algorithm 1; Sec. 4.1, Fig. 9, states S2 to S5).  The rare path: a few per cent of
// the requests of a converged trace.
template <class Slots, class AcctT>
DI void vms_alloc_rest(VmsT &V, Slots &S, u32 bsize, u32 reserved_units, const KParams &P, AcctT &A, u32 ev,
                       VmsRes &R)
{
    const u32 lane = lane_id();
    R.kind = KIND_PBLOCK;
    R.held = bsize;
    R.ref = 0;
    R.list = 0;
    // pool[lo_p, hi_p) are the pBlocks of exactly bsize chunks (all active, or S1 had taken one)
    u32 lo_p, hi_p;
    {
        const u64 k1 = ((u64)bsize << 32) | 0xFFFFFFFFu, k2 = ((u64)bsize << 32) - 1;
        if (LIKELY(V.pp.stride <= 64)) {
            // the first search level is in registers and still describes the pool: one LDS round trip
            const u32 c1 = popc64(ballot(V.pp.v > k1)), c2 = popc64(ballot(V.pp.v > k2));
            const u32 b1 = dec_sat(c1) * V.pp.stride, b2 = dec_sat(c2) * V.pp.stride;
            const u64 v1 = V.pool[b1 + lane], v2 = V.pool[b2 + lane];
            lo_p = b1 + popc64(ballot(v1 > k1));
            hi_p = b2 + popc64(ballot(v2 > k2));
        } else {
            rank_desc2(V.pool, V.np, k1, k2, &lo_p, &hi_p);
        }
    }

    // ---- Algorithm 1, second loop.  Larger blocks are pool[0, lo_p): the last inactive one in
    // pool order is the single-block candidate (state 2).
    for (u32 hi = lo_p; hi > 0;) {
        u32 lo = hi > 64 ? hi - 64 : 0;
        const bool v = lane < hi - lo;
        const u64 key = V.pool[v ? hi - 1 - lane : 0u];
        const u32 fc = v ? ~(u32)key : 0u;                  // first chunk (chunk 0 for lanes without a block)
        const u32 kw = pin(V.bmp[fc >> 5]);
        const u64 m = ballot(v && !((kw >> (fc & 31)) & 1u));
        if (m) {
            u32 l = first_lane(m), idx = hi - 1 - l;
            u64 pk = from_lane64(key, l);
            u32 psize = (u32)(pk >> 32), pstart = ~(u32)pk;
            if (UNLIKELY(psize < P.frag_limit_chunks)) {
                // below the fragmentation limit: not worth cutting, hand it out whole (Sec. 4.2.3)
                bmp_fill(V.bmp, ENT_WORD(V.e_skip), pstart, psize, true);
                R.ref = pstart;
                R.held = psize;
                R.dec_lo = C_SPLIT | (1u << 8);
                return;
            }
            if (UNLIKELY(V.np + 1 > P.cap_pblocks || V.ns + 1 > P.cap_sblocks ||
                         !arena_reserve(V, S, run_words(pstart, psize), P, A, ev))) {
                A.overflow(ev, (V.np + 1 > P.cap_pblocks ? VMS_ST_OVF_PBLOCKS : 0u) | (V.ns + 1 > P.cap_sblocks ? VMS_ST_OVF_SBLOCKS : 0u));
                R.dec_lo = C_INVALID;
                return;
            }
            // S2: Split into the request and the rest; a stitched block keeps the uncut size on record
            pool_cut(V, idx, bsize, pstart, psize - bsize, pstart + bsize, A);
            A.add(SC_N_SPLIT, 1);
            u32 n = arena_put(V, V.top, pstart, psize);
            spool_insert(V, psize, V.top, n, A, true);
            V.top += n;
            bmp_fill(V.bmp, ENT_WORD(V.e_skip), pstart, bsize, true);
            R.ref = pstart;
            R.dec_lo = C_SPLIT | B_6 | (1u << 8);
            if (stitch_free(V, P, A)) R.dec_lo |= B_7;
            return;
        }
        hi = lo;
    }

    // Smaller blocks, largest first, until the request is covered (states 3 and 4).  Blocks
    // below the fragmentation limit sit at the tail of the pool and are never stitched.
    u32 lim = V.np;
    if (UNLIKELY(P.frag_limit_chunks > 1)) lim = rank_desc(V.pool, V.np, ((u64)P.frag_limit_chunks << 32) - 1);
    u32 sum = 0, k = 0, pos = NONE32;
    for (u32 base = hi_p; base < lim; base += 64) {
        const u32 i = base + lane;
        const u64 key = V.pool[i < lim ? i : 0u];
        const u32 fc = i < lim ? ~(u32)key : 0u;
        const u32 kw = pin(V.bmp[fc >> 5]);
        const bool inact = i < lim && !((kw >> (fc & 31)) & 1u);
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
        if (UNLIKELY(reserved_units + (deficit << P.chunk_shift) > P.capacity_units)) {
            R.dec_lo = C_OOM;
            return;
        }
        if (UNLIKELY(V.n_chunks + deficit > P.cap_chunks)) {
            A.overflow(ev, VMS_ST_OVF_CHUNKS);
            R.dec_lo = C_INVALID;
            return;
        }
    }
    if (!s3 && k == 0) {
        // nothing cached is usable: the new pBlock serves the request directly (no list, no sBlock)
        if (UNLIKELY(V.np + 1 > P.cap_pblocks)) {
            A.overflow(ev, VMS_ST_OVF_PBLOCKS);
            R.dec_lo = C_INVALID;
            return;
        }
        u32 start = V.n_chunks;
        pool_insert(V, deficit, start, A);
        V.n_chunks += deficit;
        bmp_fill(V.bmp, ENT_WORD(V.e_skip), start, deficit, true);
        R.ref = start;
        R.dec_lo = C_GROW;
        return;
    }
    // list entries created below: a run of L chunks touches at most L / 32 + 2 bitmap words
    const u32 need = 2u * k + 3u * (((sum > bsize ? sum : bsize) >> 5) + 2u);
    if (UNLIKELY(V.np + 2 > P.cap_pblocks || V.ns + 2 > P.cap_sblocks || !arena_reserve(V, S, need, P, A, ev))) {
        A.overflow(ev, (V.np + 2 > P.cap_pblocks ? VMS_ST_OVF_PBLOCKS : 0u) | (V.ns + 2 > P.cap_sblocks ? VMS_ST_OVF_SBLOCKS : 0u));
        R.dec_lo = C_INVALID;
        return;
    }
    // second pass: the candidates' chunk runs (and the new pBlock's) are collected in tmp[] and
    // read back as the list
    u32 cnt;
    {
        u32 wmin = NONE32, wmax = 0;
        const u32 endi = s3 ? pos + 1 : lim;
        for (u32 base = hi_p; base < endi; base += 64) {
            const u32 i = base + lane;
            const u64 key = V.pool[i < endi ? i : 0u];
            const u32 fc = i < endi ? ~(u32)key : 0u;
            const u32 kw = pin(V.bmp[fc >> 5]);
            const bool inact = i < endi && !((kw >> (fc & 31)) & 1u);
            u32 len = (u32)(key >> 32), start = ~(u32)key;
            if (i == pos) len -= excess;
            list_mark(V, start, inact ? len : 0u, wmin, wmax);
        }
        if (!s3) list_mark(V, V.n_chunks, lane == 0 ? deficit : 0u, wmin, wmax);
        wave_sync();
        cnt = list_extract(V, wave_min_u32(wmin), wave_max_u32(wmax), V.top, P.cap_runs);
    }
    u32 used = cnt;             // arena entries consumed, including a restore block's
    R.dec_lo = 0;
    if (s3) {
        if (excess) {
            // cut the last candidate so the sum is exact; remember its uncut size (Fig. 9, sBlock 2)
            u64 qk = ld_uni(V.pool, pos);
            u32 qsize = (u32)(qk >> 32), qstart = ~(u32)qk;
            pool_cut(V, pos, qsize - excess, qstart, excess, qstart + qsize - excess, A);
            A.add(SC_N_SPLIT, 1);
            u32 n = arena_put(V, V.top + cnt, qstart, qsize);
            spool_insert(V, qsize, V.top + cnt, n, A, true);
            used += n;
            R.dec_lo |= B_6;
        }
        R.dec_lo |= C_STITCH;
    } else {
        u32 start = V.n_chunks;                 // Alloc: exactly the missing chunks
        pool_insert(V, deficit, start, A);
        V.n_chunks += deficit;
        R.dec_lo |= C_GROW;
    }
    R.ref = V.next_sid;
    spool_insert(V, bsize, V.top, cnt, A, !(s3 && excess));
    bmp_fill_entries(V, V.top, cnt, true);
    R.list = (u32)V.pack(V.top, cnt);
    V.top += used;
    A.peak(SC_HW_MEMBERS, k + (s3 ? 0u : 1u));
    R.kind = KIND_SBLOCK;
    R.dec_lo |= B_SBLOCK | (k << 8);
    if (stitch_free(V, P, A)) R.dec_lo |= B_7;
}

// Update (Sec. 3.3.2) of an sBlock that is looked up by its key (slot table in LDS)
DI void vms_free_by_key(VmsT &V, u32 ref, u32 held)
{
    const u64 key = ((u64)held << 32) | (u32)~ref;
    const u32 idx = rank_fast<false>(V.sp, V.skey, V.ns, key);
    const auto meta = ld_uni(V.smeta, idx);
    bmp_fill_entries(V, V.off(meta), V.cnt(meta), false);
}

// ---------------------------------------------------------------------------
// Hot and cold halves.  The replay loop keeps only what the two frequent paths need in registers
// (exact hit on a cached block, free).  The states S2 to S5 and the splitting pool for requests below
// one chunk sit behind unlikely branches and keep the scalars only they need in the first 256 bytes of
// LDS (SC_* above, one u32 each), where the event counters are updated in place as well.
// ---------------------------------------------------------------------------
#define LDS_SCALARS 0u
static_assert(SC_COUNT <= 64, "LDS header layout");

// stand-in for the slot table inside the rare paths: they only note that lists have moved
struct ColdSlots {
    bool compacted;
    DI void moved(u32, u32, const KParams &) { compacted = true; }
};

// the LDS scalars in registers, one LDS access for all of them: lane k holds scalar k
struct ColdState {
    u32 v;
    // pinned: every lane must load its scalar even if only one lane goes on to use them
    DI void load(const char *lds) { v = pin(((const u32 *)(lds + LDS_SCALARS))[lane_id()]); }
    DI u32 get(u32 k) const { return from_lane(v, k); }
};

DI void vms_bind(VmsT &V, char *lds, char *ws_slice, const KParams &P)
{
    V.pool = (u64 *)(lds + P.off_pool);
    V.bmp = (u32 *)(lds + P.off_bmp);
    V.skey = (u64 *)(lds + P.off_skey);
    V.smeta = (VmsT::meta_t *)(lds + P.off_smeta);
    V.sstamp = (u32 *)(lds + P.off_sstamp);
    V.swit = (u32 *)(lds + P.off_swit);
    V.tmp = (u32 *)(lds + P.off_tmp);
    V.idle = V.tmp + (P.cap_chunks + 31) / 32;
    V.e_skip = (((P.cap_chunks + 31) / 32) << 12) | WIT_NONE;
    V.bounce = (u32 *)ws_slice;                 // where arena_compact copies the lists
    V.arena = (u32 *)(lds + P.off_arena);
}

// A request for bsize chunks that no cached block fits exactly (states S2 to S5): inlined into the
// replay loop (a call would cost more in saved registers than the few per cent of the requests
// that come here can repay), working on the loop's own pool state; the three scalars that only
// this path needs (arena top, live entries, next creation number) wait in LDS in between.
// Returns false if an engine table overflowed (the trace ends).
DI bool vms_alloc_cold(char *lds, VmsT &V, const KParams &P, u32 bsize, u32 reserved_units, u32 ev, VmsRes &R,
                       bool &compacted)
{
    u32 *sc = (u32 *)(lds + LDS_SCALARS);
    ColdState C;
    C.load(lds);
    V.top = C.get(SC_TOP);
    V.live_ent = C.get(SC_LIVE);
    V.next_sid = C.get(SC_NEXT_SID);
    AcctLds A;
    A.sc = sc;
    A.idle = V.idle;
    ColdSlots S;
    S.compacted = false;
    vms_alloc_rest(V, S, bsize, reserved_units, P, A, ev, R);
    st_one(sc, (u32)SC_TOP, V.top);
    st_one(sc, (u32)SC_LIVE, V.live_ent);
    st_one(sc, (u32)SC_NEXT_SID, V.next_sid);
    wave_sync();
    compacted = S.compacted;
    return ld_uni(sc, (u32)SC_STOP) == 0;
}

// Requests below one chunk under the stitching policy: its private splitting pool (Sec. 3.1), whose
// two scalars (blocks in the list, units reserved) wait in LDS between requests.
DI void small_alloc(char *lds, const KParams &P, u32 *idle, u32 size, u32 seg, bool may_grow, u32 ev, SplitRes &r,
                    u32 &sp_reserved)
{
    u32 *sc = (u32 *)(lds + LDS_SCALARS);
    SplitPoolD sp;
    sp.fl = (u64 *)(lds + P.off_fl);
    sp.cap = P.cap_free;
    sp.n = ld_uni(sc, (u32)SC_SP_N);
    sp.reserved = sp_reserved;
    AcctLds A;
    A.sc = sc;
    A.idle = idle;
    sp_alloc(sp, size, seg, may_grow, A, ev, r);
    st_one(sc, (u32)SC_SP_N, sp.n);
    sp_reserved = sp.reserved;
    wave_sync();
}

DI void small_free(char *lds, const KParams &P, u32 *idle, u32 addr, u32 size, u32 flags, u32 ev, bool *ml, bool *mr)
{
    u32 *sc = (u32 *)(lds + LDS_SCALARS);
    SplitPoolD sp;
    sp.fl = (u64 *)(lds + P.off_fl);
    sp.cap = P.cap_free;
    sp.n = ld_uni(sc, (u32)SC_SP_N);
    sp.reserved = 0;            // not used by a release
    AcctLds A;
    A.sc = sc;
    A.idle = idle;
    sp_free(sp, addr, size, flags, ml, mr, A, ev);
    st_one(sc, (u32)SC_SP_N, sp.n);
    wave_sync();
}

// The per-tile work shared by both replay kernels: one event per lane.
struct TileOut {
    u32 n_code[8];              // events of this lane per decision code ([7]: invalid)
    u64 dig;                    // this lane's share of the digest
    DI void init()
    {
#pragma unroll
        for (u32 c = 0; c < 8; c++) n_code[c] = 0;
        dig = 0;
    }
};

// the last tile of a trace (or the tile in which a table overflowed): only the lanes below `done` store
__device__ __attribute__((noinline)) void emit_partial(u64 *dst, u64 dec, u32 done)
{
    if (lane_id() < done) dst[lane_id()] = dec;
}

DI void tile_emit(TileOut &T, u64 *dec_row, u32 base, u32 done, u32 v_dlo, u32 v_dhi, u32 v_act, u32 v_res)
{
    const u32 lane = lane_id();
    const bool valid = lane < done;
    const u64 dec = ((u64)v_dhi << 32) | v_dlo;
    if (dec_row) {
        if (done == 64) dec_row[base + lane] = dec;         // a full tile: one coalesced store, no lane off
        else emit_partial(dec_row + base, dec, done);
    }
    const u32 code = v_dlo & 15, cidx = !valid ? 8u : (code == C_INVALID ? 7u : code);
#pragma unroll
    for (u32 c = 0; c < 8; c++) T.n_code[c] += cidx == c ? 1u : 0u;
    // digest: sum over events i of (decision * K1 + (active << 32 | reserved)) * ((2 i + 1) * K2)
    const u64 term = (dec * 0x9E3779B97F4A7C15ull + (((u64)v_act << 32) | v_res)) *
                     ((2ull * (base + lane) + 1ull) * 0xD6E8FEB86659FD93ull);
    T.dig += valid ? term : 0ull;
}

// end of the trace: the lanes' shares become the totals (all lanes return the same values)
DI u64 tile_totals(const TileOut &T, u32 n_code[8])
{
#pragma unroll
    for (u32 c = 0; c < 8; c++) n_code[c] = (u32)wave_sum_u64(T.n_code[c]);
    return wave_sum_u64(T.dig);
}

// The second pass (vms_config.retry_traces): a launch of a few wavefronts with larger
// tables that replays every trace whose first replay ended in a table overflow.  The wavefronts
// share one counter over the trace numbers: each takes 64 numbers at a time, looks at their
// status words side by side and replays the flagged ones among them one after the other.
struct SecondPass {
    u64 flagged = 0;
    u32 first = 0;
    // the next flagged trace for this wavefront, or false when all have been handed out
    DI bool next(const KParams &P, const vms_trace_stats *__restrict__ st, u32 *counter, u32 &trace)
    {
        while (!flagged) {
            u32 b = 0;
            if (lane_id() == 0) b = atomicAdd(counter, 64u);
            first = from_lane(b, 0);
            if (first >= P.n_traces) return false;
            const u32 t = first + lane_id();
            flagged = ballot(t < P.n_traces && (st[t < P.n_traces ? t : 0u].status & VMS_ST_TABLE_OVERFLOW) != 0);
        }
        trace = first + first_lane(flagged);
        flagged &= flagged - 1;
        return true;
    }
};

// ---------------------------------------------------------------------------
// Replay under the stitching policy (Sec. 3, Sec. 4.1), one wavefront per trace.
// SLOT_REGS: slot table in registers (max_slots <= 64).
//
// Per event only the allocator runs; the decision word and the active / reserved totals after
// the event are parked in lane j of four registers.  Once per tile of 64 events the lanes store
// the decisions with one coalesced write, count the decision codes and fold their event into
// the digest, all 64 events side by side.
// ---------------------------------------------------------------------------
template <bool SLOT_REGS>
__global__ __launch_bounds__(64) void replay_vms_kernel(KParams P, const u64 *__restrict__ events,
                                                        const u32 *__restrict__ n_events,
                                                        u64 *__restrict__ decisions, vms_trace_stats *__restrict__ stats,
                                                        char *__restrict__ workspace)
{
    WAVE_DYNAMIC_LDS(lds);
    const u32 lane = lane_id();
    const u32 trace = blockIdx.x;
    constexpr bool USE_LIST = SLOT_REGS;
    char *ws_slice = workspace + (size_t)trace * P.ws_stride;
    // a second pass follows for traces that outgrow these tables: it counts the traces it takes on
    if (P.retry_slots && trace == 0) ((u32 *)&stats[2 * (size_t)P.n_traces])[1] = 0;     // the second pass counts from 0

    SlotsT<SLOT_REGS> S;
    S.init(lds, P);
    ((u32 *)(lds + LDS_SCALARS))[lane] = lane == SC_FIRST_OOM || lane == SC_OVF_EVENT ? NONE32 : 0u;     // LDS header
    VmsT V;
    vms_bind(V, lds, ws_slice, P);
    V.np = V.ns = V.n_chunks = V.top = V.live_ent = V.next_sid = V.clock = 0;
    V.pp.v = V.sp.v = 0;
    V.pp.stride = V.sp.stride = 1;
    for (u32 i = lane; i < (P.cap_chunks + 31) / 32; i += 64) V.bmp[i] = V.tmp[i] = 0;
    V.tmp[(P.cap_chunks + 31) / 32 + lane] = 0;             // 64 spare words: where idle lanes OR their zeros
    // the searches read up to 64 places past the live part of pool[], skey[], swit[] and arena[]
    // without clamping: zero keys there, and witnesses / entries on words that exist
    if (!P.small_regs)
        for (u32 i = lane; i < P.cap_free + 128; i += 64) ((u64 *)(lds + P.off_fl))[i] = 0;
    SplitRegs<3> Q;                                         // the pool for small requests, if it fits registers
    Q.init(lds, P);
    for (u32 i = lane; i < P.cap_pblocks + 64; i += 64) V.pool[i] = 0;
    for (u32 i = lane; i < P.cap_sblocks + 64; i += 64) {
        V.skey[i] = 0;
        V.swit[i] = WIT_NONE;
        V.smeta[i] = 0;
    }
    for (u32 i = lane; i < P.cap_runs + 64; i += 64) V.arena[i] = WIT_NONE;
    st_one(V.bmp, (P.cap_chunks + 31) / 32, 0u);                // the spare word
    wave_sync();

    u32 requested = 0, active = 0, peak_requested = 0, peak_active = 0;
    u32 sp_reserved = 0;        // small-request pool: units reserved so far
    bool stop = false;
    TileOut T;
    T.init();
    const u32 chunk_units = 1u << P.chunk_shift;
    const u32 n_ev = n_events ? min(uni(n_events[trace]), P.max_events) : P.max_events;
    const u64 *ev_row = events + (size_t)trace * P.max_events;
    u64 *dec_row = decisions ? decisions + (size_t)trace * P.max_events : nullptr;

    u32 fast_limit = P.small_limit_units;   // requests from this size on take the usual S1 route (renewed with the probe)
    u64 ev_next = lane < n_ev ? ev_row[lane] : 0;
    for (u32 base = 0; base < n_ev; base += 64) {
        const u32 tile = min(64u, n_ev - base);
        const u32 ev_lo = (u32)ev_next, ev_hi = (u32)(ev_next >> 32);
        if (base + 64 < n_ev) {                             // prefetch; lanes past the end re-read the last event
            const u32 nx = base + 64 + lane;
            const u64 x = pin64(ev_row[min(nx, n_ev - 1)]);
            ev_next = nx < n_ev ? x : 0;
        }
        u32 v_dlo = 0, v_dhi = 0, v_act = 0, v_res = 0;
        u32 done = tile, todo = tile;       // todo drops to 0 when an engine table overflows: the trace ends there
        // every path of an event ends by parking its results in lane j and going on to the next event
#define EMIT(DLO, DHI)                                                     \
    {                                                                      \
        write_lane4(v_dlo, v_dhi, v_act, v_res, (DLO), (DHI), active,      \
                    sp_reserved + (V.n_chunks << P.chunk_shift), j);       \
        wave_sync();                                                       \
        continue;                                                          \
    }
        for (u32 j = 0; j < todo; j++) {
            const u32 w = from_lane(ev_lo, j), slot = from_lane(ev_hi, j);
            if (UNLIKELY(slot >= P.max_slots)) EMIT((u32)C_INVALID, 0u)
            const u32 req = S.get_req(slot);
            if ((int)w < 0) {
                // ---- FREE.  Update (Sec. 3.3.2): only activity flips; memory stays with its pBlocks
                if (UNLIKELY(req + 1u <= 1u)) {             // unbound, or bound to a request that failed
                    if (req == SLOT_OOM) {
                        S.set_req(slot, (u32)SLOT_UNBOUND);
                        EMIT((u32)C_FREE_NOOP, 0u)
                    }
                    EMIT((u32)C_INVALID, 0u)
                }
                const u32 a = S.get_a(slot), b = S.get_b(slot);
                const u32 kind = b & 3;
                S.set_req(slot, (u32)SLOT_UNBOUND);
                requested -= req;
                if (LIKELY((kind & KIND_SBLOCK) != 0)) {    // (a bit test: the usual case stays the fall-through)
                    if (USE_LIST) {
                        const u32 list = S.get_c(slot), off = list >> 16, cnt = list & 0xFFFFu;
                        // one list read, then the entries' bits cleared without waiting for anything
                        if (LIKELY(cnt <= 64)) entries_apply(V, V.arena[off + lane], lane < cnt, false);
                        else bmp_fill_entries(V, off, cnt, false);
                    } else {
                        vms_free_by_key(V, a, b >> 2);
                    }
                    active -= (b >> 2) << P.chunk_shift;
                    EMIT(C_FREE | B_SBLOCK, a)
                }
                if (kind == KIND_PBLOCK) {
                    bmp_fill(V.bmp, ENT_WORD(V.e_skip), a, b >> 2, false);
                    active -= (b >> 2) << P.chunk_shift;
                    EMIT((u32)C_FREE, a)
                }
                if (LIKELY(P.small_regs)) {
                    AcctLds A;
                    A.sc = (u32 *)(lds + LDS_SCALARS);
                    A.idle = V.idle;
                    Q.release(a >> 2, req, a & 3, A, base + j,
                              [&](bool ml, bool mr) {
                                  active -= req;
                                  write_lane4(v_dlo, v_dhi, v_act, v_res, C_FREE | B_SMALL | (ml ? B_6 : 0u) | (mr ? B_7 : 0u),
                                              a >> 2, active, sp_reserved + (V.n_chunks << P.chunk_shift), j);
                                  wave_sync();
                              },
                              [&]() {
                                  stop = true;
                                  done = j;
                                  todo = 0;
                              });
                    continue;
                }
                bool ml, mr;
                small_free(lds, P, V.idle, a >> 2, req, a & 3, base + j, &ml, &mr);
                if (UNLIKELY(ld_uni((u32 *)(lds + LDS_SCALARS), (u32)SC_STOP) != 0)) {
                    stop = true;
                    done = j;
                    todo = 0;
                    continue;
                }
                active -= req;
                EMIT(C_FREE | B_SMALL | (ml ? B_6 : 0u) | (mr ? B_7 : 0u), a >> 2)
            }
            // ---- ALLOC
            const u32 size = w;
            if (UNLIKELY(size == 0 || req != SLOT_UNBOUND)) EMIT((u32)C_INVALID, 0u)
            if (LIKELY(size >= fast_limit)) {
                const u32 bsize = (size + chunk_units - 1) >> P.chunk_shift;
                u32 ref, list = 0;
                // Sec. 5.1: active memory is recorded at its peak; the totals only rise on an allocation
#define S1_SBLOCK_HIT                                                      \
    {                                                                      \
        S.bind(slot, size, ref, KIND_SBLOCK | (bsize << 2), list);         \
        requested += size;                                                 \
        active += bsize << P.chunk_shift;                                  \
        peak_requested = max(peak_requested, requested);                   \
        peak_active = max(peak_active, active);                            \
        EMIT(C_EXACT | B_SBLOCK | (1u << 8), ref)                          \
    }
                // S1 on stitched blocks, the usual way (see s1_sblock_from for the general route).  It is
                // written out here, not called, so that the hit leaves for the next event from where it
                // is found: returned through a function it would meet the other outcomes again and
                // cost a flag and two branches to tell them apart.
                u32 from = NONE32;              // where the general route goes on; NONE32: no inactive sBlock of this size
                switch (0) {
                default:
                    const u64 q = ((u64)bsize << 32) | 0xFFFFFFFFu;
                    // keys greater than q end at most `stride` < 64 places into the block: the first
                    // sBlock of bsize chunks, if there is one, lies inside the tile
                    const u32 c = popc64(ballot(V.sp.v > q));
                    const u32 b0 = dec_sat(c) * V.sp.stride;
                    const u32 i = b0 + lane;
                    // (pinned, after all three loads are on their way: one round trip, not the last two
                    // behind the branch)
                    const u64 key = V.skey[i];
                    const u32 wit0 = V.swit[i];
                    const auto meta0 = V.smeta[i];
                    const u32 wit = pin(wit0);
                    const auto meta = VmsT::pinm(meta0);
                    const u64 vm = ballot((u32)(key >> 32) == bsize);
                    if (UNLIKELY(!vm)) break;
                    const u32 wv = pin(V.bmp[ENT_WORD(wit)]);
                    const u64 unknown = vm & ~ballot((wv & emask(wit)) != 0);
                    if (UNLIKELY(!unknown)) {
                        if (~vm >> 63) break;   // the run of equal sizes ended inside the tile: all known active
                        from = b0 + 64;
                        break;
                    }
                    const u32 l = first_lane(unknown);
                    const auto m = from_lane_any(meta, l);
                    const u32 off = V.off(m), cnt = V.cnt(m);
                    const u32 e0 = pin(V.arena[off + lane]);
                    const u32 e = lane < cnt ? e0 : V.e_skip;
                    const u32 word = pin(V.bmp[ENT_WORD(e)]);
                    if (LIKELY(cnt <= 64 && !ballot((word & emask(e)) != 0))) {
                        entries_apply(V, e, lane < cnt, true);
                        st_one(V.sstamp, b0 + l, ++V.clock);
                        ref = ~from_lane((u32)key, l);
                        list = (u32)m;
                        S1_SBLOCK_HIT
                    }
                    from = b0 + l;
                }
                if (UNLIKELY(from != NONE32))
                    if (s1_sblock_from(V, bsize, from, ref, list)) S1_SBLOCK_HIT
#define S1_PBLOCK_TRY                                                      \
    if (s1_pblock(V, bsize, ref)) {                                        \
        bmp_fill(V.bmp, ENT_WORD(V.e_skip), ref, bsize, true);             \
        S.set_a(slot, ref);                                                \
        S.set_b(slot, KIND_PBLOCK | (bsize << 2));                         \
        S.set_req(slot, size);                                             \
        requested += size;                                                 \
        active += bsize << P.chunk_shift;                                  \
        peak_requested = max(peak_requested, requested);                   \
        peak_active = max(peak_active, active);                            \
        EMIT(C_EXACT | (1u << 8), ref)                                     \
    }
                S1_PBLOCK_TRY
            } else if (UNLIKELY(size >= P.small_limit_units)) {
                // more than 4,032 sBlocks cached: their first search level no longer selects a single
                // tile (fast_limit keeps such a trace off the route above, at no cost to the others)
                const u32 bsize = (size + chunk_units - 1) >> P.chunk_shift;
                u32 ref, list = 0;
                const u32 from = rank_fast<false>(V.sp, V.skey, V.ns, ((u64)bsize << 32) | 0xFFFFFFFFu);
                if (s1_sblock_from(V, bsize, from, ref, list)) S1_SBLOCK_HIT
                S1_PBLOCK_TRY
            }
#undef S1_PBLOCK_TRY
#undef S1_SBLOCK_HIT
            // ---- the rare cases: no exact fit (states S2 to S5), or a request below one chunk
            u32 dlo, dhi = 0, held_units = size;
            wave_sync();
            if (size >= P.small_limit_units) {
                const u32 bsize = (size + chunk_units - 1) >> P.chunk_shift;
                VmsRes R;
                bool compacted;
                const bool went = vms_alloc_cold(lds, V, P, bsize, sp_reserved + (V.n_chunks << P.chunk_shift), base + j,
                                                      R, compacted);
                // the pools may have changed: renew the first search level of both
                probe_refresh(V.sp, V.skey, V.ns);
                probe_refresh(V.pp, V.pool, V.np);
                fast_limit = V.sp.stride >= 64 ? NONE32 : P.small_limit_units;
                // lists have moved: every slot holding an sBlock looks its list up again
                if (USE_LIST && UNLIKELY(compacted)) S.relist(V.skey, (const u32 *)V.smeta, V.ns);
                if (UNLIKELY(!went)) {                                // an engine table overflowed: the trace ends here
                    stop = true;
                    done = j;
                    todo = 0;
                    continue;
                }
                dlo = R.dec_lo;
                if (LIKELY((dlo & 15) != C_OOM)) {
                    dhi = R.ref;
                    S.set_a(slot, dhi);
                    S.set_b(slot, R.kind | (R.held << 2));
                    if (USE_LIST) S.set_c(slot, R.list);
                    held_units = R.held << P.chunk_shift;
                }
            } else {
                const u32 seg = ((size + chunk_units - 1) >> P.chunk_shift) << P.chunk_shift;
                const u32 reserved = sp_reserved + (V.n_chunks << P.chunk_shift);
                if (LIKELY(P.small_regs)) {
                    AcctLds A;
                    A.sc = (u32 *)(lds + LDS_SCALARS);
                    A.idle = V.idle;
                    Q.alloc(size, seg, reserved + seg <= P.capacity_units, A, base + j,
                            [&](u32 code, u32 addr, u32 flags, bool split) {
                                sp_reserved = Q.reserved();
                                u32 d_lo = C_OOM, d_hi = 0;
                                if (code == C_OOM) {
                                    S.set_req(slot, (u32)SLOT_OOM);
                                    ColdState C;            // rare: note the first failed request
                                    C.load(lds);
                                    if (C.get(SC_FIRST_OOM) == NONE32)
                                        st_one((u32 *)(lds + LDS_SCALARS), (u32)SC_FIRST_OOM, base + j);
                                } else {
                                    S.set_a(slot, (addr << 2) | flags);
                                    S.set_b(slot, (u32)KIND_SMALL);
                                    S.set_req(slot, size);
                                    requested += size;
                                    active += size;
                                    peak_requested = max(peak_requested, requested);
                                    peak_active = max(peak_active, active);
                                    d_lo = code | B_SMALL | (split ? B_6 : 0u) | ((code == C_GROW ? 0u : 1u) << 8);
                                    d_hi = addr;
                                }
                                write_lane4(v_dlo, v_dhi, v_act, v_res, d_lo, d_hi, active,
                                            sp_reserved + (V.n_chunks << P.chunk_shift), j);
                                wave_sync();
                            },
                            [&]() {
                                stop = true;
                                done = j;
                                todo = 0;
                            });
                    continue;
                }
                SplitRes r;
                small_alloc(lds, P, V.idle, size, seg, reserved + seg <= P.capacity_units, base + j, r, sp_reserved);
                if (UNLIKELY(ld_uni((u32 *)(lds + LDS_SCALARS), (u32)SC_STOP) != 0)) {
                    stop = true;
                    done = j;
                    todo = 0;
                    continue;
                }
                dlo = C_OOM;
                if (r.code != C_OOM) {
                    const u32 af = (r.addr << 2) | r.flags;
                    S.set_a(slot, af);
                    S.set_b(slot, (u32)KIND_SMALL);
                    dlo = r.code | B_SMALL | (r.split ? B_6 : 0u) | ((r.code == C_GROW ? 0u : 1u) << 8);
                    dhi = r.addr;
                }
            }
            if (UNLIKELY((dlo & 15) == C_OOM)) {
                S.set_req(slot, (u32)SLOT_OOM);
                ColdState C;                                // rare: note the first failed request
                C.load(lds);
                if (C.get(SC_FIRST_OOM) == NONE32) st_one((u32 *)(lds + LDS_SCALARS), (u32)SC_FIRST_OOM, base + j);
                EMIT((u32)C_OOM, 0u)
            }
            S.set_req(slot, size);
            requested += size;
            active += held_units;
            peak_requested = max(peak_requested, requested);
            peak_active = max(peak_active, active);
            EMIT(dlo, dhi)
        }
#undef EMIT
        tile_emit(T, dec_row, base, done, v_dlo, v_dhi, v_act, v_res);
        if (stop) break;
    }

    wave_sync();
    u32 n_code[8];
    const u64 digest = tile_totals(T, n_code);
    ColdState C;
    C.load(lds);
    // (lane reads stay outside the one-lane block below: they are wave-wide operations)
    u32 sc[SC_COUNT];
#pragma unroll
    for (u32 k = 0; k < SC_COUNT; k++) sc[k] = C.get(k);
    if (lane == 0) {
        vms_trace_stats &s = stats[(size_t)P.n_traces + trace];
#pragma unroll
        for (u32 c = 0; c < 8; c++) s.n_code[c] = n_code[c];
        const u64 reserved = sp_reserved + (V.n_chunks << P.chunk_shift);
        s.peak_requested = (u64)peak_requested * 512;
        s.peak_active = (u64)peak_active * 512;
        s.peak_reserved = reserved * 512;           // reserved memory never shrinks: its peak is its final value
        s.final_requested = (u64)requested * 512;
        s.final_active = (u64)active * 512;
        s.final_reserved = reserved * 512;
        s.digest = digest;
        s.n_split = sc[SC_N_SPLIT];
        s.n_merge = sc[SC_N_MERGE];
        s.n_sblock_created = sc[SC_N_CREATED];
        s.n_sblock_evicted = sc[SC_N_EVICTED];
        s.first_oom_event = sc[SC_FIRST_OOM];
        s.status = sc[SC_STATUS] | (n_code[7] ? VMS_ST_INVALID_EVENT : 0u);
        s.max_pblocks = sc[SC_HW_PBLOCKS];
        s.max_sblocks = sc[SC_HW_SBLOCKS];
        s.max_free_blocks = sc[SC_HW_FREE];
        s.max_members = sc[SC_HW_MEMBERS];
        s.max_runs = sc[SC_HW_RUNS];
        s.overflow_event = sc[SC_OVF_EVENT];
        s.max_multi_pblocks = sc[SC_HW_MULTI];
        s.reserved1 = 0;
        // Sec. 5.1: fragmentation = 1 - utilisation, utilisation = peak active / peak reserved
        s.fragmentation = reserved ? 1.0 - (double)peak_active / (double)reserved : 0.0;
    }
}

// ---------------------------------------------------------------------------
// Replay under the splitting policy (Sec. 2.2), one wavefront per trace.  Both of its paths are
// hot, so everything is inline and its few scalars stay in registers.
// ---------------------------------------------------------------------------
template <bool SLOT_REGS, u32 FL_TILES>
__global__ __launch_bounds__(64) void replay_split_kernel(KParams P, const u64 *__restrict__ events,
                                                          const u32 *__restrict__ n_events, u64 *__restrict__ decisions,
                                                          vms_trace_stats *__restrict__ stats)
{
    WAVE_DYNAMIC_LDS(lds);
    const u32 lane = lane_id();
    u32 trace = blockIdx.x;
    u32 *taken = (u32 *)&stats[2 * (size_t)P.n_traces];     // [0]: trace numbers the second pass has handed out
    if (!P.retry && P.retry_slots && trace == 0) taken[0] = 0;
    SecondPass W;
    do {        // once; the second pass: once per flagged trace this wavefront takes on
    if (P.retry && !W.next(P, stats, &taken[0], trace)) return;

    SlotsT<SLOT_REGS> S;
    S.init(lds, P);
    // FL_TILES: the inactive blocks live in registers (pools of at most 64 * FL_TILES blocks), else in LDS
    typename std::conditional<FL_TILES == 0, SplitLds, SplitRegs<(FL_TILES ? FL_TILES : 1u)>>::type sp;
    sp.init(lds, P);

    AcctRegs A;
    A.init();
    u32 requested = 0, peak_requested = 0;
    TileOut T;
    T.init();
    const u32 chunk_units = 1u << P.chunk_shift;
    const u32 n_ev = n_events ? min(uni(n_events[trace]), P.max_events) : P.max_events;
    const u64 *ev_row = events + (size_t)trace * P.max_events;
    u64 *dec_row = decisions ? decisions + (size_t)trace * P.max_events : nullptr;

    u64 ev_next = lane < n_ev ? ev_row[lane] : 0;
    for (u32 base = 0; base < n_ev; base += 64) {
        const u32 tile = min(64u, n_ev - base);
        const u32 ev_lo = (u32)ev_next, ev_hi = (u32)(ev_next >> 32);
        if (base + 64 < n_ev) {                             // prefetch; lanes past the end re-read the last event
            const u32 nx = base + 64 + lane;
            const u64 x = pin64(ev_row[min(nx, n_ev - 1)]);
            ev_next = nx < n_ev ? x : 0;
        }
        u32 v_dlo = 0, v_dhi = 0, v_act = 0, v_res = 0;
        u32 done = tile, todo = tile;       // todo drops to 0 when the free list overflows: the trace ends there
        u32 w_next = from_lane(ev_lo, 0), slot_next = from_lane(ev_hi, 0);     // one event ahead
        for (u32 j = 0; j < todo; j++) {
            const u32 w = w_next, slot = slot_next;
            w_next = from_lane(ev_lo, (j + 1) & 63);
            slot_next = from_lane(ev_hi, (j + 1) & 63);
            // every path of an event ends by parking its results in lane j; none hands a result to
            // a common tail (that would cost flags to test)
            auto emit = [&](u32 dlo, u32 dhi) {
                write_lane4(v_dlo, v_dhi, v_act, v_res, dlo, dhi, requested, sp.reserved(), j);
                wave_sync();
            };
            auto overflow = [&]() {
                done = j;
                todo = 0;
            };
            if (UNLIKELY(slot >= P.max_slots)) {
                emit((u32)C_INVALID, 0u);
                continue;
            }
            const u32 req = S.get_req(slot);
            if ((int)w < 0) {
                if (UNLIKELY(req + 1u <= 1u)) {             // unbound, or bound to a request that failed
                    if (req == SLOT_OOM) {
                        S.set_req(slot, (u32)SLOT_UNBOUND);
                        emit((u32)C_FREE_NOOP, 0u);
                        continue;
                    }
                    emit((u32)C_INVALID, 0u);
                    continue;
                }
                const u32 a = S.get_a(slot);
                S.set_req(slot, (u32)SLOT_UNBOUND);
                sp.release(a >> 2, req, a & 3, A, base + j,
                           [&](bool ml, bool mr) {
                               requested -= req;
                               emit(C_FREE | (ml ? B_6 : 0u) | (mr ? B_7 : 0u), a >> 2);
                           },
                           overflow);
                continue;
            }
            const u32 size = w;
            if (UNLIKELY(size == 0 || req != SLOT_UNBOUND)) {
                emit((u32)C_INVALID, 0u);
                continue;
            }
            const u32 seg = ((size + chunk_units - 1) >> P.chunk_shift) << P.chunk_shift;
            sp.alloc(size, seg, sp.reserved() + seg <= P.capacity_units, A, base + j,
                     [&](u32 code, u32 addr, u32 flags, bool split) {
                         if (code == C_OOM) {
                             S.set_req(slot, (u32)SLOT_OOM);
                             if (A.f[SC_FIRST_OOM] == NONE32) A.f[SC_FIRST_OOM] = base + j;
                             emit((u32)C_OOM, 0u);
                             return;
                         }
                         S.set_a(slot, (addr << 2) | flags);
                         S.set_req(slot, size);
                         // blocks are cut to the request: active bytes are the requested bytes
                         requested += size;
                         peak_requested = max(peak_requested, requested);
                         emit(code | (split ? B_6 : 0u) | ((code == C_GROW ? 0u : 1u) << 8), addr);
                     },
                     overflow);
        }
        tile_emit(T, dec_row, base, done, v_dlo, v_dhi, v_act, v_res);
        if (A.stop) break;
    }

    wave_sync();
    u32 n_code[8];
    const u64 digest = tile_totals(T, n_code);
    if (lane == 0) {
        vms_trace_stats &s = stats[trace];
#pragma unroll
        for (u32 c = 0; c < 8; c++) s.n_code[c] = n_code[c];
        const u64 reserved = sp.reserved();
        s.peak_requested = (u64)peak_requested * 512;
        s.peak_active = (u64)peak_requested * 512;
        s.peak_reserved = reserved * 512;           // reserved memory never shrinks: its peak is its final value
        s.final_requested = (u64)requested * 512;
        s.final_active = (u64)requested * 512;
        s.final_reserved = reserved * 512;
        s.digest = digest;
        s.n_split = A.f[SC_N_SPLIT];
        s.n_merge = A.f[SC_N_MERGE];
        s.n_sblock_created = 0;
        s.n_sblock_evicted = 0;
        s.first_oom_event = A.f[SC_FIRST_OOM];
        s.status = A.f[SC_STATUS] | (n_code[7] ? VMS_ST_INVALID_EVENT : 0u);
        s.max_pblocks = 0;
        s.max_sblocks = 0;
        s.max_free_blocks = A.f[SC_HW_FREE];
        s.max_members = 0;
        s.max_runs = 0;
        s.overflow_event = A.f[SC_OVF_EVENT];
        s.max_multi_pblocks = 0;
        s.reserved1 = 0;
        // Sec. 5.1: fragmentation = 1 - utilisation, utilisation = peak active / peak reserved
        s.fragmentation = reserved ? 1.0 - (double)peak_requested / (double)reserved : 0.0;
    }
    wave_sync();
    } while (P.retry);
}
