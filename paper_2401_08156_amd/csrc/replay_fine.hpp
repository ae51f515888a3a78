// Replay under the stitching policy (Sec. 3, Sec. 4.1), fine-grained variant: for traces whose
// pools grow to thousands of blocks.  Offloading streams grind the pBlocks down until nearly every
// one is a single chunk, cache thousands of sBlocks, and stitch a new sBlock from a hundred
// candidates for every other request.  One wavefront still replays one trace, but its tables are
// laid out for that regime, in a quarter of the LDS the flat sorted arrays of replay_kernels.hpp
// would need, so that four such wavefronts share a compute unit:
//
//   bnd[]   one bit per physical chunk: set where a pBlock starts (and at the end of the last one).
//           pBlocks are only ever created behind the last chunk (Alloc) or cut in two (Split), so
//           the set bits are exactly the pBlock boundaries.
//   bmp[]   one bit per chunk: set while the pBlock that owns it is active.
//   A pBlock of ONE chunk is nothing but its two boundary bits: chunk c is one iff bnd has bits c
//           and c + 1.  In pool order (size descending, then first chunk ascending) these blocks
//           come last, in chunk order: Algorithm 1's scan over them is a scan over the words of
//           (singles & ~bmp), 2048 chunks per step of the wavefront.
//   pool[]  the pBlocks of two or more chunks, as in replay_kernels.hpp but with keys of twice the
//           width of a chunk number:  size << W | ~first_chunk, sorted descending.
//   ssz[] / swit[] / soff[]  the sBlocks in pool order (size descending, then creation order):
//           size in chunks, a witness chunk (one that was last seen active: while it still is, the
//           sBlock is known active after one bitmap read) and the place of its list, 6 bytes per
//           sBlock.  A new sBlock is the youngest of its size, so it enters behind the sBlocks of
//           that size and the order needs no creation number in the key.  Inserts and removals move
//           16 bytes per lane and step.
//   lists   in the trace's slice of the workspace (global memory): per sBlock two header words
//           (creation number | entries << 32,  last-use stamp) and one word per bitmap word it
//           touches (word index << 32 | chunk mask).  A list is read by an S1 test, by the FREE of
//           its sBlock (whose slot remembers the place) and by StitchFree; testing, setting and
//           clearing an sBlock is one bitmap word per lane.  Lists are bump-allocated in granules
//           and squeezed into the other half of the slice when the half in use is full.
//
// StitchFree (Sec. 3.3.2, Sec. 4.2.3) here takes one pass over the witnesses per call: every
// sBlock whose witness is no longer active is tested in full, the inactive ones are collected with
// their stamps (the 64 least recently used at most), and as many of them as the threshold asks for
// are released, least recently used first.
#ifndef VMS_REPLAY_FINE_HPP
#define VMS_REPLAY_FINE_HPP
#include "replay_kernels.hpp"

typedef uint16_t u16;

template <class IDX, int TH>
struct FineT {
    typedef typename std::conditional<sizeof(IDX) == 2, u32, u64>::type pkey_t;
    static constexpr u32 W = sizeof(IDX) * 8;
    pkey_t *pool;
    u32 *bmp, *bnd, *tmp;
    u32 *idle;                  // 64 spare words behind tmp[]: targets of lanes that have nothing to update
    IDX *ssz, *swit;
    u16 *soff;
    u64 *arena, *bounce;        // the two halves of the workspace slice
    u32 np, ns, n_chunks;       // multi-chunk pBlocks in pool[], cached sBlocks, chunks created
    u32 np_all;                 // all pBlocks
    u32 top, live;              // granules used / still referenced in the arena
    u32 next_sid, clock;
    u32 w_spare;                // a bitmap word no chunk lives in
    u32 gs, cap_grans;
    Probe2<IDX> sp;             // first level of the rank search over ssz[]
    static DI pkey_t key(u32 size, u32 start) { return ((pkey_t)size << W) | (pkey_t)(IDX)~start; }
    static DI u32 ksize(pkey_t k) { return (u32)(k >> W); }
    static DI u32 kstart(pkey_t k) { return (u32)(IDX) ~(IDX)k; }
    DI u64 *list_at(u32 place) const { return arena + ((size_t)place << gs); }
    // TH 0: ssz[] / swit[] / soff[] live in LDS.  TH 2: swit[] and soff[], TH 3: all three live in the
    // trace's workspace slice: then they are read with device-scope loads and moved by gblk_shift_*;
    // IDX is 16 bits wide there
    // before the first read of these tables after they were written (the stores must have arrived)
    DI void tables_written() const
    {
        if constexpr (TH) tbl_fence();
    }
    DI u32 sz_at(u32 i) const
    {
        if constexpr (TH == 3) return ld_tab((const u16 *)ssz + i);
        else return ssz[i];
    }
    DI u32 wit_at(u32 i) const
    {
        if constexpr (TH) return ld_tab((const u16 *)swit + i);
        else return swit[i];
    }
    DI u32 off_at(u32 i) const
    {
        if constexpr (TH) return ld_tab(soff + i);
        else return soff[i];
    }
    DI u32 grans(u32 entries) const { return (entries + 2 + (1u << gs) - 1) >> gs; }
};

template <class K>
DI K from_lane_k(K v, u32 l)
{
    if constexpr (sizeof(K) == 8) return from_lane64(v, l);
    else return (K)from_lane((u32)v, l);
}

// ---- single-chunk pBlocks --------------------------------------------------------------------
// the chunks of bitmap word w that are inactive pBlocks of one chunk (one lane per word)
template <class IDX, int TH>
DI u32 singles_free(const FineT<IDX, TH> &V, u32 w)
{
    const u32 b = V.bnd[w], bn = V.bnd[w + 1], a = V.bmp[w];
    return b & ((b >> 1) | (bn << 31)) & ~a;
}

// the chunks of bitmap word w that belong to inactive pBlocks of two or more chunks: the inactive
// chunks that exist and are not single-chunk pBlocks (an inactive pBlock has none of its bits set)
template <class IDX, int TH>
DI u32 multi_free(const FineT<IDX, TH> &V, u32 w)
{
    const u32 b = V.bnd[w], bn = V.bnd[w + 1], a = V.bmp[w];
    const u32 single = b & ((b >> 1) | (bn << 31));
    const u32 n = V.n_chunks, exist = w * 32 + 32 <= n ? 0xFFFFFFFFu : (w * 32 >= n ? 0u : (1u << (n & 31)) - 1u);
    return ~a & ~single & exist;
}

// The same for four consecutive bitmap words per lane (words 4 q .. 4 q + 3, sixteen-byte loads): the
// free single-chunk pBlocks, the chunks of free multi-chunk pBlocks and the block starts.  One step
// of the wavefront covers 8192 chunks.
struct Quad {
    u32 single[4], multi[4], start[4];
};

template <class IDX, int TH>
DI Quad quad_load(const FineT<IDX, TH> &V, u32 q)
{
    const Blk16 b = ((const Blk16 *)V.bnd)[q], a = ((const Blk16 *)V.bmp)[q];
    const u32 bn = V.bnd[4 * q + 4], n = V.n_chunks;
    Quad r;
#pragma unroll
    for (u32 k = 0; k < 4; k++) {
        const u32 w = 4 * q + k, nb = k < 3 ? b.w[k < 3 ? k + 1 : 3] : bn;
        const u32 sg = b.w[k] & ((b.w[k] >> 1) | (nb << 31));
        const u32 exist = w * 32 + 32 <= n ? 0xFFFFFFFFu : (w * 32 >= n ? 0u : (1u << (n & 31)) - 1u);
        r.single[k] = sg & ~a.w[k];
        r.multi[k] = ~a.w[k] & ~sg & exist;
        r.start[k] = b.w[k];
    }
    return r;
}

// bits of word w inside [start, end), 0 if the word lies outside
DI u32 word_mask_or0(u32 w, u32 start, u32 end)
{
    const u32 lo = max(start, w * 32), hi = min(end, w * 32 + 32);
    if (lo >= hi) return 0u;
    const u32 n = hi - lo;
    return (n == 32 ? 0xFFFFFFFFu : ((1u << n) - 1u)) << (lo & 31);
}

// S1 for a request of one chunk: the first inactive pBlock of one chunk
template <class IDX, int TH>
DI bool s1_single(const FineT<IDX, TH> &V, u32 &start)
{
    for (u32 wb = 0; wb * 32 < V.n_chunks; wb += 64) {
        const u32 w = wb + lane_id();
        const bool in = w * 32 < V.n_chunks;                    // (the bitmaps end with the word of the last chunk)
        const u32 m = in ? singles_free(V, in ? w : 0u) : 0u;
        const u64 bm = ballot(m != 0);
        if (bm) {
            const u32 l = first_lane(bm);
            start = (wb + l) * 32 + (u32)__builtin_ctz(from_lane(m, l));
            return true;
        }
    }
    return false;
}

// ---- pool[] of multi-chunk pBlocks --------------------------------------------------------------
// (4-byte keys move sixteen bytes per lane and step; the 8-byte keys of the variant with 32-bit chunk
// numbers one key per lane)
template <class IDX, int TH, class AcctT>
DI void fine_pool_insert(FineT<IDX, TH> &V, u32 size, u32 start, AcctT &A)
{
    const auto k = V.key(size, start);
    const u32 pos = rank_desc_k(V.pool, V.np, k);
    if constexpr (sizeof(IDX) == 2) blk_shift_up(V.pool, pos, V.np);
    else shift_up(V.pool, pos, V.np);
    st_one(V.pool, pos, k);
    V.np++;
    A.peak(SC_HW_MULTI, V.np);
    wave_sync();
}

template <class IDX, int TH>
DI void fine_pool_remove(FineT<IDX, TH> &V, u32 idx)
{
    if constexpr (sizeof(IDX) == 2) {
        blk_shift_down(V.pool, idx, V.np);                      // (leaves a zero key in the last place)
        V.np--;
    } else {
        shift_down(V.pool, idx, V.np);
        V.np--;
        st_one(V.pool, V.np, (typename FineT<IDX, TH>::pkey_t)0);
    }
    wave_sync();
}

// Split (Sec. 3.3.1): the pBlock at pool[idx] = [start, start + size) becomes [start, start + keep)
// and the rest.  A piece of one chunk leaves the array: its boundary bits say all there is to say.
template <class IDX, int TH, class AcctT>
DI void fine_cut(FineT<IDX, TH> &V, u32 idx, u32 start, u32 size, u32 keep, AcctT &A)
{
    fine_pool_remove(V, idx);
    const u32 cut = start + keep;
    atomicOr(lane_id() == 0 ? &V.bnd[cut >> 5] : &V.idle[lane_id()], lane_id() == 0 ? 1u << (cut & 31) : 0u);
    wave_sync();
    if (keep > 1) fine_pool_insert(V, keep, start, A);
    if (size - keep > 1) fine_pool_insert(V, size - keep, cut, A);
    V.np_all++;
    A.add(SC_N_SPLIT, 1);
    A.peak(SC_HW_PBLOCKS, V.np_all);
}

// Alloc (Sec. 3.3.1): `len` new chunks behind the last one
template <class IDX, int TH, class AcctT>
DI u32 fine_grow(FineT<IDX, TH> &V, u32 len, AcctT &A)
{
    const u32 start = V.n_chunks, end = start + len;
    atomicOr(lane_id() == 0 ? &V.bnd[end >> 5] : &V.idle[lane_id()], lane_id() == 0 ? 1u << (end & 31) : 0u);
    wave_sync();
    V.n_chunks = end;
    if (len > 1) fine_pool_insert(V, len, start, A);
    V.np_all++;
    A.peak(SC_HW_PBLOCKS, V.np_all);
    return start;
}

// S1, primitive blocks of two or more chunks: the first inactive one among pool[lo_p, hi_p), the
// pBlocks of exactly the requested number of chunks
template <class IDX, int TH>
DI bool fine_s1_pblock(const FineT<IDX, TH> &V, u32 lo_p, u32 hi_p, u32 &start)
{
    const u32 lane = lane_id();
    for (u32 base = lo_p; base < hi_p; base += 64) {
        const u32 i = base + lane;
        const auto k = V.pool[i];                               // zero keys follow the pool
        const u32 st = V.kstart(k);
        const u32 word = V.bmp[i < hi_p ? st >> 5 : V.w_spare];
        const u64 m = ballot(i < hi_p && !((word >> (st & 31)) & 1u));
        if (m) {
            start = from_lane(st, first_lane(m));
            return true;
        }
    }
    return false;
}

// ---- lists ------------------------------------------------------------------------------------
// One tile of list words (e, if live): their chunks are tested, set or cleared, one bitmap word per
// lane.  Set and clear are LDS atomics without a result; idle lanes aim at a spare word of their own.
template <class IDX, int TH>
DI u64 tile_busy(const FineT<IDX, TH> &V, u64 e, bool live, u32 &seen)
{
    const u32 word = V.bmp[live ? (u32)(e >> 32) : V.w_spare];
    seen = live ? word & (u32)e : 0u;
    return ballot(seen != 0);
}

template <class IDX, int TH>
DI void tile_apply(const FineT<IDX, TH> &V, u64 e, bool live, bool set)
{
    u32 *t = live ? &V.bmp[(u32)(e >> 32)] : &V.idle[lane_id()];
    const u32 m = live ? (u32)e : 0u;
    if (set) atomicOr(t, m);
    else atomicAnd(t, ~m);
}

// all chunks of the list at `list` (header word 0 already read: cnt entries)
template <class IDX, int TH>
DI void list_apply(const FineT<IDX, TH> &V, const u64 *list, u32 cnt, bool set)
{
    for (u32 eb = 0; eb < cnt; eb += 64) {
        const u32 k = eb + lane_id();
        const u64 e = ld_list(list + 2 + (k < cnt ? k : 0u));
        tile_apply(V, e, k < cnt, set);
    }
    wave_sync();
}

// Is any chunk of the list active?  If so *witness receives such a chunk.
template <class IDX, int TH>
DI bool list_busy(const FineT<IDX, TH> &V, const u64 *list, u32 cnt, u32 &witness)
{
    for (u32 eb = 0; eb < cnt; eb += 64) {
        const u32 k = eb + lane_id();
        const u64 e = ld_list(list + 2 + (k < cnt ? k : 0u));
        u32 seen;
        const u64 bm = tile_busy(V, e, k < cnt, seen);
        if (bm) {
            const u32 l = first_lane(bm);
            witness = (u32)(from_lane64(e, l) >> 32) * 32 + (u32)__builtin_ctz(from_lane(seen, l));
            return true;
        }
    }
    return false;
}

// ---- sBlock table -------------------------------------------------------------------------------
// the three fields of the records [pos, ns) move one place up / of (idx, ns) one place down
template <class IDX, int TH>
DI void fine_spool_shift(FineT<IDX, TH> &V, u32 pos, bool up)
{
    if constexpr (TH) {
        static_assert(sizeof(IDX) == 2, "tables in the workspace: 16-bit chunk numbers only");
        if constexpr (TH == 3) {
            u16 *const g[3] = { (u16 *)V.ssz, (u16 *)V.swit, V.soff };
            if (up) gblk_shift_up<3>(g, pos, V.ns);
            else gblk_shift_down<3>(g, pos, V.ns);
        } else {
            u16 *const g[2] = { (u16 *)V.swit, V.soff };
            if (up) {
                gblk_shift_up<2>(g, pos, V.ns);
                blk_shift_up(V.ssz, pos, V.ns);
            } else {
                gblk_shift_down<2>(g, pos, V.ns);
                blk_shift_down(V.ssz, pos, V.ns);
            }
        }
    } else if constexpr (sizeof(IDX) == 2) {
        u16 *const f[3] = { V.ssz, V.swit, V.soff };
        if (up) blk_shift_up<u16, 3>(f, pos, V.ns);
        else blk_shift_down<u16, 3>(f, pos, V.ns);
    } else {
        IDX *const f[2] = { V.ssz, V.swit };
        if (up) {
            blk_shift_up<IDX, 2>(f, pos, V.ns);
            blk_shift_up(V.soff, pos, V.ns);
        } else {
            blk_shift_down<IDX, 2>(f, pos, V.ns);
            blk_shift_down(V.soff, pos, V.ns);
        }
    }
}

// Stitch (Sec. 3.3.1): the new sBlock enters behind the cached ones of its size
template <class IDX, int TH, class AcctT>
DI void fine_spool_insert(FineT<IDX, TH> &V, u32 size, u32 place, u32 witness, AcctT &A)
{
    V.tables_written();
    V.sp.template refresh<TH == 3>(V.ssz, V.ns);
    const u32 pos = V.sp.template rank<TH == 3>(V.ssz, (IDX)(size - 1));    // sizes >= size come before it
    fine_spool_shift(V, pos, true);
    st_one(V.ssz, pos, (IDX)size);
    st_one(V.swit, pos, (IDX)witness);
    st_one(V.soff, pos, (u16)place);
    V.ns++;
    A.add(SC_N_CREATED, 1);
    wave_sync();
}

template <class IDX, int TH>
DI void fine_spool_remove(FineT<IDX, TH> &V, u32 idx)
{
    fine_spool_shift(V, idx, false);
    V.ns--;
}

// the two header words of a new list; its entries follow
template <class IDX, int TH>
DI void list_head(const FineT<IDX, TH> &V, u32 place, u32 id, u32 cnt, u32 stamp)
{
    u64 *l = V.list_at(place);
    const u32 lane = lane_id() & 1;                             // every lane stores one of the two words
    l[lane] = lane ? (u64)stamp : ((u64)cnt << 32) | id;
}

// the list of one run of chunks [start, start + len) at `place`; returns its entries
template <class IDX, int TH>
DI u32 list_put_run(const FineT<IDX, TH> &V, u32 place, u32 start, u32 len)
{
    const u32 n = run_words(start, len), w0 = start >> 5;
    u64 *l = V.list_at(place) + 2;
    for (u32 qb = 0; qb < n; qb += 64) {
        const u32 q = min(qb + lane_id(), n - 1);               // lanes past the run write its last word again
        l[q] = ((u64)(w0 + q) << 32) | word_mask(w0 + q, start, start + len);
    }
    return n;
}

// Squeeze the lists of released sBlocks out: copy the live lists, in table order, to the other
// half of the slice, which becomes the arena.  Slots that hold an sBlock learn its new place.
template <class IDX, int TH, class Slots>
DI void fine_compact(FineT<IDX, TH> &V, Slots &S)
{
    u32 top = 0;
    V.tables_written();
    for (u32 s = 0; s < V.ns; s++) {
        const u32 from = TH ? uni(V.off_at(s)) : ld_uni(V.soff, s);
        const u64 *src = V.list_at(from);
        const u32 cnt = (u32)(uni64(ld_list(src)) >> 32), words = cnt + 2;
        u64 *dst = V.bounce + ((size_t)top << V.gs);
        for (u32 rb = 0; rb < words; rb += 64) {                // lanes past the end copy the last word again
            const u32 r = min(rb + lane_id(), words - 1);
            dst[r] = ld_list(src + r);
        }
        st_one(V.soff, s, (u16)top);
        S.relocate(from, top);
        top += V.grans(cnt);
    }
    S.relocate_done();
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");      // later reads are of other lanes' global writes
    wave_sync();
    u64 *t = V.arena;
    V.arena = V.bounce;
    V.bounce = t;
    V.top = V.live = top;
}

template <class IDX, int TH, class Slots, class AcctT>
DI bool fine_reserve(FineT<IDX, TH> &V, Slots &S, u32 need_grans, AcctT &A, u32 ev)
{
    if (UNLIKELY(V.top + need_grans > V.cap_grans && V.live < V.top)) fine_compact(V, S);
    if (UNLIKELY(V.top + need_grans > V.cap_grans)) {
        A.overflow(ev, VMS_ST_OVF_RUNS);
        return false;
    }
    return true;
}

// ---- StitchFree (Sec. 3.3.2, Sec. 4.2.3) ----------------------------------------------------------
// While more sBlocks than the threshold are cached, the least recently used inactive one is
// released.  Releasing one changes nothing about the others, so the sBlocks released by one call
// are the inactive ones with the oldest stamps, as many as the excess over the threshold: one pass
// finds the inactive ones (witness first, whole list if the witness is idle), the 64 oldest of
// them wait in registers (lane v: stamp, table index, granules), the ones that must go are
// removed from the highest index down.  A call that leaves more than 64 to release goes round again.
template <class IDX, int TH, class AcctT>
DI bool fine_stitch_free(FineT<IDX, TH> &V, const KParams &P, AcctT &A)
{
    constexpr u32 E = 16 / sizeof(IDX);                         // witnesses per lane and step
    const u32 lane = lane_id();
    bool any = false;
    while (V.ns > P.spool_threshold) {
        u32 v_stamp = NONE32, v_idx = 0, v_gr = 0;              // empty places hold the youngest possible stamp
        u32 n_found = 0;
        u32 u_idx = 0, n_unk = 0;                               // lane v: table index of the v-th sBlock to test in full
        // an inactive sBlock takes an empty place, or the place of the youngest one waiting if it is older
        auto found = [&](u32 stamp, u32 idx, u32 cnt) {
            const u32 worst = ~wave_min_u32(~v_stamp);
            if (stamp < worst) {
                const u32 at = first_lane(ballot(v_stamp == worst));
                v_stamp = write_lane(v_stamp, stamp, at);
                v_idx = write_lane(v_idx, idx, at);
                v_gr = write_lane(v_gr, V.grans(cnt), at);
            }
            n_found++;
        };
        // The tests of the sBlocks noted so far.  Most of them are active through another chunk:
        // first every lane looks at the first four words of the list of one noted sBlock (all lists
        // in flight at once), which settles most; the rest are tested with all lanes on one list,
        // four lists in flight at a time.
        auto test_noted = [&]() {
            const bool mine = lane < n_unk;
            V.tables_written();
            const u32 my_place = V.off_at(mine ? u_idx : 0u);
            const u64 *ml = V.list_at(my_place);
            u64 h[6];
#pragma unroll
            for (u32 q = 0; q < 6; q++) h[q] = ld_list(ml + q);
            const u32 my_cnt = (u32)(h[0] >> 32);
            u32 wit = NONE32;                                   // an active chunk among the first four words
#pragma unroll
            for (u32 q = 0; q < 4; q++) {
                const bool live = q < my_cnt;
                const u32 word = V.bmp[live ? (u32)(h[2 + q] >> 32) : V.w_spare];
                const u32 seen = live ? word & (u32)h[2 + q] : 0u;
                wit = seen && wit == NONE32 ? (u32)(h[2 + q] >> 32) * 32 + (u32)__builtin_ctz(seen) : wit;
            }
            if (mine && wit != NONE32) V.swit[u_idx] = (IDX)wit;        // active after all: remember where
            const u64 idle_short = ballot(mine && wit == NONE32 && my_cnt <= 4);
            u64 unsettled = ballot(mine && wit == NONE32 && my_cnt > 4);
            wave_sync();
            for (u64 t = idle_short; t; t &= t - 1) {
                const u32 l = first_lane(t);
                found(from_lane((u32)h[1], l), from_lane(u_idx, l), from_lane(my_cnt, l));
            }
            while (unsettled) {
                u64 e[4];
                u32 from[4];
#pragma unroll
                for (u32 q = 0; q < 4; q++) {
                    from[q] = unsettled ? first_lane(unsettled) : NONE32;
                    unsettled &= unsettled - 1;
                    e[q] = ld_list(V.list_at(from_lane(my_place, from[q] & 63)) + lane);    // header and first 62 entries
                }
#pragma unroll
                for (u32 q = 0; q < 4; q++) {
                    if (from[q] == NONE32) break;
                    const u32 cnt = (u32)(from_lane64(e[q], 0) >> 32), stamp = (u32)from_lane64(e[q], 1);
                    const u32 idx = from_lane(u_idx, from[q]);
                    u32 seen, witness = 0;
                    const u64 bm = tile_busy(V, e[q], lane >= 2 && lane - 2 < cnt, seen);
                    bool busy = bm != 0;
                    if (busy) {
                        const u32 f = first_lane(bm);
                        witness = (u32)(from_lane64(e[q], f) >> 32) * 32 + (u32)__builtin_ctz(from_lane(seen, f));
                    } else if (UNLIKELY(cnt > 62)) {
                        busy = list_busy(V, V.list_at(from_lane(my_place, from[q])) + 62, cnt - 62, witness);
                    }
                    if (busy) st_one(V.swit, idx, (IDX)witness);
                    else found(stamp, idx, cnt);
                }
            }
            n_unk = 0;
            wave_sync();
        };
        // E witnesses per lane and step: sBlocks base + lane * E + j.  The block of the next step is on its
        // way while this one is looked at (a step renews witnesses of its own and of earlier blocks only).
        auto wit_block = [&](u32 base) {
            const u32 wblk = min(base / E + lane, (V.ns - 1) / E);                  // (lanes past the table: its last block again)
            if constexpr (TH) return gblk_load((const u16 *)V.swit, wblk);
            else return ((const Blk16 *)V.swit)[wblk];
        };
        V.tables_written();
        Blk16 wb_next;
        if constexpr (TH) wb_next = wit_block(0);
        for (u32 base = 0; base < V.ns; base += 64 * E) {
            // all the bitmap words of a step are on their way before the first is looked at
            Blk16 wb;
            if constexpr (TH) {
                wb = wb_next;
                if (base + 64 * E < V.ns) wb_next = wit_block(base + 64 * E);
            } else {
                wb = wit_block(base);
            }
            u32 word[E], wit[E];
#pragma unroll
            for (u32 j = 0; j < E; j++) {
                wit[j] = sizeof(IDX) == 2 ? (wb.w[j >> 1] >> (16 * (j & 1))) & 0xFFFFu : wb.w[j];
                word[j] = V.bmp[wit[j] >> 5];
            }
            u32 idle = 0;                                       // bit j: the witness of sBlock j of this lane is inactive
#pragma unroll
            for (u32 j = 0; j < E; j++)
                idle |= (base + lane * E + j < V.ns && !((word[j] >> (wit[j] & 31)) & 1u) ? 1u : 0u) << j;
            for (u64 todo = ballot(idle != 0); todo; todo &= todo - 1) {
                const u32 l = first_lane(todo);
                for (u32 bits = from_lane(idle, l); bits; bits &= bits - 1) {
                    u_idx = write_lane(u_idx, base + l * E + (u32)__builtin_ctz(bits), n_unk);
                    if (++n_unk == 64) test_noted();
                }
            }
        }
        if (n_unk) test_noted();
        if (!n_found) break;                                    // everything cached is in use: the threshold stays exceeded
        const u32 excess = V.ns - P.spool_threshold, have = min(n_found, 64u);
        u32 go = min(excess, have);
        // the `go` oldest of the waiting ones: a place goes if fewer than `go` places hold an older stamp
        bool sel = v_stamp != NONE32;
        if (UNLIKELY(go < have)) {
            u32 older = 0;
            for (u32 l = 0; l < 64; l++) older += from_lane(v_stamp, l) < v_stamp ? 1u : 0u;
            sel = sel && older < go;
        }
        for (; go; go--) {
            // highest table index first: the places of the others stay valid
            const u32 hi = ~wave_min_u32(sel ? ~v_idx : NONE32);
            const u32 at = first_lane(ballot(sel && v_idx == hi));
            fine_spool_remove(V, hi);
            V.live -= from_lane(v_gr, at);
            sel = sel && lane != at;
            A.add(SC_N_EVICTED, 1);
        }
        any = true;
        if (n_found <= 64) break;                               // no inactive sBlock is left unseen
    }
    A.peak(SC_HW_SBLOCKS, V.ns);     // high-water marks as seen between events
    A.peak(SC_HW_RUNS, V.live);
    return any;
}

// ---- S1 (Algorithm 1, first loop; Sec. 4.1 state S1) on stitched blocks, oldest first ------------
// Is the sBlock whose list is at `place` active?  One read of the list (header and first 62 entries,
// returned in e), more only for longer lists.  If active, *witness receives an active chunk.
template <class IDX, int TH>
DI bool sblock_busy(const FineT<IDX, TH> &V, u32 place, u64 &e, u32 &cnt, u32 &witness)
{
    const u32 lane = lane_id();
    const u64 *list = V.list_at(place);
    e = ld_list(list + lane);
    cnt = (u32)(from_lane64(e, 0) >> 32);
    u32 seen;
    const u64 bm = tile_busy(V, e, lane >= 2 && lane - 2 < cnt, seen);
    if (bm) {
        const u32 b = first_lane(bm);
        witness = (u32)(from_lane64(e, b) >> 32) * 32 + (u32)__builtin_ctz(from_lane(seen, b));
        return true;
    }
    if (UNLIKELY(cnt > 62)) return list_busy(V, list + 62, cnt - 62, witness);
    return false;
}

// hand out the (inactive) sBlock whose first list tile is e
template <class IDX, int TH>
DI void sblock_take(FineT<IDX, TH> &V, u32 place, u64 e, u32 cnt)
{
    const u32 lane = lane_id();
    u64 *list = V.list_at(place);
    tile_apply(V, e, lane >= 2 && lane - 2 < cnt, true);
    if (UNLIKELY(cnt > 62)) list_apply(V, list + 62, cnt - 62, true);
    list[1] = (u64)++V.clock;                                   // last use (every lane stores the same word)
}

// The block of 64 sizes that the rank search reads holds the first sBlock of bsize chunks, if there
// is one: it doubles as the first tile of candidates.  One lane per candidate reads its witness;
// the others are tested oldest first (table order) with all lanes over the words of one list.
template <class IDX, int TH>
DI bool fine_s1_sblock(FineT<IDX, TH> &V, u32 bsize, u32 &ref, u32 &place_out)
{
    const u32 lane = lane_id();
    u32 base = V.sp.block((IDX)bsize);
    for (;;) {
        const u32 i = base + lane;
        V.tables_written();
        const u32 wit = V.wit_at(i), so = V.off_at(i);              // (on their way while the sizes are compared)
        const u32 sz = V.sz_at(i);                                  // zero sizes follow the table
        const u64 vm = ballot(sz == bsize);
        if (!vm) return false;
        const u32 word = V.bmp[wit >> 5];
        u64 unknown = vm & ~ballot((word >> (wit & 31)) & 1u);
        while (unknown) {
            const u32 l = first_lane(unknown);
            unknown &= unknown - 1;
            const u32 place = from_lane(so, l);
            u64 e;
            u32 cnt, witness;
            if (!sblock_busy(V, place, e, cnt, witness)) {
                sblock_take(V, place, e, cnt);                  // inactive: hand it out
                ref = (u32)from_lane64(e, 0);
                place_out = place;
                return true;
            }
            st_one(V.swit, base + l, (IDX)witness);
        }
        if (~vm >> 63) return false;                            // the run of equal sizes ended inside this tile
        base += 64;
    }
}

// Update (Sec. 3.3.2) of the sBlock whose list is at `place`
template <class IDX, int TH>
DI void fine_free_sblock(const FineT<IDX, TH> &V, u32 place)
{
    const u64 *list = V.list_at(place);
    const u32 lane = lane_id();
    const u64 e = ld_list(list + lane);
    const u32 cnt = (u32)(from_lane64(e, 0) >> 32);
    tile_apply(V, e, lane >= 2 && lane - 2 < cnt, false);
    if (UNLIKELY(cnt > 62)) list_apply(V, list + 62, cnt - 62, false);
}

// No block of exactly bsize chunks is free: BestFit's second loop and the post-processing of its
// state (Algorithm 1; Sec. 4.1, Fig. 9, states S2 to S5).
template <class IDX, int TH, class Slots, class AcctT>
DI void fine_alloc_rest(FineT<IDX, TH> &V, Slots &S, u32 bsize, u32 lo_p, u32 hi_p, u32 reserved_units, const KParams &P,
                        AcctT &A, u32 ev, VmsRes &R)
{
    typedef typename FineT<IDX, TH>::pkey_t pkey_t;
    const u32 lane = lane_id();
    R.kind = KIND_PBLOCK;
    R.held = bsize;
    R.ref = 0;
    R.list = 0;
    // pool[lo_p, hi_p) are the multi-chunk pBlocks of exactly bsize chunks (all active, or S1 had taken one)

    // ---- Algorithm 1, second loop.  Larger blocks are pool[0, lo_p): the last inactive one in
    // pool order is the single-block candidate (state 2).
    for (u32 hi = lo_p; hi > 0;) {
        const u32 lo = hi > 64 ? hi - 64 : 0;
        const bool v = lane < hi - lo;
        const pkey_t k = V.pool[v ? hi - 1 - lane : 0u];
        const u32 fc = V.kstart(k);
        const u32 kw = V.bmp[v ? fc >> 5 : V.w_spare];
        const u64 m = ballot(v && !((kw >> (fc & 31)) & 1u));
        if (m) {
            const u32 l = first_lane(m), idx = hi - 1 - l;
            const pkey_t pk = from_lane_k(k, l);
            const u32 psize = V.ksize(pk), pstart = V.kstart(pk);
            if (UNLIKELY(psize < P.frag_limit_chunks)) {
                // below the fragmentation limit: not worth cutting, hand it out whole (Sec. 4.2.3)
                bmp_fill(V.bmp, V.w_spare, pstart, psize, true);
                R.ref = pstart;
                R.held = psize;
                R.dec_lo = C_SPLIT | (1u << 8);
                return;
            }
            const u32 gr = V.grans(run_words(pstart, psize));
            if (UNLIKELY(V.np + 1 > P.cap_pblocks || V.ns + 1 > P.cap_sblocks || !fine_reserve(V, S, gr, A, ev))) {
                A.overflow(ev, (V.np + 1 > P.cap_pblocks ? VMS_ST_OVF_PBLOCKS : 0u) | (V.ns + 1 > P.cap_sblocks ? VMS_ST_OVF_SBLOCKS : 0u));
                R.dec_lo = C_INVALID;
                return;
            }
            // S2: Split into the request and the rest; a stitched block keeps the uncut size on record
            fine_cut(V, idx, pstart, psize, bsize, A);
            const u32 n = list_put_run(V, V.top, pstart, psize);
            list_head(V, V.top, V.next_sid++, n, ++V.clock);
            fine_spool_insert(V, psize, V.top, pstart, A);      // its first chunk is handed out: a witness
            V.top += gr;
            V.live += gr;
            bmp_fill(V.bmp, V.w_spare, pstart, bsize, true);
            R.ref = pstart;
            R.dec_lo = C_SPLIT | B_6 | (1u << 8);
            if (fine_stitch_free(V, P, A)) R.dec_lo |= B_7;
            return;
        }
        hi = lo;
    }

    // Smaller blocks, largest first, until the request is covered (states 3 and 4): first the
    // multi-chunk ones in pool[hi_p, lim), then the single chunks in chunk order.  Blocks below the
    // fragmentation limit sit at the tail of the pool and are never stitched.
    u32 lim = V.np;
    const bool singles_ok = P.frag_limit_chunks <= 1;
    if (UNLIKELY(!singles_ok)) lim = rank_desc_k(V.pool, V.np, (pkey_t)(((pkey_t)P.frag_limit_chunks << V.W) - 1));
    u32 sum = 0, k = 0, pos = NONE32;
    // No inactive pBlock of bsize chunks or more exists at this point, so every inactive chunk that is
    // not a single-chunk pBlock belongs to a candidate.  If all of those together do not cover the
    // request, every inactive multi-chunk pBlock is taken and the order among them does not matter:
    // their chunks and their number come from the bitmaps alone, 2048 chunks per step, and pool[]
    // is not read at all.
    bool all_multi = false;
    const u32 n_quads = (V.n_chunks + 127) >> 7;                // lanes that hold chunks, four bitmap words each
    if (LIKELY(singles_ok)) {
        u32 mine = 0;                                           // chunks | blocks << 16 of this lane's words
        for (u32 qb = 0; qb < n_quads; qb += 64) {
            const u32 q = qb + lane;
            const Quad Q = quad_load(V, q < n_quads ? q : 0u);
#pragma unroll
            for (u32 t = 0; t < 4; t++)
                mine += q < n_quads ? (u32)__builtin_popcount(Q.multi[t]) | ((u32)__builtin_popcount(Q.multi[t] & Q.start[t]) << 16) : 0u;
        }
        // (at most 4096 blocks and 8192 chunks per step; larger bitmaps: the sums are taken in two halves)
        u32 t_lo, t_hi;
        wave_scan_add(mine & 0xFFFFu, &t_lo);
        wave_scan_add(mine >> 16, &t_hi);
        if (t_lo < bsize) {
            all_multi = true;
            sum = t_lo;
            k = t_hi;
        }
    }
    // The pool scan takes sixteen bytes of keys per lane and step (KE keys, all their bitmap words on
    // their way before the first is looked at).  Each candidate it passes flips two bits in tmp[]: the
    // bit of its first chunk and the bit behind its last one.  A chunk then belongs to a candidate iff
    // an odd number of flipped bits lies at or below it (runs do not overlap; where two touch, the two
    // flips of the shared place cancel): the list is read off tmp[] afterwards whatever the runs' lengths.
    constexpr u32 KE = 16 / sizeof(pkey_t);
    struct alignas(16) Keys {
        pkey_t k[KE];
    };
    u64 qk = 0;                                                 // the key of a candidate that is cut
    bool flipped = false;
    if (!all_multi) {
        for (u32 base = hi_p & ~(KE - 1); base < lim && pos == NONE32; base += 64 * KE) {
            const u32 i0 = base + lane * KE;
            const Keys K = ((const Keys *)V.pool)[i0 < lim ? i0 / KE : 0u];
            u32 kw[KE], sz[KE], mine = 0;
            bool in[KE];
#pragma unroll
            for (u32 e = 0; e < KE; e++) {
                in[e] = i0 + e >= hi_p && i0 + e < lim;
                kw[e] = V.bmp[in[e] ? V.kstart(K.k[e]) >> 5 : V.w_spare];
            }
#pragma unroll
            for (u32 e = 0; e < KE; e++) {
                in[e] = in[e] && !((kw[e] >> (V.kstart(K.k[e]) & 31)) & 1u);    // from here on: an inactive pBlock
                sz[e] = in[e] ? V.ksize(K.k[e]) : 0u;
                mine += sz[e];
            }
            u32 tot;
            const u32 incl = wave_scan_add(mine, &tot);
            u32 l_end = 64, e_end = KE, cut_by = 0;             // the last candidate: key e_end of lane l_end (none: all of them)
            if (sum + tot >= bsize) {
                // the lane, then the key inside it, at which the request is covered
                l_end = first_lane(ballot(mine && sum + incl >= bsize));
                sum += from_lane(incl - mine, l_end);
#pragma unroll
                for (u32 e = 0; e < KE; e++) k += popc64(ballot(in[e]) & ((1ull << l_end) - 1));
#pragma unroll
                for (u32 e = 0; e < KE; e++) {
                    const u32 c = from_lane(sz[e], l_end);
                    if (pos == NONE32 && c) {
                        k++;
                        sum += c;
                        if (sum >= bsize) {
                            pos = base + l_end * KE + e;
                            e_end = e;
                        }
                    }
                }
                cut_by = sum - bsize;
                if (cut_by) qk = (u64)ld_uni(V.pool, pos);
            } else {
#pragma unroll
                for (u32 e = 0; e < KE; e++) k += popc64(ballot(in[e]));
                sum += tot;
            }
#pragma unroll
            for (u32 e = 0; e < KE; e++) {
                const bool take = in[e] && (lane < l_end || (lane == l_end && e <= e_end));
                const u32 fc = V.kstart(K.k[e]);
                const u32 end = fc + V.ksize(K.k[e]) - (lane == l_end && e == e_end ? cut_by : 0u);
                atomicXor(take ? &V.tmp[fc >> 5] : &V.idle[lane], take ? 1u << (fc & 31) : 0u);
                atomicXor(take ? &V.tmp[end >> 5] : &V.idle[lane], take ? 1u << (end & 31) : 0u);
            }
            flipped = true;
        }
        wave_sync();
    }
    // single chunks, in chunk order: all free ones before word s_last, and the lowest s_take of that word
    u32 s_last = NONE32, s_take = 0, n_single = 0;
    if (pos == NONE32 && singles_ok) {
        const u32 want = bsize - sum;
        for (u32 qb = 0; qb < n_quads; qb += 64) {
            const u32 q = qb + lane;
            const Quad Q = quad_load(V, q < n_quads ? q : 0u);
            u32 pc[4], mine = 0;
#pragma unroll
            for (u32 t = 0; t < 4; t++) {
                pc[t] = q < n_quads ? (u32)__builtin_popcount(Q.single[t]) : 0u;
                mine += pc[t];
            }
            u32 tot;
            const u32 incl = wave_scan_add(mine, &tot);
            if (n_single + tot >= want) {
                const u32 l = first_lane(ballot(n_single + incl >= want));
                // inside lane l: the word in which the count is reached
                u32 before = n_single + from_lane(incl - mine, l), word = 4 * (qb + l);
#pragma unroll
                for (u32 t = 0; t < 3; t++) {
                    const u32 c = from_lane(pc[t], l);
                    const bool past = before + c < want && word == 4 * (qb + l) + t;
                    before += past ? c : 0u;
                    word += past ? 1u : 0u;
                }
                s_last = word;
                s_take = want - before;
                n_single = want;
                break;
            }
            n_single += tot;
        }
        k += n_single;
        sum += n_single;
    }
    const bool s3 = sum >= bsize;
    const u32 excess = s3 ? sum - bsize : 0, deficit = s3 ? 0 : bsize - sum;
    const u32 n_after = V.n_chunks + deficit;                   // chunks once the new pBlock exists
    // giving up from here on: the flipped bits must not stay behind in tmp[]
    auto wipe = [&]() {
        if (flipped)
            for (u32 i = lane; i < P.bmp_words; i += 64) V.tmp[i] = 0;
        wave_sync();
    };
    u32 q_gr = 0;                                               // granules of the record of a cut candidate
    if (excess) q_gr = V.grans(run_words(V.kstart((pkey_t)qk), V.ksize((pkey_t)qk)));
    if (!s3) {
        // S4 needs new physical chunks; S5 if the device cannot provide them
        if (UNLIKELY(reserved_units + (deficit << P.chunk_shift) > P.capacity_units)) {
            wipe();
            R.dec_lo = C_OOM;
            return;
        }
        if (UNLIKELY(n_after > P.cap_chunks)) {
            wipe();
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
        const u32 start = fine_grow(V, deficit, A);
        bmp_fill(V.bmp, V.w_spare, start, deficit, true);
        R.ref = start;
        R.dec_lo = C_GROW;
        return;
    }
    // room: two more pBlocks and sBlocks at most, a list of at most one word per bitmap word in use,
    // and the record of a cut candidate
    if (UNLIKELY(V.np + 2 > P.cap_pblocks || V.ns + 2 > P.cap_sblocks)) {
        A.overflow(ev, (V.np + 2 > P.cap_pblocks ? VMS_ST_OVF_PBLOCKS : 0u) | (V.ns + 2 > P.cap_sblocks ? VMS_ST_OVF_SBLOCKS : 0u));
        R.dec_lo = C_INVALID;
        return;
    }
    if (UNLIKELY(!fine_reserve(V, S, V.grans((n_after + 31) >> 5) + q_gr, A, ev))) {
        R.dec_lo = C_INVALID;
        return;
    }
    // The list, four bitmap words per lane and step: the candidates' chunks (from the flipped bits, or,
    // when every free multi-chunk pBlock is taken, straight from the bitmaps, with the chosen single
    // chunks) and the new pBlock's; one list word per bitmap word touched; the chunks become active on
    // the way and tmp[] is left zero.
    const u32 place = V.top;
    u32 cnt = 0, witness = NONE32;
    {
        u64 *l = V.list_at(place) + 2;
        u32 carry = 0;                                          // flipped bits below this step, mod 2
        for (u32 qb = 0; qb * 128 <= n_after; qb += 64) {
            const u32 q = qb + lane;
            const bool mine = q * 128 <= n_after;
            u32 out[4];
            if (all_multi) {
                const Quad Q = quad_load(V, mine ? q : 0u);
#pragma unroll
                for (u32 t = 0; t < 4; t++) {
                    const u32 w = 4 * q + t;
                    u32 sg = n_single ? Q.single[t] : 0u;
                    if (s_last != NONE32) {
                        u32 rest = sg;
                        for (u32 i = 0; i < s_take; i++) rest &= rest - 1;      // sg without its lowest s_take bits
                        sg = w < s_last ? sg : (w == s_last ? sg & ~rest : 0u);
                    }
                    out[t] = mine ? Q.multi[t] | sg : 0u;
                }
            } else {
                const Blk16 t4 = ((const Blk16 *)V.tmp)[mine ? q : 0u];
                u32 pc = 0;
#pragma unroll
                for (u32 t = 0; t < 4; t++) pc += mine ? (u32)__builtin_popcount(t4.w[t]) : 0u;
                u32 tot;
                const u32 incl = wave_scan_add(pc, &tot);
                u32 odd = (carry + incl - pc) & 1u;             // flipped bits below the word at hand, mod 2
#pragma unroll
                for (u32 t = 0; t < 4; t++) {
                    u32 x = mine ? t4.w[t] : 0u;
                    const u32 flips = (u32)__builtin_popcount(x) & 1u;
                    x ^= x << 1;
                    x ^= x << 2;
                    x ^= x << 4;
                    x ^= x << 8;
                    x ^= x << 16;                               // bit i: flipped bits 0..i of this word, mod 2
                    out[t] = odd ? ~x : x;
                    odd ^= flips;
                }
                carry += tot;
                wave_lockstep();
                if (mine) ((Blk16 *)V.tmp)[q] = Blk16{ { 0, 0, 0, 0 } };
            }
            u32 words = 0;
#pragma unroll
            for (u32 t = 0; t < 4; t++) {
                if (deficit) out[t] |= mine ? word_mask_or0(4 * q + t, V.n_chunks, n_after) : 0u;      // Alloc's chunks
                words += out[t] ? 1u : 0u;
                witness = min(witness, out[t] ? (4 * q + t) * 32 + (u32)__builtin_ctz(out[t]) : NONE32);
            }
            u32 tot;
            const u32 incl = wave_scan_add(words, &tot);
            u32 at = cnt + incl - words;
            const Blk16 a4 = ((const Blk16 *)V.bmp)[mine ? q : 0u];
            Blk16 act;
#pragma unroll
            for (u32 t = 0; t < 4; t++) {
                if (out[t]) l[at++] = ((u64)(4 * q + t) << 32) | out[t];
                act.w[t] = a4.w[t] | out[t];
            }
            wave_lockstep();
            if (mine) ((Blk16 *)V.bmp)[q] = act;
            cnt += tot;
        }
        witness = wave_min_u32(witness);
        wave_sync();
    }
    u32 used = V.grans(cnt);
    R.dec_lo = 0;
    // the record of a cut candidate is created first and is therefore the older of the two sBlocks
    u32 rid = 0, rstamp = 0;
    if (excess) {
        rid = V.next_sid++;
        rstamp = ++V.clock;
    }
    const u32 sid = V.next_sid++;
    list_head(V, place, sid, cnt, ++V.clock);
    if (s3) {
        if (excess) {
            // cut the last candidate so the sum is exact; remember its uncut size (Fig. 9, sBlock 2)
            const u32 qsize = V.ksize((pkey_t)qk), qstart = V.kstart((pkey_t)qk);
            fine_cut(V, pos, qstart, qsize, qsize - excess, A);
            const u32 n = list_put_run(V, place + used, qstart, qsize);
            list_head(V, place + used, rid, n, rstamp);
            fine_spool_insert(V, qsize, place + used, qstart, A);
            used += q_gr;
            R.dec_lo |= B_6;
        }
        R.dec_lo |= C_STITCH;
    } else {
        fine_grow(V, deficit, A);               // Alloc: exactly the missing chunks
        R.dec_lo |= C_GROW;
    }
    fine_spool_insert(V, bsize, place, witness, A);
    V.top += used;
    V.live += used;
    A.peak(SC_HW_MEMBERS, k + (s3 ? 0u : 1u));
    R.ref = sid;
    R.list = place;
    R.kind = KIND_SBLOCK;
    R.dec_lo |= B_SBLOCK | (k << 8);
    if (fine_stitch_free(V, P, A)) R.dec_lo |= B_7;
}

// The rare path of the replay loop (see vms_alloc_cold): its scalars wait in the LDS header.
template <class IDX, int TH, class Slots>
DI bool fine_alloc_cold(char *lds, FineT<IDX, TH> &V, Slots &S, const KParams &P, u32 bsize, u32 lo_p, u32 hi_p,
                        u32 reserved_units, u32 ev, VmsRes &R)
{
    u32 *sc = (u32 *)(lds + LDS_SCALARS);
    ColdState C;
    C.load(lds);
    V.top = C.get(SC_TOP);
    V.live = C.get(SC_LIVE);
    V.next_sid = C.get(SC_NEXT_SID);
    V.np_all = C.get(SC_NP_ALL);
    AcctLds A;
    A.sc = sc;
    A.idle = V.idle;
    fine_alloc_rest(V, S, bsize, lo_p, hi_p, reserved_units, P, A, ev, R);
    st_one(sc, (u32)SC_TOP, V.top);
    st_one(sc, (u32)SC_LIVE, V.live);
    st_one(sc, (u32)SC_NEXT_SID, V.next_sid);
    st_one(sc, (u32)SC_NP_ALL, V.np_all);
    wave_sync();
    return ld_uni(sc, (u32)SC_STOP) == 0;
}

// ---------------------------------------------------------------------------
// The kernel: same event loop, slot table, small-request pool and per-tile accounting as
// replay_vms_kernel; the pools are the ones above.  IDX: the type of a chunk number.
// ---------------------------------------------------------------------------
template <bool SLOT_REGS, class IDX, int TH>
__global__ __launch_bounds__(64) void replay_vms_fine_kernel(KParams P, const u64 *__restrict__ events,
                                                             const u32 *__restrict__ n_events,
                                                             u64 *__restrict__ decisions, vms_trace_stats *__restrict__ stats,
                                                             char *__restrict__ workspace)
{
    WAVE_DYNAMIC_LDS(lds);
    wave_priority<2>();
    typedef typename FineT<IDX, TH>::pkey_t pkey_t;
    const u32 lane = lane_id();
    u32 trace = blockIdx.x;
    char *ws_slice = workspace + (size_t)trace * P.ws_stride;
    u32 *taken = (u32 *)&stats[2 * (size_t)P.n_traces];     // [1]: trace numbers the second pass has handed out
    if (!P.retry && P.retry_slots && trace == 0) taken[1] = 0;
    SecondPass W;
    do {        // once; the second pass: once per flagged trace this wavefront takes on
    if (P.retry) {
        // larger tables, a workspace slice per wavefront of this launch behind those of the first pass
        if (!W.next(P, stats + P.n_traces, &taken[1], trace)) return;
        ws_slice = workspace + P.retry_ws_off + (size_t)blockIdx.x * P.ws_stride;
    }

    SlotsT<SLOT_REGS> S;
    S.init(lds, P);
    ((u32 *)(lds + LDS_SCALARS))[lane] = lane == SC_FIRST_OOM || lane == SC_OVF_EVENT ? NONE32 : 0u;     // LDS header
    FineT<IDX, TH> V;
    V.pool = (pkey_t *)(lds + P.off_pool);
    V.bmp = (u32 *)(lds + P.off_bmp);
    V.bnd = (u32 *)(lds + P.off_bnd);
    V.tmp = (u32 *)(lds + P.off_tmp);
    V.idle = V.tmp + P.bmp_words;
    V.ssz = TH == 3 ? (IDX *)(ws_slice + 2 * P.ws_half + 2 * (size_t)P.ws_tbl_bytes) : (IDX *)(lds + P.off_skey);
    if constexpr (TH) {
        V.swit = (IDX *)(ws_slice + 2 * P.ws_half);
        V.soff = (u16 *)(ws_slice + 2 * P.ws_half + P.ws_tbl_bytes);
    } else {
        V.swit = (IDX *)(lds + P.off_swit);
        V.soff = (u16 *)(lds + P.off_soff);
    }
    V.gs = P.gran_shift;
    V.cap_grans = P.cap_grans;
    V.arena = (u64 *)ws_slice;
    V.bounce = (u64 *)(ws_slice + P.ws_half);
    V.w_spare = P.bmp_words;
    V.np = V.ns = V.n_chunks = V.np_all = V.top = V.live = V.next_sid = V.clock = 0;
    for (u32 i = lane; i < P.bmp_words + 1; i += 64) V.bmp[i] = V.bnd[i] = 0;
    for (u32 i = lane; i < P.bmp_words + 64; i += 64) V.tmp[i] = 0;
    if (!P.small_regs)
        for (u32 i = lane; i < P.cap_free + 128; i += 64) ((u64 *)(lds + P.off_fl))[i] = 0;
    SplitRegs<3> Q;                                         // the pool for small requests, if it fits registers
    Q.init(lds, P);
    for (u32 i = lane; i < P.cap_pblocks + 80; i += 64) V.pool[i] = 0;
    for (u32 i = lane; i < P.cap_sblocks + 80; i += 64) {
        V.ssz[i] = 0;
        if constexpr (!TH) {        // (in the workspace nothing reads a place before it was written)
            V.swit[i] = 0;
            V.soff[i] = 0;
        }
    }
    wave_sync();
    st_one(V.bnd, 0u, 1u);                                  // no chunk yet: the end of the last pBlock is chunk 0
    V.tables_written();
    V.sp.template refresh<TH == 3>(V.ssz, 0u);
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
                if (LIKELY((kind & KIND_SBLOCK) != 0)) {
                    fine_free_sblock(V, S.get_c(slot));
                    active -= (b >> 2) << P.chunk_shift;
                    EMIT(C_FREE | B_SBLOCK, a)
                }
                if (kind == KIND_PBLOCK) {
                    bmp_fill(V.bmp, V.w_spare, a, b >> 2, false);
                    active -= (b >> 2) << P.chunk_shift;
                    EMIT((u32)C_FREE, a)
                }
                if (LIKELY(P.small_regs)) {
                    // (each outcome parks its results and goes on from where it is found: handed back
                    // through a record they would meet in flags that are tested again)
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
                bool ml = false, mr = false;
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
            u32 dlo, dhi = 0, held_units = size;
            if (LIKELY(size >= P.small_limit_units)) {
                const u32 bsize = (size + chunk_units - 1) >> P.chunk_shift;
                u32 ref, place;
                // S1: stitched blocks first, then primitive blocks (Algorithm 1, first loop)
                if (fine_s1_sblock(V, bsize, ref, place)) {
                    S.bind(slot, size, ref, KIND_SBLOCK | (bsize << 2), place);
                    if (!SLOT_REGS) S.set_c(slot, place);
                    requested += size;
                    active += bsize << P.chunk_shift;
                    peak_requested = max(peak_requested, requested);
                    peak_active = max(peak_active, active);
                    EMIT(C_EXACT | B_SBLOCK | (1u << 8), ref)
                }
                // pool[lo_p, hi_p): the multi-chunk pBlocks of exactly bsize chunks
                u32 lo_p, hi_p;
                rank_desc2_k(V.pool, V.np, V.key(bsize, 0), (pkey_t)(((pkey_t)bsize << V.W) - 1), &lo_p, &hi_p);
                if (bsize > 1 ? fine_s1_pblock(V, lo_p, hi_p, ref) : s1_single(V, ref)) {
                    bmp_fill(V.bmp, V.w_spare, ref, bsize, true);
                    S.bind(slot, size, ref, KIND_PBLOCK | (bsize << 2), 0u);
                    requested += size;
                    active += bsize << P.chunk_shift;
                    peak_requested = max(peak_requested, requested);
                    peak_active = max(peak_active, active);
                    EMIT(C_EXACT | (1u << 8), ref)
                }
                // ---- no exact fit: states S2 to S5
                VmsRes R;
                const bool went = fine_alloc_cold(lds, V, S, P, bsize, lo_p, hi_p, sp_reserved + (V.n_chunks << P.chunk_shift), base + j, R);
                V.tables_written();
                V.sp.template refresh<TH == 3>(V.ssz, V.ns);        // the sBlock table may have changed
                if (UNLIKELY(!went)) {                      // an engine table overflowed: the trace ends here
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
                    S.set_c(slot, R.list);
                    held_units = R.held << P.chunk_shift;
                }
            } else {
                // ---- a request below one chunk: the policy's own splitting pool (Sec. 3.1)
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
                    S.set_a(slot, (r.addr << 2) | r.flags);
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
    wave_sync();
    } while (P.retry);
}

#endif
