// TEST INFRASTRUCTURE ONLY.  Plain, slow CPU replay of alloc/free traces under
// the two allocator policies of the GMLake paper.  Nothing in the product path
// may include, link or call this file; only the tests, the smoke check and the
// CPU-baseline leg of the benchmark do.  It shares no code with the GPU path.
//
// What is replayed (all sizes are multiples of 512 B):
//   * the splitting caching allocator (Sec. 2.2, "Caching Allocator": best fit,
//     split, lazy free, merge with inactive neighbours), and
//   * the virtual-memory-stitching allocator: pBlock / sBlock pools (Sec. 3.2),
//     Alloc / Split / Stitch (Sec. 3.3.1), BestFit (Algorithm 1), Update and
//     StitchFree (Sec. 3.3.2), the four-state strategy (Sec. 4.1, Fig. 9) and
//     the fragmentation limit (Sec. 4.2.3).
// Metrics follow Sec. 5.1 "Metric": utilisation = peak active / peak reserved,
// fragmentation = 1 - utilisation.
//
// Both policies are online heuristics, so the oracle is the algorithm itself
// in the paper's order; every tie the paper leaves open is broken by a fixed
// total order written next to the code that needs it.
//
// Pins (tests with "not gpu"): the paper's 1 GB + 2 GB stitch example and the
// worked 4 MiB + 2 MiB example; closed forms for peak requested bytes and for
// the stitching allocator's reserved bytes; per-event invariants checked by an
// independent checker over the decision stream; exhaustive best-fit and
// minimal-stitch enumeration on tiny pools; an independent naive Python
// implementation on thousands of small random traces; hand-derived examples of
// what StitchFree releases (Sec. 3.3.2: the least recently used sBlock, and only
// an inactive one; a hand-out renews the use) and of the stitched block that
// records a candidate cut in state S3 (Sec. 4.1, Fig. 9).
// Parity unpinned (the paper fixes no order): which of several equal-sized
// blocks is taken, the StitchFree threshold's exact form, and the numeric ids
// reported in the decision words.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstring>
#include <map>
#include <set>
#include <thread>
#include <utility>
#include <vector>

namespace {

typedef uint64_t u64;
typedef uint32_t u32;

const u64 UNIT = 512;                       // all event sizes are in these units
const u64 ENGINE_MAX_BYTES = 1ull << 39;    // capacity 0 means this (512 GiB)

// decision codes
enum { C_FREE = 0, C_EXACT = 1, C_SPLIT = 2, C_STITCH = 3, C_GROW = 4, C_OOM = 5, C_FREE_NOOP = 6,
       C_INVALID = 15 };
const u64 B_SMALL = 1u << 4, B_SBLOCK = 1u << 5, B_6 = 1u << 6, B_7 = 1u << 7;

struct Params {                 // mirrors the fields the tests pass in
    u64 chunk_bytes;            // physical chunk, 2 MiB in the paper (Sec. 3.1)
    u64 small_limit_bytes;      // requests below this use the splitting pool (Sec. 3.1)
    u64 frag_limit_bytes;       // blocks below this are neither split nor stitched (Sec. 4.2.3)
    u64 capacity_bytes;         // 0 = engine maximum
    u32 spool_threshold;        // StitchFree runs while more sBlocks than this are cached
    u32 max_slots;
};

struct Stats {
    u64 peak_requested, peak_active, peak_reserved;
    u64 final_requested, final_active, final_reserved;
    u64 digest;
    u32 n_code[8];              // events per code 0..6, [7] = invalid
    u32 n_split, n_merge, n_sblock_created, n_sblock_evicted;
    u32 first_oom_event, status;
    u32 max_pblocks, max_sblocks, max_free_blocks, max_members;
    u32 max_total_members, reserved0;   // members summed over all cached sBlocks (high-water mark)
    double fragmentation;
};

// ---------------------------------------------------------------------------
// Splitting pool: best fit with split and neighbour merge (Sec. 2.2, steps 1-4).
// Segments come from the "native allocator": placed one after another in the
// pool's own address space and never returned.  Blocks of different segments
// are never merged (the links exist only between the two halves of a split).
// ---------------------------------------------------------------------------
struct SplitBlock {
    u64 size;       // units
    bool active;
    bool seg_first; // no left neighbour in its segment
    bool seg_last;  // no right neighbour in its segment
};

struct SplitPool {
    std::map<u64, SplitBlock> blocks;           // by address (units): every block, active or not
    std::set<std::pair<u64, u64>> free_blocks;  // (size, address) of the inactive ones
    u64 reserved_units = 0;

    struct Result { int code; bool split; u64 addr; };

    // seg_units: size of a fresh segment if one is needed; may_grow: capacity check result
    Result alloc(u64 size, u64 seg_units, bool may_grow)
    {
        // step 1: the smallest inactive block that fits; equal sizes -> lowest address
        std::map<u64, SplitBlock>::iterator best = blocks.end();
        auto fit = free_blocks.lower_bound(std::make_pair(size, (u64)0));
        if (fit != free_blocks.end()) best = blocks.find(fit->second);
        bool grew = false;
        if (best == blocks.end()) {
            if (!may_grow) return { C_OOM, false, 0 };
            SplitBlock seg = { seg_units, false, true, true };
            best = blocks.insert(std::make_pair(reserved_units, seg)).first;
            reserved_units += seg_units;
            grew = true;
        } else {
            free_blocks.erase(fit);
        }
        // step 2: split off the remainder, which stays cached as the right neighbour
        bool split = false;
        if (best->second.size > size) {
            SplitBlock rest = { best->second.size - size, false, false, best->second.seg_last };
            best->second.size = size;
            best->second.seg_last = false;
            blocks.insert(std::make_pair(best->first + size, rest));
            free_blocks.insert(std::make_pair(rest.size, best->first + size));
            split = true;
        }
        best->second.active = true;
        return { grew ? C_GROW : (split ? C_SPLIT : C_EXACT), split, best->first };
    }

    // steps 3 and 4: mark inactive, merge with inactive neighbours of the same segment
    void release(u64 addr, bool *merged_left, bool *merged_right)
    {
        auto it = blocks.find(addr);
        it->second.active = false;
        *merged_left = *merged_right = false;
        if (!it->second.seg_last) {
            auto r = std::next(it);
            if (!r->second.active) {
                free_blocks.erase(std::make_pair(r->second.size, r->first));
                it->second.size += r->second.size;
                it->second.seg_last = r->second.seg_last;
                blocks.erase(r);
                *merged_right = true;
            }
        }
        if (!it->second.seg_first) {
            auto l = std::prev(it);
            if (!l->second.active) {
                free_blocks.erase(std::make_pair(l->second.size, l->first));
                l->second.size += it->second.size;
                l->second.seg_last = it->second.seg_last;
                blocks.erase(it);
                it = l;
                *merged_left = true;
            }
        }
        free_blocks.insert(std::make_pair(it->second.size, it->first));
    }
};

// ---------------------------------------------------------------------------
// Virtual memory pool (Sec. 3.2).  Physical chunks are numbered in the order
// Alloc creates them.  A pBlock owns a run of consecutive chunk numbers (Alloc
// creates a run, Split cuts a run in two, nothing ever joins runs).  An sBlock
// is an ordered list of chunk runs under one new virtual range; it owns no
// memory.  When a member pBlock is later split the sBlock still denotes the
// same chunks, i.e. its member list is read as "the pBlocks now covering these
// chunks".  It is active as soon as one of its chunks belongs to an active
// pBlock (Sec. 3.2, "if even one pBlock is active").
// ---------------------------------------------------------------------------
struct Run { u32 start, len; };     // in chunks

struct SBlock {
    u32 size;                   // chunks
    u32 id;                     // creation number
    u64 stamp;                  // last use, for LRU
    std::vector<Run> runs;
};

struct PKey {                   // pool order: size descending, then start ascending
    u32 size, start;
    bool operator<(const PKey &o) const { return size != o.size ? size > o.size : start < o.start; }
};
struct SKey {                   // pool order: size descending, then creation number ascending
    u32 size, id;
    bool operator<(const SKey &o) const { return size != o.size ? size > o.size : id < o.id; }
};

// Algorithm 1, over blocks that are already known to be inactive, each range
// in pool order.  The exact-match loop is done by the caller (it needs to know
// which sBlocks are inactive); this is the second loop and the state decision.
// Blocks below the fragmentation limit are never stitched (Sec. 4.2.3), so the
// append branch passes over them.
template <class It>
int best_fit_scan(u32 bsize, It first, It last, u32 frag_limit, std::vector<PKey> *cb)
{
    cb->clear();
    u64 cb_size = 0;
    for (It it = first; it != last; ++it) {
        if (it->size >= bsize) {
            cb->assign(1, *it);
            cb_size = it->size;
        } else if (cb_size < bsize) {
            if (it->size < frag_limit) continue;
            cb->push_back(*it);
            cb_size += it->size;
        } else {
            break;
        }
    }
    if (cb->size() == 1 && cb_size > bsize) return 2;
    if (cb_size >= bsize) return 3;
    return 4;
}

struct VmsPool {
    std::map<u32, u32> pblocks;             // start chunk -> length: all pBlocks (pPool image)
    std::set<PKey> inactive;                // inactive pBlocks in pool order
    std::vector<uint8_t> chunk_active;      // per physical chunk
    std::map<SKey, SBlock> spool;           // sPool in pool order
    std::map<u32, SKey> by_id;              // creation number -> key in spool
    std::map<u64, SKey> by_stamp;           // last-use stamp -> key in spool (LRU order)
    u32 total_members = 0;                  // sum of member counts over the sPool
    u32 n_chunks = 0;                       // chunks created so far (large path)
    u32 next_sblock_id = 0;
    u64 clock = 0;

    bool sblock_inactive(const SBlock &s) const
    {
        for (const Run &r : s.runs)
            for (u32 c = r.start; c < r.start + r.len; c++)
                if (chunk_active[c]) return false;
        return true;
    }
    void set_pblock(u32 start, u32 len, bool active)
    {
        for (u32 c = start; c < start + len; c++) chunk_active[c] = active;
        if (active) inactive.erase(PKey{ len, start });
        else inactive.insert(PKey{ len, start });
    }
    // every pBlock now covering the sBlock's chunks changes state together
    void set_sblock(const SBlock &s, bool active)
    {
        for (const Run &r : s.runs)
            for (auto it = pblocks.lower_bound(r.start); it != pblocks.end() && it->first < r.start + r.len; ++it)
                set_pblock(it->first, it->second, active);
    }
    // Alloc: the only place physical chunks are created (Sec. 3.3.1)
    PKey alloc_pblock(u32 len)
    {
        u32 start = n_chunks;
        n_chunks += len;
        chunk_active.resize(n_chunks, 0);
        pblocks[start] = len;
        inactive.insert(PKey{ len, start });
        return PKey{ len, start };
    }
    // Split an inactive pBlock: first `keep` chunks and the rest become two new pBlocks
    void split_pblock(PKey p, u32 keep)
    {
        inactive.erase(p);
        pblocks[p.start] = keep;
        pblocks[p.start + keep] = p.size - keep;
        inactive.insert(PKey{ keep, p.start });
        inactive.insert(PKey{ p.size - keep, p.start + keep });
    }
    // Stitch: the only place sBlocks are created
    SBlock &stitch(const std::vector<Run> &runs)
    {
        SBlock s;
        s.size = 0;
        for (const Run &r : runs) s.size += r.len;
        s.id = next_sblock_id++;
        s.stamp = ++clock;
        s.runs = runs;
        total_members += (u32)runs.size();
        by_id[s.id] = SKey{ s.size, s.id };
        by_stamp[s.stamp] = SKey{ s.size, s.id };
        return spool.insert(std::make_pair(SKey{ s.size, s.id }, s)).first->second;
    }
    void touch(SBlock &s)
    {
        by_stamp.erase(s.stamp);
        s.stamp = ++clock;
        by_stamp[s.stamp] = SKey{ s.size, s.id };
    }
    void drop(SKey k)
    {
        SBlock &s = spool.at(k);
        total_members -= (u32)s.runs.size();
        by_id.erase(s.id);
        by_stamp.erase(s.stamp);
        spool.erase(k);
    }
};

struct Slot {
    enum Kind { UNBOUND = 0, SPLIT_POOL, PBLOCK, SBLOCK, OOM } kind = UNBOUND;
    u64 req_units = 0;      // requested size
    u64 addr = 0;           // split pool address (units) / pBlock start chunk / sBlock id
    u64 held_units = 0;     // size of the block handed out
};

struct Replay {
    const Params &P;
    int policy;             // 0 = splitting allocator, 1 = stitching allocator
    Stats st;
    u64 requested = 0, active = 0;  // units
    SplitPool sp;           // whole allocator for policy 0; small-request pool for policy 1
    VmsPool vp;
    std::vector<Slot> slots;
    u64 chunk_units, capacity_units;
    std::vector<u64> *handout;      // optional: (event, start chunk, chunks) of large-path hand-outs

    Replay(const Params &p, int pol) : P(p), policy(pol), handout(nullptr)
    {
        memset(&st, 0, sizeof st);
        st.first_oom_event = 0xFFFFFFFFu;
        slots.resize(p.max_slots);
        chunk_units = p.chunk_bytes / UNIT;
        capacity_units = (p.capacity_bytes ? std::min(p.capacity_bytes, ENGINE_MAX_BYTES) : ENGINE_MAX_BYTES) / UNIT;
    }
    u64 reserved() const { return sp.reserved_units + (u64)vp.n_chunks * chunk_units; }

    u64 alloc_split_pool(Slot &s, u64 size, bool small)
    {
        u64 seg = (size + chunk_units - 1) / chunk_units * chunk_units;
        bool may_grow = reserved() + seg <= capacity_units;
        SplitPool::Result r = sp.alloc(size, seg, may_grow);
        if (r.code == C_OOM) return C_OOM;
        if (r.split) st.n_split++;
        s.kind = Slot::SPLIT_POOL;
        s.addr = r.addr;
        s.held_units = size;
        u64 ncb = r.code == C_GROW ? 0 : 1;
        return (u64)r.code | (small ? B_SMALL : 0) | (r.split ? B_6 : 0) | (ncb << 8) | (r.addr << 32);
    }

    void stitch_free(u64 *dec)
    {
        // release least-recently-used inactive sBlocks while above the threshold (Sec. 4.2.3)
        while (vp.spool.size() > P.spool_threshold) {
            auto victim = vp.by_stamp.begin();      // oldest stamp first
            while (victim != vp.by_stamp.end() && !vp.sblock_inactive(vp.spool.at(victim->second))) ++victim;
            if (victim == vp.by_stamp.end()) break;
            vp.drop(victim->second);
            st.n_sblock_evicted++;
            *dec |= B_7;
        }
    }

    void note_handout(u32 ev, const std::vector<Run> &runs)
    {
        if (!handout) return;
        for (const Run &r : runs) {
            handout->push_back(ev);
            handout->push_back(r.start);
            handout->push_back(r.len);
        }
    }

    u64 alloc_vms(Slot &s, u64 size, u32 ev)
    {
        const u32 bsize = (u32)((size + chunk_units - 1) / chunk_units);   // chunks (Sec. 3.1: uniform chunks)
        const u32 frag_limit = (u32)(P.frag_limit_bytes / P.chunk_bytes);

        // S1: exact match, stitched blocks first, then primitive blocks, each in pool order
        for (auto it = vp.spool.lower_bound(SKey{ bsize, 0 }); it != vp.spool.end() && it->first.size == bsize; ++it) {
            SBlock &sb = it->second;
            if (!vp.sblock_inactive(sb)) continue;
            std::vector<Run> now;       // the pBlocks currently covering it
            for (const Run &r : sb.runs)
                for (auto p = vp.pblocks.lower_bound(r.start); p != vp.pblocks.end() && p->first < r.start + r.len; ++p)
                    now.push_back(Run{ p->first, p->second });
            vp.set_sblock(sb, true);
            vp.touch(sb);
            s.kind = Slot::SBLOCK;
            s.addr = sb.id;
            s.held_units = (u64)bsize * chunk_units;
            note_handout(ev, now);
            return C_EXACT | B_SBLOCK | (1ull << 8) | ((u64)sb.id << 32);
        }
        {
            auto it = vp.inactive.lower_bound(PKey{ bsize, 0 });
            if (it != vp.inactive.end() && it->size == bsize) {
                PKey p = *it;
                vp.set_pblock(p.start, p.size, true);
                s.kind = Slot::PBLOCK;
                s.addr = p.start;
                s.held_units = (u64)bsize * chunk_units;
                note_handout(ev, { Run{ p.start, p.size } });
                return C_EXACT | (1ull << 8) | ((u64)p.start << 32);
            }
        }

        std::vector<PKey> cb;
        int state = best_fit_scan(bsize, vp.inactive.begin(), vp.inactive.end(), frag_limit, &cb);
        u64 dec;

        if (state == 2) {
            // S2: one larger block
            PKey p = cb[0];
            if (p.size < frag_limit) {
                // too small to be worth splitting: hand it out whole
                vp.set_pblock(p.start, p.size, true);
                s.kind = Slot::PBLOCK;
                s.addr = p.start;
                s.held_units = (u64)p.size * chunk_units;
                note_handout(ev, { Run{ p.start, p.size } });
                return C_SPLIT | (1ull << 8) | ((u64)p.start << 32);
            }
            vp.split_pblock(p, bsize);
            st.n_split++;
            vp.stitch({ Run{ p.start, p.size } });      // remembers the size that was just cut (Fig. 9, sBlock 1)
            st.n_sblock_created++;
            vp.set_pblock(p.start, bsize, true);
            s.kind = Slot::PBLOCK;
            s.addr = p.start;
            s.held_units = (u64)bsize * chunk_units;
            note_handout(ev, { Run{ p.start, bsize } });
            dec = C_SPLIT | B_6 | (1ull << 8) | ((u64)p.start << 32);
        } else {
            u64 cb_size = 0;
            for (const PKey &p : cb) cb_size += p.size;
            std::vector<Run> runs;
            dec = 0;
            if (state == 3) {
                // S3: several blocks; cut the last one so the sum is exact
                PKey last = cb.back();
                u32 excess = (u32)(cb_size - bsize);
                if (excess) {
                    vp.split_pblock(last, last.size - excess);
                    st.n_split++;
                    vp.stitch({ Run{ last.start, last.size } });
                    st.n_sblock_created++;
                    cb.back() = PKey{ last.size - excess, last.start };
                    dec |= B_6;
                }
                dec |= C_STITCH;
            } else {
                // S4: not enough cached memory; create exactly the missing chunks
                u32 deficit = (u32)(bsize - cb_size);
                if (reserved() + (u64)deficit * chunk_units > capacity_units) return C_OOM;   // S5
                dec |= C_GROW;
                PKey fresh = vp.alloc_pblock(deficit);
                if (cb.empty()) {
                    vp.set_pblock(fresh.start, fresh.size, true);
                    s.kind = Slot::PBLOCK;
                    s.addr = fresh.start;
                    s.held_units = (u64)bsize * chunk_units;
                    note_handout(ev, { Run{ fresh.start, fresh.size } });
                    return dec | ((u64)fresh.start << 32);
                }
                cb.push_back(fresh);
            }
            for (const PKey &p : cb) runs.push_back(Run{ p.start, p.size });
            u32 n_cand = (u32)cb.size() - (state == 4 ? 1 : 0);
            SBlock &sb = vp.stitch(runs);
            st.n_sblock_created++;
            if (runs.size() > st.max_members) st.max_members = (u32)runs.size();
            vp.set_sblock(sb, true);
            s.kind = Slot::SBLOCK;
            s.addr = sb.id;
            s.held_units = (u64)bsize * chunk_units;
            note_handout(ev, runs);
            dec |= B_SBLOCK | ((u64)n_cand << 8) | ((u64)sb.id << 32);
        }
        stitch_free(&dec);
        return dec;
    }

    u64 step(u64 word, u32 ev)
    {
        const u64 size = word & 0x7FFFFFFFull;
        const bool is_free = (word >> 31) & 1;
        const u64 slot = word >> 32;
        if (slot >= slots.size()) { st.status |= 1; return C_INVALID; }
        Slot &s = slots[slot];

        if (!is_free) {
            if (size == 0 || s.kind != Slot::UNBOUND) { st.status |= 1; return C_INVALID; }
            u64 dec;
            if (policy == 0) dec = alloc_split_pool(s, size, false);
            else if (size * UNIT < P.small_limit_bytes) dec = alloc_split_pool(s, size, true);
            else dec = alloc_vms(s, size, ev);
            if ((dec & 15) == C_OOM) {
                s.kind = Slot::OOM;
                if (st.first_oom_event == 0xFFFFFFFFu) st.first_oom_event = ev;
                return dec;
            }
            s.req_units = size;
            requested += size;
            active += s.held_units;
            return dec;
        }

        switch (s.kind) {
        case Slot::UNBOUND:
            st.status |= 1;
            return C_INVALID;
        case Slot::OOM:
            s.kind = Slot::UNBOUND;
            return C_FREE_NOOP;
        case Slot::SPLIT_POOL: {
            bool ml, mr;
            sp.release(s.addr, &ml, &mr);
            st.n_merge += (ml ? 1 : 0) + (mr ? 1 : 0);
            u64 dec = C_FREE | (policy == 1 ? B_SMALL : 0) | (ml ? B_6 : 0) | (mr ? B_7 : 0) | (s.addr << 32);
            requested -= s.req_units;
            active -= s.held_units;
            s.kind = Slot::UNBOUND;
            return dec;
        }
        case Slot::PBLOCK: {
            // Update: only the state flips; the memory stays with its pBlock (Sec. 3.3.2)
            vp.set_pblock((u32)s.addr, (u32)(s.held_units / chunk_units), false);
            u64 dec = C_FREE | (s.addr << 32);
            requested -= s.req_units;
            active -= s.held_units;
            s.kind = Slot::UNBOUND;
            return dec;
        }
        case Slot::SBLOCK: {
            vp.set_sblock(vp.spool.at(vp.by_id.at((u32)s.addr)), false);
            u64 dec = C_FREE | B_SBLOCK | (s.addr << 32);
            requested -= s.req_units;
            active -= s.held_units;
            s.kind = Slot::UNBOUND;
            return dec;
        }
        }
        return C_INVALID;
    }

    void run(const u64 *events, u32 n, u64 *decisions, u64 *series)
    {
        for (u32 i = 0; i < n; i++) {
            u64 dec = step(events[i], i);
            u32 code = (u32)(dec & 15);
            st.n_code[code == C_INVALID ? 7 : code]++;
            u64 res = reserved();
            st.peak_requested = std::max(st.peak_requested, requested * UNIT);
            st.peak_active = std::max(st.peak_active, active * UNIT);
            st.peak_reserved = std::max(st.peak_reserved, res * UNIT);
            st.max_free_blocks = std::max(st.max_free_blocks, (u32)sp.free_blocks.size());
            st.max_pblocks = std::max(st.max_pblocks, (u32)vp.pblocks.size());
            st.max_sblocks = std::max(st.max_sblocks, (u32)vp.spool.size());
            st.max_total_members = std::max(st.max_total_members, vp.total_members);
            // checksum of the whole stream (defined here; the paper defines none): every event
            // adds a term that depends on its position, its decision and the totals after it
            st.digest += (dec * 0x9E3779B97F4A7C15ull + ((active << 32) | res)) *
                         ((2 * (u64)i + 1) * 0xD6E8FEB86659FD93ull);
            if (decisions) decisions[i] = dec;
            if (series) { series[2 * i] = active * UNIT; series[2 * i + 1] = res * UNIT; }
        }
        st.final_requested = requested * UNIT;
        st.final_active = active * UNIT;
        st.final_reserved = reserved() * UNIT;
        // Sec. 5.1 "Metric"
        st.fragmentation = st.peak_reserved ? 1.0 - (double)st.peak_active / (double)st.peak_reserved : 0.0;
    }
};

bool params_ok(const Params &p)
{
    return p.chunk_bytes >= UNIT && p.chunk_bytes % UNIT == 0 && p.frag_limit_bytes % p.chunk_bytes == 0 &&
           p.small_limit_bytes <= p.chunk_bytes && p.max_slots > 0;
}

} // namespace

extern "C" {

// Replay n_traces rows of events[n_traces][max_events] under one policy
// (0 splitting, 1 stitching).  n_events may be NULL (every row is full).
// decisions (nullable) has the shape of events; stats has n_traces entries.
// Returns 0, or -1 on bad parameters.
int oracle_replay(const uint64_t *events, uint32_t n_traces, uint32_t max_events, const uint32_t *n_events,
                  const Params *params, int policy, uint64_t *decisions, Stats *stats, int n_threads)
{
    if (!events || !params || !stats || !params_ok(*params) || policy < 0 || policy > 1) return -1;
    if (n_threads < 1) n_threads = 1;
    std::atomic<uint32_t> next(0);
    auto work = [&]() {
        for (;;) {
            uint32_t t = next.fetch_add(1);
            if (t >= n_traces) break;
            Replay r(*params, policy);
            uint32_t n = n_events ? std::min(n_events[t], max_events) : max_events;
            r.run(events + (size_t)t * max_events, n, decisions ? decisions + (size_t)t * max_events : nullptr, nullptr);
            stats[t] = r.st;
        }
    };
    std::vector<std::thread> th;
    for (int i = 1; i < n_threads; i++) th.emplace_back(work);
    work();
    for (auto &t : th) t.join();
    return 0;
}

// One trace with extra outputs for the invariant checks:
//   series[n][2]   active and reserved bytes after every event (nullable)
//   handout        (event, start chunk, chunks) triples for every chunk run handed
//                  out on the stitching allocator's large path; at most handout_cap
//                  triples are stored, *n_handout receives the number produced
int oracle_replay_verbose(const uint64_t *events, uint32_t n, const Params *params, int policy,
                          uint64_t *decisions, Stats *stats, uint64_t *series,
                          uint64_t *handout, uint64_t handout_cap, uint64_t *n_handout)
{
    if (!events || !params || !stats || !params_ok(*params) || policy < 0 || policy > 1) return -1;
    Replay r(*params, policy);
    std::vector<u64> h;
    r.handout = &h;
    r.run(events, n, decisions, series);
    *stats = r.st;
    if (n_handout) *n_handout = h.size() / 3;
    if (handout) memcpy(handout, h.data(), std::min<u64>(h.size(), handout_cap * 3) * sizeof(u64));
    return 0;
}

// Algorithm 1 on a bare pool of inactive blocks (sizes in chunks, any order:
// they are put into pool order here).  Returns the state 1..4; cb_index
// receives, for each candidate, its index in pblock_sizes (for state 1 a
// stitched block is reported as -(index+1)); *n_cb their number.
int oracle_bestfit(uint32_t bsize, const uint32_t *sblock_sizes, uint32_t n_s, const uint32_t *pblock_sizes,
                   uint32_t n_p, uint32_t frag_limit, int32_t *cb_index, uint32_t *n_cb)
{
    std::set<SKey> s;
    for (u32 i = 0; i < n_s; i++) s.insert(SKey{ sblock_sizes[i], i });
    std::set<PKey> p;
    for (u32 i = 0; i < n_p; i++) p.insert(PKey{ pblock_sizes[i], i });   // "start" carries the index
    for (const SKey &k : s)
        if (k.size == bsize) { cb_index[0] = -(int32_t)k.id - 1; *n_cb = 1; return 1; }
    for (const PKey &k : p)
        if (k.size == bsize) { cb_index[0] = (int32_t)k.start; *n_cb = 1; return 1; }
    std::vector<PKey> cb;
    int state = best_fit_scan(bsize, p.begin(), p.end(), frag_limit, &cb);
    for (size_t i = 0; i < cb.size(); i++) cb_index[i] = (int32_t)cb[i].start;
    *n_cb = (u32)cb.size();
    return state;
}

uint32_t oracle_stats_size(void) { return (uint32_t)sizeof(Stats); }

} // extern "C"
