// The stitching allocator as a live device allocator over HIP's virtual memory management
// API: the decisions of the paper's allocation strategy (Sec. 3.2 - 3.3, Algorithm 1, Sec. 4.1,
// Sec. 4.2.3) taken on the host, every Alloc / Stitch / StitchFree carried out with real
// mappings.  Host code only.
//
// Physical chunks are numbered in the order they are created.  A pBlock is a run of
// consecutive chunk numbers; the run an Alloc created is mapped once, into a range of its own
// ("origin"), and the pBlocks later cut out of it keep their places inside that range, so Split
// needs no driver call.  An sBlock is a list of chunk runs mapped a second time into a range of
// its own; it stays valid when a member pBlock is cut later, because it names chunks, not
// pBlocks, and it is in use as soon as one of its chunks is.
#include <hip/hip_runtime.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>
#include <iterator>
#include <map>
#include <mutex>
#include <new>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

#include "../../include/vms_live.h"

namespace {

typedef uint32_t u32;
typedef uint64_t u64;

const u64 UNIT = 512;
const u64 ENGINE_MAX_BYTES = 1ull << 39;

// decision word (vms_replay.h)
enum : u64 { D_FREE = 0, D_EXACT = 1, D_SPLIT = 2, D_STITCH = 3, D_GROW = 4, D_OOM = 5, D_FREE_NOOP = 6, D_INVALID = 15 };
const u64 D_SMALL = 1u << 4, D_SBLOCK = 1u << 5, D_BIT6 = 1u << 6, D_BIT7 = 1u << 7;

struct Stopwatch {
    double *acc;
    uint64_t *n;
    std::chrono::steady_clock::time_point t0;
    Stopwatch(double *a, uint64_t *c) : acc(a), n(c), t0(std::chrono::steady_clock::now()) {}
    ~Stopwatch()
    {
        *acc += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        if (n) ++*n;
    }
};

// pool order of both pools: larger blocks first; equal sizes by first chunk (pBlocks) or by
// creation number (sBlocks), ascending
struct Rank {
    u32 size, tie;
    bool operator<(const Rank &o) const { return size != o.size ? size > o.size : tie < o.tie; }
};

typedef std::pair<u32, u32> Run;        // (first chunk, chunks)

struct Origin {                         // the range an Alloc mapped its new chunks into
    char *va;
    u32 chunks;
};
struct PBlock {
    u32 len;
    bool active;
};
struct SBlock {
    u32 id;
    u64 stamp;                          // creation or last hand-out: the LRU order of StitchFree
    std::vector<Run> runs;
    char *va;
};
struct SmallBlock {                     // a block of the splitting pool, keyed by its address (units)
    u64 size;
    bool active, seg_first, seg_last;
};
struct SmallSeg {                       // one chunk-sized segment of the splitting pool
    char *va;
    hipMemGenericAllocationHandle_t handle;
    u64 units;
};
struct Held {
    enum Kind { SMALL, PBLOCK, SBLOCK } kind;
    u64 ref;                            // pool address / first chunk / creation number
    u64 req_units, held_units;
};

}  // namespace

struct vms_live {
    vms_live_config cfg;
    int device = 0;
    hipMemAllocationProp prop;
    hipMemAccessDesc access;
    u64 chunk_units = 0, capacity_units = 0, small_limit_units = 0;
    u32 frag_chunks = 0;
    std::mutex lock;
    bool broken = false;                // a driver call failed half-way through an operation

    // large path
    std::vector<hipMemGenericAllocationHandle_t> chunks;
    std::vector<uint8_t> chunk_busy;
    std::map<u32, Origin> origins;      // by first chunk
    std::map<u32, PBlock> pblocks;      // by first chunk
    std::set<Rank> idle;                // inactive pBlocks in pool order
    std::map<Rank, SBlock> spool;       // cached sBlocks in pool order
    std::map<u64, Rank> lru;            // stamp -> sBlock
    std::unordered_map<u32, u32> size_of_sblock;   // creation number -> chunks
    u32 next_sid = 0;
    u64 clock = 0;

    // small path
    std::map<u64, SmallBlock> small_blocks;
    std::set<std::pair<u64, u64>> small_idle;       // (size, address)
    std::map<u64, SmallSeg> small_segs;             // by first address (units)
    u64 small_units = 0;

    std::unordered_map<void *, Held> held;
    // the trace served by vms_live_run_trace
    std::vector<void *> slot_ptr;
    std::vector<uint8_t> slot_state;    // 0 unbound, 1 bound, 2 its request failed
    std::vector<u64> slot_bytes;

    vms_trace_stats st;
    vms_live_api_report api;
    u64 requested = 0, active = 0;      // units
    u32 n_events = 0;

    u64 reserved_units() const { return small_units + (u64)chunks.size() * chunk_units; }
    size_t chunk_bytes() const { return (size_t)cfg.chunk_bytes; }

    bool hip_ok(hipError_t e)
    {
        if (e != hipSuccess) api.hip_error = (int)e;
        return e == hipSuccess;
    }

    // ---- driver calls ------------------------------------------------------------------------

    // new physical chunks; all or none
    bool create_chunks(u32 n, std::vector<hipMemGenericAllocationHandle_t> &out)
    {
        out.clear();
        for (u32 i = 0; i < n; i++) {
            hipMemGenericAllocationHandle_t h;
            hipError_t e;
            {
                Stopwatch t(&api.ms_create, &api.n_create);
                e = hipMemCreate(&h, chunk_bytes(), &prop, 0);
            }
            if (e != hipSuccess) {
                api.hip_error = (int)e;
                (void)hipGetLastError();
                for (auto g : out) {
                    Stopwatch t(&api.ms_release, &api.n_release);
                    (void)hipMemRelease(g);
                }
                out.clear();
                return false;
            }
            out.push_back(h);
        }
        return true;
    }

    // one virtual range over the given handles, in order, readable and writable
    char *map_handles(const std::vector<hipMemGenericAllocationHandle_t> &hs)
    {
        const size_t bytes = hs.size() * chunk_bytes();
        void *va = nullptr;
        {
            Stopwatch t(&api.ms_reserve, &api.n_reserve);
            if (!hip_ok(hipMemAddressReserve(&va, bytes, 0, nullptr, 0))) return nullptr;
        }
        size_t done = 0;
        bool good = true;
        for (; done < hs.size() && good; done++) {
            Stopwatch t(&api.ms_map, &api.n_map);
            good = hip_ok(hipMemMap((char *)va + done * chunk_bytes(), chunk_bytes(), 0, hs[done], 0));
        }
        if (!good) done--;
        if (good) {
            Stopwatch t(&api.ms_set_access, &api.n_set_access);
            good = hip_ok(hipMemSetAccess(va, bytes, &access, 1));
        }
        if (!good) {
            for (size_t i = 0; i < done; i++) (void)hipMemUnmap((char *)va + i * chunk_bytes(), chunk_bytes());
            (void)hipMemAddressFree(va, bytes);
            return nullptr;
        }
        return (char *)va;
    }

    void unmap_range(char *va, size_t n_chunks)
    {
        if (!va) return;
        {
            Stopwatch t(&api.ms_unmap, &api.n_unmap);
            hip_ok(hipMemUnmap(va, n_chunks * chunk_bytes()));
        }
        Stopwatch t(&api.ms_address_free, &api.n_address_free);
        hip_ok(hipMemAddressFree(va, n_chunks * chunk_bytes()));
    }

    // ---- the pools ---------------------------------------------------------------------------

    char *pblock_va(u32 first_chunk) const
    {
        auto it = origins.upper_bound(first_chunk);
        --it;
        return it->second.va + (size_t)(first_chunk - it->first) * (size_t)cfg.chunk_bytes;
    }

    void mark_pblock(u32 first, bool active)
    {
        PBlock &p = pblocks.at(first);
        p.active = active;
        for (u32 c = first; c < first + p.len; c++) chunk_busy[c] = active;
        if (active) idle.erase(Rank{ p.len, first });
        else idle.insert(Rank{ p.len, first });
    }

    // every pBlock that now covers a chunk of the sBlock changes state with it
    void mark_sblock(const SBlock &s, bool active)
    {
        for (const Run &r : s.runs)
            for (auto it = pblocks.lower_bound(r.first); it != pblocks.end() && it->first < r.first + r.second; ++it)
                mark_pblock(it->first, active);
    }

    bool sblock_idle(const SBlock &s) const
    {
        for (const Run &r : s.runs)
            for (u32 c = r.first; c < r.first + r.second; c++)
                if (chunk_busy[c]) return false;
        return true;
    }

    // Split (Sec. 3.3.1) of an inactive pBlock into its first `keep` chunks and the rest
    void cut_pblock(u32 first, u32 keep)
    {
        const u32 len = pblocks.at(first).len;
        idle.erase(Rank{ len, first });
        pblocks[first] = PBlock{ keep, false };
        pblocks[first + keep] = PBlock{ len - keep, false };
        idle.insert(Rank{ keep, first });
        idle.insert(Rank{ len - keep, first + keep });
        st.n_split++;
    }

    // Stitch (Sec. 3.3.1): a second mapping of the runs' chunks under one new range
    SBlock *stitch(const std::vector<Run> &runs)
    {
        std::vector<hipMemGenericAllocationHandle_t> hs;
        for (const Run &r : runs)
            for (u32 c = r.first; c < r.first + r.second; c++) hs.push_back(chunks[c]);
        char *va = map_handles(hs);
        // the driver keeps a limited number of mappings: make room by releasing cached sBlocks that are
        // not in use, oldest first, whatever the threshold says, and try again
        for (int attempt = 0; !va && attempt < 16 && release_oldest(32); attempt++) va = map_handles(hs);
        if (!va) {
            broken = true;
            return nullptr;
        }
        SBlock s;
        s.id = next_sid++;
        s.stamp = ++clock;
        s.runs = runs;
        s.va = va;
        const Rank key{ (u32)hs.size(), s.id };
        lru[s.stamp] = key;
        size_of_sblock[s.id] = key.size;
        st.n_sblock_created++;
        return &spool.emplace(key, std::move(s)).first->second;
    }

    // release up to `most` cached sBlocks that are not in use, least recently used first, while
    // more than `keep` are cached; returns how many went
    u32 release_oldest(u32 most, size_t keep = 0)
    {
        u32 gone = 0;
        auto it = lru.begin();
        while (gone < most && spool.size() > keep && it != lru.end()) {
            const Rank key = it->second;
            SBlock &s = spool.at(key);
            if (!sblock_idle(s)) {
                ++it;
                continue;
            }
            if (cfg.sync_before_unmap && !gone) hip_ok(hipDeviceSynchronize());
            unmap_range(s.va, key.size);
            size_of_sblock.erase(s.id);
            it = lru.erase(it);
            spool.erase(key);
            st.n_sblock_evicted++;
            gone++;
        }
        return gone;
    }

    // StitchFree (Sec. 3.3.2, Sec. 4.2.3): back to the threshold, as far as idle sBlocks allow
    bool stitch_free() { return spool.size() > cfg.spool_threshold && release_oldest(0xFFFFFFFFu, cfg.spool_threshold) > 0; }

    // ---- requests of one chunk or more (Sec. 4.1) -----------------------------------------------

    u64 serve_large(u64 size_units, Held &out, void **ptr)
    {
        const u32 want = (u32)((size_units + chunk_units - 1) / chunk_units);
        out.held_units = (u64)want * chunk_units;

        // S1: a cached block of exactly this size: stitched blocks before primitive ones
        for (auto it = spool.lower_bound(Rank{ want, 0 }); it != spool.end() && it->first.size == want; ++it) {
            SBlock &s = it->second;
            if (!sblock_idle(s)) continue;
            mark_sblock(s, true);
            lru.erase(s.stamp);
            s.stamp = ++clock;
            lru[s.stamp] = it->first;
            out.kind = Held::SBLOCK;
            out.ref = s.id;
            *ptr = s.va;
            return D_EXACT | D_SBLOCK | (1ull << 8) | ((u64)s.id << 32);
        }
        auto below = idle.lower_bound(Rank{ want, 0 });      // first idle pBlock that is not larger
        if (below != idle.end() && below->size == want) {
            const u32 first = below->tie;
            mark_pblock(first, true);
            out.kind = Held::PBLOCK;
            out.ref = first;
            *ptr = pblock_va(first);
            return D_EXACT | (1ull << 8) | ((u64)first << 32);
        }

        // BestFit, second loop: the last block in pool order that is large enough on its own ...
        if (below != idle.begin()) {
            const Rank big = *std::prev(below);
            u64 dec = D_SPLIT | (1ull << 8) | ((u64)big.tie << 32);
            out.kind = Held::PBLOCK;
            out.ref = big.tie;
            *ptr = pblock_va(big.tie);
            if (big.size < frag_chunks) {
                // S2 under the fragmentation limit: too small to cut, handed out whole
                mark_pblock(big.tie, true);
                out.held_units = (u64)big.size * chunk_units;
                return dec;
            }
            // S2: cut it; an sBlock over both halves keeps the old size on offer (Fig. 9)
            cut_pblock(big.tie, want);
            if (!stitch({ Run(big.tie, big.size) })) return D_INVALID;
            mark_pblock(big.tie, true);
            dec |= D_BIT6;
            if (stitch_free()) dec |= D_BIT7;
            return dec;
        }
        // ... else the largest blocks, as many as needed, none below the fragmentation limit
        std::vector<Run> take;
        u64 have = 0;
        for (auto it = below; it != idle.end() && have < want; ++it) {
            if (it->size < frag_chunks) continue;
            take.push_back(Run(it->tie, it->size));
            have += it->size;
        }
        u64 dec;
        const u32 n_taken = (u32)take.size();
        if (have >= want) {
            // S3: stitch them; the last one is cut so that the sum is exact
            dec = D_STITCH;
            const u32 spare = (u32)(have - want);
            if (spare) {
                Run &last = take.back();
                cut_pblock(last.first, last.second - spare);
                if (!stitch({ last })) return D_INVALID;
                last.second -= spare;
                dec |= D_BIT6;
            }
        } else {
            // S4: the cache is short; Alloc creates exactly the missing chunks (S5 if it cannot)
            const u32 missing = (u32)(want - have);
            if (reserved_units() + (u64)missing * chunk_units > capacity_units) return D_OOM;
            std::vector<hipMemGenericAllocationHandle_t> fresh;
            if (!create_chunks(missing, fresh)) return D_OOM;
            char *va = map_handles(fresh);
            if (!va) {
                for (auto h : fresh) (void)hipMemRelease(h);
                return D_OOM;
            }
            const u32 first = (u32)chunks.size();
            chunks.insert(chunks.end(), fresh.begin(), fresh.end());
            chunk_busy.resize(chunks.size(), 0);
            origins[first] = Origin{ va, missing };
            pblocks[first] = PBlock{ missing, false };
            idle.insert(Rank{ missing, first });
            dec = D_GROW;
            if (take.empty()) {
                mark_pblock(first, true);
                out.kind = Held::PBLOCK;
                out.ref = first;
                *ptr = va;
                return dec | ((u64)first << 32);
            }
            take.push_back(Run(first, missing));
        }
        SBlock *s = stitch(take);
        if (!s) return D_INVALID;
        if (take.size() > st.max_members) st.max_members = (u32)take.size();
        mark_sblock(*s, true);
        out.kind = Held::SBLOCK;
        out.ref = s->id;
        *ptr = s->va;
        dec |= D_SBLOCK | ((u64)n_taken << 8) | ((u64)s->id << 32);
        if (stitch_free()) dec |= D_BIT7;
        return dec;
    }

    // ---- requests below one chunk: best fit with split and neighbour merge (Sec. 2.2, Sec. 3.1) --

    char *small_va(u64 addr) const
    {
        auto it = small_segs.upper_bound(addr);
        --it;
        return it->second.va + (size_t)(addr - it->first) * UNIT;
    }

    u64 serve_small(u64 size_units, Held &out, void **ptr)
    {
        u64 addr;
        bool grew = false, cut = false;
        auto fit = small_idle.lower_bound(std::make_pair(size_units, (u64)0));
        if (fit != small_idle.end()) {
            addr = fit->second;
            small_idle.erase(fit);
        } else {
            const u64 seg_units = (size_units + chunk_units - 1) / chunk_units * chunk_units;
            if (reserved_units() + seg_units > capacity_units) return D_OOM;
            std::vector<hipMemGenericAllocationHandle_t> fresh;
            if (!create_chunks((u32)(seg_units / chunk_units), fresh)) return D_OOM;
            char *va = map_handles(fresh);
            if (!va || fresh.size() != 1) {         // a segment is one chunk: small requests are below one
                for (auto h : fresh) (void)hipMemRelease(h);
                return D_OOM;
            }
            addr = small_units;
            small_segs[addr] = SmallSeg{ va, fresh[0], seg_units };
            small_blocks[addr] = SmallBlock{ seg_units, false, true, true };
            small_units += seg_units;
            grew = true;
        }
        SmallBlock &b = small_blocks.at(addr);
        if (b.size > size_units) {
            small_blocks[addr + size_units] = SmallBlock{ b.size - size_units, false, false, b.seg_last };
            small_idle.insert(std::make_pair(b.size - size_units, addr + size_units));
            b.size = size_units;
            b.seg_last = false;
            cut = true;
            st.n_split++;
        }
        b.active = true;
        out.kind = Held::SMALL;
        out.ref = addr;
        out.held_units = size_units;
        *ptr = small_va(addr);
        const u64 code = grew ? D_GROW : (cut ? D_SPLIT : D_EXACT);
        return code | D_SMALL | (cut ? D_BIT6 : 0) | ((grew ? 0ull : 1ull) << 8) | (addr << 32);
    }

    u64 release_small(u64 addr)
    {
        auto it = small_blocks.find(addr);
        it->second.active = false;
        u64 flags = 0;
        if (!it->second.seg_last) {
            auto right = std::next(it);
            if (!right->second.active) {
                small_idle.erase(std::make_pair(right->second.size, right->first));
                it->second.size += right->second.size;
                it->second.seg_last = right->second.seg_last;
                small_blocks.erase(right);
                flags |= D_BIT7;
                st.n_merge++;
            }
        }
        if (!it->second.seg_first) {
            auto left = std::prev(it);
            if (!left->second.active) {
                small_idle.erase(std::make_pair(left->second.size, left->first));
                left->second.size += it->second.size;
                left->second.seg_last = it->second.seg_last;
                small_blocks.erase(it);
                it = left;
                flags |= D_BIT6;
                st.n_merge++;
            }
        }
        small_idle.insert(std::make_pair(it->second.size, it->first));
        return D_FREE | D_SMALL | flags | (addr << 32);
    }

    // ---- one request ---------------------------------------------------------------------------

    // totals, high-water marks and checksum after the event (same definitions as the replay's)
    void account(u64 dec)
    {
        const u32 code = (u32)(dec & 15);
        st.n_code[code == D_INVALID ? 7 : code]++;
        if (code == D_INVALID) st.status |= VMS_ST_INVALID_EVENT;
        if (code == D_OOM && st.first_oom_event == 0xFFFFFFFFu) st.first_oom_event = n_events;
        const u64 res = reserved_units();
        if (requested * UNIT > st.peak_requested) st.peak_requested = requested * UNIT;
        if (active * UNIT > st.peak_active) st.peak_active = active * UNIT;
        if (res * UNIT > st.peak_reserved) st.peak_reserved = res * UNIT;
        if (small_idle.size() > st.max_free_blocks) st.max_free_blocks = (u32)small_idle.size();
        if (pblocks.size() > st.max_pblocks) st.max_pblocks = (u32)pblocks.size();
        if (spool.size() > st.max_sblocks) st.max_sblocks = (u32)spool.size();
        st.digest += (dec * 0x9E3779B97F4A7C15ull + ((active << 32) | res)) * ((2 * (u64)n_events + 1) * 0xD6E8FEB86659FD93ull);
        n_events++;
    }

    u64 do_malloc(u64 size_units, void **ptr)
    {
        Stopwatch t(&api.ms_malloc, &api.n_malloc);
        *ptr = nullptr;
        Held h;
        h.req_units = size_units;
        u64 dec = size_units < small_limit_units ? serve_small(size_units, h, ptr) : serve_large(size_units, h, ptr);
        if ((dec & 15) == D_OOM || (dec & 15) == D_INVALID) {
            *ptr = nullptr;
            dec &= 15;
        } else {
            held[*ptr] = h;
            requested += h.req_units;
            active += h.held_units;
        }
        account(dec);
        return dec;
    }

    bool do_free(void *ptr, u64 *dec_out)
    {
        Stopwatch t(&api.ms_free, &api.n_free);
        auto it = held.find(ptr);
        if (it == held.end()) return false;
        const Held h = it->second;
        held.erase(it);
        u64 dec;
        if (h.kind == Held::SMALL) {
            dec = release_small(h.ref);
        } else if (h.kind == Held::PBLOCK) {
            mark_pblock((u32)h.ref, false);             // Update: only the state flips (Sec. 3.3.2)
            dec = D_FREE | (h.ref << 32);
        } else {
            mark_sblock(spool.at(Rank{ size_of_sblock.at((u32)h.ref), (u32)h.ref }), false);
            dec = D_FREE | D_SBLOCK | (h.ref << 32);
        }
        requested -= h.req_units;
        active -= h.held_units;
        account(dec);
        *dec_out = dec;
        return true;
    }

    void finish_stats(vms_trace_stats *out) const
    {
        *out = st;
        out->final_requested = requested * UNIT;
        out->final_active = active * UNIT;
        out->final_reserved = reserved_units() * UNIT;
        out->max_runs = 0;
        out->overflow_event = 0xFFFFFFFFu;
        out->fragmentation = st.peak_reserved ? 1.0 - (double)st.peak_active / (double)st.peak_reserved : 0.0;
    }

    void teardown()
    {
        (void)hipDeviceSynchronize();
        for (auto &s : spool) unmap_range(s.second.va, s.first.size);
        for (auto &o : origins) unmap_range(o.second.va, o.second.chunks);
        for (auto &g : small_segs) unmap_range(g.second.va, (size_t)(g.second.units / chunk_units));
        for (auto h : chunks) {
            Stopwatch t(&api.ms_release, &api.n_release);
            (void)hipMemRelease(h);
        }
        for (auto &g : small_segs) {
            Stopwatch t(&api.ms_release, &api.n_release);
            (void)hipMemRelease(g.second.handle);
        }
    }
};

extern "C" void vms_live_config_default(vms_live_config *cfg)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->struct_size = (uint32_t)sizeof *cfg;
    cfg->spool_threshold = 512;
    cfg->chunk_bytes = 2ull << 20;
    cfg->small_limit_bytes = cfg->chunk_bytes;
    cfg->frag_limit_bytes = cfg->chunk_bytes;
    cfg->capacity_bytes = 0;
    cfg->sync_before_unmap = 1;
}

extern "C" int vms_live_create(const vms_live_config *cfg, vms_live **out)
{
    if (!cfg || !out) return VMS_EINVAL;
    if (cfg->struct_size != sizeof(vms_live_config)) return VMS_ESTRUCT;
    const u64 chunk = cfg->chunk_bytes;
    if (chunk < UNIT || (chunk & (chunk - 1)) || cfg->small_limit_bytes > chunk || cfg->frag_limit_bytes % chunk ||
        cfg->small_limit_bytes % UNIT)
        return VMS_EINVAL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return VMS_EHIP;
    vms_live *h = new (std::nothrow) vms_live;
    if (!h) return VMS_ENOMEM;
    h->cfg = *cfg;
    h->device = dev;
    memset(&h->prop, 0, sizeof h->prop);
    h->prop.type = hipMemAllocationTypePinned;
    h->prop.location.type = hipMemLocationTypeDevice;
    h->prop.location.id = dev;
    memset(&h->access, 0, sizeof h->access);
    h->access.location = h->prop.location;
    h->access.flags = hipMemAccessFlagsProtReadWrite;
    size_t gran = 0;
    if (hipMemGetAllocationGranularity(&gran, &h->prop, hipMemAllocationGranularityMinimum) != hipSuccess) {
        delete h;
        return VMS_EHIP;
    }
    if (gran == 0 || chunk % gran) {
        delete h;
        return VMS_EINVAL;
    }
    h->chunk_units = chunk / UNIT;
    const u64 cap = cfg->capacity_bytes ? (cfg->capacity_bytes < ENGINE_MAX_BYTES ? cfg->capacity_bytes : ENGINE_MAX_BYTES)
                                        : ENGINE_MAX_BYTES;
    h->capacity_units = cap / UNIT;
    h->small_limit_units = cfg->small_limit_bytes / UNIT;
    h->frag_chunks = (u32)(cfg->frag_limit_bytes / chunk);
    memset(&h->st, 0, sizeof h->st);
    h->st.first_oom_event = 0xFFFFFFFFu;
    memset(&h->api, 0, sizeof h->api);
    *out = h;
    return VMS_OK;
}

extern "C" int vms_live_malloc(vms_live *h, uint64_t bytes, void **d_ptr, uint64_t *decision)
{
    if (!h || !d_ptr || bytes == 0 || bytes > ENGINE_MAX_BYTES) return VMS_EINVAL;
    std::lock_guard<std::mutex> g(h->lock);
    if (h->broken) return VMS_EHIP;
    const u64 dec = h->do_malloc((bytes + UNIT - 1) / UNIT, d_ptr);
    if (decision) *decision = dec;
    return h->broken ? VMS_EHIP : VMS_OK;
}

extern "C" int vms_live_free(vms_live *h, void *d_ptr, uint64_t *decision)
{
    if (!h || !d_ptr) return VMS_EINVAL;
    std::lock_guard<std::mutex> g(h->lock);
    u64 dec = 0;
    if (!h->do_free(d_ptr, &dec)) return VMS_EINVAL;
    if (decision) *decision = dec;
    return VMS_OK;
}

extern "C" int vms_live_run_trace(vms_live *h, const uint64_t *h_events, uint32_t n_events, uint32_t max_slots,
                                  uint64_t *h_decisions)
{
    if (!h || (!h_events && n_events) || !h_decisions || max_slots == 0) return VMS_EINVAL;
    std::lock_guard<std::mutex> g(h->lock);
    if (h->n_events || !h->slot_state.empty()) return VMS_ESTATE;
    h->slot_ptr.assign(max_slots, nullptr);
    h->slot_state.assign(max_slots, 0);
    h->slot_bytes.assign(max_slots, 0);
    for (uint32_t i = 0; i < n_events; i++) {
        const u64 word = h_events[i], size = word & 0x7FFFFFFFull, slot = word >> 32;
        const bool is_free = (word >> 31) & 1;
        u64 dec = D_INVALID;
        if (slot < max_slots) {
            uint8_t &state = h->slot_state[slot];
            if (!is_free && size && state == 0) {
                void *p = nullptr;
                dec = h->do_malloc(size, &p);
                if (h->broken) return VMS_EHIP;
                state = p ? 1 : 2;
                h->slot_ptr[slot] = p;
                h->slot_bytes[slot] = size * UNIT;
                h_decisions[i] = dec;
                continue;                           // accounted inside
            }
            if (is_free && state == 1) {
                h->do_free(h->slot_ptr[slot], &dec);
                state = 0;
                h->slot_ptr[slot] = nullptr;
                h_decisions[i] = dec;
                continue;
            }
            if (is_free && state == 2) {
                state = 0;
                dec = D_FREE_NOOP;
            }
        }
        h->account(dec);
        h_decisions[i] = dec;
    }
    return VMS_OK;
}

extern "C" int vms_live_slot(vms_live *h, uint32_t slot, void **d_ptr, uint64_t *bytes)
{
    if (!h || !d_ptr) return VMS_EINVAL;
    std::lock_guard<std::mutex> g(h->lock);
    if (slot >= h->slot_ptr.size()) return VMS_EINVAL;
    *d_ptr = h->slot_state[slot] == 1 ? h->slot_ptr[slot] : nullptr;
    if (bytes) *bytes = h->slot_state[slot] == 1 ? h->slot_bytes[slot] : 0;
    return VMS_OK;
}

extern "C" int vms_live_stats(vms_live *h, vms_trace_stats *out, vms_live_api_report *api)
{
    if (!h || !out) return VMS_EINVAL;
    if (api && api->struct_size != sizeof(vms_live_api_report)) return VMS_ESTRUCT;
    std::lock_guard<std::mutex> g(h->lock);
    h->finish_stats(out);
    if (api) {
        *api = h->api;
        api->struct_size = (uint32_t)sizeof *api;
    }
    return VMS_OK;
}

extern "C" void vms_live_destroy(vms_live *h)
{
    if (!h) return;
    {
        std::lock_guard<std::mutex> g(h->lock);
        h->teardown();
    }
    delete h;
}

// ---- one allocator per device for PyTorch's pluggable-allocator hooks ---------------------------

namespace {
const int MAX_DEVICES = 16;
std::mutex g_torch_lock;
vms_live *g_torch[MAX_DEVICES];

u64 env_mb(const char *name, u64 fallback_bytes)
{
    const char *v = getenv(name);
    if (!v || !*v) return fallback_bytes;
    return strtoull(v, nullptr, 10) << 20;
}

vms_live *torch_allocator(int device, bool create)
{
    if (device < 0 || device >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> g(g_torch_lock);
    if (g_torch[device] || !create) return g_torch[device];
    int before = 0;
    if (hipGetDevice(&before) != hipSuccess || hipSetDevice(device) != hipSuccess) return nullptr;
    vms_live_config cfg;
    vms_live_config_default(&cfg);
    cfg.chunk_bytes = env_mb("VMS_LIVE_CHUNK_MB", cfg.chunk_bytes);
    cfg.small_limit_bytes = cfg.chunk_bytes;
    cfg.frag_limit_bytes = env_mb("VMS_LIVE_FRAG_LIMIT_MB", cfg.chunk_bytes);
    cfg.capacity_bytes = env_mb("VMS_LIVE_CAPACITY_MB", 0);
    if (const char *t = getenv("VMS_LIVE_SPOOL_THRESHOLD"))
        if (*t) cfg.spool_threshold = (uint32_t)strtoul(t, nullptr, 10);
    vms_live *h = nullptr;
    if (vms_live_create(&cfg, &h) != VMS_OK) h = nullptr;
    (void)hipSetDevice(before);
    g_torch[device] = h;
    return h;
}
}  // namespace

extern "C" void *vms_torch_malloc(ptrdiff_t size, int device, void *)
{
    vms_live *h = torch_allocator(device, true);
    if (!h) return nullptr;
    void *p = nullptr;
    if (vms_live_malloc(h, size > 0 ? (uint64_t)size : 1, &p, nullptr) != VMS_OK) return nullptr;
    return p;
}

extern "C" void vms_torch_free(void *d_ptr, ptrdiff_t, int device, void *)
{
    vms_live *h = torch_allocator(device, false);
    if (h && d_ptr) (void)vms_live_free(h, d_ptr, nullptr);
}

extern "C" vms_live *vms_torch_allocator(int device) { return torch_allocator(device, false); }
