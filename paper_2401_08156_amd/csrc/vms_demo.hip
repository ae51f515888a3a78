// Functional demonstration of virtual memory stitching with real device mappings.
//
// One trace's decision stream of the stitching policy (as written by vms_replay_run) is
// executed on the host with HIP's virtual memory management API: Alloc = hipMemCreate per
// chunk + hipMemAddressReserve + hipMemMap + hipMemSetAccess (Sec. 3.1, Sec. 2.5), Split = two
// new virtual ranges over the same chunks, Stitch = one new virtual range mapped onto the
// chunks of the member blocks while their own mappings stay in place (Sec. 3.3.1: a physical
// chunk may be mapped by several virtual addresses), StitchFree = unmap + release of the range.
//
// The decision words do not list the candidate blocks, so this file keeps its own books of
// pBlocks and sBlocks and re-derives them ("the first k inactive pBlocks in pool order");
// every decision is cross-checked against those books and VMS_EINVAL is returned if they
// disagree.  Call latencies are accumulated per API, and a 2 GiB allocation in 2 MiB chunks
// is timed against hipMalloc for comparison with the paper's Table 1.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <chrono>
#include <map>
#include <set>
#include <string.h>
#include <vector>

#include "../../include/vms_replay.h"

namespace {

typedef uint32_t u32;
typedef uint64_t u64;

struct Timer {
    double *acc;
    u64 *n;
    std::chrono::steady_clock::time_point t0;
    Timer(double *a, u64 *c) : acc(a), n(c), t0(std::chrono::steady_clock::now()) {}
    ~Timer()
    {
        *acc += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        ++*n;
    }
};

struct PBlock {
    u32 len;
    bool active;
    char *va;
};
struct SBlock {
    u32 size;
    u64 stamp;
    std::vector<std::pair<u32, u32>> runs;   // (first chunk, chunks) in mapping order
    char *va;
};
struct PoolKey {
    u32 size, start;
    bool operator<(const PoolKey &o) const { return size != o.size ? size > o.size : start < o.start; }
};
struct Held {
    int kind;       // 0 none, 1 pBlock, 2 sBlock, 3 not tracked (small pool / failed request)
    u32 ref, chunks;
};

struct Demo {
    const vms_config &cfg;
    vms_demo_report &rep;
    hipMemAllocationProp prop;
    hipMemAccessDesc access;
    size_t chunk_bytes;
    std::vector<hipMemGenericAllocationHandle_t> chunks;
    std::map<u32, PBlock> pblocks;           // by first chunk
    std::set<PoolKey> inactive;              // inactive pBlocks in pool order
    std::map<u32, SBlock> sblocks;           // by creation number
    std::vector<Held> slots;
    u32 next_sid = 0;
    u64 clock = 0;
    hipError_t err = hipSuccess;
    bool dry = false;                        // books only: no driver call, mappings are counted
    u64 mapped_now = 0;                      // chunks mapped at this moment, over all live ranges

    Demo(const vms_config &c, vms_demo_report &r) : cfg(c), rep(r), chunk_bytes(c.chunk_bytes), slots(c.max_slots) {}

    bool ok(hipError_t e, u32 api)
    {
        if (e != hipSuccess && err == hipSuccess) {
            err = e;
            rep.failed_api = api;
        }
        return e == hipSuccess;
    }

    // reserve a virtual range and map the given chunk runs into it, in order
    char *map_runs(const std::vector<std::pair<u32, u32>> &runs, u32 total_chunks)
    {
        void *va = nullptr;
        u64 covered = 0;
        for (auto &r : runs) {
            if (r.second == 0 || (u64)r.first + r.second > chunks.size()) return nullptr;   // not chunks we own
            covered += r.second;
        }
        if (covered != total_chunks) return nullptr;
        mapped_now += total_chunks;
        rep.peak_mapped_chunks = std::max<u64>(rep.peak_mapped_chunks, mapped_now);
        if (dry) {
            rep.n_reserve++;
            rep.n_map += total_chunks;
            rep.n_set_access += total_chunks;
            return (char *)chunk_bytes;      // any non-null value: never dereferenced
        }
        {
            Timer t(&rep.ms_reserve, &rep.n_reserve);
            if (!ok(hipMemAddressReserve(&va, (size_t)total_chunks * chunk_bytes, 0, nullptr, 0), 1)) {
                mapped_now -= total_chunks;
                return nullptr;
            }
        }
        // a call that fails leaves nothing of this range behind: what was mapped so far is unmapped
        // and the range returned (the first error is the one reported)
        size_t off = 0, mapped = 0;
        auto undo = [&]() -> char * {
            for (size_t i = 0; i < mapped; i++) (void)hipMemUnmap((char *)va + i * chunk_bytes, chunk_bytes);
            (void)hipMemAddressFree(va, (size_t)total_chunks * chunk_bytes);
            mapped_now -= total_chunks;
            return nullptr;
        };
        for (auto &r : runs)
            for (u32 c = r.first; c < r.first + r.second; c++, off += chunk_bytes) {
                Timer t(&rep.ms_map, &rep.n_map);
                if (!ok(hipMemMap((char *)va + off, chunk_bytes, 0, chunks[c], 0), 3)) return undo();
                mapped++;
            }
        // the paper enables access chunk by chunk (Sec. 2.5); one call per mapped chunk here too
        off = 0;
        for (u32 i = 0; i < total_chunks; i++, off += chunk_bytes) {
            Timer t(&rep.ms_set_access, &rep.n_set_access);
            if (!ok(hipMemSetAccess((char *)va + off, chunk_bytes, &access, 1), 4)) return undo();
        }
        return (char *)va;
    }

    void unmap(char *va, u32 total_chunks)
    {
        if (!va) return;
        mapped_now -= total_chunks;
        if (dry) {
            rep.n_unmap++;
            rep.n_address_free++;
            return;
        }
        {
            Timer t(&rep.ms_unmap, &rep.n_unmap);
            ok(hipMemUnmap(va, (size_t)total_chunks * chunk_bytes), 5);
        }
        Timer t(&rep.ms_address_free, &rep.n_address_free);
        ok(hipMemAddressFree(va, (size_t)total_chunks * chunk_bytes), 7);
    }

    // Alloc: new physical chunks under a new pBlock
    bool alloc_pblock(u32 len)
    {
        u32 start = (u32)chunks.size();
        for (u32 i = 0; i < len; i++) {
            hipMemGenericAllocationHandle_t h;
            if (dry) {
                memset(&h, 0, sizeof h);
                chunks.push_back(h);
                rep.n_create++;
                continue;
            }
            Timer t(&rep.ms_create, &rep.n_create);
            if (!ok(hipMemCreate(&h, chunk_bytes, &prop, 0), 2)) return false;
            chunks.push_back(h);
        }
        char *va = map_runs({ { start, len } }, len);
        if (!va) return false;
        pblocks[start] = PBlock{ len, false, va };
        inactive.insert(PoolKey{ len, start });
        rep.n_pblocks_created++;
        return true;
    }

    // Split: the pBlock's range is replaced by two ranges over the same chunks
    bool split(u32 start, u32 keep)
    {
        auto found = pblocks.find(start);
        if (found == pblocks.end() || keep == 0 || keep >= found->second.len || found->second.active) return false;
        PBlock p = found->second;
        inactive.erase(PoolKey{ p.len, start });
        unmap(p.va, p.len);
        pblocks.erase(found);                // its range is gone: no record may keep the address
        char *a = map_runs({ { start, keep } }, keep);
        char *b = a ? map_runs({ { start + keep, p.len - keep } }, p.len - keep) : nullptr;
        if (!a || !b) {
            unmap(a, keep);
            return false;
        }
        pblocks[start] = PBlock{ keep, false, a };
        pblocks[start + keep] = PBlock{ p.len - keep, false, b };
        inactive.insert(PoolKey{ keep, start });
        inactive.insert(PoolKey{ p.len - keep, start + keep });
        rep.n_splits++;
        return true;
    }

    // Stitch: a new range over chunks that stay mapped where they are
    u32 stitch(const std::vector<std::pair<u32, u32>> &runs)
    {
        SBlock s;
        s.size = 0;
        for (auto &r : runs) s.size += r.second;
        s.stamp = ++clock;
        s.runs = runs;
        s.va = map_runs(runs, s.size);
        u32 id = next_sid++;
        sblocks[id] = s;
        rep.n_stitches++;
        return id;
    }

    void set_pblock(u32 start, bool active)
    {
        PBlock &p = pblocks.at(start);
        p.active = active;
        if (active) inactive.erase(PoolKey{ p.len, start });
        else inactive.insert(PoolKey{ p.len, start });
    }
    void set_sblock(const SBlock &s, bool active)
    {
        for (auto &r : s.runs)
            for (auto it = pblocks.lower_bound(r.first); it != pblocks.end() && it->first < r.first + r.second; ++it)
                set_pblock(it->first, active);
    }
    bool sblock_inactive(const SBlock &s)
    {
        for (auto &r : s.runs)
            for (auto it = pblocks.lower_bound(r.first); it != pblocks.end() && it->first < r.first + r.second; ++it)
                if (it->second.active) return false;
        return true;
    }

    // StitchFree: release least-recently-used inactive sBlocks above the threshold
    bool stitch_free()
    {
        bool any = false;
        while (sblocks.size() > cfg.spool_threshold) {
            auto victim = sblocks.end();
            for (auto it = sblocks.begin(); it != sblocks.end(); ++it)
                if ((victim == sblocks.end() || it->second.stamp < victim->second.stamp) && sblock_inactive(it->second))
                    victim = it;
            if (victim == sblocks.end()) break;
            unmap(victim->second.va, victim->second.size);
            sblocks.erase(victim);
            rep.n_sblocks_released++;
            any = true;
        }
        return any;
    }

    // A stitched range must alias its members: write through the first member pBlock's own
    // range, read back through the sBlock's range.
    void check_alias(const SBlock &s)
    {
        if (dry || !s.va || rep.alias_checks >= 64) return;
        const PBlock &p = pblocks.at(s.runs[0].first);
        u64 pattern = 0xA5A5000000000000ull | ((u64)rep.alias_checks << 32) | s.runs[0].first, back = 0;
        if (!ok(hipMemcpy(p.va, &pattern, sizeof pattern, hipMemcpyHostToDevice), 8)) return;
        if (!ok(hipMemcpy(&back, s.va, sizeof back, hipMemcpyDeviceToHost), 8)) return;
        rep.alias_checks++;
        if (back != pattern) rep.alias_failures++;
    }

    // returns false if the decision contradicts the books kept here
    bool step(u64 ev, u64 dec)
    {
        const u32 code = (u32)dec & 15, slot = (u32)(ev >> 32), where = (u32)(dec >> 32);
        const bool is_free = (ev >> 31) & 1, small = (dec >> 4) & 1, is_s = (dec >> 5) & 1, cut = (dec >> 6) & 1;
        const u32 k = (u32)(dec >> 8) & 0xFFFFFF;
        if (code == 15) return true;
        if (slot >= slots.size()) return false;
        Held &h = slots[slot];
        if (is_free) {
            if (h.kind == 1) {
                if (code != 0 || is_s || where != h.ref) return false;
                set_pblock(h.ref, false);
            } else if (h.kind == 2) {
                if (code != 0 || !is_s || where != h.ref) return false;
                set_sblock(sblocks.at(h.ref), false);
            }
            h.kind = 0;
            return true;
        }
        if (code == 5 || small) {
            h.kind = 3;
            return true;
        }
        const u64 units = (ev & 0x7FFFFFFF) * 512;
        const u32 bsize = (u32)((units + chunk_bytes - 1) / chunk_bytes);
        const u32 frag_limit = (u32)(cfg.frag_limit_bytes / cfg.chunk_bytes);
        bool created = false;
        if (code == 1) {
            if (is_s) {
                auto it = sblocks.find(where);
                if (it == sblocks.end() || it->second.size != bsize || !sblock_inactive(it->second)) return false;
                set_sblock(it->second, true);
                it->second.stamp = ++clock;
                h = Held{ 2, where, bsize };
            } else {
                auto it = pblocks.find(where);
                if (it == pblocks.end() || it->second.len != bsize || it->second.active) return false;
                set_pblock(where, true);
                h = Held{ 1, where, bsize };
            }
        } else if (code == 2) {
            auto it = pblocks.find(where);
            if (it == pblocks.end() || it->second.active || it->second.len <= bsize) return false;
            u32 len = it->second.len;
            if (cut) {
                if (!split(where, bsize)) return false;
                stitch({ { where, len } });
                created = true;
                len = bsize;
            }
            set_pblock(where, true);
            h = Held{ 1, where, len };
        } else if (code == 3 || code == 4) {
            // the candidates: the first k inactive pBlocks smaller than the request, in pool order
            std::vector<PoolKey> cb;
            u64 sum = 0;
            for (auto it = inactive.begin(); it != inactive.end() && cb.size() < k; ++it) {
                if (it->size >= bsize) return false;            // would have been state S1 or S2
                if (it->size < frag_limit) continue;
                cb.push_back(*it);
                sum += it->size;
            }
            if (cb.size() != k) return false;
            std::vector<std::pair<u32, u32>> runs;
            for (auto &p : cb) runs.push_back({ p.start, p.size });
            if (code == 3) {
                if (sum < bsize || (sum > bsize) != cut || k < 2) return false;
                if (sum - cb.back().size >= bsize) return false;     // the last candidate was not needed
                if (cut) {
                    PoolKey last = cb.back();
                    u32 keep = last.size - (u32)(sum - bsize);
                    if (!split(last.start, keep)) return false;
                    stitch({ { last.start, last.size } });
                    runs.back().second = keep;
                }
            } else {
                if (sum >= bsize) return false;
                u32 deficit = bsize - (u32)sum, start = (u32)chunks.size();
                if (!alloc_pblock(deficit)) return false;
                if (k == 0) {
                    if (is_s || where != start) return false;
                    set_pblock(start, true);
                    h = Held{ 1, start, bsize };
                    return true;
                }
                runs.push_back({ start, deficit });
            }
            if (!is_s || where != next_sid) return false;
            u32 id = stitch(runs);
            created = true;
            set_sblock(sblocks.at(id), true);
            check_alias(sblocks.at(id));
            h = Held{ 2, id, bsize };
        } else {
            return false;
        }
        if (created) {
            bool any = stitch_free();
            if (any != (bool)((dec >> 7) & 1)) return false;
        }
        return err == hipSuccess;
    }

    void teardown()
    {
        for (auto &s : sblocks) unmap(s.second.va, s.second.size);
        for (auto &p : pblocks) unmap(p.second.va, p.second.len);
        if (dry) {
            rep.n_release += chunks.size();
            return;
        }
        for (auto h : chunks) {
            Timer t(&rep.ms_release, &rep.n_release);
            ok(hipMemRelease(h), 6);
        }
    }
};

// Table 1 of the paper on this device: one block of `bytes` built from chunks of `chunk` bytes,
// each step timed, against hipMalloc of the same size.
void table1(vms_demo_report &rep, const hipMemAllocationProp &prop, const hipMemAccessDesc &access, size_t bytes,
            size_t chunk)
{
    using clk = std::chrono::steady_clock;
    auto ms = [](clk::time_point a, clk::time_point b) { return std::chrono::duration<double, std::milli>(b - a).count(); };
    double best = 1e30;
    for (int i = 0; i < 3; i++) {
        void *p = nullptr;
        auto t0 = clk::now();
        if (hipMalloc(&p, bytes) != hipSuccess) return;
        auto t1 = clk::now();
        (void)hipFree(p);
        best = std::min(best, ms(t0, t1));
    }
    rep.table1_hipmalloc_ms = best;
    size_t n = bytes / chunk;
    std::vector<hipMemGenericAllocationHandle_t> hs(n);
    void *va = nullptr;
    auto t0 = clk::now();
    if (hipMemAddressReserve(&va, bytes, 0, nullptr, 0) != hipSuccess) return;
    auto t1 = clk::now();
    size_t made = 0;
    for (; made < n; made++)
        if (hipMemCreate(&hs[made], chunk, &prop, 0) != hipSuccess) break;
    auto t2 = clk::now();
    bool good = made == n;
    for (size_t i = 0; good && i < n; i++) good = hipMemMap((char *)va + i * chunk, chunk, 0, hs[i], 0) == hipSuccess;
    auto t3 = clk::now();
    for (size_t i = 0; good && i < n; i++) good = hipMemSetAccess((char *)va + i * chunk, chunk, &access, 1) == hipSuccess;
    auto t4 = clk::now();
    if (good) {
        rep.table1_reserve_ms = ms(t0, t1);
        rep.table1_create_ms = ms(t1, t2);
        rep.table1_map_ms = ms(t2, t3);
        rep.table1_set_access_ms = ms(t3, t4);
        rep.table1_bytes = bytes;
    }
    (void)hipMemUnmap(va, bytes);
    for (size_t i = 0; i < made; i++) (void)hipMemRelease(hs[i]);
    (void)hipMemAddressFree(va, bytes);
}

}  // namespace

// What vms_demo_run would do, without touching the device: the same books, every driver call
// counted instead of made.  Tells whether a trace fits the device before anything is mapped.
extern "C" int vms_demo_plan(const vms_config *cfg, const uint64_t *h_events, const uint64_t *h_dec_vms,
                             uint32_t n_events, vms_demo_report *out)
{
    if (!cfg || !h_events || !h_dec_vms || !out) return VMS_EINVAL;
    if (cfg->struct_size != sizeof(vms_config) || out->struct_size != sizeof(vms_demo_report)) return VMS_ESTRUCT;
    memset((char *)out + sizeof(uint32_t), 0, sizeof *out - sizeof(uint32_t));
    Demo d(*cfg, *out);
    d.dry = true;
    int rc = VMS_OK;
    for (uint32_t i = 0; i < n_events; i++) {
        if (!d.step(h_events[i], h_dec_vms[i])) {
            out->failed_event = i;
            rc = VMS_EINVAL;
            break;
        }
        out->events_replayed = i + 1;
    }
    out->chunks_created = d.chunks.size();
    out->sblocks_cached = (uint32_t)d.sblocks.size();
    d.teardown();
    return rc;
}

extern "C" int vms_demo_run(const vms_config *cfg, const uint64_t *h_events, const uint64_t *h_dec_vms,
                            uint32_t n_events, vms_demo_report *out)
{
    if (!cfg || !h_events || !h_dec_vms || !out) return VMS_EINVAL;
    if (cfg->struct_size != sizeof(vms_config) || out->struct_size != sizeof(vms_demo_report)) return VMS_ESTRUCT;
    memset((char *)out + sizeof(uint32_t), 0, sizeof *out - sizeof(uint32_t));
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return VMS_EHIP;
    Demo d(*cfg, *out);
    memset(&d.prop, 0, sizeof d.prop);
    d.prop.type = hipMemAllocationTypePinned;
    d.prop.location.type = hipMemLocationTypeDevice;
    d.prop.location.id = dev;
    memset(&d.access, 0, sizeof d.access);
    d.access.location = d.prop.location;
    d.access.flags = hipMemAccessFlagsProtReadWrite;
    size_t gran = 0;
    if (hipMemGetAllocationGranularity(&gran, &d.prop, hipMemAllocationGranularityMinimum) != hipSuccess) {
        out->hip_error = (int)hipGetLastError();
        return VMS_EHIP;
    }
    out->granularity_bytes = gran;
    if (gran == 0 || cfg->chunk_bytes % gran) return VMS_EINVAL;   // the model's chunk must be mappable

    int rc = VMS_OK;
    for (uint32_t i = 0; i < n_events; i++) {
        if (!d.step(h_events[i], h_dec_vms[i])) {
            out->failed_event = i;
            rc = d.err != hipSuccess ? VMS_EHIP : VMS_EINVAL;
            break;
        }
        out->events_replayed = i + 1;
    }
    out->chunks_created = d.chunks.size();
    out->sblocks_cached = (uint32_t)d.sblocks.size();
    d.teardown();
    if (rc == VMS_OK && d.err != hipSuccess) rc = VMS_EHIP;
    out->hip_error = (int)d.err;
    if (d.err != hipSuccess) (void)hipGetLastError();   // reported here; not left for the caller's next HIP call to trip over
    if (rc == VMS_OK) table1(*out, d.prop, d.access, (size_t)2 << 30, cfg->chunk_bytes);
    return rc;
}

// The latency table of Sec. 2.5 (Fig. 6, Table 1) on this device: one block of block_bytes built
// from chunks of chunk_bytes, each driver call class timed and the best of `repeats` rounds kept,
// beside hipMalloc + hipFree of the same size.
extern "C" int vms_vmm_latency(uint64_t block_bytes, uint64_t chunk_bytes, uint32_t repeats, vms_vmm_latency_report *out)
{
    if (!out || out->struct_size != sizeof(vms_vmm_latency_report)) return out ? VMS_ESTRUCT : VMS_EINVAL;
    memset((char *)out + sizeof(uint32_t), 0, sizeof *out - sizeof(uint32_t));
    if (!block_bytes || !chunk_bytes || block_bytes % chunk_bytes || !repeats || block_bytes / chunk_bytes > (1u << 20))
        return VMS_EINVAL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return VMS_EHIP;
    hipMemAllocationProp prop;
    memset(&prop, 0, sizeof prop);
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = dev;
    hipMemAccessDesc access;
    memset(&access, 0, sizeof access);
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
    size_t gran = 0;
    hipError_t e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityMinimum);
    if (e != hipSuccess) {
        out->hip_error = (int)e;
        return VMS_EHIP;
    }
    out->granularity_bytes = gran;
    if (gran == 0 || chunk_bytes % gran) return VMS_EINVAL;
    out->block_bytes = block_bytes;
    out->chunk_bytes = chunk_bytes;
    out->n_chunks = block_bytes / chunk_bytes;

    using clk = std::chrono::steady_clock;
    auto ms = [](clk::time_point a, clk::time_point b) { return std::chrono::duration<double, std::milli>(b - a).count(); };
    const size_t n = (size_t)out->n_chunks, bytes = (size_t)block_bytes, chunk = (size_t)chunk_bytes;
    std::vector<hipMemGenericAllocationHandle_t> hs(n);
    double best[8];
    for (double &b : best) b = 1e300;
    for (uint32_t round = 0; round < repeats; round++) {
        void *p = nullptr;
        auto a0 = clk::now();
        e = hipMalloc(&p, bytes);
        auto a1 = clk::now();
        if (e != hipSuccess) {
            out->hip_error = (int)e;
            return VMS_EHIP;
        }
        (void)hipFree(p);
        auto a2 = clk::now();
        best[0] = std::min(best[0], ms(a0, a1));
        best[1] = std::min(best[1], ms(a1, a2));

        void *va = nullptr;
        auto t0 = clk::now();
        e = hipMemAddressReserve(&va, bytes, 0, nullptr, 0);
        auto t1 = clk::now();
        if (e != hipSuccess) {
            out->hip_error = (int)e;
            return VMS_EHIP;
        }
        size_t made = 0, mapped = 0;
        for (; made < n && e == hipSuccess; made++) e = hipMemCreate(&hs[made], chunk, &prop, 0);
        if (e != hipSuccess) made--;
        auto t2 = clk::now();
        for (; mapped < n && e == hipSuccess; mapped++) e = hipMemMap((char *)va + mapped * chunk, chunk, 0, hs[mapped], 0);
        if (e != hipSuccess && mapped) mapped--;
        auto t3 = clk::now();
        for (size_t i = 0; i < n && e == hipSuccess; i++) e = hipMemSetAccess((char *)va + i * chunk, chunk, &access, 1);
        auto t4 = clk::now();
        // give everything back, whatever happened
        for (size_t i = 0; i < mapped; i++) (void)hipMemUnmap((char *)va + i * chunk, chunk);
        auto t5 = clk::now();
        for (size_t i = 0; i < made; i++) (void)hipMemRelease(hs[i]);
        auto t6 = clk::now();
        (void)hipMemAddressFree(va, bytes);
        if (e != hipSuccess) {
            out->hip_error = (int)e;
            (void)hipGetLastError();
            return VMS_EHIP;
        }
        best[2] = std::min(best[2], ms(t0, t1));
        best[3] = std::min(best[3], ms(t1, t2));
        best[4] = std::min(best[4], ms(t2, t3));
        best[5] = std::min(best[5], ms(t3, t4));
        best[6] = std::min(best[6], ms(t4, t5));
        best[7] = std::min(best[7], ms(t5, t6));
    }
    out->hipmalloc_ms = best[0];
    out->hipfree_ms = best[1];
    out->reserve_ms = best[2];
    out->create_ms = best[3];
    out->map_ms = best[4];
    out->set_access_ms = best[5];
    out->unmap_ms = best[6];
    out->release_ms = best[7];
    return VMS_OK;
}
