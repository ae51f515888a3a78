// TEST INFRASTRUCTURE ONLY.  Compiles the replay kernels for the host on top of wave_hw_emu.hpp
// (64 lanes as cooperative fibers) so that their indexing and results can be checked on the CPU:
// every device buffer and the LDS get guard bands that are verified after each wavefront.  The
// product never loads this; it exists to find out-of-bounds accesses and wrong decisions without a GPU.
#include "wave_hw_emu.hpp"

#include "../../paper_2401_08156_amd/csrc/replay_kernels.hpp"
#include "../../paper_2401_08156_amd/csrc/replay_fine.hpp"
#include "../../paper_2401_08156_amd/csrc/selftest.hpp"

#include <vector>

namespace emu {
int cur;
ucontext_t ctx[LANES], back;
u64 xchg[2][LANES];
u64 n_coll;
u64 coll_of[LANES];
bool trace_on = getenv("VMS_EMU_TRACE") != nullptr;
static std::vector<void *> g_sites[LANES];
void note(void *site) { g_sites[cur].push_back(site); }
static void (*g_body)(void *);
static void *g_arg;
static std::vector<char> g_stacks;

static void trampoline(int lane)
{
    g_body(g_arg);
    cur = lane + 1;         // this lane is done: the next one runs on from where it last switched
}

void launch(void (*body)(void *), void *arg, u32 block)
{
    const size_t STACK = 1 << 20;
    if (g_stacks.empty()) g_stacks.resize(STACK * LANES);
    g_body = body;
    g_arg = arg;
    blockIdx.x = block;
    for (int l = 0; l < LANES; l++) {
        coll_of[l] = 0;
        g_sites[l].clear();
        getcontext(&ctx[l]);
        ctx[l].uc_stack.ss_sp = g_stacks.data() + STACK * l;
        ctx[l].uc_stack.ss_size = STACK;
        ctx[l].uc_link = l + 1 < LANES ? &ctx[l + 1] : &back;
        makecontext(&ctx[l], (void (*)())trampoline, 1, l);
    }
    cur = 0;
    swapcontext(&back, &ctx[0]);
    for (int l = 1; l < LANES; l++)
        if (coll_of[l] != coll_of[0]) {
            if (trace_on) {
                size_t i = 0;
                while (i < g_sites[0].size() && i < g_sites[l].size() && g_sites[0][i] == g_sites[l][i]) i++;
                fprintf(stderr, "emu: first difference at operation %zu: lane 0 at %p, lane %d at %p (previous %p)\n", i,
                        i < g_sites[0].size() ? g_sites[0][i] : nullptr, l, i < g_sites[l].size() ? g_sites[l][i] : nullptr,
                        i ? g_sites[0][i - 1] : nullptr);
            }
            fprintf(stderr, "emu: lane %d passed %llu wave-wide operations, lane 0 %llu: divergent control flow\n", l,
                    (unsigned long long)coll_of[l], (unsigned long long)coll_of[0]);
            abort();
        }
}
}  // namespace emu

emu::Dim blockIdx;
const size_t LDS_MAX = 160 * 1024, GUARD = 4096;
alignas(16) char lds[LDS_MAX + GUARD];

namespace {

const unsigned char CANARY = 0xA5;

// a device buffer with guard bands on both sides
struct Guarded {
    std::vector<char> mem;
    size_t bytes;
    Guarded(size_t n) : mem(n + 2 * GUARD + 256, (char)CANARY), bytes(n) {}
    char *ptr() { return (char *)(((uintptr_t)mem.data() + GUARD + 255) & ~(uintptr_t)255); }
    bool intact()
    {
        char *p = ptr();
        for (char *q = mem.data(); q < p; q++)
            if ((unsigned char)*q != CANARY) return false;
        for (char *q = p + bytes; q < mem.data() + mem.size(); q++)
            if ((unsigned char)*q != CANARY) return false;
        return true;
    }
};

struct Args {
    KParams P;
    const u64 *events;
    const u32 *n_events;
    u64 *dec;
    vms_trace_stats *stats;
    char *ws;
    int variant;
};

void body_vms(void *p)
{
    Args &a = *(Args *)p;
    switch (a.variant) {
    case 0: replay_vms_kernel<true>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 1: replay_vms_kernel<false>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 2: replay_vms_fine_kernel<true, uint16_t, 0>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 3: replay_vms_fine_kernel<false, uint16_t, 0>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 4: replay_vms_fine_kernel<true, u32, 0>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 5: replay_vms_fine_kernel<false, u32, 0>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 6: replay_vms_fine_kernel<true, uint16_t, 2>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 7: replay_vms_fine_kernel<false, uint16_t, 2>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 8: replay_vms_fine_kernel<true, uint16_t, 3>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    case 9: replay_vms_fine_kernel<false, uint16_t, 3>(a.P, a.events, a.n_events, a.dec, a.stats, a.ws); break;
    }
}

void body_split(void *p)
{
    Args &a = *(Args *)p;
    switch (a.variant) {
    case 0: replay_split_kernel<true, 3>(a.P, a.events, a.n_events, a.dec, a.stats); break;
    case 1: replay_split_kernel<false, 3>(a.P, a.events, a.n_events, a.dec, a.stats); break;
    case 2: replay_split_kernel<true, 0>(a.P, a.events, a.n_events, a.dec, a.stats); break;
    case 3: replay_split_kernel<false, 0>(a.P, a.events, a.n_events, a.dec, a.stats); break;
    case 4: replay_split_kernel<true, 5>(a.P, a.events, a.n_events, a.dec, a.stats); break;
    case 5: replay_split_kernel<false, 5>(a.P, a.events, a.n_events, a.dec, a.stats); break;
    }
}

u32 g_selftest_fail;
void body_selftest(void *) { selftest_kernel(&g_selftest_fail); }

}  // namespace

extern "C" {

// Replays every trace under the policies of cfg->policy_mask with the kernels the library would
// launch.  dec_split / dec_vms: [n_traces][max_events] or NULL; stats: [2][n_traces].
// Returns 0, a VMS_E* code from planning, or -100 - k if guard band k was written
// (1 LDS, 2 decisions, 3 statistics, 4 workspace).
int emu_replay(const vms_config *cfg, const uint64_t *events, const uint32_t *n_events, uint64_t *dec_split,
               uint64_t *dec_vms, vms_trace_stats *stats)
{
    ReplayPlan plan;
    int rc = replay_plan_make(cfg, plan);
    if (rc != VMS_OK) return rc;
    ReplayPlan again;
    rc = replay_plan_retry(cfg, plan, again);
    if (rc != VMS_OK) return rc;
    if (again.has_retry)
        for (int pol = 0; pol < 2; pol++) plan.kp[pol].retry_slots = cfg->retry_traces;
    const size_t n = (size_t)cfg->n_traces * cfg->max_events, ws_bytes = plan.ws_bytes + again.ws_bytes;
    Guarded g_dec(n * 8), g_stats(sizeof(vms_trace_stats) * (2 * cfg->n_traces + 1)), g_ws(ws_bytes ? ws_bytes : 256);
    memset(g_stats.ptr(), 0, g_stats.bytes);
    for (int pol = 0; pol < 2; pol++) {
        if (!(cfg->policy_mask & (1u << pol))) continue;
        Args a;
        a.P = plan.kp[pol];
        a.events = events;
        a.n_events = n_events;
        uint64_t *out = pol ? dec_vms : dec_split;
        a.dec = out ? (u64 *)g_dec.ptr() : nullptr;
        a.stats = (vms_trace_stats *)g_stats.ptr();
        a.ws = g_ws.ptr();
        if (pol) a.variant = plan.fine ? (plan.wide ? 4 : plan.tbl_ws == 3 ? 8 : plan.tbl_ws ? 6 : 2) + (plan.slot_regs ? 0 : 1) : (plan.slot_regs ? 0 : 1);
        else a.variant = (plan.fl_tiles == 3 ? 0 : plan.fl_tiles == 5 ? 4 : 2) + (plan.slot_regs ? 0 : 1);
        if (out) memset(g_dec.ptr(), 0xFF, n * 8);
        for (int pass = 0; pass < (again.has_retry ? 2 : 1); pass++) {
            const ReplayPlan &pl = pass ? again : plan;
            a.P = pl.kp[pol];
            if (pol) a.variant = pl.fine ? (pl.wide ? 4 : pl.tbl_ws == 3 ? 8 : pl.tbl_ws ? 6 : 2) + (pl.slot_regs ? 0 : 1) : (pl.slot_regs ? 0 : 1);
            else a.variant = (pl.fl_tiles == 3 ? 0 : pl.fl_tiles == 5 ? 4 : 2) + (pl.slot_regs ? 0 : 1);
            // the second pass is a launch of retry_traces wavefronts that share out the flagged traces
            const u32 waves = pass ? std::min(cfg->retry_traces, cfg->n_traces) : cfg->n_traces;
            for (u32 t = 0; t < waves; t++) {
                memset(lds, CANARY, sizeof lds);
                emu::launch(pol ? body_vms : body_split, &a, t);
                for (size_t i = a.P.lds_bytes; i < sizeof lds; i++)
                    if ((unsigned char)lds[i] != CANARY) return -101;
            }
        }
        if (!g_dec.intact()) return -102;
        if (!g_stats.intact()) return -103;
        if (!g_ws.intact()) return -104;
        if (out) memcpy(out, g_dec.ptr(), n * 8);
    }
    memcpy(stats, g_stats.ptr(), sizeof(vms_trace_stats) * 2 * cfg->n_traces);
    return 0;
}

// the wave primitives' self-test kernel on the host lanes: 0, or its failure bits
unsigned emu_selftest(void)
{
    g_selftest_fail = 0xFFFFFFFFu;
    emu::launch(body_selftest, nullptr, 0);
    return g_selftest_fail;
}

}  // extern "C"
