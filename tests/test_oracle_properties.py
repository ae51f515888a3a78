"""Closed forms, invariants and brute-force checks that pin the CPU oracle.

None of the expected values here comes from the oracle itself: they are prefix
sums over the raw trace, set arithmetic over the decision stream, or exhaustive
enumeration on tiny pools.
"""
import itertools

import numpy as np
import pytest

import naive_alloc
import oracle
from paper_2401_08156_amd import tracegen as tg

MiB = 1 << 20
CHUNK = 2 * MiB


def live_series(events, round_to=1):
    """Running sum of live request bytes (each rounded up to round_to)."""
    is_free, size, slot = tg.decode(events)
    held = {}
    cur, out = 0, []
    for f, s, k in zip(is_free.tolist(), size.tolist(), slot.tolist()):
        if f:
            cur -= held.pop(k)
        else:
            held[k] = -(-s // round_to) * round_to
            cur += held[k]
        out.append(cur)
    return np.array(out, dtype=np.int64)


def small_random_trace(rng, n, size_choices, p_free=0.45):
    ops, live, free_slots, nxt = [], [], [], 0
    for _ in range(n):
        if live and rng.random() < p_free:
            k = live.pop(rng.integers(len(live)))
            ops.append(("F", k))
            free_slots.append(k)
        else:
            if free_slots:
                k = min(free_slots)
                free_slots.remove(k)
            else:
                k, nxt = nxt, nxt + 1
            live.append(k)
            ops.append(("A", k, int(rng.choice(size_choices))))
    return tg.make_events(ops), max(nxt, 1)


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("cfg,nt,ne", [(1, 1, 2000), (2, 3, 3000), (3, 2, 1500), (4, 2, 4000), (6, 5, 3000)])
def test_peak_requested_and_split_active_are_prefix_sums(cfg, nt, ne):
    ev, ms = tg.generate(cfg, n_traces=nt, n_events=ne)
    P = oracle.make_params(ms)
    for pol in (oracle.SPLIT, oracle.VMS):
        _, st = oracle.replay(ev, P, pol)
        for t in range(nt):
            live = live_series(ev[t])
            assert st["peak_requested"][t] == live.max()
            assert st["final_requested"][t] == live[-1]
            if pol == oracle.SPLIT:     # blocks are cut to exactly the request
                assert st["peak_active"][t] == live.max()


@pytest.mark.parametrize("cfg,nt,ne", [(2, 3, 3000), (3, 2, 1500)])
def test_stitching_reserves_exactly_the_peak_of_live_chunks(cfg, nt, ne):
    # Sec. 4.2.1: at every new peak the pool cannot serve the request, every cached block is
    # consumed and only the missing chunks are created -> reserved == active at each growth.
    # With all requests >= 2 MiB and no fragmentation limit the reserved peak is therefore the
    # running maximum of live bytes rounded up to chunks, computed here without any allocator.
    ev, ms = tg.generate(cfg, n_traces=nt, n_events=ne)
    _, st = oracle.replay(ev, oracle.make_params(ms), oracle.VMS)
    for t in range(nt):
        want = live_series(ev[t], CHUNK).max()
        assert st["peak_reserved"][t] == want
        assert st["peak_active"][t] == want
        assert st["fragmentation"][t] == 0.0


def test_degenerate_traces():
    P = oracle.make_params(64)
    # all sizes equal: both policies reuse blocks perfectly
    ops = []
    for rep in range(3):
        ops += [("A", i, 6 * MiB) for i in range(10)] + [("F", i) for i in range(10)]
    ev = tg.make_events(ops)
    for pol in (oracle.SPLIT, oracle.VMS):
        _, st = oracle.replay(ev, P, pol)
        assert st["peak_reserved"][0] == 60 * MiB and st["fragmentation"][0] == 0.0
    # alloc only, chunk multiples: reserved is the plain sum
    sizes = [2, 4, 6, 8, 10, 2, 2, 64]
    ev = tg.make_events([("A", i, s * MiB) for i, s in enumerate(sizes)])
    for pol in (oracle.SPLIT, oracle.VMS):
        _, st = oracle.replay(ev, P, pol)
        assert st["peak_reserved"][0] == sum(sizes) * MiB == st["final_active"][0]
    # strict LIFO: reserved is the deepest stack
    ops = [("A", 0, 4 * MiB), ("A", 1, 8 * MiB), ("A", 2, 2 * MiB), ("F", 2), ("F", 1), ("A", 1, 8 * MiB),
           ("A", 2, 2 * MiB), ("F", 2), ("F", 1), ("F", 0)]
    for pol in (oracle.SPLIT, oracle.VMS):
        _, st = oracle.replay(tg.make_events(ops), P, pol)
        assert st["peak_reserved"][0] == 14 * MiB and st["final_active"][0] == 0


def test_periodic_trace_converges_to_exact_matches():
    # Sec. 4.2.2: after a few identical iterations only state S1 remains and nothing new is reserved.
    rng = np.random.default_rng(7)
    sizes = [int(s) * MiB for s in rng.integers(1, 40, size=24) * 2]
    order = rng.permutation(24).tolist()
    it = [("A", i, s) for i, s in enumerate(sizes)] + [("F", i) for i in order]
    warm = [("A", 30, 100 * MiB), ("A", 31, 36 * MiB), ("F", 30), ("F", 31)]      # pre-fragment the pool
    ev = tg.make_events(warm + it * 6)
    dec, st, series, _ = oracle.replay_verbose(ev, oracle.make_params(64), oracle.VMS)
    codes = (dec & np.uint64(15)).reshape(-1)
    per_it = codes[len(warm):].reshape(6, len(it))
    assert set(per_it[2:].reshape(-1).tolist()) <= {0, 1}
    assert series[len(warm) + len(it):, 1].min() == series[-1, 1]          # reserved constant after iteration 1
    # the splitting allocator keeps splitting and merging on the same trace
    dec2, _ = oracle.replay(ev, oracle.make_params(64), oracle.SPLIT)
    assert 2 in set((dec2[0][-len(it):] & np.uint64(15)).tolist())


# ---------------------------------------------------------------- invariants

def check_invariants(ev, pol, P):
    """Independent checker: rebuilds what is live from the decision words alone."""
    dec, st, series, hand = oracle.replay_verbose(ev, P, pol)
    is_free, size, slot = tg.decode(ev)
    chunk = P.chunk_bytes
    live_req = live_series(ev) if st["n_code"][5] == 0 and st["n_code"][7] == 0 else None
    hand_by_ev = {}
    for e, s, n in hand.tolist():
        hand_by_ev.setdefault(e, []).append((s, n))
    live = {}                      # slot -> list of (space, lo, hi) byte/chunk intervals
    prev_res = 0
    for i, d in enumerate(dec.tolist()):
        code, small, sb, where = d & 15, (d >> 4) & 1, (d >> 5) & 1, d >> 32
        act, res = int(series[i, 0]), int(series[i, 1])
        assert res >= act, "reserved below active"
        assert res >= prev_res, "reserved shrank"
        if res > prev_res:
            assert code == 4, "only growth may raise reserved memory (Sec. 4.2.1, Interface)"
        prev_res = res
        if live_req is not None:
            assert act >= live_req[i]
        if code in (1, 2, 3, 4):
            s = int(size[i])
            if pol == oracle.SPLIT or small:
                iv = [("split", where * 512, where * 512 + s)]
            else:
                runs = hand_by_ev[i]
                got = sum(n for _, n in runs) * chunk
                bsize = -(-s // chunk) * chunk
                if code == 2 and not (d >> 6) & 1:
                    assert got >= bsize       # whole block below the fragmentation limit
                else:
                    assert got == bsize, "a served block matches the chunk-rounded request exactly"
                if sb:
                    assert code in (1, 3, 4), "stitched blocks only by exact match or as a fresh stitch"
                else:
                    assert len(runs) == 1 and runs[0][0] == where
                iv = [("chunk", a, a + n) for a, n in runs]
            for other in live.values():
                for (sp1, lo1, hi1) in other:
                    for (sp2, lo2, hi2) in iv:
                        assert sp1 != sp2 or hi1 <= lo2 or hi2 <= lo1, "two live allocations overlap"
            live[int(slot[i])] = iv
        elif code == 0:
            live.pop(int(slot[i]))
        total = 0
        for ivs in live.values():
            for (sp_, lo, hi) in ivs:
                total += (hi - lo) * (chunk if sp_ == "chunk" else 1)
        assert total == act, "active bytes are exactly the bytes of live blocks"
    return st


@pytest.mark.parametrize("seed", range(6))
def test_invariants_random_small(seed):
    rng = np.random.default_rng(seed)
    sizes = [512, 4096, 300 * 1024, MiB, 2 * MiB, 3 * MiB, 5 * MiB + 512, 8 * MiB, 16 * MiB, 30 * MiB]
    ev, ms = small_random_trace(rng, 400, sizes)
    for pol in (oracle.SPLIT, oracle.VMS):
        check_invariants(ev, pol, oracle.make_params(ms))
    check_invariants(ev, oracle.VMS, oracle.make_params(ms, frag_limit_bytes=4 * MiB))
    check_invariants(ev, oracle.VMS, oracle.make_params(ms, spool_threshold=3))
    check_invariants(ev, oracle.VMS, oracle.make_params(ms, capacity_bytes=64 * MiB))
    check_invariants(ev, oracle.SPLIT, oracle.make_params(ms, capacity_bytes=64 * MiB))


def test_invariants_config1():
    ev, ms = tg.generate(1)
    for pol in (oracle.SPLIT, oracle.VMS):
        st = check_invariants(ev[0], pol, oracle.make_params(ms))
        assert st["status"] == 0


def test_invariants_transformer_slices():
    for cfg in (2, 3, 4, 6):
        ev, ms = tg.generate(cfg, n_traces=1, n_events=1200, first_trace=3)
        check_invariants(ev[0], oracle.VMS, oracle.make_params(ms))
        check_invariants(ev[0], oracle.SPLIT, oracle.make_params(ms))


def test_split_pool_never_leaves_mergeable_neighbours():
    # Sec. 2.2 step 4: after a free, adjacent inactive halves are merged.  Observable consequence:
    # freeing everything returns each segment to one block, so replaying the same allocations
    # again is served without growth.
    rng = np.random.default_rng(3)
    sizes = [int(x) * 512 for x in rng.integers(1, 20000, size=40)]
    order = rng.permutation(40).tolist()
    once = [("A", i, s) for i, s in enumerate(sizes)] + [("F", i) for i in order]
    ev = tg.make_events(once * 2)
    dec, st = oracle.replay(ev, oracle.make_params(64), oracle.SPLIT)
    codes = (dec[0] & np.uint64(15)).tolist()
    assert 4 not in codes[len(once):]
    assert st["n_merge"][0] > 0


# ---------------------------------------------------------------- brute force

def test_bestfit_states_on_hand_built_pools():
    # Algorithm 1: the four states.  Pools are given unsorted; candidates are indices.
    assert oracle.bestfit(5, [7, 5], [5, 9]) == (1, [-2])                 # stitched exact match wins
    assert oracle.bestfit(5, [7], [9, 5, 3]) == (1, [1])
    assert oracle.bestfit(5, [], [9, 6, 7, 3]) == (2, [1])               # smallest block that is larger
    assert oracle.bestfit(10, [], [4, 3, 6, 2]) == (3, [2, 0])           # largest first until the sum reaches
    assert oracle.bestfit(10, [], [4, 3, 2]) == (4, [0, 1, 2])           # everything, still short
    assert oracle.bestfit(10, [], []) == (4, [])
    assert oracle.bestfit(10, [], [9, 9, 1]) == (3, [0, 1])              # stops once satisfied
    assert oracle.bestfit(10, [10], [4, 6]) == (1, [-1])
    # fragmentation limit (Sec. 4.2.3): blocks below it are not stitched
    assert oracle.bestfit(10, [], [6, 3, 3, 2], frag_limit=3) == (3, [0, 1, 2])
    assert oracle.bestfit(10, [], [6, 2, 2, 3], frag_limit=3) == (4, [0, 3])


def test_bestfit_against_exhaustive_enumeration():
    rng = np.random.default_rng(11)
    for _ in range(300):
        n = int(rng.integers(0, 11))
        pool = rng.integers(1, 12, size=n).tolist()
        bsize = int(rng.integers(1, 30))
        state, cb = oracle.bestfit(bsize, [], pool)
        fits = [s for s in pool if s >= bsize]
        if bsize in pool:
            assert state == 1 and pool[cb[0]] == bsize
        elif fits:
            # exhaustive best fit: the minimum over all blocks that are large enough
            assert state == 2 and len(cb) == 1 and pool[cb[0]] == min(fits)
        elif sum(pool) >= bsize:
            # minimal stitch: no subset with fewer blocks reaches the request
            assert state == 3
            got = [pool[i] for i in cb]
            assert sum(got) >= bsize and len(set(cb)) == len(cb)
            k_min = min(k for k in range(1, n + 1)
                        if any(sum(c) >= bsize for c in itertools.combinations(pool, k)))
            assert len(cb) == k_min
            assert sum(got[:-1]) < bsize
        else:
            assert state == 4 and sorted(cb) == list(range(n))


# ---------------------------------------------------------------- independent naive implementation

@pytest.mark.parametrize("seed", range(40))
def test_against_naive_implementation(seed):
    rng = np.random.default_rng(1000 + seed)
    sizes = [512, 1536, 100 * 1024, MiB, 2 * MiB - 512, 2 * MiB, 2 * MiB + 512, 4 * MiB, 6 * MiB,
             7 * MiB, 10 * MiB, 12 * MiB, 20 * MiB]
    n = int(rng.integers(50, 200))
    ev, ms = small_random_trace(rng, n, sizes, p_free=float(rng.choice([0.3, 0.45, 0.55])))
    variants = [dict(), dict(frag_limit_bytes=4 * MiB), dict(spool_threshold=2), dict(capacity_bytes=48 * MiB)]
    kw = variants[seed % len(variants)]
    P = oracle.make_params(ms, **kw)
    for pol in (oracle.SPLIT, oracle.VMS):
        dec, st, series, _ = oracle.replay_verbose(ev, P, pol)
        ref = naive_alloc.replay(ev, pol, max_slots=ms, **kw)
        assert dec.tolist() == ref["decisions"]
        assert series[:, 0].tolist() == ref["active"]
        assert series[:, 1].tolist() == ref["reserved"]
        assert st["peak_active"] == max(ref["active"]) and st["peak_reserved"] == max(ref["reserved"])


def test_digest_definition():
    # sum over events i of (decision * K1 + (active units << 32 | reserved units)) * ((2 i + 1) * K2) mod 2^64
    ev, ms = tg.generate(1, n_events=300)
    dec, st, series, _ = oracle.replay_verbose(ev[0], oracle.make_params(ms), oracle.VMS)
    d, K1, K2, M = 0, 0x9E3779B97F4A7C15, 0xD6E8FEB86659FD93, (1 << 64) - 1
    for i in range(300):
        a, r = int(series[i, 0]) // 512, int(series[i, 1]) // 512
        d = (d + ((int(dec[i]) * K1 + ((a << 32) | r)) & M) * (((2 * i + 1) * K2) & M)) & M
    assert d == int(st["digest"])
