"""Independent, deliberately naive replay of both allocator policies.

Written separately from oracle/oracle.cpp to pin it: flat Python lists, linear
scans, everything re-sorted on every event, one entry per physical chunk.  It
is only usable on traces of a few hundred events.

Policies follow the GMLake paper: the splitting caching allocator of Sec. 2.2
and the stitching allocator of Sec. 3 / Sec. 4.1 (Algorithm 1, Fig. 9).
"""

UNIT = 512
FREE_BIT = 1 << 31


class NaiveSplit:
    """Best fit + split + merge over one flat list of [addr, size, active, seg_id]."""

    def __init__(self, chunk_units):
        self.blocks = []
        self.chunk = chunk_units
        self.reserved = 0
        self.n_seg = 0

    def n_free(self):
        return sum(1 for b in self.blocks if not b[2])

    def alloc(self, size, may_grow):
        fits = [b for b in self.blocks if not b[2] and b[1] >= size]
        grew = False
        if fits:
            b = min(fits, key=lambda x: (x[1], x[0]))
        else:
            if not may_grow(self.seg_size(size)):
                return None
            b = [self.reserved, self.seg_size(size), False, self.n_seg]
            self.n_seg += 1
            self.reserved += b[1]
            self.blocks.append(b)
            grew = True
        split = b[1] > size
        if split:
            self.blocks.append([b[0] + size, b[1] - size, False, b[3]])
            b[1] = size
        b[2] = True
        return b[0], grew, split

    def seg_size(self, size):
        return -(-size // self.chunk) * self.chunk

    def free(self, addr):
        b = next(x for x in self.blocks if x[0] == addr and x[2])
        b[2] = False
        right = [x for x in self.blocks if x[0] == b[0] + b[1] and x[3] == b[3] and not x[2]]
        mr = bool(right)
        if mr:
            b[1] += right[0][1]
            self.blocks.remove(right[0])
        left = [x for x in self.blocks if x[0] + x[1] == b[0] and x[3] == b[3] and not x[2]]
        ml = bool(left)
        if ml:
            left[0][1] += b[1]
            self.blocks.remove(b)
        return ml, mr


class NaiveVms:
    """Per-chunk bookkeeping: owner[c] = index of the pBlock holding chunk c."""

    def __init__(self):
        self.pb = []            # [start, len, active] ; never removed, len 0 = dead
        self.sb = []            # dict(id, chunks=[...], stamp) ; order of creation
        self.n_chunks = 0
        self.next_id = 0
        self.clock = 0

    def live_pblocks(self):
        return [p for p in self.pb if p[1] > 0]

    def chunk_is_active(self, c):
        for p in self.pb:
            if p[1] > 0 and p[0] <= c < p[0] + p[1]:
                return p[2]
        raise AssertionError("chunk without owner")

    def sblock_inactive(self, s):
        return not any(self.chunk_is_active(c) for c in s["chunks"])

    def pblocks_under(self, chunks):
        cs = set(chunks)
        out = [p for p in self.pb if p[1] > 0 and p[0] in cs]
        for p in out:
            assert all(c in cs for c in range(p[0], p[0] + p[1]))
        return out

    def inactive_sorted(self):
        return sorted([p for p in self.pb if p[1] > 0 and not p[2]], key=lambda p: (-p[1], p[0]))

    def stitch(self, plist):
        chunks = []
        for p in plist:
            chunks.extend(range(p[0], p[0] + p[1]))
        self.clock += 1
        s = dict(id=self.next_id, chunks=chunks, stamp=self.clock)
        self.next_id += 1
        self.sb.append(s)
        return s

    def split(self, p, keep):
        a = [p[0], keep, False]
        b = [p[0] + keep, p[1] - keep, False]
        p[1] = 0
        self.pb.extend([a, b])
        return a, b


def replay(events, policy, chunk_bytes=2 << 20, small_limit_bytes=None, frag_limit_bytes=None,
           capacity_bytes=0, spool_threshold=512, max_slots=1 << 20):
    """Returns dict(decisions=[...], active=[...], reserved=[...]) with byte counts per event."""
    chunk = chunk_bytes // UNIT
    small_limit = chunk if small_limit_bytes is None else small_limit_bytes // UNIT
    frag_limit = 1 if frag_limit_bytes is None else frag_limit_bytes // chunk_bytes
    cap = (min(capacity_bytes, 1 << 39) if capacity_bytes else 1 << 39) // UNIT

    sp = NaiveSplit(chunk)
    vm = NaiveVms()
    slots = {}
    active = 0
    out = dict(decisions=[], active=[], reserved=[])

    def reserved():
        return sp.reserved + vm.n_chunks * chunk

    def may_grow(extra):
        return reserved() + extra <= cap

    def do_split_pool(size, small):
        r = sp.alloc(size, may_grow)
        if r is None:
            return 5, None
        addr, grew, split = r
        code = 4 if grew else (2 if split else 1)
        dec = code | (16 if small else 0) | (64 if split else 0) | ((0 if grew else 1) << 8) | (addr << 32)
        return dec, ("split", addr, size)

    def do_vms(size):
        bsize = -(-size // chunk)
        # exact match: stitched blocks in (size desc, id asc) order, then primitive ones
        for s in sorted(vm.sb, key=lambda s: (-len(s["chunks"]), s["id"])):
            if len(s["chunks"]) == bsize and vm.sblock_inactive(s):
                for p in vm.pblocks_under(s["chunks"]):
                    p[2] = True
                vm.clock += 1
                s["stamp"] = vm.clock
                return 1 | 32 | (1 << 8) | (s["id"] << 32), ("s", s["id"], bsize * chunk)
        pool = vm.inactive_sorted()
        for p in pool:
            if p[1] == bsize:
                p[2] = True
                return 1 | (1 << 8) | (p[0] << 32), ("p", p[0], bsize * chunk)
        # Algorithm 1, second loop
        cb, cbsize = [], 0
        for p in pool:
            if p[1] >= bsize:
                cb, cbsize = [p], p[1]
            elif cbsize < bsize:
                if p[1] >= frag_limit:
                    cb.append(p)
                    cbsize += p[1]
            else:
                break
        created = False
        if len(cb) == 1 and cbsize > bsize:
            p = cb[0]
            if p[1] < frag_limit:
                p[2] = True
                return 2 | (1 << 8) | (p[0] << 32), ("p", p[0], p[1] * chunk)
            old = [p[0], p[1], False]
            a, b = vm.split(p, bsize)
            vm.stitch([old])
            a[2] = True
            dec = 2 | 64 | (1 << 8) | (a[0] << 32)
            held = ("p", a[0], bsize * chunk)
            created = True
        elif cbsize >= bsize:
            dec = 3
            if cbsize > bsize:
                last = cb[-1]
                old = [last[0], last[1], False]
                a, b = vm.split(last, last[1] - (cbsize - bsize))
                vm.stitch([old])
                cb[-1] = a
                dec |= 64
            s = vm.stitch(cb)
            for p in cb:
                p[2] = True
            dec |= 32 | (len(cb) << 8) | (s["id"] << 32)
            held = ("s", s["id"], bsize * chunk)
            created = True
        else:
            deficit = bsize - cbsize
            if not may_grow(deficit * chunk):
                return 5, None
            fresh = [vm.n_chunks, deficit, False]
            vm.n_chunks += deficit
            vm.pb.append(fresh)
            if not cb:
                fresh[2] = True
                return 4 | (fresh[0] << 32), ("p", fresh[0], bsize * chunk)
            s = vm.stitch(cb + [fresh])
            for p in cb + [fresh]:
                p[2] = True
            dec = 4 | 32 | (len(cb) << 8) | (s["id"] << 32)
            held = ("s", s["id"], bsize * chunk)
            created = True
        if created:
            while len(vm.sb) > spool_threshold:
                idle = [s for s in vm.sb if vm.sblock_inactive(s)]
                if not idle:
                    break
                vm.sb.remove(min(idle, key=lambda s: s["stamp"]))
                dec |= 128
        return dec, held

    for w in events:
        w = int(w)
        size, is_free, slot = w & 0x7FFFFFFF, (w >> 31) & 1, w >> 32
        dec = 15
        if slot < max_slots:
            if not is_free:
                if size > 0 and slot not in slots:
                    if policy == 0:
                        dec, held = do_split_pool(size, False)
                    elif size < small_limit:
                        dec, held = do_split_pool(size, True)
                    else:
                        dec, held = do_vms(size)
                    if held is None:
                        slots[slot] = ("oom",)
                    else:
                        slots[slot] = held
                        active += held[2]
            elif slot in slots:
                h = slots.pop(slot)
                if h[0] == "oom":
                    dec = 6
                elif h[0] == "split":
                    ml, mr = sp.free(h[1])
                    dec = (16 if policy == 1 else 0) | (64 if ml else 0) | (128 if mr else 0) | (h[1] << 32)
                    active -= h[2]
                elif h[0] == "p":
                    p = next(x for x in vm.pb if x[1] > 0 and x[0] == h[1])
                    assert p[2] and p[1] * chunk == h[2]
                    p[2] = False
                    dec = h[1] << 32
                    active -= h[2]
                else:
                    s = next(x for x in vm.sb if x["id"] == h[1])
                    for p in vm.pblocks_under(s["chunks"]):
                        assert p[2]
                        p[2] = False
                    dec = 32 | (h[1] << 32)
                    active -= h[2]
        out["decisions"].append(dec)
        out["active"].append(active * UNIT)
        out["reserved"].append(reserved() * UNIT)
    return out
