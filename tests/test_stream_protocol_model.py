"""A model of the streaming kernels' workgroup protocol (csrc/expert_stream.hip, small tiles), run on the CPU.

In that kernel four waves of a workgroup only load (they issue the DMA of slot k + AHEAD after barrier k) and four
only multiply (they use slot k after barrier k); a ring of AHEAD + 1 slots sits between them.  When the line of small
tiles is long, its tail is drawn from a counter in units: wave 0 of the multiplying waves draws unit n + 1 during the
first step of unit n and leaves it in a four-word mailbox, the loading waves pick it up when the first slot of unit
n + 1 is due.  The kernel cannot be stepped on a CPU, so this file restates the two loops and the schedule
arithmetic and checks what the design relies on:

  * both roles execute the same sequence of barriers (a mismatch would hang the workgroup),
  * a ring slot is refilled only after the multiplying waves have passed the barrier that ends its step,
  * a mailbox word is read only in a barrier interval after the one it was written in,
  * every tile of the line is processed exactly once, whatever order the workgroups run in.

It also shows that the checks bite: with units of two slots the mailbox is read too early.
"""
import random

import pytest

AHEAD = 2
RING = AHEAD + 1


class Line:
    """Schedule arithmetic of one small line: the fixed ranges and the units of the drawn part."""

    def __init__(self, n_tiles, G, nkb, rng, pct=60, min_slots=3, dynamic=True):
        self.n_tiles, self.G, self.nkb = n_tiles, G, nkb
        ut = max(1, (min_slots + nkb - 1) // nkb)  # tiles per unit: at least min_slots slots
        ns = (n_tiles * pct // 100) // ut * ut
        nq = (n_tiles - ns) // ut
        self.dyn = dynamic and ns >= G * ut and nq >= G
        if not self.dyn:
            ns, ut = n_tiles, 1
        self.ut, self.pool0 = ut, ns
        n_single = min(nq, 2 * G) if self.dyn else 0
        if self.dyn and (nq - n_single) & 1:
            n_single += 1
        self.n_double = (nq - n_single) // 2 if self.dyn else 0
        self.n_units = self.n_double + n_single
        # the fixed cut: arbitrary non-decreasing positions (the kernel takes them from a cost estimate),
        # rounded down to multiples of ut; some ranges are empty
        w = [rng.choice([0, 0, 1, 1, 1, 2]) for _ in range(G)]
        tot = sum(w) or 1
        cum, self.cuts = 0, [0]
        for b in range(G - 1):
            cum += w[b]
            self.cuts.append(min(int(ns * cum / tot), ns) // ut * ut)
        self.cuts.append(ns)
        self.counter = 0

    def fixed_range(self, b):
        return self.cuts[b], self.cuts[b + 1]

    def unit_range(self, u):
        if u < 0 or u >= self.n_units:
            return 0, 0
        if u < self.n_double:
            t0 = self.pool0 + u * 2 * self.ut
            return t0, t0 + 2 * self.ut
        t0 = self.pool0 + self.n_double * 2 * self.ut + (u - self.n_double) * self.ut
        return t0, (self.n_tiles if u == self.n_units - 1 else t0 + self.ut)

    def draw(self):
        self.counter += 1
        return self.counter - 1


class Workgroup:
    """The two roles as generators that yield at every barrier."""

    def __init__(self, line, b, done):
        self.line, self.done = line, done
        self.mbox = [None] * 4
        self.mbox_interval = [None] * 4
        self.issued, self.used = [], []          # tile of every slot, per role
        self.issue_interval, self.use_interval = {}, {}
        first = line.fixed_range(b)
        if line.dyn and first[0] >= first[1]:    # empty fixed range: the first unit is drawn before the roles split
            first = line.unit_range(line.draw())
        self.first = first

    def loading(self):
        line, nkb = self.line, self.line.nkb
        if self.first[0] >= self.first[1]:
            return
        st = dict(n=0, t=self.first[0], end=self.first[1], kb=0, slot=0, live=True, need=False, single=0)

        def advance(interval):
            if line.dyn and st["need"]:
                st["n"] += 1
                word = st["n"] & 3
                assert self.mbox[word] is not None and self.mbox_interval[word] < interval, "mailbox read too early"
                st["t"], st["end"] = line.unit_range(self.mbox[word])
                if st["t"] >= st["end"]:
                    st["live"] = False
                    return
                st["need"] = False
            self.issued.append(st["t"])
            self.issue_interval[st["slot"]] = interval
            bit = 1 << (st["slot"] & 63)
            st["single"] = (st["single"] & ~bit) | (bit if nkb == 1 else 0)
            st["slot"] += 1
            st["kb"] += 1
            if st["kb"] == nkb:
                st["kb"] = 0
                st["t"] += 1
                if st["t"] == st["end"]:
                    if line.dyn:
                        st["need"] = True
                    else:
                        st["live"] = False

        for _ in range(AHEAD):
            if st["live"]:
                advance(0)
        k = 0
        while k < st["slot"]:
            yield ("slot", k)
            if st["live"]:
                advance(k + 1)
            if (st["single"] >> (k & 63)) & 1:
                yield ("one-slot tile", k)
            k += 1
        yield ("last reduction",)
        yield ("end of class",)

    def multiplying(self):
        line, nkb = self.line, self.line.nkb
        if self.first[0] >= self.first[1]:
            return
        n, t, end = 0, self.first[0], self.first[1]
        kb = slot = 0
        first_step = line.dyn
        while True:
            yield ("slot", slot)
            interval = slot + 1
            if first_step:
                word = (n + 1) & 3
                self.mbox[word], self.mbox_interval[word] = line.draw(), interval
                first_step = False
            self.used.append(t)
            self.use_interval[slot] = interval
            kb += 1
            slot += 1
            if kb == nkb:
                kb = 0
                if nkb == 1:
                    yield ("one-slot tile", slot - 1)
                self.done[t] += 1
                t += 1
                if t == end:
                    if not line.dyn:
                        break
                    n += 1
                    # (wave 0 wrote it, the other multiplying waves read it: a barrier must lie between)
                    assert self.mbox_interval[n & 3] < interval, "mailbox read too early"
                    t, end = line.unit_range(self.mbox[n & 3])
                    if t >= end:
                        break
                    first_step = True
        yield ("last reduction",)
        yield ("end of class",)


def run_line(n_tiles, G, nkb, seed, **kw):
    rng = random.Random(seed)
    line = Line(n_tiles, G, nkb, rng, **kw)
    done = [0] * n_tiles
    wgs = [Workgroup(line, b, done) for b in range(G)]
    gens = [(w.loading(), w.multiplying()) for w in wgs]
    alive = list(range(G))
    while alive:  # workgroups advance one barrier interval at a time, in random order; so do the two roles inside one
        b = rng.choice(alive)
        order = [0, 1]
        rng.shuffle(order)
        ev = [None, None]
        for r in order:
            try:
                ev[r] = next(gens[b][r])
            except StopIteration:
                ev[r] = "stop"
        assert ev[0] == ev[1], f"workgroup {b}: the roles disagree on a barrier: {ev}"
        if ev[0] == "stop":
            alive.remove(b)
    for w in wgs:
        assert w.issued == w.used
        for s, iv in w.issue_interval.items():
            if s >= RING:  # its ring position held slot s - RING, used in interval use_interval[s - RING]
                assert iv > w.use_interval[s - RING], "ring slot refilled before its step was over"
            assert w.use_interval[s] > iv, "slot used before the interval after its issue"
    assert all(d == 1 for d in done), "a tile was skipped or taken twice"
    return line.dyn


@pytest.mark.parametrize("dynamic", [False, True])
def test_roles_agree_and_every_tile_is_taken_once(dynamic):
    rng = random.Random(5)
    n_dyn = 0
    for trial in range(1500):
        G = rng.choice([2, 3, 8, 16])
        nkb = rng.choice([1, 2, 3, 4, 7])
        n_tiles = rng.randint(1, 40 * G)
        n_dyn += run_line(n_tiles, G, nkb, trial, dynamic=dynamic)
    assert (n_dyn > 1000) == dynamic


def test_units_of_two_slots_would_read_the_mailbox_too_early():
    # the reason for "at least three slots per unit" with loads two slots ahead
    rng = random.Random(6)
    with pytest.raises(AssertionError, match="mailbox read too early"):
        for trial in range(400):
            G = rng.choice([2, 3, 8])
            run_line(rng.randint(10 * G, 40 * G), G, rng.choice([1, 2]), trial, min_slots=2)


def test_units_cover_the_drawn_part_exactly():
    rng = random.Random(7)
    for _ in range(300):
        G, nkb = rng.choice([4, 16, 256]), rng.choice([1, 2, 3, 5, 14])
        line = Line(rng.randint(1, 60 * G), G, nkb, rng)
        if not line.dyn:
            continue
        at = line.pool0
        for u in range(line.n_units):
            t0, t1 = line.unit_range(u)
            assert t0 == at and (t1 - t0) * nkb >= 3
            at = t1
        assert at == line.n_tiles and line.unit_range(line.n_units) == (0, 0)
