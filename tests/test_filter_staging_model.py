"""Host model of how the blocks of the top-k filter pass (Definition 2) hand their candidates to a row's
list: a stage per block in LDS whose positions an LDS counter hands out, a small stage per wave once the
block's is used up, list slots reserved with atomics on the low half of the row's 64-bit counter word (one
per emptied wave stage, one per finished block, which also adds the block's keys above the band to the
high half), and a per-block flag that stops the listing once a reservation has passed the list's capacity.

The model states the protocol, not the device code.  Blocks and waves take their steps in a seeded random
interleaving; every step that is one atomic on the device is one step here.  Checked: while the list has
room every candidate ends up in it exactly once, slots 0 .. n - 1 are all written and the counter word
reads (n, keys above the band); once more candidates arrive than the list holds, the counter stays above
the capacity, no slot is written twice and nothing is written beyond the capacity.
"""
import random

import pytest

STAGE, WAVE_STAGE = 1024, 256          # the kernel's capacities; the model also runs smaller ones


class Row:
    def __init__(self, cap):
        self.cap = cap
        self.count = 0                 # low half of the counter word
        self.sure = 0                  # high half
        self.slots = {}                # list slot -> entry

    def reserve(self, n, sure=0):      # one 64-bit atomic add
        at = self.count
        self.count += n
        self.sure += sure
        return at

    def write(self, at, entry):
        if at < self.cap:
            assert at not in self.slots, f"slot {at} written twice"
            self.slots[at] = entry


class Block:
    def __init__(self, row, stage_cap, wave_cap):
        self.row, self.stage_cap, self.wave_cap = row, stage_cap, wave_cap
        self.staged = 0                # LDS counter of stage positions handed out
        self.full = False              # the list is full: stop listing
        self.stage = {}
        self.wave = [[] for _ in range(4)]

    def flush_wave(self, w):
        entries = self.wave[w]
        at = self.row.reserve(len(entries))
        if at + len(entries) > self.row.cap:
            self.full = True
        for s, entry in enumerate(entries):
            self.row.write(at + s, entry)
        self.wave[w] = []

    def hit(self, w, entries):
        """Wave w found these candidates in one chunk (at most wave_cap of them)."""
        if self.full:
            return
        m = len(entries)
        pos = self.staged
        self.staged += m
        first_spill = max(pos, self.stage_cap)
        if pos + m > self.stage_cap:
            nsp = pos + m - first_spill
            if len(self.wave[w]) + nsp > self.wave_cap:
                self.flush_wave(w)
            wbase = len(self.wave[w])
            self.wave[w].extend([None] * nsp)
        for o, entry in enumerate(entries):
            p = pos + o
            if p < self.stage_cap:
                assert p not in self.stage
                self.stage[p] = entry
            else:
                self.wave[w][wbase + (p - first_spill)] = entry

    def finish(self, sure):
        for w in range(4):
            if self.wave[w]:
                self.flush_wave(w)
        n = min(self.staged, self.stage_cap)
        at = self.row.reserve(n, sure) if (n or sure) else 0
        for s in range(n):
            self.row.write(at + s, self.stage[s])


def _run(seed, blocks, cap, stage_cap, wave_cap, mean_hit):
    rng = random.Random(seed)
    row = Row(cap)
    blks = [Block(row, stage_cap, wave_cap) for _ in range(blocks)]
    # every wave has its own sequence of hits; the interleaving across waves and blocks is random
    plans, serial, sure_total = [], 0, 0
    for b in range(blocks):
        for w in range(4):
            hits = []
            for _ in range(rng.randrange(0, 12)):
                m = min(wave_cap, max(1, int(rng.expovariate(1.0 / mean_hit))))
                hits.append([(b, serial + i) for i in range(m)])
                serial += m
            plans.append([b, w, hits])
    order = [i for i, p in enumerate(plans) for _ in p[2]]
    rng.shuffle(order)
    cursor = [0] * len(plans)
    for i in order:
        b, w, hits = plans[i]
        blks[b].hit(w, hits[cursor[i]])
        cursor[i] += 1
    finishing = list(range(blocks))
    rng.shuffle(finishing)
    for b in finishing:
        s = rng.randrange(0, 1000)
        sure_total += s
        blks[b].finish(s)
    return row, serial, sure_total, any(bl.full for bl in blks)


@pytest.mark.parametrize("seed", range(40))
def test_every_candidate_is_listed_once_while_the_list_has_room(seed):
    stage_cap, wave_cap = [(STAGE, WAVE_STAGE), (8, 4), (16, 16), (0, 4)][seed % 4]
    mean = [3, 40, 200][seed % 3] if stage_cap == STAGE else 3
    row, total, sure, full = _run(seed, blocks=1 + seed % 7, cap=10**9, stage_cap=stage_cap, wave_cap=wave_cap, mean_hit=mean)
    assert not full
    assert row.count == total and row.sure == sure
    assert sorted(row.slots) == list(range(total)), "the slots 0 .. n - 1 are all written"
    assert len(set(row.slots.values())) == total, "every candidate once"


@pytest.mark.parametrize("seed", range(40))
def test_an_overflowed_list_keeps_its_count_above_the_capacity(seed):
    stage_cap, wave_cap = [(STAGE, WAVE_STAGE), (8, 4), (16, 16)][seed % 3]
    mean = 150 if stage_cap == STAGE else 3
    probe, total, _, _ = _run(seed, blocks=2 + seed % 5, cap=10**9, stage_cap=stage_cap, wave_cap=wave_cap, mean_hit=mean)
    if total < 4:
        pytest.skip("nothing to overflow")
    cap = max(1, total // 3)
    row, total2, sure, _ = _run(seed, blocks=2 + seed % 5, cap=cap, stage_cap=stage_cap, wave_cap=wave_cap, mean_hit=mean)
    assert total2 == total
    assert row.count > cap, "the count must say that the list overflowed"
    assert row.count <= total and row.sure == sure
    assert all(at < cap for at in row.slots), "nothing is written beyond the capacity"
    assert len(set(row.slots.values())) == len(row.slots), "no candidate twice"
