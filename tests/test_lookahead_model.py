"""A CPU model of the look-ahead kernel's block phase (plain Python, no GPU): the window of stream words a lane
carries through a block, and the hand-overs between the decoding, expanding and storing wavefronts of a chunk
(who may join a block, room in the ring, reuse of log slots, tags, the last pass), run on the library's own
tables and containers under a random scheduler.  The kernel's invariants are asserted at every step:

  * at the start of a block a lane's four words hold at least 97 bits ahead of its position, and the registers the
    kernel still shifts deliver the true next T+1 bits to each of the 8 look-ups;
  * a lane joins a block only if the 8 entries of 8 symbols it may emit fit between what has been stored and the
    ring's size, so no ring slot ever holds two elements, and a slab is stored only when it is final;
  * a log slot is written only after both expanding wavefronts have moved past the block that used it before;
  * the positions the storing wavefronts see (the smaller of the two rows) never run ahead of what is expanded;
  * every wait ends: some wavefront can always make progress until the chunk is complete.

The decoding wavefront publishes a block late (beside the first look-up of the next block, or when it starts to
wait, or when it is done): the other wavefronts see the count of blocks as published, not as logged.
"""
import random

import numpy as np
import pytest

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

BLOCK = 8            # look-ups per block
MAX_SYMBOLS = 8      # symbols per entry
MAX_BITS = 12        # stream bits per entry
SHIFTED = [3, 3, 2, 2, 2, 1, 1, 0]      # window registers the kernel shifts after look-up 0..7


def test_window_registers_deliver_the_next_bits():
    # the schedule follows from the reach of the look-ups still to come: with j to follow, 12 j + 1 bits matter
    for i in range(BLOCK):
        j = BLOCK - 1 - i
        assert SHIFTED[i] == (0 if j == 0 else max(r + 1 for r in range(4) if MAX_BITS * j + 1 > 32 * r))
    rng = random.Random(5)
    for trial in range(6000):
        stream = rng.getrandbits(128 + 64)
        a = rng.choice([31, 31, rng.randrange(32)])                       # position inside the first word
        assert 128 - a >= BLOCK * MAX_BITS + 1 == 97
        full = (stream >> a) & ((1 << (128 - a)) - 1)                     # the four words, aligned (zeros above)
        w = [(full >> (32 * k)) & 0xFFFFFFFF for k in range(4)]
        Ts = [MAX_BITS] * BLOCK if trial % 3 == 0 else [rng.randrange(MAX_BITS + 1) for _ in range(BLOCK)]
        pos = 0
        for i, T in enumerate(Ts):
            assert w[0] & ((1 << (T + 1)) - 1) == (stream >> (a + pos)) & ((1 << (T + 1)) - 1), (trial, i, Ts)
            for k in range(SHIFTED[i]):                                    # a funnel shift per register, low to high:
                up = w[k + 1] if k + 1 < 4 else 0                          # a register that is no longer shifted goes stale
                w[k] = ((w[k] >> T) | (up << (32 - T))) & 0xFFFFFFFF if T else w[k]
            pos += T


class Chunk:
    """One chunk as the look-ahead kernel sees it, and the state its wavefronts hand over."""

    def __init__(self, h, ci, table, ring, slab, slots, storers):
        c = h.chunks[ci]
        self.N, self.n = h.n_streams, int(c["n_symbols"])
        self.t = table
        N = self.N
        hdr = h.stream_hdr[int(c["stream_offset"]):int(c["stream_offset"]) + N].astype(np.int64)
        self.n_words = [int(x >> 16) for x in hdr]
        first = np.cumsum(self.n_words) - self.n_words
        words = h.payload[int(c["payload_offset"]):int(c["payload_offset"]) + int(c["payload_words"])]
        self.payload_words = len(words)
        self.bits = int.from_bytes(np.concatenate([words, np.zeros(8, np.uint32)]).tobytes(), "little")   # 8 zero words behind
        self.first_bit = [32 * min(int(f), self.payload_words) for f in first]
        self.lane_end = [k + ((self.n - k + N - 1) // N if self.n > k else 0) * N for k in range(N)]
        self.ring, self.slab, self.slots, self.storers = ring, slab, slots, storers
        self.reach = BLOCK * MAX_SYMBOLS * N
        assert self.reach < ring and ring % slab == 0
        L2 = len(table["la_bits"])
        # decoding wavefront
        self.pos = list(self.first_bit)
        self.ne = [k if k < self.n else self.lane_end[k] for k in range(N)]
        self.idx = [2 * int(hdr[k] & (L2 // 2 - 1)) + self.peek(self.pos[k], 1) for k in range(N)]
        self.logged, self.published, self.over = 0, 0, False
        self.seen_stored, self.seen_next = 0, 0            # hand-over words as read when the previous block began
                                                           # (the kernel reads them later in that block: newer values are only larger)
        self.log = [None] * slots
        self.bit_row = [[0xFFFFFFFF] * N for _ in range(slots)]
        # expanding wavefronts
        self.next = [0, 1]
        self.prog = [[k if k < self.n else 0xFFFFFFF0 for k in range(N)] for _ in range(2)]
        self.done_x = [False, False]
        self.err = 0
        # storing wavefronts
        self.mine = [s * slab for s in range(storers)]
        self.done_s = [False] * storers
        self.ring_elem = {}                                # ring slot -> (element, symbol); absent: background
        self.out = np.full(self.n, 255, dtype=np.uint8)
        self.stored_elems = 0
        self.dominant = int(table["sym"][-1])

    def peek(self, pos, k):                                # next k stream bits, first bit on top
        v = 0
        for i in range(k):
            v = (v << 1) | ((self.bits >> (pos + i)) & 1)
        return v

    # ---- decoding wavefront: one block, or a wait
    def decode(self):
        if self.over:
            return False
        N = self.N
        newly_published = self.published != self.logged
        self.published = self.logged                        # the block before: published whatever this pass does next
        if not any(self.ne[k] < self.lane_end[k] for k in range(N)):
            self.over = True
            return True
        stored_now, next_now = min(self.mine), min(self.next)           # what this pass reads; used for the block after this one
        limit = [min(self.lane_end[k], self.seen_stored + self.ring - self.reach) for k in range(N)]
        joins = [self.ne[k] < limit[k] for k in range(N)]
        if not any(joins) or self.logged - self.seen_next >= self.slots:
            progress = (self.seen_stored, self.seen_next) != (stored_now, next_now)
            self.seen_stored, self.seen_next = stored_now, next_now
            return progress or newly_published
        # the slot is free: both expanding wavefronts are past the block that used it
        assert self.logged - min(self.next) < self.slots
        slot = self.logged % self.slots
        entries, row8 = [[None] * BLOCK for _ in range(N)], [0] * N
        pos_row = list(self.ne)
        for k in range(N):
            if not joins[k]:
                continue
            # four words from the lane's word, clamped to the chunk's last: in the payload or the zero words behind it
            word = min(self.pos[k] >> 5, self.payload_words)
            assert self.pos[k] - 32 * word + BLOCK * MAX_BITS + 1 <= 128 or word == self.payload_words
            for i in range(BLOCK):
                e = self.idx[k]
                T, c = int(self.t["la_bits"][e]), int(self.t["la_count"][e])
                assert T <= MAX_BITS and 1 <= c <= MAX_SYMBOLS
                entries[k][i] = (int(self.t["la_sym"][e]), T, c, int(self.t["la_state0"][e]))
                self.idx[k] = int(self.t["la_base"][e]) + self.peek(self.pos[k], T + 1)
                assert 0 <= self.idx[k] < len(self.t["la_bits"])            # any bits keep the index in the table
                self.pos[k] += T
                self.ne[k] += c * N
            row8[k] = self.idx[k]
            self.bit_row[slot][k] = (self.pos[k] & 0x3FFFFF) | ((self.logged & 0x3FF) << 22)
            assert self.pos[k] < 1 << 22
        self.log[slot] = (self.logged, entries, row8, pos_row)
        self.logged += 1
        self.seen_stored, self.seen_next = stored_now, next_now
        return True

    # ---- expanding wavefront e: its next block, or a wait
    def expand(self, e):
        if self.done_x[e]:
            return False
        b = self.next[e]
        if self.published <= b:
            if self.over:
                self.done_x[e] = True
                return True
            return False
        slot = b % self.slots
        block, entries, row8, pos_row = self.log[slot]
        assert block == b                                   # not logged over
        N = self.N
        ne = list(pos_row)
        stored_true = min(self.mine)
        for k in range(N):
            took_part = (self.bit_row[slot][k] >> 22) == (b & 0x3FF) and pos_row[k] < self.lane_end[k]
            assert took_part == (entries[k][0] is not None)
            if not took_part:
                continue
            bits_before = (self.bit_row[slot][k] & 0x3FFFFF) - sum(en[1] for en in entries[k])
            pos, bits, found = pos_row[k], bits_before, False
            for i, (sym, T, c, _) in enumerate(entries[k]):
                last = ne[k] + (c - 1) * N
                if last < self.lane_end[k]:                 # (beyond the stream's end the kernel writes slots nobody reads)
                    assert stored_true <= last < stored_true + self.ring, "ring room"
                    s = last % self.ring
                    assert s not in self.ring_elem, "two elements in one ring slot"
                    self.ring_elem[s] = (last, sym)
                ne[k] = last + N
                after = pos + c * N
                bits += T
                if not found and after >= self.lane_end[k]:
                    found = True
                    in_state_0 = entries[k][i + 1][3] != 0 if i + 1 < BLOCK else row8[k] < 2
                    if after != self.lane_end[k] or not in_state_0:
                        self.err |= B.ST_BAD_STATE
                    if (bits - self.first_bit[k] + 31) // 32 != self.n_words[k]:
                        self.err |= B.ST_BAD_LENGTH
                pos = after
        self.prog[e] = ne
        self.next[e] = b + 2
        return True

    # ---- storing wavefront s: the slabs it can take, or a wait
    def store(self, s):
        if self.done_s[s]:
            return False
        last_pass = self.over and self.published <= min(self.next)
        nxt = [0xFFFFFFFF] * self.N if last_pass else [min(a, b) for a, b in zip(self.prog[0], self.prog[1])]
        # the smaller of the two rows never runs ahead of what both wavefronts have expanded
        moved = False
        while self.mine[s] + self.slab <= self.n and all(p >= self.mine[s] + self.slab for p in nxt):
            for j in range(self.mine[s], self.mine[s] + self.slab):
                held = self.ring_elem.pop(j % self.ring, None)
                assert held is None or held[0] == j, "a slab taken while another element sits in its slots"
                self.out[j] = held[1] if held else self.dominant
            self.stored_elems += self.slab
            self.mine[s] += self.storers * self.slab
            moved = True
        if last_pass:
            rest = self.n // self.slab * self.slab
            if (rest // self.slab) % self.storers == s:
                for j in range(rest, self.n):
                    held = self.ring_elem.pop(j % self.ring, None)
                    assert held is None or held[0] == j
                    self.out[j] = held[1] if held else self.dominant
            self.done_s[s] = True
            return True
        return moved

    def finished(self):
        return self.over and all(self.done_x) and all(self.done_s)


def _run(w, ring, slab, slots, storers, seed, corrupt=None):
    h = B.pack_workload(w)
    if corrupt:
        corrupt(h)
    tables = B.build_tables_host(h.freqs, h.table_log)
    syms = np.concatenate(w.symbols())
    rng = random.Random(seed)
    errs = 0
    for ci in range(len(h.chunks)):
        t = B.split_table(tables[int(h.chunks[ci]["layer_id"])])
        ch = Chunk(h, ci, t, ring, slab, slots, storers)
        roles = [("d", 0), ("x", 0), ("x", 1)] + [("s", s) for s in range(storers)]
        idle = 0
        while not ch.finished():
            kind, i = rng.choice(roles) if rng.random() < 0.8 else roles[rng.randrange(len(roles))]
            moved = ch.decode() if kind == "d" else ch.expand(i) if kind == "x" else ch.store(i)
            idle = 0 if moved else idle + 1
            assert idle < 400 * len(roles), "no wavefront can make progress"
        errs |= ch.err
        if not corrupt:
            o = int(h.chunks[ci]["out_offset"])
            assert np.array_equal(ch.out, syms[o:o + ch.n])
    return errs


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("geometry", [(2048, 128, 4, 3), (1024, 64, 2, 4), (4096, 256, 8, 2)])
def test_hand_overs_keep_their_invariants_under_any_schedule(geometry, seed):
    ring, slab, slots, storers = geometry
    # 8 streams, chunks of 6,000 symbols and a ragged last one; reach of a block = 8 * 8 * 8 = 512 elements
    w = W.tiny(seed=seed, n=14000 + 37 * seed, bitwidth=4, n_streams=8, chunk_size=6000, table_log=9, p0=0.55 + 0.1 * seed)
    assert _run(w, ring, slab, slots, storers, seed) == 0


def test_streams_that_end_wrong_are_flagged_by_the_model_too():
    def corrupt(h):
        h.stream_hdr[3] ^= 0x11                  # another initial state: the stream ends elsewhere
    w = W.tiny(seed=4, n=9000, bitwidth=3, n_streams=8, chunk_size=9000, table_log=8, p0=0.7)
    assert _run(w, 2048, 128, 4, 3, 9, corrupt) != 0
