"""Host-side model of the slot kernel's op-window protocol.

A lane stages its row through a ring of kRing words that is topped up every kSyncRounds rounds with
the kChunk-word load requested at the previous top-up; a request goes out when at most kRefillAt words
are unread.  The kernel relies on two facts, checked here for the constants its source defines: when
a lane issues the op at position k the ring already holds word k + 2, and the word at the cursor is
never overwritten.  (Pure Python, no GPU: the model only moves words around.)
"""
import os
import random
import re

import pytest

SRC = os.path.join(os.path.dirname(__file__), "..", "paper_2510_05112_amd", "csrc", "eval_slots.hip")


def kernel_constants():
    text = open(SRC).read()
    out = {}
    for name in ("kRing", "kChunk", "kSyncRounds", "kRefillAt", "kPrimeChunks"):
        m = re.search(r"constexpr\s+(?:int|unsigned)\s+%s\s*=\s*(\d+)" % name, text)
        assert m, name
        out[name] = int(m.group(1))
    return out


def run_lane(stride, length, rnd, ring_n, chunk, sync, refill_at, prime_chunks):
    row = [rnd.randrange(1, 60000) for _ in range(length)] + [0] * (stride - length)

    def expect(i):
        return row[i] if i < stride else 0

    ring = [None] * ring_n
    loaded = 0
    for _ in range(prime_chunks):
        if loaded < stride:
            for i in range(chunk):
                ring[(loaded + i) % ring_n] = row[loaded + i]
            loaded += chunk
    if loaded >= stride:
        ring[stride % ring_n] = 0          # END planted behind a full row
    w, w_next = ring[0], ring[1 % ring_n]
    cursor, pend = 0, None
    p_move = rnd.choice([0.2, 0.5, 0.9, 1.0])
    r = rnd.randrange(sync)
    for _ in range(50 * stride + 100):
        if r % sync == 0:
            if pend is not None:
                q = loaded % ring_n
                for i in range(chunk):
                    ring[q + i] = pend[i]
                loaded += chunk
                pend = None
                if loaded >= stride:
                    ring[stride % ring_n] = 0
            if loaded - cursor <= refill_at and loaded < stride:
                pend = row[loaded:loaded + chunk]
        assert cursor >= stride or ring[cursor % ring_n] == expect(cursor), "cursor word overwritten"
        if w != 0 and rnd.random() < p_move:
            assert w == row[cursor]
            assert w_next == expect(cursor + 1), "stale next word"
            two_ahead = ring[(cursor + 2) % ring_n]
            cursor, w, w_next = cursor + 1, w_next, two_ahead
        if w == 0:
            return
        r += 1
    raise AssertionError("lane did not finish")


@pytest.mark.parametrize("stride", [8, 16, 24, 32, 40, 64, 896])
def test_two_ahead_word_is_always_in_the_ring(stride):
    k = kernel_constants()
    assert k["kChunk"] >= k["kSyncRounds"] and k["kRing"] & (k["kRing"] - 1) == 0
    rnd = random.Random(stride)
    lengths = sorted({0, 1, 2, 3, 4, 7, 8, 9, 11, 12, 13, 15, 16, 23, 24, 25, stride - 2, stride - 1, stride})
    for length in lengths:
        if 0 <= length <= stride:
            for _ in range(40):
                run_lane(stride, length, rnd, k["kRing"], k["kChunk"], k["kSyncRounds"], k["kRefillAt"],
                         k["kPrimeChunks"])


def test_a_smaller_refill_threshold_would_fail():
    # the model is sharp: one word less of look-ahead and a lane meets a word that has not landed
    k = kernel_constants()
    rnd = random.Random(1)
    with pytest.raises(AssertionError):
        for _ in range(400):
            run_lane(16, 12, rnd, k["kRing"], k["kChunk"], k["kSyncRounds"], k["kRefillAt"] - 1, k["kPrimeChunks"])
