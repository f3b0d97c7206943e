"""Pins of the pack / unpack / exchange oracle against what fixes it from
outside: numpy.concatenate for gap-free layouts, round trips, and hand-written
swaps."""

import numpy as np

from oracle import pack_oracle as po


def _segments(seed, n, sizes=(1, 15, 16, 17, 100, 4096, 33000)):
    rng = np.random.default_rng(seed)
    nb = rng.choice(np.asarray(sizes), size=n)
    return [rng.integers(0, 256, size=int(b), dtype=np.uint8) for b in nb]


def test_gap_free_pack_is_concatenation():
    ts = _segments(0, 40)
    off = np.concatenate([[0], np.cumsum([t.size for t in ts])[:-1]])
    slab = po.pack(ts, off, np.zeros(sum(t.size for t in ts), dtype=np.uint8))
    assert np.array_equal(slab, np.concatenate(ts))


def test_pack_leaves_gaps_untouched_and_unpack_inverts_it():
    ts = _segments(1, 25)
    off, at = [], 7
    for t in ts:
        off.append(at)
        at += t.size + 5
    slab = np.full(at, 0xEE, dtype=np.uint8)
    po.pack(ts, off, slab)
    back = po.unpack(slab, [t.size for t in ts], off)
    assert all(np.array_equal(a, b) for a, b in zip(ts, back))
    covered = np.zeros(at, dtype=bool)
    for t, o in zip(ts, off):
        covered[o:o + t.size] = True
    assert np.all(slab[~covered] == 0xEE)


def test_exchange_swaps_in_place_and_handles_one_sided_units():
    mem = np.arange(64, dtype=np.uint8)
    ref = mem.copy()
    # unit 0: A=[0,16) and B=[16,32) swap: out A->B, in B->A
    # unit 1: only an incoming half [32,40) -> [48,56)
    po.exchange(mem, [(0, 16, 16, 0, 16), (-1, 0, 32, 48, 8)])
    assert np.array_equal(mem[0:16], ref[16:32]) and np.array_equal(mem[16:32], ref[0:16])
    assert np.array_equal(mem[48:56], ref[32:40]) and np.array_equal(mem[32:48], ref[32:48])
    # a planted write-before-read order would have duplicated one half
    assert not np.array_equal(mem[0:16], mem[16:32])
