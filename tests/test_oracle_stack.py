"""Pins of the slot-cache model the stacked-decode GPU tests compare the library's counters with
(CPU only): a sequence worked out by hand, and properties that hold for any sequence."""
import numpy as np
import pytest

from oracle.stack_model import SlotCache


def test_hand_worked_sequence():
    # 3 slots, 2 layers of 4 experts, k = 2, n = 1, factors in use; two decode steps with prefetch.
    c = SlotCache(3)
    guess = np.array([[1, 3]])                   # layer 1's gate on layer 0's input: expert 1 first
    # step 1, layer 0: experts 0 and 2 have rows, expert 0 a Top-n row -> two misses (slots 0, 1),
    # one factor copy
    c.layer(0, rows=[1, 0, 1, 0], comp=[1, 0, 0, 0], factors_used=True)
    assert c.key == [(0, 0), (0, 2), None] and c.has_f == [True, False, False]
    # copies ahead for layer 1: expert 1 takes the last free slot with its factors (first in the
    # guessed list); for expert 3 every slot is spoken for
    c.prefetch(1, guess, 4, 1, True)
    assert c.key == [(0, 0), (0, 2), (1, 1)] and c.fresh == [False, False, True]
    assert c.c["prefetched"] == 1 and c.c["factor_copies"] == 2
    # step 1, layer 1: expert 1 hits the slot filled ahead; expert 3 misses and evicts the least
    # recently used slot (slot 0, used before slot 1), with a factor copy
    c.layer(1, rows=[0, 1, 0, 1], comp=[0, 0, 0, 1], factors_used=True)
    assert c.key == [(1, 3), (0, 2), (1, 1)]
    assert c.c["hits"] == 1 and c.c["prefetch_hits"] == 1 and c.c["misses"] == 3 and c.c["factor_copies"] == 3
    # step 2, layer 0: expert 0 was evicted -> miss; least recently used is slot 1
    c.layer(0, rows=[1, 0, 0, 0], comp=[1, 0, 0, 0], factors_used=True)
    assert c.key == [(1, 3), (0, 0), (1, 1)] and c.c["misses"] == 4 and c.c["factor_copies"] == 4
    c.prefetch(1, guess, 4, 1, True)             # both guessed experts are already in slots
    assert c.c["prefetched"] == 1 and c.c["factor_copies"] == 4
    c.layer(1, rows=[0, 1, 0, 1], comp=[0, 0, 0, 1], factors_used=True)
    assert c.c == dict(expert_uses=7, hits=3, misses=4, prefetched=1, prefetch_hits=1, factor_copies=4,
                       weight_copies=5)


def test_factor_pair_follows_only_top_n_rows():
    c = SlotCache(4)
    c.layer(0, rows=[2, 3, 0, 0], comp=[0, 0, 0, 0], factors_used=True)
    assert c.c["factor_copies"] == 0             # no Top-n row: packed weights only (Section 3.2)
    c.layer(0, rows=[2, 3, 0, 0], comp=[0, 1, 0, 0], factors_used=True)
    assert c.c["hits"] == 2 and c.c["factor_copies"] == 1 and c.has_f[c.where[(0, 1)]]
    c.layer(0, rows=[2, 3, 0, 0], comp=[1, 1, 0, 0], factors_used=False)   # rank 0 or n = 0
    assert c.c["factor_copies"] == 1


def test_too_few_slots_for_one_layer():
    c = SlotCache(2)
    with pytest.raises(RuntimeError):
        c.layer(0, rows=[1, 1, 1], comp=[0, 0, 0], factors_used=False)


@pytest.mark.parametrize("n_slots,prefetch", [(4, False), (4, True), (7, True), (24, True), (24, False)])
def test_properties_on_random_sequences(n_slots, prefetch):
    rng = np.random.default_rng(n_slots * 2 + prefetch)
    L, E, k, n, T = 3, 8, 2, 1, 2
    c = SlotCache(n_slots)
    ever = set()
    for step in range(40):
        for l in range(L):
            idx = np.stack([rng.permutation(E)[:k] for _ in range(T)])
            rows = np.bincount(idx.ravel(), minlength=E)
            comp = np.bincount(idx[:, :n].ravel(), minlength=E)
            before = dict(c.where)
            c.layer(l, rows, comp, True)
            for e in np.flatnonzero(rows):
                s = c.where[(l, e)]                         # everything needed is in a slot, its own
                assert c.key[s] == (l, e)
                assert c.has_f[s] or comp[e] == 0           # with the factors if it has a Top-n row
                ever.add((l, int(e)))
            for key, s in before.items():                   # a hit keeps its slot
                if key[0] == l and rows[key[1]] > 0:
                    assert c.where[key] == s
            if prefetch and l + 1 < L:
                g = np.stack([rng.permutation(E)[:k] for _ in range(T)])
                needed_now = {c.where[(l, int(e))] for e in np.flatnonzero(rows)}
                c.prefetch(l + 1, g, E, n, True)
                for e in np.flatnonzero(rows):              # copies ahead never take a slot in use
                    assert c.where[(l, int(e))] in needed_now
                ever.update((l + 1, int(e)) for e in g.ravel() if (l + 1, int(e)) in c.where)
        assert len(c.where) == sum(k is not None for k in c.key) <= n_slots
        assert sorted(c.where.values()) == sorted(i for i, k in enumerate(c.key) if k is not None)
    cc = c.c
    assert cc["hits"] + cc["misses"] == cc["expert_uses"]
    assert cc["weight_copies"] == cc["misses"] + cc["prefetched"]
    assert cc["prefetch_hits"] <= cc["prefetched"]
    if n_slots >= L * E:                                    # room for everything: each expert is copied once
        assert cc["weight_copies"] == len(ever)
    if not prefetch:
        assert cc["prefetched"] == 0 and cc["prefetch_hits"] == 0
