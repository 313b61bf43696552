"""TEST INFRASTRUCTURE — model of a stack of MoE layers decoding from host-resident experts through
a shared device slot cache (Section 4.3, case study 1: experts and compensators are loaded on
demand; Section 3.2: the packed experts of every activated pair, the compensators of Top-n pairs
only), plus the stack's arithmetic: the layer oracle applied layer after layer.

The paper fixes what is transferred, not how slots are reused; the policy modelled here is the one
this build states in its design notes, written out step by step:

  per layer l, with rows[e] = routed rows of expert e and comp[e] = its Top-n rows:
    1. every expert with rows that sits in a slot is a hit: its slot is pinned for this layer and
       becomes the most recently used; a slot filled ahead of time and not used since counts as a
       prefetch hit;
    2. every expert with rows that sits in no slot is a miss: it takes, among the slots that are not
       pinned, an empty one, else the least recently used (lowest index on ties), which is pinned
       and becomes the most recently used; its packed weights are copied;
    3. an expert with Top-n rows whose slot lacks the factor pair gets the pair copied;
    4. with prefetching, the experts that layer l+1's gate selects on layer l's input are treated
       likewise in ascending order, as long as an unpinned slot is left: absent ones take a slot
       (pinned for this layer, marked as filled ahead, and ranked as never used until their own layer
       uses them, so that a wrong guess is the first to be evicted) and are copied, with the factor
       pair if the guess puts them in a token's first n slots.

Nothing here is shared with the HIP library; the tests compare the library's counters with this.
"""
from __future__ import annotations

import numpy as np

from . import moe_lrc_oracle as orc


class SlotCache:
    def __init__(self, n_slots: int):
        self.n = int(n_slots)
        self.key = [None] * self.n          # (layer, expert) or None
        self.has_f = [False] * self.n
        self.fresh = [False] * self.n
        self.tick = [0] * self.n
        self.pin = [0] * self.n
        self.where = {}
        self.clock = 0
        self.epoch = 0
        self.c = dict(expert_uses=0, hits=0, misses=0, prefetched=0, prefetch_hits=0, factor_copies=0,
                      weight_copies=0)

    def _victim(self):
        best = None
        for i in range(self.n):
            if self.pin[i] == self.epoch:
                continue
            rank = (self.key[i] is not None, self.tick[i])          # empty slots first, then by last use
            if best is None or rank < (self.key[best] is not None, self.tick[best]):
                best = i
        return best

    def _take(self, slot, key, fresh):
        if self.key[slot] is not None:
            del self.where[self.key[slot]]
        self.key[slot] = key
        self.has_f[slot] = False
        self.fresh[slot] = fresh
        self.pin[slot] = self.epoch
        if fresh:                       # filled ahead: counts as never used until its layer uses it
            self.tick[slot] = 0
        else:
            self.clock += 1
            self.tick[slot] = self.clock
        self.where[key] = slot
        self.c["weight_copies"] += 1

    def layer(self, l: int, rows, comp, factors_used: bool) -> None:
        """Steps 1-3 for layer l."""
        self.epoch += 1
        E = len(rows)
        for e in range(E):
            if rows[e] <= 0:
                continue
            self.c["expert_uses"] += 1
            s = self.where.get((l, e))
            if s is None:
                continue
            self.pin[s] = self.epoch
            self.clock += 1
            self.tick[s] = self.clock
            self.c["hits"] += 1
            if self.fresh[s]:
                self.c["prefetch_hits"] += 1
                self.fresh[s] = False
        for e in range(E):
            if rows[e] <= 0:
                continue
            s = self.where.get((l, e))
            if s is None:
                s = self._victim()
                if s is None:
                    raise RuntimeError("fewer slots than one layer's active experts")
                self._take(s, (l, e), fresh=False)
                self.c["misses"] += 1
            if factors_used and comp[e] > 0 and not self.has_f[s]:
                self.has_f[s] = True
                self.c["factor_copies"] += 1

    def prefetch(self, l_next: int, guess_idx: np.ndarray, n_experts: int, top_n: int, factors_used: bool) -> None:
        """Step 4: guess_idx [T][k] is layer l_next's routing of the current layer's input."""
        want = np.zeros(n_experts, dtype=np.int64)
        T, k = guess_idx.shape
        for t in range(T):
            for j in range(k):
                want[guess_idx[t, j]] |= 1 | (2 if (factors_used and j < top_n) else 0)
        for e in range(n_experts):
            if not want[e]:
                continue
            s = self.where.get((l_next, e))
            if s is None:
                s = self._victim()
                if s is None:
                    break
                self._take(s, (l_next, e), fresh=True)
                self.c["prefetched"] += 1
            self.pin[s] = self.epoch
            if (want[e] & 2) and not self.has_f[s]:
                self.has_f[s] = True
                self.c["factor_copies"] += 1


def layer_output_bits(cfg, layer: dict, x_bits: np.ndarray, residual: bool, forward) -> np.ndarray:
    """What the next layer sees: the layer's output (plus its input, with `residual`), rounded once
    to bf16.  `forward(cfg, layer, x_bits)` is the single-layer oracle (fixtures.oracle_forward)."""
    from . import compress
    out = forward(cfg, layer, x_bits)["out"]
    if residual:
        out = out + orc.bf16_to_f64(x_bits)
    return compress.round_to_bf16_bits(out)
