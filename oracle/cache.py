"""K/V-carrying cache simulators (oracle, test only).

Two independent forms of the same process (Alg. 1, Sec. 3.1):

* ``FlatCache``     - one Python list per sequence: the eviction step of Alg. 1 as
                      "remove the window's entries, put the beacon in their place".
                      No bookkeeping besides the list.
* ``BatchCache``    - the structured form [prompt | beacons | window] (Fig. 1)
                      for a batch with per-sequence ratio c, with the state and
                      capacity rules a fixed-capacity implementation must
                      enforce.  Its counters (nb, w) and sticky error bits are
                      what the library's device tables are compared with.

Rows are whatever array objects the caller passes ([Hkv, d] each for K and V);
they are stored, never modified, so a bit-exact comparison is meaningful.
"""
from __future__ import annotations

import numpy as np

ERR_STATE = 1       # operation not allowed in the sequence's current state
ERR_CAPACITY = 2    # the sequence's slab is full


class FlatCache:
    """One sequence; Alg. 1 with a flat list.  c <= 0: never compress."""

    def __init__(self, prompt_k, prompt_v, c: int):
        self.c = int(c)
        self.kv = [(prompt_k[j], prompt_v[j]) for j in range(len(prompt_k))]

    def append(self, k, v):
        self.kv.append((k, v))

    def beacon_and_evict(self, bk, bv):
        # what is left of the window after the step is its beacon: the c newest entries go,
        # the beacon's pair takes their place behind the prompt and the earlier beacons
        del self.kv[len(self.kv) - self.c:]
        self.kv.append((bk, bv))

    def resident(self):
        K = np.stack([r[0] for r in self.kv])
        V = np.stack([r[1] for r in self.kv])
        return K, V


class BatchCache:
    """Structured per-sequence caches with fixed capacities.

    P[s], c[s], cap[s] are fixed; nb[s] (beacons so far) and w[s] (entries after
    the beacons: window tokens, plus one when a beacon sits at the tail waiting
    for the eviction) change.  L[s] = P[s] + nb[s] + w[s].

    Rules (mirrored by the library header):
      append token   : needs w < c (when c > 0) else ERR_STATE; needs L < cap
                       else ERR_CAPACITY; on error the sequence is untouched.
      append beacon  : acts only on sequences with c > 0 and w == c; needs
                       L < cap else ERR_CAPACITY; afterwards w == c + 1.
      compress, beacon supplied : acts on sequences with c > 0 and w == c
                       (or 1 <= w <= c when require_full is False); w == c + 1
                       is ERR_STATE.  The beacon replaces the whole window.
      compress, beacon at tail  : acts on sequences with c > 0 and w == c + 1:
                       the tail entry is kept, the c before it are dropped.
    Inactive sequences are never touched.
    """

    def __init__(self, prompts_k, prompts_v, c, cap):
        self.B = len(prompts_k)
        self.P = [len(pk) for pk in prompts_k]
        self.c = [int(x) for x in c]
        self.cap = [int(x) for x in cap]
        self.prompt = [[(pk[j], pv[j]) for j in range(len(pk))]
                       for pk, pv in zip(prompts_k, prompts_v)]
        self.beacons = [[] for _ in range(self.B)]
        self.window = [[] for _ in range(self.B)]
        self.err = 0
        for s in range(self.B):
            assert self.P[s] <= self.cap[s]

    # -- tables -------------------------------------------------------------
    @property
    def nb(self):
        return [len(b) for b in self.beacons]

    @property
    def w(self):
        return [len(x) for x in self.window]

    def L(self, s):
        return self.P[s] + len(self.beacons[s]) + len(self.window[s])

    # -- operations ---------------------------------------------------------
    def _active(self, active, s):
        return active is None or bool(active[s])

    def append(self, k, v, active=None, beacon=False):
        """k, v: [B, Hkv, d].  beacon=True is the 'encode b' step of Alg. 1."""
        for s in range(self.B):
            if not self._active(active, s):
                continue
            c, w = self.c[s], len(self.window[s])
            if beacon:
                if c <= 0 or w != c:
                    continue
            elif c > 0 and w >= c:
                self.err |= ERR_STATE
                continue
            if self.L(s) >= self.cap[s]:
                self.err |= ERR_CAPACITY
                continue
            self.window[s].append((k[s], v[s]))

    def compress_evict(self, bk=None, bv=None, active=None, require_full=True):
        """Beacon append + window eviction.  bk/bv [B, Hkv, d] or None (tail form)."""
        for s in range(self.B):
            if not self._active(active, s):
                continue
            c, w = self.c[s], len(self.window[s])
            if c <= 0:
                continue
            if bk is None:
                if w != c + 1:
                    continue
                self.beacons[s].append(self.window[s][-1])
                self.window[s] = []
            else:
                if w == c + 1:
                    self.err |= ERR_STATE
                    continue
                if w == c or (not require_full and 1 <= w <= c):
                    self.beacons[s].append((bk[s], bv[s]))
                    self.window[s] = []

    def set_ratio(self, new_c, active=None):
        """Mid-generation ratio change (the paper fixes c per generation; dynamic ratios are its
        stated future work, Sec. 6): allowed when the current window fits the new ratio."""
        for s in range(self.B):
            if not self._active(active, s):
                continue
            nc, w = int(new_c[s]), len(self.window[s])
            if nc > 0 and w >= nc and w != 0:
                self.err |= ERR_STATE
                continue
            self.c[s] = nc

    def apply_budget(self, budget, live):
        """Evaluation rule (Sec. 4, Evaluation): generation is interrupted when the cache cap is
        reached.  Called at attention time; budget caps the generation entries nb + w."""
        for s in range(self.B):
            if live[s] and len(self.beacons[s]) + len(self.window[s]) >= budget[s]:
                live[s] = 0

    def admit(self, admit, prompts_k, prompts_v, new_c=None, live=None):
        """A new sequence takes over a slot whose generation is over (the evaluation rule of
        Sec. 4 ends generations at different times; the slot's capacity stays).  Equivalent to
        Alg. 1's initialisation for that slot alone: prompt entries, no beacons, empty window.
        A prompt longer than the slot is a capacity error and leaves the slot as it was."""
        for s in range(self.B):
            if not admit[s]:
                continue
            if len(prompts_k[s]) > self.cap[s]:
                self.err |= ERR_CAPACITY
                continue
            self.P[s] = len(prompts_k[s])
            self.prompt[s] = [(prompts_k[s][j], prompts_v[s][j]) for j in range(self.P[s])]
            self.beacons[s] = []
            self.window[s] = []
            if new_c is not None:
                self.c[s] = int(new_c[s])
            if live is not None:
                live[s] = 1

    # -- views --------------------------------------------------------------
    def resident(self, s):
        """(K, V) [L, Hkv, d] of sequence s in cache order."""
        rows = self.prompt[s] + self.beacons[s] + self.window[s]
        K = np.stack([r[0] for r in rows])
        V = np.stack([r[1] for r in rows])
        return K, V
