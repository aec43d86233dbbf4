"""Which KV-cache entries are resident at each generation step (oracle, test only).

Follows Alg. 1 and Sec. 3.1 of the paper.  Entry ids are tuples:
``('q', j)`` prompt token j, ``('x', i)`` generated token x_i, ``('b', m)`` the
m-th beacon (m = 1, 2, ...).

Reading of Alg. 1 used here (Sec. 3.1, last sentences): x_i is *sampled* at
iteration i but only *encoded* (its K/V written) by the forward pass that
samples x_{i+1}; after a beacon the next input is the last sampled token, so
generation continues as normal.  Hence when the test ``i > 0 and i mod c == 0``
fires, the cache tail holds x_{i-c} .. x_{i-1}: exactly c window entries.

Step numbering used by the whole repo: decode step t (t = 1, 2, ...) is the
forward pass that encodes x_{t-1} and samples x_t.  Compression fires after
step t when t mod c == 0 (this is iteration i = t of Alg. 1).
"""
from __future__ import annotations


def alg1_literal(P: int, c: int, G: int):
    """Alg. 1 written as one flat Python list with the slice of its eviction line.

    Yields, for t = 1..G, ``(t, at_attention, after_step)``: the list of entry
    ids the decode attention of step t sees, and the list left once the step
    (including a possible beacon + eviction) has finished.  ``c <= 0`` means the
    uncompressed model: the test never fires.
    """
    kv = [("q", j) for j in range(P)]          # Initialize: encode the prompt
    i = 0
    while i < G:
        i += 1                                  # iteration i of Alg. 1 (i >= 1 here;
        kv.append(("x", i - 1))                 # i = 0 samples from the prefill logits)
        at_attention = list(kv)                 # forward pass that samples x_i
        if c > 0 and i > 0 and i % c == 0:
            kv.append(("b", i // c))            # encode the beacon: its entry joins the cache
            kv = kv[: -c - 1] + kv[-1:]         # drop the c entries before it, keep the beacon
        yield i, at_attention, list(kv)


def structured(P: int, c: int, G: int):
    """Same process kept as three lists [prompt | beacons | window] (Fig. 1)."""
    prompt = [("q", j) for j in range(P)]
    beacons: list = []
    window: list = []
    for t in range(1, G + 1):
        window.append(("x", t - 1))
        at_attention = prompt + beacons + window
        if c > 0 and len(window) == c:
            beacons.append(("b", len(beacons) + 1))
            window = []
        yield t, at_attention, prompt + beacons + window


def len_at_attention(P: int, c: int, t: int) -> int:
    """Closed form: entries seen by the attention of step t (t >= 1)."""
    if c <= 0:
        return P + t
    return P + (t - 1) // c + (t - 1) % c + 1


def len_after_step(P: int, c: int, t: int) -> int:
    """Closed form: entries left after step t: P + floor(t/c) + (t mod c)."""
    if c <= 0:
        return P + t
    return P + t // c + t % c


def tables_after_step(c: int, t: int):
    """(number of beacons, window length) after step t."""
    if c <= 0:
        return 0, t
    return t // c, t % c


def tables_at_attention(c: int, t: int):
    """(number of beacons, window length) when the attention of step t runs."""
    if c <= 0:
        return 0, t
    return (t - 1) // c, (t - 1) % c + 1


def first_step_reaching(budget: int, c: int) -> int:
    """First step whose attention sees `budget` generation entries (beacons + window).

    The paper's evaluation interrupts generation when the generation cache
    reaches 1,000 entries (Sec. 4, Evaluation); with ratio c this allows
    roughly c times more tokens (Sec. 5; Table 3 caption).
    """
    t = 1
    while len_at_attention(0, c, t) < budget:
        t += 1
    return t
