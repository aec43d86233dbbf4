"""Seeded synthetic workloads shaped like the paper's reasoning rollouts.

Input generation only: shapes, lengths, ratios and N(0,1) values.  Every array
is a pure function of (seed, workload id, stream id, counter), so any step of
any rollout can be regenerated without storing the stream; the same arrays are
handed to the HIP library and to the CPU oracle by the tests and the benchmark.
Nothing here computes attention, eviction or masks.

These inputs stand in for the paper's workloads (rollouts of Qwen2.5-1.5B /
Phi-4-mini on Countdown, LinSys and StarGraph with ratios c in {2,4,8,16,32},
Sec. 4), whose prompts, trajectories and weights are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20251013

_STREAM_PROMPT, _STREAM_TOKEN, _STREAM_BEACON, _STREAM_SHAPE, _STREAM_PREFILL = range(5)
_BLOCK = 128      # decode steps whose K/V are drawn together


# ---------------------------------------------------------------------------
# bf16 helpers (round-to-nearest-even on the upper 16 bits of an fp32)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array whose values are exactly representable in `dtype`."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    return x


def device_format(x: np.ndarray, dtype: str) -> np.ndarray:
    """Array in the memory format the library reads: fp32, or bf16 bit patterns (uint16)."""
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32)


# ---------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    wid: int                    # workload id, part of every rng key
    B: int
    Hq: int
    Hkv: int
    d: int
    dtype: str                  # "f32" | "bf16"
    P: np.ndarray               # [B] prompt lengths
    G: np.ndarray               # [B] generated tokens per sequence
    c: np.ndarray               # [B] compression ratio, <= 0: never compress
    peak_every: int = 0         # every peak_every-th written K row is scaled (0: off)
    peak_scale: float = 4.0
    seed: int = BASE_SEED
    extra: dict = field(default_factory=dict)
    _blocks: dict = field(default_factory=dict, repr=False)

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    def capacity(self, tail_beacon: bool = True) -> np.ndarray:
        """Rows a sequence's slab needs: prompt + one per finished window + one
        window (+ one transient slot when the beacon is appended before eviction)."""
        cc = np.maximum(self.c, 1)
        comp = self.P + self.G // cc + self.c + (1 if tail_beacon else 0)
        return np.where(self.c > 0, comp, self.P + self.G).astype(np.int32)

    def _rng(self, stream: int, *counter: int):
        return np.random.default_rng([self.seed, self.wid, stream, *counter])

    # write-order counter of a K row, used only for the "every n-th key" scaling
    def _peak_mask_tokens(self, t: int) -> np.ndarray:
        cc = np.maximum(self.c, 1)
        beacons_before = np.where(self.c > 0, (t - 1) // cc, 0)
        a = self.P + (t - 1) + beacons_before
        return a % self.peak_every == self.peak_every - 1

    def _peak_mask_beacons(self, t: int) -> np.ndarray:
        cc = np.maximum(self.c, 1)
        a = self.P + t + (t // cc - 1)
        return a % self.peak_every == self.peak_every - 1

    def prompt_kv(self, s: int):
        """(k, v) [P_s, Hkv, d] of sequence s."""
        r = self._rng(_STREAM_PROMPT, s)
        n = int(self.P[s])
        k = r.standard_normal((n, self.Hkv, self.d), dtype=np.float32)
        v = r.standard_normal((n, self.Hkv, self.d), dtype=np.float32)
        if self.peak_every:
            j = np.arange(n)
            k[j % self.peak_every == self.peak_every - 1] *= self.peak_scale
        return round_to_dtype(k, self.dtype), round_to_dtype(v, self.dtype)

    def _kv_block(self, stream: int, blk: int):
        """K/V of `_BLOCK` consecutive steps drawn at once (key: stream, block index)."""
        key = (stream, blk)
        hit = self._blocks.get(key)
        if hit is None:
            r = self._rng(stream, blk, 0)
            k = r.standard_normal((_BLOCK, self.B, self.Hkv, self.d), dtype=np.float32)
            v = r.standard_normal((_BLOCK, self.B, self.Hkv, self.d), dtype=np.float32)
            hit = (round_to_dtype(k, self.dtype), round_to_dtype(v, self.dtype))
            if len(self._blocks) >= 4:
                self._blocks.pop(next(iter(self._blocks)))
            self._blocks[key] = hit
        return hit

    def step_kv(self, t: int):
        """(k, v) [B, Hkv, d]: K/V of the token encoded at decode step t (t >= 1)."""
        kb, vb = self._kv_block(_STREAM_TOKEN, t // _BLOCK)
        k, v = kb[t % _BLOCK].copy(), vb[t % _BLOCK].copy()
        if self.peak_every:
            k[self._peak_mask_tokens(t)] *= self.peak_scale     # x4 keeps bf16 values exact
        return k, v

    def step_q(self, t: int):
        """q [B, Hq, d] of decode step t."""
        r = self._rng(_STREAM_TOKEN, t, 1, 1)
        q = r.standard_normal((self.B, self.Hq, self.d), dtype=np.float32)
        return round_to_dtype(q, self.dtype)

    def beacon_kv(self, t: int):
        """(k, v) [B, Hkv, d] of the beacons encoded after decode step t."""
        kb, vb = self._kv_block(_STREAM_BEACON, t // _BLOCK)
        k, v = kb[t % _BLOCK].copy(), vb[t % _BLOCK].copy()
        if self.peak_every:
            k[self._peak_mask_beacons(t)] *= self.peak_scale
        return k, v

    def beacon_q(self, t: int):
        """q [B, Hq, d] of the beacon token's own forward pass after step t."""
        r = self._rng(_STREAM_BEACON, t, 1, 1)
        return round_to_dtype(r.standard_normal((self.B, self.Hq, self.d), dtype=np.float32), self.dtype)


def _const(B, x):
    return np.full(B, x, dtype=np.int32)


def tiny(seed: int = BASE_SEED) -> Workload:
    """Config 1: batch 2, 4 query / 1 KV head, d 64, fp32, P 32, G 256, c 16."""
    B = 2
    return Workload("tiny", 1, B, 4, 1, 64, "f32", _const(B, 32), _const(B, 256), _const(B, 16), seed=seed)


def batch64(c: int = 16, G: int = 4096, B: int = 64, seed: int = BASE_SEED) -> Workload:
    """Config 2: batch 64, 12 query / 2 KV heads, d 128, bf16, P 256, G 4096, c 16
    (c = 0 is the uncompressed control at the same shapes)."""
    return Workload("batch64_c%d" % c if c > 0 else "batch64_cinf", 2, B, 12, 2, 128, "bf16",
                    _const(B, 256), _const(B, G), _const(B, c), seed=seed)


def ragged256(B: int = 256, g_lo: int = 1024, g_hi: int = 16384, seed: int = BASE_SEED) -> Workload:
    """Config 3: ragged batch, P ~ U[64,512], G ~ U[g_lo,g_hi], c from {2,4,8,16,32};
    `extra['T']` is the step the snapshot is taken at (uniform in [1, g_hi])."""
    r = np.random.default_rng([seed, 3, _STREAM_SHAPE])
    P = r.integers(64, 513, size=B).astype(np.int32)
    G = r.integers(g_lo, g_hi + 1, size=B).astype(np.int32)
    c = r.choice(np.array([2, 4, 8, 16, 32], dtype=np.int32), size=B).astype(np.int32)
    T = int(r.integers(1, g_hi + 1))
    return Workload("ragged256", 3, B, 12, 2, 128, "bf16", P, G, c, seed=seed, extra={"T": T})


def long_reasoning(G: int = 32768, B: int = 32, seed: int = BASE_SEED) -> Workload:
    """Config 4: batch 32, 32 query / 8 KV heads, d 128, bf16, P 512, G 32768, c 32,
    every 64th written K row scaled by 4 (peaked softmax rows)."""
    return Workload("long_reasoning", 4, B, 32, 8, 128, "bf16", _const(B, 512), _const(B, G),
                    _const(B, 32), peak_every=64, seed=seed)


@dataclass
class PrefillWorkload:
    name: str
    wid: int
    B: int
    Hq: int
    Hkv: int
    d: int
    dtype: str
    P: np.ndarray               # [B] prompt rows
    R: np.ndarray               # [B] response tokens (beacons not counted)
    c: np.ndarray               # [B]
    seed: int = BASE_SEED

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def S(self) -> np.ndarray:
        """Rows per trajectory: prompt + response tokens + one beacon per c response tokens."""
        cc = np.maximum(self.c, 1)
        return (self.P + self.R + np.where(self.c > 0, self.R // cc, 0)).astype(np.int64)

    def qkv(self, b: int):
        """(q [S,Hq,d], k [S,Hkv,d], v [S,Hkv,d]) of trajectory b."""
        r = np.random.default_rng([self.seed, self.wid, _STREAM_PREFILL, b])
        S = int(self.S[b])
        q = r.standard_normal((S, self.Hq, self.d), dtype=np.float32)
        k = r.standard_normal((S, self.Hkv, self.d), dtype=np.float32)
        v = r.standard_normal((S, self.Hkv, self.d), dtype=np.float32)
        return (round_to_dtype(q, self.dtype), round_to_dtype(k, self.dtype),
                round_to_dtype(v, self.dtype))

    def dout(self, b: int):
        """Upstream gradient dO [S, Hq, d] of trajectory b (N(0,1), as the rest)."""
        r = np.random.default_rng([self.seed, self.wid, _STREAM_PREFILL, b, 1])
        return round_to_dtype(r.standard_normal((int(self.S[b]), self.Hq, self.d), dtype=np.float32),
                              self.dtype)


def prefill_train(B: int = 16, tokens: int = 8192, P: int = 256, c: int = 16,
                  seed: int = BASE_SEED) -> PrefillWorkload:
    """Config 5: batch 16, 12 query / 2 KV heads, d 128, bf16; `tokens` regular
    tokens of which the first P are the prompt, one beacon after every c
    response tokens (8192, 256, 16 -> 496 beacons, 8688 rows)."""
    return PrefillWorkload("prefill_train", 5, B, 12, 2, 128, "bf16", _const(B, P),
                           _const(B, tokens - P), _const(B, c), seed=seed)


_STREAM_DISTILL = 7


@dataclass
class DistillWorkload:
    """Inputs of the distillation loss (Eq. 1; App. A): student logits over a vocabulary of V
    entries for T tokens, and the teacher's k largest logits per token with their ids.  Synthetic:
    student logits N(0, 2^2); the teacher is the student plus N(0, 1) noise (a trained student
    is close to its teacher), and its k largest entries are kept.  Rows are generated one token
    at a time, so any subset of tokens can be drawn without the rest."""
    name: str
    T: int
    V: int
    k: int
    dtype: str
    seed: int = BASE_SEED

    def token(self, t: int):
        """(student logits [V] fp32 exact in dtype, teacher logits [k] fp32, teacher ids [k] int32)."""
        r = np.random.default_rng([self.seed, _STREAM_DISTILL, self.V, t])
        z = 2.0 * r.standard_normal(self.V, dtype=np.float32)
        teacher = z + r.standard_normal(self.V, dtype=np.float32)
        if self.k < self.V:
            idx = np.argpartition(-teacher, self.k - 1)[: self.k]
        else:
            idx = np.arange(self.V)
        idx = idx[np.argsort(-teacher[idx], kind="stable")].astype(np.int32)
        return round_to_dtype(z, self.dtype), teacher[idx].astype(np.float32), idx

    def tokens(self, ts):
        rows = [self.token(int(t)) for t in ts]
        return (np.stack([x[0] for x in rows]), np.stack([x[1] for x in rows]),
                np.stack([x[2] for x in rows]))


def distill(T: int = 4096, V: int = 151936, k: int = 100, dtype: str = "bf16",
            seed: int = BASE_SEED) -> DistillWorkload:
    """Loss inputs at the paper's shape: vocabulary of the Qwen2.5 family (151,936 logits per
    token), top-100 teacher logits (App. A); T tokens of a micro-batch."""
    return DistillWorkload("distill", T, V, k, dtype, seed)
