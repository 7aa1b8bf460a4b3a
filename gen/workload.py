"""Synthetic verification workloads: target logits + draft tokens, seeded.

Each decode step of a workload is a batch of B sequences; a sequence has k
draft tokens and k+1 rows of vocab-wide target logits (one per draft position
plus the bonus row).  Rows are generated independently from a counter-based
generator (Philox) keyed on (seed, config, step, sequence, position), so any
row can be regenerated alone.

Recipe per draft row (probabilities from ``mix``):
  * match    : the planted top token is also the draft token;
  * synonym  : a (target, draft) divergence pair is drawn by Zipf rank from a
               fixed seeded map; target is planted on top and the draft's
               logit sits ``delta ~ U(0,3)`` below it;
  * uniform  : target planted on top, the draft is another uniform token whose
               logit stays background noise.
Background is i.i.d. N(0, sigma^2); the planted top is 8 above the noise
maximum of the row.  Values are rounded to the storage type first (bf16:
round-to-nearest-even), and ``delta`` is re-drawn while the ratio
exp(logit[draft] - logit[top]) of the *stored* values lies within 1e-4 of the
gating threshold, so that a threshold decision never depends on rounding.

The "two_peak" recipe plants a second peak ``g ~ U(0,1)`` below the first
(``g = 0`` exactly with probability ``p_exact_tie``) to stress argmax ties.

Nothing here computes a verification result; this module only makes inputs.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

MARGIN = 1e-4          # generated ratios stay this far from tau
SPIKE = 8.0            # planted top = row noise maximum + SPIKE
DELTA_MAX = 3.0        # synonym logit gap ~ U(0, DELTA_MAX)

BRANCH_MATCH, BRANCH_SYNONYM, BRANCH_UNIFORM, BRANCH_BONUS = 0, 1, 2, 3

_STREAM_PAIRS = (1 << 63)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round finite float32 values to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.asarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def pack_pair(draft, target):
    """Pack an ordered (draft, target) pair of token ids (< 2^20 each) into one integer key."""
    return (np.asarray(draft, dtype=np.uint64) << np.uint64(20)) | np.asarray(target, dtype=np.uint64)


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int
    B: int
    k: int
    V: int
    dtype: str                # "f32" or "bf16" (storage type of the logits)
    steps: int
    sigma: float
    n_pairs: int
    zipf_s: float
    mix: Tuple[float, float, float]   # P(match), P(synonym), P(uniform)
    tau: float
    lam: int
    capacity: int
    two_peak: bool = False
    p_exact_tie: float = 0.0
    seed: int = 0

    @property
    def K1(self) -> int:
        return self.k + 1

    @property
    def rows(self) -> int:
        return self.B * (self.k + 1)

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def bytes_per_step(self) -> int:
        return self.rows * self.V * self.itemsize


CONFIGS = (
    WorkloadConfig("cfg0_tiny_f32", 0, B=1, k=4, V=32000, dtype="f32", steps=1000, sigma=3.0,
                   n_pairs=512, zipf_s=1.1, mix=(0.7, 0.2, 0.1), tau=0.3, lam=2, capacity=4096),
    WorkloadConfig("cfg1_llama3_bf16", 1, B=8, k=5, V=128256, dtype="bf16", steps=2000, sigma=3.0,
                   n_pairs=2048, zipf_s=1.1, mix=(0.7, 0.2, 0.1), tau=0.3, lam=2, capacity=65536),
    WorkloadConfig("cfg2_qwen25_bf16", 2, B=32, k=7, V=151936, dtype="bf16", steps=2000, sigma=3.0,
                   n_pairs=4096, zipf_s=1.0, mix=(0.6, 0.3, 0.1), tau=0.25, lam=3, capacity=262144),
    WorkloadConfig("cfg3_large_f32_twopeak", 3, B=64, k=8, V=152064, dtype="f32", steps=1000, sigma=2.0,
                   n_pairs=16384, zipf_s=1.0, mix=(0.7, 0.2, 0.1), tau=0.4, lam=2, capacity=1048576,
                   two_peak=True, p_exact_tie=0.05),
    WorkloadConfig("cfg4_contention_bf16", 4, B=256, k=4, V=256000, dtype="bf16", steps=500, sigma=3.0,
                   n_pairs=64, zipf_s=1.5, mix=(0.5, 0.45, 0.05), tau=0.3, lam=2, capacity=1048576),
)


class Workload:
    """A seeded stream of decode steps for one configuration."""

    def __init__(self, cfg: WorkloadConfig, **overrides):
        if overrides:
            cfg = dataclasses.replace(cfg, **overrides)
        if cfg.dtype not in ("f32", "bf16"):
            raise ValueError("dtype must be 'f32' or 'bf16'")
        if cfg.V < 4 or cfg.V > (1 << 20):
            raise ValueError("V out of range")
        if abs(sum(cfg.mix) - 1.0) > 1e-9:
            raise ValueError("mix must sum to 1")
        self.cfg = cfg
        self._key0 = ((cfg.seed & 0xFFFFFFFF) << 32) | (cfg.index & 0xFFFFFFFF)
        self.pair_target, self.pair_draft = self._make_pair_map()
        w = np.arange(1, len(self.pair_target) + 1, dtype=np.float64) ** (-cfg.zipf_s)
        self._zipf_cdf = np.cumsum(w) / np.sum(w)

    # ------------------------------------------------------------------ pair map
    def _make_pair_map(self):
        cfg = self.cfg
        n = min(cfg.n_pairs, cfg.V * (cfg.V - 1))
        rng = np.random.Generator(np.random.Philox(key=[self._key0, _STREAM_PAIRS]))
        seen = set()
        tgt, drf = [], []
        while len(tgt) < n:
            t = int(rng.integers(cfg.V))
            d = int(rng.integers(cfg.V))
            if t == d or (t, d) in seen:
                continue
            seen.add((t, d))
            tgt.append(t)
            drf.append(d)
        return np.asarray(tgt, dtype=np.int64), np.asarray(drf, dtype=np.int64)

    # ------------------------------------------------------------------ storage helpers
    def _quant_scalar(self, x: float) -> float:
        """Round one value to the storage type and return it as a Python float."""
        f = np.float32(x)
        if self.cfg.dtype == "bf16":
            f = bf16_bits_to_f32(f32_to_bf16_bits(np.array([f], dtype=np.float32)))[0]
        return float(f)

    def _store(self, row: np.ndarray, idx: int, value: float) -> None:
        if self.cfg.dtype == "bf16":
            row[idx] = f32_to_bf16_bits(np.array([value], dtype=np.float32))[0]
        else:
            row[idx] = np.float32(value)

    def empty_step(self):
        cfg = self.cfg
        dt = np.float32 if cfg.dtype == "f32" else np.uint16
        return (np.empty((cfg.B, cfg.K1, cfg.V), dtype=dt), np.empty((cfg.B, cfg.k), dtype=np.int32))

    # ------------------------------------------------------------------ one row
    def _row(self, step: int, b: int, i: int, out_row: np.ndarray):
        """Fill one logits row; returns (draft token or -1 for the bonus row, branch)."""
        cfg = self.cfg
        V = cfg.V
        rowkey = (step << 34) | (b << 10) | i
        rs = np.random.Generator(np.random.Philox(key=[self._key0, 2 * rowkey + 1]))
        rn = np.random.Generator(np.random.Philox(key=[self._key0, 2 * rowkey]))

        # -- scalar draws first (independent of the noise stream)
        if i < cfg.k:
            u = rs.random()
            if u < cfg.mix[0]:
                branch = BRANCH_MATCH
                t = int(rs.integers(V))
                d = t
            elif u < cfg.mix[0] + cfg.mix[1]:
                branch = BRANCH_SYNONYM
                r = int(np.searchsorted(self._zipf_cdf, rs.random(), side="left"))
                r = min(r, len(self.pair_target) - 1)
                t = int(self.pair_target[r])
                d = int(self.pair_draft[r])
            else:
                branch = BRANCH_UNIFORM
                t = int(rs.integers(V))
                d = int(rs.integers(V - 1))
                if d >= t:
                    d += 1
        else:
            branch = BRANCH_BONUS
            t = int(rs.integers(V))
            d = -1

        # -- background noise, rounded to storage
        noise = rn.standard_normal(V, dtype=np.float32)
        noise *= np.float32(cfg.sigma)
        nmax = float(noise.max())
        if cfg.dtype == "bf16":
            out_row[:] = f32_to_bf16_bits(noise)
        else:
            out_row[:] = noise

        top = self._quant_scalar(nmax + SPIKE)
        self._store(out_row, t, top)

        if cfg.two_peak:
            # second peak g below the first; in the synonym branch it is the draft token
            if branch == BRANCH_SYNONYM:
                second = d
            else:
                while True:
                    second = int(rs.integers(V))
                    if second != t and second != d:
                        break
            while True:
                g = 0.0 if rs.random() < cfg.p_exact_tie else float(rs.random())
                zs = self._quant_scalar(top - g)
                if branch != BRANCH_SYNONYM:
                    break
                ratio = math.exp(zs - top)
                if abs(ratio - cfg.tau) >= MARGIN:
                    break
            self._store(out_row, second, zs)
        elif branch == BRANCH_SYNONYM:
            while True:
                delta = float(rs.random()) * DELTA_MAX
                zd = self._quant_scalar(top - delta)
                ratio = math.exp(zd - top)
                if abs(ratio - cfg.tau) >= MARGIN:
                    break
            self._store(out_row, d, zd)
        return d, branch

    # ------------------------------------------------------------------ one step
    def step(self, step: int, threads: int = 1, out=None, return_meta: bool = False):
        """Generate decode step ``step``: (logits[B][k+1][V], draft[B][k]).

        logits dtype is float32, or uint16 holding bf16 bit patterns.
        """
        cfg = self.cfg
        logits, draft = out if out is not None else self.empty_step()
        meta = np.empty((cfg.B, cfg.K1), dtype=np.int8)

        def work(job):
            b, i = job
            d, br = self._row(step, b, i, logits[b, i])
            if i < cfg.k:
                draft[b, i] = d
            meta[b, i] = br

        jobs = [(b, i) for b in range(cfg.B) for i in range(cfg.K1)]
        if threads > 1 and len(jobs) > 1:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(work, jobs))
        else:
            for j in jobs:
                work(j)
        if return_meta:
            return logits, draft, meta
        return logits, draft

    def logits_as_f32(self, logits: np.ndarray) -> np.ndarray:
        """Widen stored logits to float32 (exact)."""
        if self.cfg.dtype == "bf16":
            return bf16_bits_to_f32(logits)
        return logits


class SampledWorkload(Workload):
    """Decode steps for verification at a sampling temperature: target logits and draft tokens as in
    Workload, plus the draft model's logits and the uniform random numbers of the step.

    Draft row of position i: independent N(0, sigma^2) noise, the drafted token planted 8 above the noise
    maximum (the draft model is confident of what it drafted), and - when the drafted token is not the
    target's top token - the target's top token planted ``U(0,3)`` below that (the draft model also gives
    it weight, so that the residual max(0, p - q) is concentrated but not a single spike).
    u_accept [B][k] and u_draw [B][k+1] are uniform in [0, 1) (float32).  Nothing here evaluates the
    acceptance test or a distribution: keeping the random numbers away from decision boundaries is the
    test harness's job, with the oracle."""

    def empty_sampled_step(self):
        cfg = self.cfg
        dt = np.float32 if cfg.dtype == "f32" else np.uint16
        return (np.empty((cfg.B, cfg.K1, cfg.V), dtype=dt), np.empty((cfg.B, cfg.k, cfg.V), dtype=dt),
                np.empty((cfg.B, cfg.k), dtype=np.int32))

    def _draft_row(self, step: int, b: int, i: int, d: int, target_row: np.ndarray, out_row: np.ndarray) -> None:
        cfg = self.cfg
        rowkey = (step << 34) | (b << 10) | i
        key0 = self._key0 | (1 << 31)
        rn = np.random.Generator(np.random.Philox(key=[key0, 2 * rowkey]))
        rs = np.random.Generator(np.random.Philox(key=[key0, 2 * rowkey + 1]))
        noise = rn.standard_normal(cfg.V, dtype=np.float32)
        noise *= np.float32(cfg.sigma)
        nmax = float(noise.max())
        if cfg.dtype == "bf16":
            out_row[:] = f32_to_bf16_bits(noise)
        else:
            out_row[:] = noise
        top = self._quant_scalar(nmax + SPIKE)
        self._store(out_row, d, top)
        t = int(np.argmax(self.logits_as_f32(target_row)))        # the planted top of the target row
        if t != d:
            self._store(out_row, t, self._quant_scalar(top - float(rs.random()) * DELTA_MAX))

    def sampled_step(self, step: int, threads: int = 1, out=None):
        """(target logits [B][k+1][V], draft logits [B][k][V], draft [B][k], u_accept [B][k], u_draw [B][k+1])."""
        cfg = self.cfg
        zp, zq, draft = out if out is not None else self.empty_sampled_step()

        def work(job):
            b, i = job
            d, _ = self._row(step, b, i, zp[b, i])
            if i < cfg.k:
                draft[b, i] = d
                self._draft_row(step, b, i, d, zp[b, i], zq[b, i])

        jobs = [(b, i) for b in range(cfg.B) for i in range(cfg.K1)]
        if threads > 1 and len(jobs) > 1:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(work, jobs))
        else:
            for j in jobs:
                work(j)
        ru = np.random.Generator(np.random.Philox(key=[self._key0 | (1 << 31), (1 << 62) | step]))
        u_accept = ru.random((cfg.B, cfg.k), dtype=np.float32)
        u_draw = ru.random((cfg.B, cfg.K1), dtype=np.float32)
        return zp, zq, draft, u_accept, u_draw
