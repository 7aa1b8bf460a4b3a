"""CPU oracle for CSD verification at a sampling temperature T > 0 (fp64, step by step).

TEST INFRASTRUCTURE ONLY: this module is what the GPU library is checked against.  It shares no
code with the GPU path, and the GPU path never calls it.

The procedure is the verification loop of Algorithm 1 as printed, with the random numbers it draws
passed in as inputs (so that two implementations can be compared value by value):

  * per draft position i, with p_i = softmax(target logits / T) and q_i = softmax(draft logits / T):
    the draft token x~ is accepted when r <= alpha, alpha = min(1, p_i(x~) / q_i(x~))   (Eq. 2);
  * otherwise a correction token t* is drawn from the normalised residual
    norm(max(0, p_i - q_i)) by inverting its cumulative sum at u (tokens in ascending id:
    t* = the smallest v whose cumulative residual mass exceeds u * R, R the total mass);
  * then the memory is consulted (T[(x~, t*)] >= lambda), the gate is evaluated on the
    temperature-1 probabilities of the TARGET model, p^(T=1)(x~) / p^(T=1)(t*) >= tau, which is
    exp(z(x~) - z(t*)) on the raw logits (Eq. 3), the pair is counted whatever the outcome, and
    the position is rescued (both true: x~ is kept) or the loop ends with t* as the emitted token;
  * if all draft tokens were kept, the emitted token is drawn from p_{k+1} (inverse cumulative sum at u).

Batches read the memory as it stood when the step began and add their counts afterwards, as in the
greedy oracle (csd_oracle.py), whose table class is reused here.

Conventions where the paper is silent: "r <= alpha" is inclusive as printed; a draft id outside [0, V)
ends the loop uncounted; when the residual has no mass at all (p_i == q_i in floating point) t* is the
target row's lowest-id argmax - a branch no r in [0, 1] reaches, because alpha is then 1 and the token is
accepted; it is there so that an r outside the range still gives a defined answer.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

from .csd_oracle import (CSDOracle, FLAG_ACCEPTED, FLAG_COUNTED, FLAG_FREQ, FLAG_MATCH, FLAG_SAFE)


def widen(z: np.ndarray) -> np.ndarray:
    """Stored logits (float32, or uint16 holding bfloat16 bit patterns) widened exactly to float64."""
    if z.dtype == np.uint16:
        return (z.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if z.dtype == np.float32:
        return z.astype(np.float64)
    raise TypeError("logits must be float32, or uint16 holding bfloat16 bit patterns")


def softmax_T(z64: np.ndarray, T: float) -> np.ndarray:
    """softmax(z / T) of one row, in double: exp((z - max) / T) / sum."""
    m = np.max(z64)
    e = np.exp((z64 - m) / T)
    return e / np.sum(e)


def inverse_cdf(w: np.ndarray, u: float) -> Tuple[int, float, float]:
    """Draw from the distribution proportional to the non-negative weights w by inverting the running
    sum at u in [0, 1): the smallest v with cumsum(w)[v] > u * sum(w).

    Returns (v, total mass, margin) where margin is the distance, in units of probability mass, from
    u * total to the nearer end of v's interval - how far u is from changing the outcome."""
    c = np.cumsum(w)
    R = float(c[-1])
    if not (R > 0.0):
        return -1, R, 0.0
    target = u * R
    v = int(np.searchsorted(c, target, side="right"))
    v = min(v, len(w) - 1)
    lo = float(c[v - 1]) if v > 0 else 0.0
    return v, R, float(min(target - lo, float(c[v]) - target))


@dataclass
class SampledStepResult:
    accept_len: np.ndarray      # [B]
    next_token: np.ndarray      # [B]  t* of the stopping position, or the bonus draw
    alpha: np.ndarray           # [B][k]  min(1, p(x~)/q(x~)); 0 for an invalid draft id
    p_draft: np.ndarray         # [B][k]  p_i(x~) at temperature T
    q_draft: np.ndarray         # [B][k]  q_i(x~) at temperature T
    rejected: np.ndarray        # [B][k]  bool: the acceptance test failed (r > alpha), whether or not the loop got there
    tstar: np.ndarray           # [B][k]  residual draw where `rejected`, else -1
    res_mass: np.ndarray        # [B][k]  total residual mass R where `rejected`, else 0
    ratio: np.ndarray           # [B][k]  exp(z(x~) - z(t*)) on the raw target logits where `rejected`, else 0
    bonus_token: np.ndarray     # [B]     draw from p_{k+1} (defined for every sequence)
    flags: np.ndarray           # [B][k]  FLAG_* bits of processed positions
    accept_margin: np.ndarray   # [B][k]  |r - alpha|
    draw_margin: np.ndarray     # [B][k+1] inverse-cdf margin of the residual draws (and of the bonus draw at [k])
    log: List[List[Tuple[int, int]]] = field(default_factory=list)
    rescued: int = 0


def verify_step_sampled(orc: CSDOracle, zp: np.ndarray, zq: np.ndarray, draft: np.ndarray, temperature: float,
                        u_accept: np.ndarray, u_draw: np.ndarray, tau: float, lam: int, apply_updates: bool = True,
                        use_ocm: bool = True) -> SampledStepResult:
    """One decode step for a batch at temperature T.  zp: [B][k+1][V] target logits, zq: [B][k][V] draft
    logits (stored type), draft: [B][k] ids, u_accept: [B][k] the r of the acceptance test, u_draw: [B][k+1]
    the uniforms of the residual draws (positions 0..k-1) and of the bonus draw (index k)."""
    B, K1, V = zp.shape
    k = K1 - 1
    assert zq.shape == (B, k, V) and draft.shape == (B, k) and u_accept.shape == (B, k) and u_draw.shape == (B, K1)
    T = float(temperature)
    assert T > 0.0
    res = SampledStepResult(
        accept_len=np.zeros(B, np.int64), next_token=np.zeros(B, np.int64), alpha=np.zeros((B, k)),
        p_draft=np.zeros((B, k)), q_draft=np.zeros((B, k)), rejected=np.zeros((B, k), bool),
        tstar=np.full((B, k), -1, np.int64), res_mass=np.zeros((B, k)), ratio=np.zeros((B, k)),
        bonus_token=np.zeros(B, np.int64), flags=np.zeros((B, k), np.uint8), accept_margin=np.zeros((B, k)),
        draw_margin=np.zeros((B, K1)))
    snapshot = orc.T

    for b in range(B):
        # quantities that are functions of the inputs alone, for every position
        for i in range(k):
            d = int(draft[b, i])
            if not (0 <= d < V):
                res.rejected[b, i] = True
                continue
            z = widen(zp[b, i])
            p = softmax_T(z, T)
            q = softmax_T(widen(zq[b, i]), T)
            res.p_draft[b, i], res.q_draft[b, i] = p[d], q[d]
            res.alpha[b, i] = 1.0 if q[d] <= 0.0 else min(1.0, p[d] / q[d])
            r = float(u_accept[b, i])
            res.accept_margin[b, i] = abs(r - res.alpha[b, i])
            if r <= res.alpha[b, i]:
                continue
            res.rejected[b, i] = True
            w = np.maximum(0.0, p - q)
            t, R, margin = inverse_cdf(w, float(u_draw[b, i]))
            if t < 0:
                t = int(np.argmax(z))                 # no residual mass: the target's own choice
            res.tstar[b, i], res.res_mass[b, i], res.draw_margin[b, i] = t, R, margin
            res.ratio[b, i] = np.exp(z[d] - z[t])
        pk = softmax_T(widen(zp[b, k]), T)
        t, _, margin = inverse_cdf(pk, float(u_draw[b, k]))
        res.bonus_token[b], res.draw_margin[b, k] = t, margin

        # the verification loop
        n = 0
        pending: List[Tuple[int, int]] = []
        stopped = False
        for i in range(k):
            d = int(draft[b, i])
            if not res.rejected[b, i]:
                res.flags[b, i] = FLAG_MATCH | FLAG_ACCEPTED      # kept by the acceptance test
                n += 1
                continue
            if not (0 <= d < V):
                orc.bad_draft += 1
                res.next_token[b] = int(np.argmax(widen(zp[b, i])))
                stopped = True
                break
            ts = int(res.tstar[b, i])
            is_freq = use_ocm and (snapshot.get((d, ts), 0) >= lam)
            is_safe = res.ratio[b, i] >= tau
            pending.append((d, ts))
            f = FLAG_COUNTED | (FLAG_FREQ if is_freq else 0) | (FLAG_SAFE if is_safe else 0)
            if is_freq and is_safe:
                res.flags[b, i] = f | FLAG_ACCEPTED
                n += 1
                res.rescued += 1
            else:
                res.flags[b, i] = f
                res.next_token[b] = ts
                stopped = True
                break
        res.accept_len[b] = n
        if not stopped:
            res.next_token[b] = res.bonus_token[b]
        res.log.append(pending)

    if apply_updates and use_ocm:
        for pending in res.log:
            orc.ocm_update(pending)
    return res
