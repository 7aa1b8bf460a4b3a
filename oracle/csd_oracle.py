"""CPU oracle for Calibrated Speculative Decoding verification (fp64, step by step).

TEST INFRASTRUCTURE ONLY: this module is what the GPU library is checked
against.  It shares no code with the GPU path, and the GPU path never calls it.

The verification step is a heuristic procedure, so the oracle is the procedure
itself, taken in the order of Algorithm 1 (verification loop) with greedy
decoding, which is how the method is evaluated:

  * at temperature 0 both distributions are one-hot, so the acceptance test of
    Eq. 2 accepts exactly when the draft token equals the target's argmax, and
    the token drawn from the residual distribution is that argmax, ``t*``;
  * on a mismatch the Online Correction Memory is consulted first
    (``T[(draft, t*)] >= lambda``), then the Semantic Consistency Gate
    (``p(draft) / p(t*) >= tau`` on the raw, temperature-1 logits, Eq. 3),
    then the pair's count is incremented whatever the outcome, and only then
    is the position rescued (both tests true) or the loop left;
  * the emitted extra token is ``t*`` of the stopping position, or the argmax
    of the bonus row when every draft token was kept.

Batches: every lookup of a step reads the table as it stood when the step
began; the step's increments are applied afterwards (sums commute).  For one
sequence this equals the sequential order of Algorithm 1, because a later
position is reached only if every earlier mismatch already had count >= lambda.

Row statistics (max, first argmax, sum of exponentials) come from the plain C
loops in ``csd_oracle_rows.c``; the table is a Python dict.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Iterable, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csd_oracle_rows.c")
_LIB = os.path.join(_HERE, "libcsd_oracle.so")

DTYPE_F32 = 0
DTYPE_BF16 = 1
COUNT_MAX = (1 << 24) - 1      # counts saturate here (the table stores 24-bit counts)

FLAG_MATCH = 1                 # draft token == t*
FLAG_FREQ = 2                  # T[(draft, t*)] >= lambda (evaluated on a mismatch only)
FLAG_SAFE = 4                  # ratio >= tau           (evaluated on a mismatch only)
FLAG_ACCEPTED = 8              # position kept (match or rescued)
FLAG_COUNTED = 16              # the pair was handed to UpdateMemory


def build_oracle_lib(force: bool = False) -> str:
    """Compile the C part with gcc (-O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle_lib())
        lib.csd_oracle_logit.restype = ctypes.c_double
        lib.csd_oracle_logit.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64]
        lib.csd_oracle_rows.restype = None
        lib.csd_oracle_rows.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p]
        _lib = lib
    return _lib


def _storage_dtype(z: np.ndarray) -> int:
    if z.dtype == np.float32:
        return DTYPE_F32
    if z.dtype == np.uint16:
        return DTYPE_BF16
    raise TypeError("logits must be float32, or uint16 holding bfloat16 bit patterns")


def row_stats(z: np.ndarray, threads: int = 1):
    """(m, t*, S) for every row of a C-contiguous [..., V] logits array, in fp64."""
    lib = _load()
    dt = _storage_dtype(z)
    if not z.flags.c_contiguous:
        raise ValueError("logits must be C-contiguous")
    V = z.shape[-1]
    rows = int(np.prod(z.shape[:-1], dtype=np.int64))
    m = np.empty(rows, dtype=np.float64)
    t = np.empty(rows, dtype=np.int64)
    S = np.empty(rows, dtype=np.float64)

    def run(r0, r1):
        lib.csd_oracle_rows(z.ctypes.data, dt, V, V, r0, r1, m.ctypes.data, t.ctypes.data, S.ctypes.data)

    threads = max(1, min(threads, rows))
    if threads == 1:
        run(0, rows)
    else:
        cuts = [rows * j // threads for j in range(threads + 1)]
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda j: run(cuts[j], cuts[j + 1]), range(threads)))
    shp = z.shape[:-1]
    return m.reshape(shp), t.reshape(shp), S.reshape(shp)


def logit(z_row: np.ndarray, v: int) -> float:
    """One stored logit widened to double."""
    return float(_load().csd_oracle_logit(z_row.ctypes.data, _storage_dtype(z_row), int(v)))


@dataclass
class StepResult:
    accept_len: np.ndarray      # [B]    n in [0, k]
    next_token: np.ndarray      # [B]    t* of the stopping row, or argmax of the bonus row
    argmax: np.ndarray          # [B][k+1]
    row_max: np.ndarray         # [B][k+1] fp64
    row_sumexp: np.ndarray      # [B][k+1] fp64
    ratio: np.ndarray           # [B][k] p(draft)/p(t*)
    p_draft: np.ndarray         # [B][k]
    flags: np.ndarray           # [B][k] uint8, FLAG_* bits; 0 for positions after the stop
    log: List[List[Tuple[int, int]]] = field(default_factory=list)   # per sequence: counted (draft, t*) pairs
    rescued: int = 0


class CSDOracle:
    """Verification state: the correction memory T : (draft, target) -> count."""

    def __init__(self, capacity: Optional[int] = None):
        self.T: Dict[Tuple[int, int], int] = {}
        self.capacity = capacity
        self.dropped = 0        # increments lost because the table was full
        self.bad_draft = 0      # draft ids outside [0, V)

    def reset(self) -> None:
        self.T.clear()

    # UpdateMemory (Algorithm 1) / prior calibration load (Online Correction Memory, phase 1)
    def ocm_update(self, pairs: Iterable[Tuple[int, int]], weights: Optional[Iterable[int]] = None) -> None:
        pairs = list(pairs)
        ws = [1] * len(pairs) if weights is None else [int(w) for w in weights]
        for (d, t), w in zip(pairs, ws):
            if w == 0:
                continue
            key = (int(d), int(t))
            if key not in self.T:
                if self.capacity is not None and len(self.T) >= self.capacity:
                    self.dropped += w
                    continue
                self.T[key] = 0
            self.T[key] = min(self.T[key] + w, COUNT_MAX)

    # Memory life cycle around runs (the calibrated prior is an offline product that later runs start from):
    # folding another memory in, and the memory as a plain list of (pair, count).
    def ocm_merge(self, other: "CSDOracle") -> None:
        for key, cnt in other.T.items():
            self.ocm_update([key], [cnt])

    def ocm_export(self) -> Dict[Tuple[int, int], int]:
        return dict(self.T)

    def verify_step(self, z: np.ndarray, draft: np.ndarray, tau: float, lam: int, apply_updates: bool = True,
                    use_ocm: bool = True, threads: int = 1) -> StepResult:
        """One decode step for a batch.  z: [B][k+1][V] stored logits, draft: [B][k] token ids."""
        B, K1, V = z.shape
        k = K1 - 1
        assert draft.shape == (B, k)
        m, t, S = row_stats(z, threads=threads)

        accept_len = np.zeros(B, dtype=np.int64)
        next_token = np.zeros(B, dtype=np.int64)
        ratio = np.zeros((B, k), dtype=np.float64)
        p_draft = np.zeros((B, k), dtype=np.float64)
        flags = np.zeros((B, k), dtype=np.uint8)
        log: List[List[Tuple[int, int]]] = []
        rescued = 0
        snapshot = self.T            # not modified until every sequence has been scanned

        for b in range(B):
            # quantities defined for every draft position
            for i in range(k):
                d = int(draft[b, i])
                if 0 <= d < V:
                    ratio[b, i] = math.exp(logit(z[b, i], d) - m[b, i])
                    p_draft[b, i] = ratio[b, i] / S[b, i]
            # the verification loop
            n = 0
            pending: List[Tuple[int, int]] = []
            for i in range(k):
                d = int(draft[b, i])
                ts = int(t[b, i])
                if d == ts:                                   # accepted by the greedy acceptance test
                    flags[b, i] = FLAG_MATCH | FLAG_ACCEPTED
                    n += 1
                    continue
                if not (0 <= d < V):                          # invalid id: a mismatch that is never rescued or counted
                    self.bad_draft += 1
                    break
                is_freq = use_ocm and (snapshot.get((d, ts), 0) >= lam)
                is_safe = ratio[b, i] >= tau
                pending.append((d, ts))                       # UpdateMemory: every processed divergence
                f = FLAG_COUNTED | (FLAG_FREQ if is_freq else 0) | (FLAG_SAFE if is_safe else 0)
                if is_freq and is_safe:
                    flags[b, i] = f | FLAG_ACCEPTED           # rescued: the draft token is kept
                    n += 1
                    rescued += 1
                else:
                    flags[b, i] = f
                    break
            accept_len[b] = n
            next_token[b] = t[b, n]
            log.append(pending)

        if apply_updates and use_ocm:
            for pending in log:
                self.ocm_update(pending)

        return StepResult(accept_len, next_token, t, m, S, ratio, p_draft, flags, log, rescued)
