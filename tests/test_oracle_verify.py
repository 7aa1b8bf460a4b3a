"""Pins for the oracle's verification loop, memory and scan.

Independent checks: a literal single-sequence transcription of Algorithm 1 with
one-hot (temperature-0) distributions and full-softmax ratios; the hand-worked
fixture; reductions to strict greedy matching; brute-force recounts on tiny
vocabularies; ordering invariants that follow from the rescue predicate being
a conjunction (ablation rows of Table 3).
"""
import json
import os

import numpy as np
import pytest
import scipy.special

from oracle import csd_oracle as O


# --------------------------------------------------------------------------- helpers
def rand_stream(rng, steps, B, k, V, scale=1.0, p_match=0.5):
    """Tiny random workload: logits N(0, scale^2); drafts equal the argmax with probability p_match."""
    for _ in range(steps):
        z = (rng.standard_normal((B, k + 1, V)) * scale).astype(np.float32)
        draft = rng.integers(0, V, size=(B, k)).astype(np.int32)
        hit = rng.random((B, k)) < p_match
        am = z[:, :k, :].argmax(axis=-1)
        draft = np.where(hit, am, draft).astype(np.int32)
        yield z, draft


def strict_prefix(z, draft):
    """Longest prefix of draft tokens equal to the row argmax (plain speculative decoding, greedy)."""
    B, K1, V = z.shape
    out = np.zeros(B, dtype=np.int64)
    am = z.astype(np.float64).argmax(axis=-1)
    for b in range(B):
        n = 0
        while n < K1 - 1 and draft[b, n] == am[b, n]:
            n += 1
        out[b] = n
    return out, am


def algorithm1_literal(z, draft, table, tau, lam, rng):
    """Algorithm 1's verification loop for ONE sequence, as printed, at temperature 0.

    p_i and q_i are one-hot (greedy target / the drafted token); r ~ U(0,1]; the
    residual distribution is normalised max(0, p - q); the gate uses the ratio of
    full temperature-1 softmax probabilities; the memory is updated immediately.
    Returns (n, emitted extra token)."""
    K1, V = z.shape
    gamma = K1 - 1
    n = 0
    for i in range(gamma):
        x = int(draft[i])
        p = np.zeros(V)
        p[int(np.argmax(z[i]))] = 1.0
        q = np.zeros(V)
        q[x] = 1.0
        r = 1.0 - rng.random()                  # in (0, 1]
        alpha = min(1.0, p[x] / q[x])
        if r <= alpha:
            n += 1
        else:
            res = np.maximum(0.0, p - q)
            res /= res.sum()
            t_star = int(rng.choice(V, p=res))
            is_freq = table.get((x, t_star), 0) >= lam
            p1 = scipy.special.softmax(z[i].astype(np.float64))
            is_safe = (p1[x] / p1[t_star]) >= tau
            table[(x, t_star)] = table.get((x, t_star), 0) + 1
            if is_freq and is_safe:
                n += 1
            else:
                return n, t_star
    return n, int(np.argmax(z[gamma]))


# --------------------------------------------------------------------------- fixture from the paper's algorithm
def test_worked_example(golden_dir):
    with open(os.path.join(golden_dir, "worked_example.json")) as f:
        g = json.load(f)
    orc = O.CSDOracle()
    tol = g["tolerance"]
    for st in g["steps"]:
        z = np.asarray(st["rows"], dtype=np.float32).reshape(1, g["k"] + 1, g["V"])
        d = np.asarray(st["draft"], dtype=np.int32).reshape(1, g["k"])
        res = orc.verify_step(z, d, tau=g["tau"], lam=g["lambda"])
        e = st["expect"]
        assert list(res.argmax[0]) == e["argmax"], e["why"]
        assert res.accept_len[0] == e["accept_len"], e["why"]
        assert res.next_token[0] == e["next_token"], e["why"]
        assert res.ratio[0, 0] == pytest.approx(e["ratio0"], abs=tol)
        assert res.row_sumexp[0, 0] == pytest.approx(e["S0"], abs=tol)
        assert 1.0 / res.row_sumexp[0, 0] == pytest.approx(e["p_target0"], abs=tol)
        assert res.p_draft[0, 0] == pytest.approx(e["p_draft0"], abs=tol)
        assert orc.T[(1, 0)] == e["count_after"], e["why"]
        assert len(orc.T) == 1


# --------------------------------------------------------------------------- literal Algorithm 1, B = 1
@pytest.mark.parametrize("V,k,lam,tau", [(6, 4, 2, 0.3), (12, 6, 3, 0.25), (4, 15, 6, 0.01), (16, 5, 0, 0.6),
                                          (8, 3, 1, 0.0)])
def test_matches_literal_algorithm1_single_sequence(V, k, lam, tau):
    rng = np.random.default_rng(1000 + V * 7 + k)
    r2 = np.random.default_rng(7)
    orc = O.CSDOracle()
    lit = {}
    for z, draft in rand_stream(rng, 400, 1, k, V, scale=1.0, p_match=0.4):
        res = orc.verify_step(z, draft, tau=tau, lam=lam)
        n, tok = algorithm1_literal(z[0], draft[0], lit, tau, lam, r2)
        assert res.accept_len[0] == n
        assert res.next_token[0] == tok
        assert orc.T == lit
    assert sum(orc.T.values()) > 100          # the stream really exercised the memory


# --------------------------------------------------------------------------- reductions to strict greedy matching
def test_empty_frozen_memory_is_strict_matching():
    rng = np.random.default_rng(21)
    orc = O.CSDOracle()
    for z, draft in rand_stream(rng, 100, 5, 5, 9):
        res = orc.verify_step(z, draft, tau=0.0, lam=1, apply_updates=False)
        n, am = strict_prefix(z, draft)
        np.testing.assert_array_equal(res.accept_len, n)
        np.testing.assert_array_equal(res.next_token, am[np.arange(5), n])
        assert res.rescued == 0 and not orc.T


def test_tau_above_every_ratio_is_strict_matching():
    rng = np.random.default_rng(22)
    orc = O.CSDOracle()
    for z, draft in rand_stream(rng, 150, 4, 6, 7):
        res = orc.verify_step(z, draft, tau=1.0 + 1e-9, lam=0)        # ratios never exceed 1
        n, am = strict_prefix(z, draft)
        np.testing.assert_array_equal(res.accept_len, n)
        np.testing.assert_array_equal(res.next_token, am[np.arange(4), n])
        assert res.rescued == 0
    assert orc.T                                                       # rejections were still counted


def test_unreachable_lambda_and_no_memory_are_strict_matching():
    rng = np.random.default_rng(23)
    orc = O.CSDOracle()
    orc2 = O.CSDOracle()
    for z, draft in rand_stream(rng, 100, 3, 4, 6):
        n, _ = strict_prefix(z, draft)
        res = orc.verify_step(z, draft, tau=0.0, lam=2 ** 32 - 1)
        np.testing.assert_array_equal(res.accept_len, n)
        res2 = orc2.verify_step(z, draft, tau=0.0, lam=0, use_ocm=False)
        np.testing.assert_array_equal(res2.accept_len, n)
    assert not orc2.T


# --------------------------------------------------------------------------- bounds and monotonicity
def test_accept_len_bounded_by_strict_plus_rescues_and_flag_accounting():
    rng = np.random.default_rng(24)
    orc = O.CSDOracle()
    total_rescued = 0
    for z, draft in rand_stream(rng, 300, 6, 5, 8):
        res = orc.verify_step(z, draft, tau=0.3, lam=2)
        n, am = strict_prefix(z, draft)
        fl = res.flags
        resc = ((fl & O.FLAG_ACCEPTED) != 0) & ((fl & O.FLAG_MATCH) == 0)
        acc = (fl & O.FLAG_ACCEPTED) != 0
        assert np.all(res.accept_len >= n)
        # every kept position is a strict match or a rescue, so the accept length is bounded by the
        # number of strictly matching positions plus the number of rescues, and equals the strict
        # prefix when nothing was rescued
        n_match_total = (draft == am[:, :5]).sum(axis=1)
        assert np.all(res.accept_len <= n_match_total + resc.sum(axis=1))
        matched_kept = (((fl & O.FLAG_MATCH) != 0) & acc).sum(axis=1)
        np.testing.assert_array_equal(res.accept_len, matched_kept + resc.sum(axis=1))
        none = resc.sum(axis=1) == 0
        np.testing.assert_array_equal(res.accept_len[none], n[none])
        np.testing.assert_array_equal(res.accept_len, acc.sum(axis=1))
        # accepted positions form a prefix; rescued implies frequent and safe
        for b in range(6):
            assert acc[b, :res.accept_len[b]].all() and not acc[b, res.accept_len[b]:].any()
        assert np.all((fl[resc] & (O.FLAG_FREQ | O.FLAG_SAFE)) == (O.FLAG_FREQ | O.FLAG_SAFE))
        assert res.rescued == resc.sum()
        total_rescued += res.rescued
    assert total_rescued > 50


def test_monotone_in_tau_and_lambda_and_ablation_ordering():
    """For a fixed table: accept length falls as tau or lambda rise; and
    strict <= CSD <= min(memory-only, gate-only) position-wise (Table 3's ordering)."""
    rng = np.random.default_rng(25)
    warm = O.CSDOracle()
    stream = list(rand_stream(rng, 200, 4, 6, 8))
    for z, draft in stream[:100]:
        warm.verify_step(z, draft, tau=0.3, lam=2)
    table = dict(warm.T)

    def run(z, draft, tau, lam, use_ocm=True):
        o = O.CSDOracle()
        o.T = dict(table)
        return o.verify_step(z, draft, tau=tau, lam=lam, apply_updates=False, use_ocm=use_ocm).accept_len

    for z, draft in stream[100:]:
        strict = run(z, draft, 0.3, 2, use_ocm=False)
        prev = None
        for tau in (0.0, 0.01, 0.1, 0.3, 0.6, 1.0, 1.5):
            a = run(z, draft, tau, 2)
            if prev is not None:
                assert np.all(a <= prev)
            prev = a
        prev = None
        for lam in (0, 1, 2, 3, 6, 50, 10 ** 6):
            a = run(z, draft, 0.3, lam)
            if prev is not None:
                assert np.all(a <= prev)
            prev = a
        csd = run(z, draft, 0.3, 2)
        ocm_only = run(z, draft, 0.0, 2)         # gate always true
        scg_only = run(z, draft, 0.3, 0)         # every pair counts as frequent
        assert np.all(strict <= csd)
        assert np.all(csd <= np.minimum(ocm_only, scg_only))


# --------------------------------------------------------------------------- memory: recount, timing, snapshot
@pytest.mark.parametrize("V,B,k", [(4, 1, 3), (8, 5, 4), (16, 7, 6)])
def test_counts_equal_bruteforce_recount_of_logged_rejections(V, B, k):
    rng = np.random.default_rng(300 + V)
    orc = O.CSDOracle()
    dense = np.zeros((V, V), dtype=np.int64)
    n_logged = 0
    for z, draft in rand_stream(rng, 250, B, k, V):
        res = orc.verify_step(z, draft, tau=0.3, lam=2)
        _, am = strict_prefix(z, draft)
        for b in range(B):
            n = int(res.accept_len[b])
            # the logged pairs are exactly the mismatches among processed positions 0..min(n, k-1)
            want = [(int(draft[b, i]), int(am[b, i])) for i in range(min(n + 1, k)) if draft[b, i] != am[b, i]]
            assert res.log[b] == want
            for d, t in res.log[b]:
                dense[d, t] += 1
                n_logged += 1
    for d in range(V):
        for t in range(V):
            assert orc.T.get((d, t), 0) == dense[d, t]
    assert np.all(np.diag(dense) == 0)
    assert sum(orc.T.values()) == n_logged and n_logged > 200


def test_first_possible_rescue_is_occurrence_lambda_plus_one():
    """With an empty memory, occurrences 1..lambda of a pair are never rescued; the next one can be."""
    V, k = 5, 1
    z = np.zeros((1, 2, V), dtype=np.float32)
    z[0, 0, 3] = 2.0
    z[0, 0, 1] = 1.5            # ratio exp(-0.5) = 0.61
    z[0, 1, 4] = 1.0
    draft = np.array([[1]], dtype=np.int32)
    for lam in (0, 1, 2, 6):
        orc = O.CSDOracle()
        for occ in range(1, lam + 4):
            res = orc.verify_step(z, draft, tau=0.5, lam=lam)
            assert res.accept_len[0] == (1 if occ > lam else 0)
            assert res.next_token[0] == (4 if occ > lam else 3)
            assert orc.T[(1, 3)] == occ


def test_pair_is_ordered_draft_then_target():
    V = 6
    z = np.zeros((1, 2, V), dtype=np.float32)
    z[0, 0, 2] = 1.0
    draft = np.array([[5]], dtype=np.int32)
    orc = O.CSDOracle()
    orc.verify_step(z, draft, tau=0.0, lam=1)
    assert orc.T == {(5, 2): 1}
    # the reversed pair does not make it frequent
    orc2 = O.CSDOracle()
    orc2.ocm_update([(2, 5)], [10])
    assert orc2.verify_step(z, draft, tau=0.0, lam=1).accept_len[0] == 0
    orc3 = O.CSDOracle()
    orc3.ocm_update([(5, 2)], [1])
    assert orc3.verify_step(z, draft, tau=0.0, lam=1).accept_len[0] == 1


def test_positions_after_the_stop_are_neither_tested_nor_counted():
    V = 6
    z = np.zeros((1, 4, V), dtype=np.float32)
    z[0, :, 0] = 3.0
    draft = np.array([[1, 2, 3]], dtype=np.int32)          # three mismatches
    orc = O.CSDOracle()
    res = orc.verify_step(z, draft, tau=0.0, lam=5)
    assert res.accept_len[0] == 0 and orc.T == {(1, 0): 1}
    assert list(res.flags[0]) == [O.FLAG_COUNTED | O.FLAG_SAFE, 0, 0]
    # ratios and probabilities are still reported for every position
    assert np.all(res.ratio[0] > 0) and np.all(res.p_draft[0] > 0)


def test_batch_snapshot_lookups_precede_all_updates_of_the_step():
    """Two sequences hit the same pair in one step with count = lambda - 1: neither may be rescued."""
    V = 5
    z = np.zeros((2, 2, V), dtype=np.float32)
    z[:, 0, 3] = 1.0
    draft = np.array([[1], [1]], dtype=np.int32)
    orc = O.CSDOracle()
    orc.ocm_update([(1, 3)], [1])
    res = orc.verify_step(z, draft, tau=0.0, lam=2)
    np.testing.assert_array_equal(res.accept_len, [0, 0])
    assert orc.T[(1, 3)] == 3
    res = orc.verify_step(z, draft, tau=0.0, lam=2)
    np.testing.assert_array_equal(res.accept_len, [1, 1])


def test_snapshot_equals_sequential_within_a_sequence():
    """A sequence repeating one pair several times: deferred and immediate updates agree (B = 1)."""
    V, k = 4, 5
    z = np.zeros((1, k + 1, V), dtype=np.float32)
    z[0, :, 0] = 1.0
    draft = np.full((1, k), 2, dtype=np.int32)
    orc = O.CSDOracle()
    lit = {}
    r2 = np.random.default_rng(1)
    for _ in range(6):
        res = orc.verify_step(z, draft, tau=0.1, lam=2)
        n, tok = algorithm1_literal(z[0], draft[0], lit, 0.1, 2, r2)
        assert (res.accept_len[0], res.next_token[0]) == (n, tok)
        assert orc.T == lit


def test_capacity_drop_and_saturation_and_bad_ids():
    orc = O.CSDOracle(capacity=2)
    orc.ocm_update([(1, 2), (3, 4), (5, 6), (1, 2)], [1, 2, 3, 4])
    assert orc.T == {(1, 2): 5, (3, 4): 2} and orc.dropped == 3
    orc.ocm_update([(1, 2)], [O.COUNT_MAX])
    assert orc.T[(1, 2)] == O.COUNT_MAX
    orc.ocm_update([(9, 9)], [0])
    assert (9, 9) not in orc.T and orc.dropped == 3
    # out-of-range draft id: mismatch, zero ratio, not counted
    z = np.zeros((1, 3, 4), dtype=np.float32)
    z[0, :, 1] = 1.0
    o2 = O.CSDOracle()
    res = o2.verify_step(z, np.array([[1, 7]], dtype=np.int32), tau=0.0, lam=0)
    assert res.accept_len[0] == 1 and res.next_token[0] == 1
    assert res.ratio[0, 1] == 0.0 and res.p_draft[0, 1] == 0.0 and not o2.T and o2.bad_draft == 1


def test_memory_merge_and_export_are_plain_dictionary_sums():
    """Folding one memory into another adds counts pair by pair (saturating, same drop rule as an update);
    the export is the table itself."""
    a, b = O.CSDOracle(capacity=4), O.CSDOracle()
    a.ocm_update([(1, 2), (3, 4)], [5, 7])
    b.ocm_update([(3, 4), (5, 6), (7, 8), (9, 10)], [1, O.COUNT_MAX, 2, 3])
    a.ocm_merge(b)
    assert a.ocm_export() == {(1, 2): 5, (3, 4): 8, (5, 6): O.COUNT_MAX, (7, 8): 2}
    assert a.dropped == 3                      # the fifth distinct pair found the four slots taken
    a.ocm_merge(b)
    assert a.T[(5, 6)] == O.COUNT_MAX and a.T[(3, 4)] == 9
