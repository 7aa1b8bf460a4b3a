"""Pins for the sampling-temperature oracle (oracle/csd_oracle_sampled.py).

What fixes it from outside: the hand-worked fixture; the theorem that speculative sampling leaves the
target distribution unchanged (Section 2.1: accepted-or-resampled tokens follow p exactly), checked by
exact integration over the random numbers on tiny vocabularies; the greedy oracle (already pinned) as the
limit of small temperature; a brute-force inverse-cumulative-sum; brute-force recounts of the memory.
"""
import json
import os

import numpy as np
import pytest

from oracle import csd_oracle as O
from oracle import csd_oracle_sampled as OS

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _logits(prob):
    return np.log(np.asarray(prob, dtype=np.float64)).astype(np.float32)


def test_worked_example():
    fx = json.load(open(os.path.join(GOLDEN, "sampled_example.json")))
    T = fx["temperature"]
    for case in fx["cases"]:
        zp = np.stack([_logits(case["p"]), _logits(case["p_bonus"])])[None]
        zq = _logits(case["q"])[None, None]
        d = case["draft"]
        for run in case["runs"]:
            orc = O.CSDOracle()
            tgt = run.get("pair_target", 0)
            if run["count_before"]:
                orc.ocm_update([(d, tgt)], [run["count_before"]])
            r = OS.verify_step_sampled(orc, zp, zq, np.array([[d]], np.int32), T, np.array([[run["r"]]]),
                                       np.array([[run["u"], run["u_bonus"]]]), tau=run["tau"], lam=run["lambda"])
            assert r.alpha[0, 0] == pytest.approx(case["alpha"], abs=2e-6), run["why"]
            assert int(r.accept_len[0]) == run["accept_len"], run["why"]
            assert int(r.next_token[0]) == run["next_token"], run["why"]
            assert orc.T.get((d, tgt), 0) == run["count_after"], run["why"]
            if r.rejected[0, 0]:
                assert r.res_mass[0, 0] == pytest.approx(case["res_mass"], abs=2e-6)
                assert r.ratio[0, 0] == pytest.approx(run.get("ratio", case.get("ratio")), abs=2e-6)


def _brute_inverse_cdf(w, u):
    total = 0.0
    for x in w:
        total += x
    acc = 0.0
    for v, x in enumerate(w):
        acc += x
        if acc > u * total:
            return v
    return len(w) - 1


def test_inverse_cdf_against_a_plain_loop_and_its_edges():
    rng = np.random.default_rng(1)
    for _ in range(200):
        V = int(rng.integers(1, 40))
        w = rng.random(V) * (rng.random(V) < 0.6)
        if w.sum() == 0:
            w[int(rng.integers(V))] = 1.0
        u = float(rng.random())
        v, R, margin = OS.inverse_cdf(w, u)
        assert v == _brute_inverse_cdf(w, u) and w[v] > 0 and margin >= 0
        assert R == pytest.approx(w.sum())
    w = np.array([0.0, 0.0, 0.2, 0.0, 0.3, 0.5, 0.0])
    assert OS.inverse_cdf(w, 0.0)[0] == 2                        # first token that has mass
    assert OS.inverse_cdf(w, np.nextafter(1.0, 0.0))[0] == 5     # last token that has mass
    assert OS.inverse_cdf(w, 0.2)[0] == 4                        # exactly on a boundary: strictly-greater rule
    assert [OS.inverse_cdf(w, u)[0] for u in np.linspace(0, 0.999, 50)] == sorted(
        OS.inverse_cdf(w, u)[0] for u in np.linspace(0, 0.999, 50))
    assert OS.inverse_cdf(np.zeros(4), 0.3)[0] == -1


@pytest.mark.parametrize("V,T,seed", [(5, 1.0, 0), (7, 0.6, 1), (4, 1.7, 2)])
def test_emitted_token_follows_the_target_distribution(V, T, seed):
    """No memory (plain speculative sampling): integrating the first emitted token over the draft token
    x ~ q, the acceptance number r and the residual draw u gives p exactly.  r is integrated in closed form
    (the outcome only depends on whether r <= alpha), u on a fine grid of interval midpoints."""
    rng = np.random.default_rng(seed)
    zp = (rng.standard_normal((1, 2, V)) * 2).astype(np.float32)
    zq = (rng.standard_normal((1, 1, V)) * 2).astype(np.float32)
    p = OS.softmax_T(zp[0, 0].astype(np.float64), T)
    q = OS.softmax_T(zq[0, 0].astype(np.float64), T)
    N = 4000
    us = (np.arange(N) + 0.5) / N
    out = np.zeros(V)
    for x in range(V):
        d = np.array([[x]], np.int32)
        acc = OS.verify_step_sampled(O.CSDOracle(), zp, zq, d, T, np.array([[0.0]]), np.array([[0.5, 0.5]]), 0.0, 2 ** 40,
                                     use_ocm=False)
        assert int(acc.accept_len[0]) == 1                       # r = 0 is always accepted
        alpha = float(acc.alpha[0, 0])
        assert alpha == pytest.approx(min(1.0, p[x] / q[x]), rel=1e-12)
        out[x] += q[x] * alpha
        if alpha < 1.0:
            hist = np.zeros(V)
            for u in us:
                rej = OS.verify_step_sampled(O.CSDOracle(), zp, zq, d, T, np.array([[1.0]]), np.array([[u, 0.5]]), 0.0,
                                             2 ** 40, use_ocm=False)
                assert int(rej.accept_len[0]) == 0
                hist[int(rej.next_token[0])] += 1.0 / N
            out += q[x] * (1.0 - alpha) * hist
    np.testing.assert_allclose(out, p, atol=2.0 / N)


def test_bonus_token_follows_p_of_the_last_row():
    rng = np.random.default_rng(5)
    V, T = 6, 0.8
    zp = (rng.standard_normal((1, 2, V)) * 2).astype(np.float32)
    zq = zp[:, :1].copy()                                        # q == p: alpha = 1, always accepted
    pk = OS.softmax_T(zp[0, 1].astype(np.float64), T)
    N = 5000
    hist = np.zeros(V)
    for u in (np.arange(N) + 0.5) / N:
        r = OS.verify_step_sampled(O.CSDOracle(), zp, zq, np.array([[2]], np.int32), T, np.array([[1.0]]),
                                   np.array([[0.3, u]]), 0.3, 2)
        assert int(r.accept_len[0]) == 1 and r.alpha[0, 0] == 1.0
        hist[int(r.next_token[0])] += 1.0 / N
    np.testing.assert_allclose(hist, pk, atol=2.0 / N)


def test_small_temperature_reduces_to_the_greedy_oracle():
    """As T -> 0 both distributions become one-hot: with the draft model certain of its token the loop is
    the greedy one (match = accepted, t* = target argmax), whatever the random numbers."""
    rng = np.random.default_rng(7)
    B, k, V, T = 3, 4, 12, 0.02
    og, osmp = O.CSDOracle(), O.CSDOracle()
    for step in range(60):
        zp = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
        top = rng.integers(0, V, (B, k + 1))
        np.put_along_axis(zp, top[..., None], zp.max(-1, keepdims=True) + 3.0, axis=-1)      # a clear top
        am = zp[:, :k].argmax(-1)
        draft = np.where(rng.random((B, k)) < 0.5, am, rng.integers(0, V, (B, k))).astype(np.int32)
        zq = np.zeros((B, k, V), np.float32)
        np.put_along_axis(zq, draft[..., None].astype(np.int64), 5.0, axis=-1)
        g = og.verify_step(zp, draft, tau=np.float32(0.05), lam=2)
        s = OS.verify_step_sampled(osmp, zp, zq, draft, T, rng.random((B, k)) * 0.98 + 0.01,
                                   rng.random((B, k + 1)) * 0.98 + 0.01, tau=np.float32(0.05), lam=2)
        np.testing.assert_array_equal(s.accept_len, g.accept_len)
        np.testing.assert_array_equal(s.next_token, g.next_token)
        np.testing.assert_array_equal(s.flags, g.flags)
        assert s.log == g.log
    assert osmp.T == og.T and len(og.T) > 5 and og.T


def test_gate_uses_raw_logits_whatever_the_temperature():
    """Eq. 3: the gate ratio is exp(z(draft) - z(t*)) on the target's raw logits; the sampling temperature
    changes alpha and the residual, never the ratio of a given pair."""
    zp = np.array([[[2.0, 1.0, 0.0, -1.0], [0, 0, 0, 0]]], np.float32)
    zq = np.array([[[0.0, 3.0, 0.0, 0.0]]], np.float32)
    d = np.array([[1]], np.int32)
    seen = []
    for T in (0.5, 1.0, 2.0):
        r = OS.verify_step_sampled(O.CSDOracle(), zp, zq, d, T, np.array([[0.999]]), np.array([[0.01, 0.5]]), 0.3, 0)
        assert r.rejected[0, 0] and int(r.tstar[0, 0]) == 0
        assert r.ratio[0, 0] == pytest.approx(np.exp(-1.0), rel=1e-12)
        seen.append(float(r.alpha[0, 0]))
    assert seen[0] < seen[1] < seen[2]                            # alpha does move with T
    assert int(r.accept_len[0]) == 1                              # e^-1 >= 0.3 and lambda = 0: rescued


def test_counts_equal_bruteforce_recount_and_snapshot_rule():
    rng = np.random.default_rng(11)
    B, k, V, T, lam = 6, 4, 8, 0.9, 2
    orc = O.CSDOracle()
    dense = np.zeros((V, V), np.int64)
    rescued = 0
    for step in range(80):
        zp = (rng.standard_normal((B, k + 1, V)) * 1.5).astype(np.float32)
        zq = (zp[:, :k] + rng.standard_normal((B, k, V)).astype(np.float32)).astype(np.float32)
        draft = rng.integers(0, V, (B, k)).astype(np.int32)
        before = dict(orc.T)
        r = OS.verify_step_sampled(orc, zp, zq, draft, T, rng.random((B, k)), rng.random((B, k + 1)), 0.2, lam)
        for b in range(B):
            n_by_test = 0
            for i in range(k):
                f = int(r.flags[b, i])
                if i > int(r.accept_len[b]):
                    assert f == 0                                 # nothing after the stop is touched
                if f & O.FLAG_COUNTED:
                    d, t = int(draft[b, i]), int(r.tstar[b, i])
                    assert d != t
                    dense[d, t] += 1
                    assert bool(f & O.FLAG_FREQ) == (before.get((d, t), 0) >= lam)     # table as of the step's start
                    assert bool(f & O.FLAG_SAFE) == (r.ratio[b, i] >= 0.2)
                    rescued += bool(f & O.FLAG_ACCEPTED)
                elif f:
                    assert f == (O.FLAG_MATCH | O.FLAG_ACCEPTED) and not r.rejected[b, i]
                    n_by_test += 1
            kept = sum(1 for i in range(k) if int(r.flags[b, i]) & O.FLAG_ACCEPTED)
            assert int(r.accept_len[b]) == kept
    for d in range(V):
        for t in range(V):
            assert orc.T.get((d, t), 0) == dense[d, t]
    assert rescued > 0                                            # pairs recur on 8 tokens: some cross the threshold
    assert sum(orc.T.values()) == dense.sum() > 100


def test_invalid_draft_id_ends_the_loop_uncounted():
    """Hand-stated: V = 4, k = 3.  Position 0 is accepted (r = 0); position 1 carries an id outside the
    vocabulary (4, then -1): the loop ends there, nothing is counted, nothing is looked up, the emitted token is
    the argmax of that position's target row, and position 2 is never processed - although its own acceptance
    test and draw are still reported.  The memory and the rescue counter are untouched; bad_draft counts one."""
    zp = np.array([[[3.0, 0.0, 0.0, 0.0], [0.0, 0.0, 5.0, 0.0], [0.0, 4.0, 0.0, 0.0], [1.0, 0.0, 0.0, 0.0]]], np.float32)
    zq = np.array([[[3.0, 0.0, 0.0, 0.0], [0.0, 0.0, 0.0, 0.0], [0.0, 0.0, 0.0, 6.0]]], np.float32)
    for bad in (4, -1, 2 ** 31 - 1):
        orc = O.CSDOracle()
        orc.ocm_update([(3, 1)], [9])
        draft = np.array([[0, bad, 3]], np.int32)
        r = OS.verify_step_sampled(orc, zp, zq, draft, 1.0, np.array([[0.0, 0.0, 0.999]]), np.array([[0.5, 0.5, 0.5, 0.5]]),
                                   tau=0.0, lam=0)
        assert r.accept_len.tolist() == [1] and r.next_token.tolist() == [2]        # argmax of target row 1
        assert r.flags[0].tolist() == [O.FLAG_MATCH | O.FLAG_ACCEPTED, 0, 0]
        assert r.log == [[]] and r.rescued == 0 and orc.T == {(3, 1): 9} and orc.bad_draft == 1
        assert bool(r.rejected[0, 1]) and int(r.tstar[0, 1]) == -1 and r.alpha[0, 1] == 0.0 and r.ratio[0, 1] == 0.0
        # position 2 (never reached): q puts its mass on token 3, p on token 1 -> rejected, residual on token 1
        assert bool(r.rejected[0, 2]) and int(r.tstar[0, 2]) == 1
    # the same id behind a stop is never reached, hence not counted as bad: at position 0 the draft model is sure
    # of token 3 (q = 0.99) which the target gives 0.04, so r = 0.999 rejects; the residual's mass sits on token 0
    # (0.87 of 0.95), u = 0.5 draws it; the gate ratio e^-3 is below tau = 0.9: not rescued, the loop stops
    zq2 = zq.copy()
    zq2[0, 0] = [0.0, 0.0, 0.0, 6.0]
    orc = O.CSDOracle()
    r = OS.verify_step_sampled(orc, zp, zq2, np.array([[3, 4, 0]], np.int32), 1.0, np.array([[0.999, 0.0, 0.0]]),
                               np.array([[0.5, 0.5, 0.5, 0.5]]), tau=0.9, lam=0)
    assert r.accept_len.tolist() == [0] and r.next_token.tolist() == [0] and orc.bad_draft == 0 and r.log == [[(3, 0)]]
    assert r.ratio[0, 0] == pytest.approx(np.exp(-3.0), rel=1e-12) and orc.T == {(3, 0): 1}


def test_residual_without_mass_reports_the_target_argmax():
    """p == q leaves max(0, p - q) without any mass.  With r in [0, 1] that case is never drawn from (alpha = 1
    accepts); an r above 1 - outside the interface's range, used here only to reach the branch - shows what it
    reports: the target row's lowest-id argmax, with a gate ratio of exp(z(draft) - z(argmax))."""
    zp = np.array([[[1.0, 4.0, 4.0, 0.0], [0.0, 0.0, 0.0, 2.0]]], np.float32)
    r = OS.verify_step_sampled(O.CSDOracle(), zp, zp[:, :1].copy(), np.array([[0]], np.int32), 0.7, np.array([[1.5]]),
                               np.array([[0.3, 0.3]]), tau=0.01, lam=0)
    assert bool(r.rejected[0, 0]) and r.alpha[0, 0] == 1.0 and r.res_mass[0, 0] == 0.0
    assert int(r.tstar[0, 0]) == 1                                  # tokens 1 and 2 tie: the lower id
    assert r.ratio[0, 0] == pytest.approx(np.exp(-3.0), rel=1e-12)
    assert r.log == [[(0, 1)]] and r.accept_len.tolist() == [1]     # e^-3 >= 0.01 and lambda = 0: rescued


def test_equal_models_accept_everything():
    rng = np.random.default_rng(3)
    zp = (rng.standard_normal((2, 4, 9)) * 3).astype(np.float32)
    r = OS.verify_step_sampled(O.CSDOracle(), zp, zp[:, :3].copy(), rng.integers(0, 9, (2, 3)).astype(np.int32), 0.7,
                               np.ones((2, 3)), rng.random((2, 4)), 0.3, 2)
    assert r.accept_len.tolist() == [3, 3] and not r.rejected.any() and np.all(r.alpha == 1.0)
    np.testing.assert_array_equal(r.next_token, r.bonus_token)


def test_bf16_storage_is_widened_exactly():
    from gen import f32_to_bf16_bits
    rng = np.random.default_rng(4)
    z32 = (rng.standard_normal((1, 3, 10)) * 2).astype(np.float32)
    bits = f32_to_bf16_bits(z32).reshape(z32.shape)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    d = rng.integers(0, 10, (1, 2)).astype(np.int32)
    ua, ud = rng.random((1, 2)), rng.random((1, 3))
    a = OS.verify_step_sampled(O.CSDOracle(), bits, bits[:, :2][:, ::-1].copy(), d, 0.8, ua, ud, 0.3, 0)
    b = OS.verify_step_sampled(O.CSDOracle(), back, back[:, :2][:, ::-1].copy(), d, 0.8, ua, ud, 0.3, 0)
    np.testing.assert_array_equal(a.alpha, b.alpha)
    np.testing.assert_array_equal(a.next_token, b.next_token)
