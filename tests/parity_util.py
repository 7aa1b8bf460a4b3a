"""Shared helpers of the GPU parity tests: run one step on both sides and compare to the bar.

Bar: bit-exact for argmax, accept lengths, emitted tokens, flags, the rejection log and memory
counts; row maxima equal as floats; normalisers, ratios and probabilities within 1e-5 relative of
the fp64 oracle (values below the smallest normal float32 are compared absolutely, since a
float32 output cannot hold them to a relative bar).
"""
import numpy as np
import torch

from gen.device import to_device_logits  # noqa: F401  (re-exported for the tests)
from oracle import csd_oracle as O
from paper_2604_13634_amd import binding as csd

RTOL = 1e-5
ATOL = 1.1754944e-38          # FLT_MIN


def assert_close(gpu: np.ndarray, ref: np.ndarray, what: str):
    gpu = gpu.astype(np.float64)
    assert np.all(np.isfinite(gpu)), "%s: non-finite value from the GPU" % what
    err = np.abs(gpu - ref)
    tol = RTOL * np.abs(ref) + ATOL
    bad = ~(err <= tol)                       # a NaN on either side fails
    if bad.any():
        i = int(np.argmax(err - tol))
        raise AssertionError("%s: %d values beyond 1e-5 relative; worst gpu=%r oracle=%r" %
                             (what, int(bad.sum()), gpu.ravel()[i], ref.ravel()[i]))


def compare_step(res: O.StepResult, bf: csd.VerifyBuffers, where: str = ""):
    """Compare one step's GPU outputs (already synchronised) with the oracle's."""
    g = lambda t: t.cpu().numpy()
    np.testing.assert_array_equal(g(bf.argmax), res.argmax, err_msg=where + " argmax")
    np.testing.assert_array_equal(g(bf.accept_len), res.accept_len, err_msg=where + " accept_len")
    np.testing.assert_array_equal(g(bf.next_token), res.next_token, err_msg=where + " next_token")
    assert np.all(g(bf.row_max).astype(np.float64) == res.row_max), where + " row_max"
    assert_close(g(bf.row_sumexp), res.row_sumexp, where + " row_sumexp")
    assert_close(g(bf.ratio), res.ratio, where + " ratio")
    assert_close(g(bf.p_draft), res.p_draft, where + " p_draft")
    np.testing.assert_array_equal(g(bf.pos_flags), res.flags, err_msg=where + " pos_flags")
    log = g(bf.rej_log).view(np.uint64)
    B, k = res.flags.shape
    for b in range(B):
        got = [(int(x >> np.uint64(20)), int(x & np.uint64(0xFFFFF))) for x in log[b]
               if (x & np.uint64(csd.CSD_OCM_KEY_MASK)) != np.uint64(csd.CSD_OCM_EMPTY)]
        assert got == res.log[b], "%s rej_log of sequence %d: %r != %r" % (where, b, got, res.log[b])


def decode_ocm(ocm: torch.Tensor):
    """Copy a table to the host and unpack its slots into {(draft, target): count} (slot layout of csd.h)."""
    raw = ocm.detach().cpu().numpy().view(np.uint64)
    key = raw & np.uint64(csd.CSD_OCM_KEY_MASK)
    used = key != np.uint64(csd.CSD_OCM_EMPTY)
    key = key[used]
    cnt = (raw[used] >> np.uint64(csd.CSD_OCM_KEY_BITS)).astype(np.int64)
    d = (key >> np.uint64(20)).astype(np.int64)
    t = (key & np.uint64((1 << 20) - 1)).astype(np.int64)
    out = {}
    for a, b, c in zip(d.tolist(), t.tolist(), cnt.tolist()):
        assert (a, b) not in out, "a key occupies two slots"
        out[(a, b)] = c
    return out


def compare_table(ocm: torch.Tensor, orc: O.CSDOracle, where: str = ""):
    got = decode_ocm(ocm)
    assert got == orc.T, "%s: memory differs (gpu %d keys, oracle %d keys)" % (where, len(got), len(orc.T))


def run_stream(workload, steps, tau=None, lam=None, capacity=None, prior=None, check_table_every=50,
               threads=8, apply_updates=True, progress_every=0):
    """Drive `steps` decode steps through csd_verify and the oracle; compare every step."""
    cfg = workload.cfg
    tau = cfg.tau if tau is None else tau
    lam = cfg.lam if lam is None else lam
    capacity = cfg.capacity if capacity is None else capacity
    orc = O.CSDOracle(capacity=capacity)
    ocm = csd.new_ocm(capacity)
    if prior is not None:
        pairs, weights = prior
        orc.ocm_update(pairs, weights)
        keys = torch.tensor([(d << 20) | t for d, t in pairs], dtype=torch.int64, device="cuda")
        csd.csd_ocm_update(ocm, keys, torch.tensor(weights, dtype=torch.int32, device="cuda"))
    bf = None
    rescued = counted = 0
    out = workload.empty_step()
    for step in steps:
        z, draft = workload.step(step, threads=threads, out=out)
        zt = to_device_logits(z)
        dt = torch.from_numpy(draft).cuda()
        bf = csd.csd_verify(zt, dt, tau, lam, ocm, csd.CSD_APPLY_UPDATES if apply_updates else 0, buffers=bf)
        torch.cuda.synchronize()
        res = orc.verify_step(z, draft, tau=np.float32(tau), lam=lam, apply_updates=apply_updates, threads=threads)
        where = "%s step %d" % (cfg.name, step)
        compare_step(res, bf, where)
        rescued += res.rescued
        counted += sum(len(l) for l in res.log)
        if check_table_every and (step % check_table_every == 0):
            compare_table(ocm, orc, where)
        if progress_every and (step % progress_every == 0):
            print("%s ok, %d rescued, %d counted, %d pairs" % (where, rescued, counted, len(orc.T)), flush=True)
    compare_table(ocm, orc, cfg.name + " final")
    st = bf.status.cpu().numpy().view(np.uint32)
    assert st[csd.CSD_STATUS_RESCUED] == rescued and st[csd.CSD_STATUS_COUNTED] == counted
    assert st[csd.CSD_STATUS_DROPPED] == orc.dropped and st[csd.CSD_STATUS_BAD_DRAFT] == orc.bad_draft
    return orc, ocm, rescued, counted


# --------------------------------------------------------------------------- verification at a sampling temperature
from oracle import csd_oracle_sampled as OS   # noqa: E402

TOL_ACCEPT = 1e-4      # |r - alpha| of every acceptance test
TOL_DRAW = 1e-5        # probability mass: a draw whose u * R lies this close to a boundary of the running sum may
                       # fall on either side in float32 (the kernel's running sums are good to about 1e-6 of mass)


def settle_uniforms(zp, zq, draft, T, u_accept, u_draw, seed, tries=12):
    """Move the acceptance numbers r away from their decision boundary, |r - alpha| >= TOL_ACCEPT, so that a
    float32 evaluation and the float64 oracle must agree on every acceptance test; offending numbers are re-drawn
    (always possible: alpha is one point of [0, 1]).  The draws u_draw are left exactly as generated, however
    finely the residual is divided: check_sampled_step deals with draws near a boundary.  Returns float32 copies."""
    rng = np.random.default_rng(seed)
    ua, ud = u_accept.astype(np.float32).copy(), u_draw.astype(np.float32).copy()
    V = zp.shape[-1]
    valid = (draft >= 0) & (draft < V)
    for attempt in range(tries + 1):
        r = OS.verify_step_sampled(O.CSDOracle(), zp, zq, draft, T, ua, ud, tau=0.0, lam=0, apply_updates=False)
        bad_acc = valid & (r.accept_margin < TOL_ACCEPT)
        if not bad_acc.any():
            return ua, ud
        ua[bad_acc] = rng.random(int(bad_acc.sum()), dtype=np.float32)
    raise AssertionError("could not settle the acceptance numbers of a step")


def _draw_weights(zp, zq, b, i, k, T):
    """The weights a draw inverts, from the oracle's own functions: the residual of position i < k, or p_{k+1}."""
    p = OS.softmax_T(OS.widen(zp[b, i]), T)
    if i == k:
        return p
    return np.maximum(0.0, p - OS.softmax_T(OS.widen(zq[b, i]), T))


def _tokens_within_tolerance(w, u, tol):
    """{token: a u' at the middle of its interval} for every token with mass whose interval of the running sum of
    w comes within tol (probability mass, as the oracle's draw margin) of u * R: the draws correct at that tolerance."""
    c = np.cumsum(w)
    R = float(c[-1])
    target = float(u) * R
    lo = int(np.searchsorted(c, target - tol, side="right"))
    hi = min(int(np.searchsorted(c, target + tol, side="right")), len(w) - 1)
    out = {}
    for v in range(max(lo - 1, 0), hi + 1):
        if w[v] > 0.0 and c[v] - w[v] <= target + tol and c[v] >= target - tol:
            out[v] = (float(c[v]) - 0.5 * float(w[v])) / R
    return out


class DrawStats:
    """How many draws of a run sat within TOL_DRAW of a boundary, and how many of those the GPU resolved the other way."""
    def __init__(self):
        self.draws = self.near_boundary = self.other_neighbour = 0


def check_sampled_step(orc, zp, zq, draft, T, ua, ud, tau, lam, bf, where="", stats=None, apply_updates=True):
    """Run the oracle on the step, compare every output of the GPU with it, and apply the step's updates to the
    oracle's memory.  A draw whose u * R lies within TOL_DRAW of a boundary of the running sum has two correct
    outcomes (csd.h says so).  For such a draw the GPU's token must be one of the tokens whose interval - by the
    oracle's running sum - comes within the tolerance; if it is not the oracle's own, the oracle is run again on
    that sequence with the draw moved to the middle of that token's interval, and everything downstream (gate,
    lookup, accept length, emitted token, log, memory) is compared on that branch.  No case is dropped."""
    B, K1, V = zp.shape
    k = K1 - 1
    view = O.CSDOracle(capacity=orc.capacity)        # same table, own counters: sequences may be run twice
    view.T = orc.T
    res = OS.verify_step_sampled(view, zp, zq, draft, T, ua, ud, tau=tau, lam=lam, apply_updates=False)
    g_tstar, g_bonus = bf.tstar.cpu().numpy(), bf.bonus_token.cpu().numpy()
    valid = (draft >= 0) & (draft < V)
    drawn = np.zeros((B, K1), bool)
    drawn[:, :k] = res.rejected & valid
    drawn[:, k] = True
    near = drawn & (res.draw_margin < TOL_DRAW)
    if stats is not None:
        stats.draws += int(drawn.sum())
        stats.near_boundary += int(near.sum())
    for b in np.nonzero(near.any(axis=1))[0]:
        ud_b = ud[b].astype(np.float64)
        moved = False
        for i in np.nonzero(near[b])[0]:
            mine = int(res.tstar[b, i]) if i < k else int(res.bonus_token[b])
            theirs = int(g_tstar[b, i]) if i < k else int(g_bonus[b])
            if theirs == mine:
                continue
            ok = _tokens_within_tolerance(_draw_weights(zp, zq, b, i, k, T), ud[b, i], TOL_DRAW)
            assert theirs in ok, "%s sequence %d draw %d: token %d is not within %g of mass of u*R (oracle %d, valid %r)" % (
                where, b, i, theirs, TOL_DRAW, mine, sorted(ok))
            ud_b[i] = ok[theirs]
            moved = True
            if stats is not None:
                stats.other_neighbour += 1
        if moved:
            rb = OS.verify_step_sampled(view, zp[b:b + 1], zq[b:b + 1], draft[b:b + 1], T, ua[b:b + 1], ud_b[None], tau=tau,
                                        lam=lam, apply_updates=False)
            res.rescued += rb.rescued - sum(1 for i in range(k) if (res.flags[b, i] & O.FLAG_COUNTED) and (res.flags[b, i] & O.FLAG_ACCEPTED))
            for name in ("accept_len", "next_token", "alpha", "p_draft", "q_draft", "rejected", "tstar", "ratio", "bonus_token",
                         "flags"):
                getattr(res, name)[b] = getattr(rb, name)[0]
            res.log[b] = rb.log[0]
    compare_sampled_step(res, bf, where)
    # what the loop of each sequence ended on: an id outside the vocabulary is counted once per sequence that reached it
    for b in range(B):
        n = int(res.accept_len[b])
        if n < k and not valid[b, n]:
            orc.bad_draft += 1
    if apply_updates:
        for pending in res.log:
            orc.ocm_update(pending)
    return res


def compare_sampled_step(res, bf, where: str = ""):
    g = lambda t: t.cpu().numpy()
    np.testing.assert_array_equal(g(bf.accept_len), res.accept_len, err_msg=where + " accept_len")
    np.testing.assert_array_equal(g(bf.tstar), res.tstar, err_msg=where + " tstar")
    np.testing.assert_array_equal(g(bf.bonus_token), res.bonus_token, err_msg=where + " bonus_token")
    np.testing.assert_array_equal(g(bf.next_token), res.next_token, err_msg=where + " next_token")
    np.testing.assert_array_equal(g(bf.pos_flags), res.flags, err_msg=where + " pos_flags")
    assert_close(g(bf.alpha), res.alpha, where + " alpha")
    assert_close(g(bf.p_draft), res.p_draft, where + " p_draft")
    assert_close(g(bf.q_draft), res.q_draft, where + " q_draft")
    assert_close(g(bf.ratio), np.minimum(res.ratio, 3.0e38), where + " ratio")
    k = res.flags.shape[1]
    log = g(bf.rej_log).view(np.uint64)
    for b, pending in enumerate(res.log):
        got = [int(x) for x in log[b] if int(x) & csd.CSD_OCM_KEY_MASK != csd.CSD_OCM_EMPTY]
        assert got == [(d << 20) | t for d, t in pending], "%s rej_log of sequence %d" % (where, b)


def run_sampled_stream(workload, steps, T, tau=None, lam=None, capacity=None, prior=None, check_table_every=10,
                       threads=8, progress_every=0):
    """Drive decode steps through csd_verify_sampled and the oracle; compare every step and the memory."""
    cfg = workload.cfg
    tau = cfg.tau if tau is None else tau
    lam = cfg.lam if lam is None else lam
    capacity = cfg.capacity if capacity is None else capacity
    orc = O.CSDOracle(capacity=capacity)
    ocm = csd.new_ocm(capacity)
    if prior is not None:
        pairs, weights = prior
        orc.ocm_update(pairs, weights)
        keys = torch.tensor([(d << 20) | t for d, t in pairs], dtype=torch.int64, device="cuda")
        csd.csd_ocm_update(ocm, keys, torch.tensor(weights, dtype=torch.int32, device="cuda"))
    bf = None
    rescued = counted = rejected = 0
    stats = DrawStats()
    for step in steps:
        zp, zq, draft, ua, ud = workload.sampled_step(step, threads=threads)
        ua, ud = settle_uniforms(zp, zq, draft, T, ua, ud, seed=step)
        bf = csd.csd_verify_sampled(to_device_logits(zp), to_device_logits(zq), torch.from_numpy(draft).cuda(), T,
                                    torch.from_numpy(ua).cuda(), torch.from_numpy(ud).cuda(), tau, lam, ocm, buffers=bf)
        torch.cuda.synchronize()
        where = "%s T=%g step %d" % (cfg.name, T, step)
        res = check_sampled_step(orc, zp, zq, draft, T, ua, ud, np.float32(tau), lam, bf, where, stats)
        rescued += res.rescued
        counted += sum(len(l) for l in res.log)
        rejected += int(res.rejected.sum())
        if check_table_every and (step % check_table_every == 0):
            compare_table(ocm, orc, where)
        if progress_every and (step % progress_every == 0):
            print("%s ok, %d rejected, %d rescued, %d counted, %d pairs" % (where, rejected, rescued, counted, len(orc.T)),
                  flush=True)
    compare_table(ocm, orc, cfg.name + " final")
    st = bf.status.cpu().numpy().view(np.uint32)
    assert st[csd.CSD_STATUS_RESCUED] == rescued and st[csd.CSD_STATUS_COUNTED] == counted
    print("%s T=%g: %d draws, %d within %g of a boundary, %d of those resolved to the other neighbour" % (
        cfg.name, T, stats.draws, stats.near_boundary, TOL_DRAW, stats.other_neighbour))
    return orc, ocm, rescued, counted, rejected
