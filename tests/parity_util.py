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
TOL_DRAW = 1e-5        # probability mass between u * R and the nearer end of the drawn token's interval


def settle_uniforms(zp, zq, draft, T, u_accept, u_draw, seed, tries=12):
    """Move the step's random numbers away from decision boundaries, so that a float32 evaluation and the
    float64 oracle must agree: every |r - alpha| >= TOL_ACCEPT, every draw at least TOL_DRAW of probability
    mass inside its token's interval.  Offending numbers are re-drawn; a rejected position whose residual is
    too finely divided for any draw to have that margin (mass spread over thousands of tail tokens) is
    turned into an accepted one (r = 0).  Returns float32 copies."""
    rng = np.random.default_rng(seed)
    ua, ud = u_accept.astype(np.float32).copy(), u_draw.astype(np.float32).copy()
    B, k = draft.shape
    V = zp.shape[-1]
    valid = (draft >= 0) & (draft < V)
    for attempt in range(tries + 1):
        r = OS.verify_step_sampled(O.CSDOracle(), zp, zq, draft, T, ua, ud, tau=0.0, lam=0, apply_updates=False)
        bad_acc = valid & (r.accept_margin < TOL_ACCEPT) & (ua != 0)
        bad_draw = np.zeros((B, k + 1), bool)
        bad_draw[:, :k] = valid & r.rejected & (r.draw_margin[:, :k] < TOL_DRAW)
        bad_draw[:, k] = r.draw_margin[:, k] < TOL_DRAW
        if not bad_acc.any() and not bad_draw.any():
            return ua, ud
        if attempt >= tries - 2:
            ua[bad_draw[:, :k]] = 0.0                       # give up on these residuals: accept the position
            ua[bad_acc] = 0.0
        else:
            ua[bad_acc] = rng.random(int(bad_acc.sum()), dtype=np.float32)
        ud[bad_draw] = rng.random(int(bad_draw.sum()), dtype=np.float32)
    raise AssertionError("could not settle the random numbers of a step")


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
    for step in steps:
        zp, zq, draft, ua, ud = workload.sampled_step(step, threads=threads)
        ua, ud = settle_uniforms(zp, zq, draft, T, ua, ud, seed=step)
        bf = csd.csd_verify_sampled(to_device_logits(zp), to_device_logits(zq), torch.from_numpy(draft).cuda(), T,
                                    torch.from_numpy(ua).cuda(), torch.from_numpy(ud).cuda(), tau, lam, ocm, buffers=bf)
        torch.cuda.synchronize()
        res = OS.verify_step_sampled(orc, zp, zq, draft, T, ua, ud, tau=np.float32(tau), lam=lam)
        where = "%s T=%g step %d" % (cfg.name, T, step)
        compare_sampled_step(res, bf, where)
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
    return orc, ocm, rescued, counted, rejected
