"""Shared helpers of the GPU parity tests: run one step on both sides and compare to the bar.

Bar: bit-exact for argmax, accept lengths, emitted tokens, flags, the rejection log and memory
counts; row maxima equal as floats; normalisers, ratios and probabilities within 1e-5 relative of
the fp64 oracle (values below the smallest normal float32 are compared absolutely, since a
float32 output cannot hold them to a relative bar).
"""
import numpy as np
import torch

from oracle import csd_oracle as O
from paper_2604_13634_amd import binding as csd

RTOL = 1e-5
ATOL = 1.1754944e-38          # FLT_MIN


def to_device_logits(z: np.ndarray) -> torch.Tensor:
    """Host logits (float32, or uint16 bf16 bit patterns) -> device tensor (float32 / bfloat16).

    The library wants every row 16-byte aligned: when V * itemsize is not a multiple of 16 the rows
    are laid out with a padded pitch (padding filled with a large value that must never be read) and
    a [..., :V] view is returned."""
    if z.dtype == np.float32:
        t = torch.from_numpy(z)
        per16, big = 4, 1e30
    else:
        assert z.dtype == np.uint16
        t = torch.from_numpy(z.view(np.int16)).view(torch.bfloat16)
        per16, big = 8, 1e30
    V = z.shape[-1]
    if V % per16 == 0:
        return t.cuda()
    pitch = (V + per16 - 1) // per16 * per16
    padded = torch.full(z.shape[:-1] + (pitch,), big, dtype=t.dtype, device="cuda")
    padded[..., :V] = t.cuda()
    return padded[..., :V]


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


def compare_table(ocm: torch.Tensor, orc: O.CSDOracle, where: str = ""):
    got = csd.decode_ocm(ocm)
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
