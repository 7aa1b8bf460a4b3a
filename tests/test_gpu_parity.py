"""GPU parity: csd_verify / csd_ocm_* through the C ABI against the fp64 oracle (needs an MI355X)."""
import os

import numpy as np
import pytest
import torch

from gen import CONFIGS, Workload, f32_to_bf16_bits
from oracle import csd_oracle as O
from paper_2604_13634_amd import binding as csd
from parity_util import compare_step, compare_table, decode_ocm, run_stream, to_device_logits

pytestmark = pytest.mark.gpu


def _prior_from_pairs(w, lam, n=64):
    """A calibrated prior: the head of the divergence-pair map, already at the frequency threshold."""
    pairs = [(int(d), int(t)) for t, d in zip(w.pair_target[:n], w.pair_draft[:n])]
    return pairs, [lam] * len(pairs)


# --------------------------------------------------------------------------- streams with an evolving memory
def test_config0_full_stream():
    """Config 0 exactly: B=1, k=4, V=32000, fp32, 1000 steps, empty memory at start."""
    w = Workload(CONFIGS[0])
    orc, ocm, rescued, counted = run_stream(w, range(w.cfg.steps), check_table_every=100)
    assert rescued > 20 and counted > 500


@pytest.mark.parametrize("ci,V,steps", [(1, 4099, 400), (2, 8200, 150), (3, 3001, 100), (4, 2048 + 6, 120)])
def test_long_streams_reduced_vocab(ci, V, steps):
    """Configs 1-4 with their batch, k, tau, lambda, pair skew and storage type over many steps,
    on a reduced ragged vocabulary so that the oracle keeps up; the memory evolves from empty."""
    cfg = CONFIGS[ci]
    w = Workload(cfg, V=V, n_pairs=min(cfg.n_pairs, 1024))
    orc, ocm, rescued, counted = run_stream(w, range(steps), check_table_every=25)
    assert rescued > 0 and counted > steps


@pytest.mark.parametrize("ci,steps", [(1, 6), (2, 3), (3, 2), (4, 2)])
def test_full_size_steps_with_prior(ci, steps):
    """Configs 1-4 at full size (the shapes bench.py times) for a few steps, memory pre-loaded with a
    prior so that rescues happen from the first step."""
    w = Workload(CONFIGS[ci])
    prior = _prior_from_pairs(w, w.cfg.lam, n=min(512, w.cfg.n_pairs))
    orc, ocm, rescued, counted = run_stream(w, range(steps), prior=prior, check_table_every=1, threads=16)
    assert rescued > 0


@pytest.mark.parametrize("ci,steps", [(1, 600), (2, 250), (3, 120), (4, 100)])
def test_full_size_streams_from_an_empty_memory(ci, steps):
    """Configs 1-4 at full size (the shapes and launch configuration bench.py times), the memory evolving
    from empty: pairs cross the frequency threshold and are rescued without any prior.  Every step is
    compared, the memory every 10 steps."""
    w = Workload(CONFIGS[ci])
    orc, ocm, rescued, counted = run_stream(w, range(steps), check_table_every=10, threads=16)
    print("%s: %d steps from empty, %d rescued, %d counted, %d pairs" % (w.cfg.name, steps, rescued, counted, len(orc.T)))
    assert rescued > 0 and counted > steps


@pytest.mark.skipif(os.environ.get("CSD_FULL_STREAMS") != "1",
                    reason="several minutes of oracle time per configuration: set CSD_FULL_STREAMS=1 and run with -s")
@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_full_streams_every_step(ci):
    """Configs 1-4 exactly as stated: full size, every step of the stream (2000/2000/1000/500), memory
    evolving from empty, every step compared and the memory compared every 100 steps."""
    w = Workload(CONFIGS[ci])
    orc, ocm, rescued, counted = run_stream(w, range(w.cfg.steps), check_table_every=100, threads=16, progress_every=20)
    assert rescued > 0 and counted > w.cfg.steps


# --------------------------------------------------------------------------- row statistics: shapes, ties, ranges
def _verify_rows(z_np, draft_np=None, tau=0.3, lam=2, ocm=None, flags=0):
    B, K1, V = z_np.shape
    if draft_np is None:
        draft_np = np.zeros((B, K1 - 1), dtype=np.int32)
    zt = to_device_logits(z_np)
    bf = csd.csd_verify(zt, torch.from_numpy(draft_np).cuda(), tau, lam, ocm, flags)
    torch.cuda.synchronize()
    return bf


def _check_against_oracle(z_np, draft_np=None, tau=0.3, lam=2):
    B, K1, V = z_np.shape
    if draft_np is None:
        draft_np = np.zeros((B, K1 - 1), dtype=np.int32)
    bf = _verify_rows(z_np, draft_np, tau, lam)
    res = O.CSDOracle().verify_step(np.ascontiguousarray(z_np), draft_np, tau=np.float32(tau), lam=lam, use_ocm=False)
    compare_step(res, bf, "V=%d" % V)
    return bf, res


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 255, 1023, 1024, 1025, 4095, 4097, 8191, 8193,
                               16385, 40000, 70001])
def test_ragged_vocab_sizes(dtype, V):
    rng = np.random.default_rng(V)
    z = (rng.standard_normal((3, 3, V)) * 3).astype(np.float32)
    if dtype == "bf16":
        z = f32_to_bf16_bits(z).reshape(3, 3, V)
    draft = rng.integers(0, V, size=(3, 2)).astype(np.int32)
    _check_against_oracle(z, draft)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_stride_larger_than_vocab(dtype):
    rng = np.random.default_rng(7)
    V, pitch = 3000, 3016
    zp = (rng.standard_normal((2, 4, pitch)) * 3).astype(np.float32)
    zp[..., V:] = 100.0                       # padding must never be read as logits
    if dtype == "bf16":
        zp = f32_to_bf16_bits(zp).reshape(2, 4, pitch)
    draft = rng.integers(0, V, size=(2, 3)).astype(np.int32)
    zt = to_device_logits(zp)[..., :V]
    bf = csd.csd_verify(zt, torch.from_numpy(draft).cuda(), 0.3, 2, None, 0)
    torch.cuda.synchronize()
    res = O.CSDOracle().verify_step(np.ascontiguousarray(zp[..., :V]), draft, tau=np.float32(0.3), lam=2, use_ocm=False)
    compare_step(res, bf, "strided")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ties_resolve_to_lowest_id_everywhere(dtype):
    """Equal maxima inside one 16-byte chunk, across lanes, waves, tiles and row segments."""
    V = 150000
    rng = np.random.default_rng(3)
    spots = [(0, 1), (5, 6), (3, 64 * 8 + 3), (1000, 1001), (2047, 2048), (4095, 4096), (8191, 8192), (100, 140000),
             (70000, 70001), (V - 2, V - 1), (65535, 65536), (32767, 98304)]
    z = (rng.standard_normal((len(spots), 2, V))).astype(np.float32)
    for r, (a, b) in enumerate(spots):
        z[r, 0, a] = 9.0
        z[r, 0, b] = 9.0
        z[r, 1, b] = 9.0
        z[r, 1, a] = 9.0 if r % 2 else 8.5
    if dtype == "bf16":
        z = f32_to_bf16_bits(z).reshape(z.shape)
    bf, res = _check_against_oracle(z)
    assert [int(x) for x in bf.argmax[:, 0].cpu()] == [a for a, _ in spots]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_constant_rows_and_signed_zero(dtype):
    V = 20000
    z = np.full((2, 2, V), 1.5, dtype=np.float32)
    z[1, 0, :] = -0.0
    z[1, 0, 77] = 0.0
    z[1, 1, :] = -3.0
    z[1, 1, 5000] = -0.0
    z[1, 1, 9000] = 0.0
    if dtype == "bf16":
        z = f32_to_bf16_bits(z).reshape(z.shape)
    bf, res = _check_against_oracle(z)
    assert bf.argmax.cpu().tolist() == [[0, 0], [0, 5000]]
    assert float(bf.row_sumexp[0, 0]) == pytest.approx(V, rel=1e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_masked_vocab_and_extreme_ranges(dtype):
    """-inf entries, maxima that climb steeply along the row (reference rescaling), huge and tiny magnitudes."""
    V = 50000
    rng = np.random.default_rng(9)
    z = (rng.standard_normal((1, 8, V)) * 2).astype(np.float32)
    z[0, 0, rng.random(V) < 0.7] = -np.inf                       # mostly masked
    z[0, 1, :] = -np.inf
    z[0, 1, 43210] = -5.0                                        # a single finite value, late in the row
    z[0, 2, :] = np.linspace(-300.0, 300.0, V)                   # ascending ramp: many rescales
    z[0, 3, :] = np.linspace(300.0, -300.0, V)                   # descending ramp
    z[0, 4, :] *= 1000.0                                         # spread of thousands
    z[0, 5, :] = z[0, 5, :] * 1e-3 + 1e4                         # large offset, tiny spread
    z[0, 6, :] = -5e8                                            # the largest magnitude the interface admits
    z[0, 6, 123] = -4.95e8
    z[0, 7, : V // 2] = -np.inf                                  # first segments hold nothing finite
    if dtype == "bf16":
        fin = np.isfinite(z)
        zb = np.where(fin, z, 0).astype(np.float32)
        bits = f32_to_bf16_bits(zb).reshape(z.shape)
        bits[~fin] = 0xFF80
        z = bits
    draft = np.array([[1, 43210, V - 1, 0, 17, 99, 123]], dtype=np.int32)
    _check_against_oracle(z, draft)


@pytest.mark.parametrize("dtype,B,k,V", [("f32", 1, 4, 1 << 20), ("bf16", 1, 6, 1000003), ("f32", 2, 7, 600011),
                                         ("bf16", 257, 3, 4100), ("f32", 1030, 2, 2500)])
def test_few_sequences_over_huge_vocabularies_and_batches_past_the_barrier(dtype, B, k, V):
    """Shapes off the benchmark's beaten path of the single-launch step: one or two sequences over a vocabulary so
    large that a row is cut into more than a hundred workgroups (a sequence wave then takes its rows' records in
    several rounds and re-reads them for the sums), and batches of more than 256 sequences (more sequence
    workgroups than may wait for each other: the updates go through the log and a second launch).  Three steps
    each, memory evolving, everything compared with the oracle."""
    rng = np.random.default_rng(B * 1000 + k)
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    bf = None
    pool = rng.integers(0, V, 24)                                   # few tokens, so that pairs recur and get rescued
    for step in range(3):
        z = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
        top = pool[rng.integers(0, 24, (B, k + 1))]
        np.put_along_axis(z, top[..., None], z.max(-1, keepdims=True) + 4.0, axis=-1)
        draft = np.where(rng.random((B, k)) < 0.5, top[:, :k], pool[rng.integers(0, 24, (B, k))]).astype(np.int32)
        zd = z[:, :k]                                               # a view: a divergent draft token sits 0.5 below the top
        off = np.where(draft == top[:, :k], 0.0, 0.5).astype(np.float32)
        np.put_along_axis(zd, draft[..., None].astype(np.int64), (zd.max(-1) - off)[..., None], axis=-1)
        if dtype == "bf16":
            z = f32_to_bf16_bits(z).reshape(z.shape)
        bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), 0.3, 1, ocm, buffers=bf)
        torch.cuda.synchronize()
        res = orc.verify_step(np.ascontiguousarray(z), draft, tau=np.float32(0.3), lam=1)
        compare_step(res, bf, "%s B=%d k=%d V=%d step %d" % (dtype, B, k, V, step))
        compare_table(ocm, orc, "B=%d V=%d step %d" % (B, V, step))
    assert int(bf.status[csd.CSD_STATUS_STALLED]) == 0 and len(orc.T) > 0


def test_waits_that_run_out_are_reported_and_leave_everything_usable():
    """The waits inside the single-launch step are bounded.  A test hook of the library (not part of csd.h) makes
    the sequence waves look for records under another per-call number than the streaming workgroups publish them
    under, and cuts the bound to 64 polls: every wait runs out.  The kernels end normally, status[CSD_STATUS_STALLED]
    counts one wait per sequence (its rows' records) and one per sequence workgroup of four (the barrier before the
    updates), every sequence reports accept_len 0 / next_token -1, the memory is untouched - and the next
    ordinary call on the same buffers and workspace agrees with the oracle again.  Same for the sampled step."""
    import ctypes
    from gen.workload import SampledWorkload
    from parity_util import check_sampled_step, settle_uniforms
    lib = csd.load_library()
    lib.csd_test_set_wait_rules.restype = None
    lib.csd_test_set_wait_rules.argtypes = [ctypes.c_uint32, ctypes.c_uint64]
    w = Workload(CONFIGS[1], V=9001, B=10, n_pairs=16)
    ws = SampledWorkload(CONFIGS[1], V=9001, B=10, n_pairs=16)
    cfg = w.cfg
    ocm, ocm_s = csd.new_ocm(1 << 10), csd.new_ocm(1 << 10)
    orc, orc_s = O.CSDOracle(), O.CSDOracle()
    bf = sb = None
    for step in range(4):
        z, draft = w.step(step)
        zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
        zp, zq, sdraft, ua, ud = ws.sampled_step(step)
        ua, ud = settle_uniforms(zp, zq, sdraft, 0.9, ua, ud, seed=step)
        sargs = (to_device_logits(zp), to_device_logits(zq), torch.from_numpy(sdraft).cuda(), 0.9, torch.from_numpy(ua).cuda(),
                 torch.from_numpy(ud).cuda(), cfg.tau, 1, ocm_s)
        if step == 2:                                   # in the middle of the stream: both paths stall once
            before, before_s = decode_ocm(ocm), decode_ocm(ocm_s)
            lib.csd_test_set_wait_rules(64, 0x5EEDF00D)
            try:
                bf.status.zero_()
                sb.status.zero_()
                csd.csd_verify(zt, dt, cfg.tau, 1, ocm, buffers=bf)
                csd.csd_verify_sampled(*sargs, buffers=sb)
                torch.cuda.synchronize()
            finally:
                lib.csd_test_set_wait_rules(0, 0)
            for b_, name in ((bf, "greedy"), (sb, "sampled")):
                st = b_.status.cpu().numpy().view(np.uint32)
                assert st[csd.CSD_STATUS_STALLED] == cfg.B + (cfg.B + 3) // 4 and st[csd.CSD_STATUS_COUNTED] == 0, (name, st)
                assert b_.accept_len.cpu().tolist() == [0] * cfg.B and b_.next_token.cpu().tolist() == [-1] * cfg.B, name
            assert decode_ocm(ocm) == before and decode_ocm(ocm_s) == before_s
            bf.status.zero_()
            sb.status.zero_()
        bf = csd.csd_verify(zt, dt, cfg.tau, 1, ocm, buffers=bf)
        sb = csd.csd_verify_sampled(*sargs, buffers=sb)
        torch.cuda.synchronize()
        compare_step(orc.verify_step(z, draft, tau=np.float32(cfg.tau), lam=1), bf, "greedy step %d" % step)
        check_sampled_step(orc_s, zp, zq, sdraft, 0.9, ua, ud, np.float32(cfg.tau), 1, sb, "sampled step %d" % step)
        compare_table(ocm, orc, "greedy step %d" % step)
        compare_table(ocm_s, orc_s, "sampled step %d" % step)
    assert int(bf.status[csd.CSD_STATUS_STALLED]) == 0 and int(sb.status[csd.CSD_STATUS_STALLED]) == 0


def test_many_rows_and_k_limits():
    rng = np.random.default_rng(21)
    for B, k, V in [(1, 0, 5000), (3, 63, 700), (700, 1, 300), (33, 15, 2500)]:
        z = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
        draft = rng.integers(0, V, size=(B, k)).astype(np.int32)
        am = z[:, :k].argmax(axis=-1)
        draft = np.where(rng.random((B, k)) < 0.8, am, draft).astype(np.int32)
        bf = _verify_rows(z, draft, tau=0.2, lam=0, ocm=csd.new_ocm(1 << 12), flags=0)
        res = O.CSDOracle().verify_step(z, draft, tau=np.float32(0.2), lam=0, apply_updates=False)
        compare_step(res, bf, "B=%d k=%d" % (B, k))
    # an empty batch is a no-op that must not fail
    zt = torch.empty((0, 3, 100), dtype=torch.float32, device="cuda")
    rc = csd.load_library().csd_verify(None, 0, 100, None, 0, 2, 100, 0.3, 2, None, 0, 0, None, None, None, None, None,
                                       None, None, None, None, None, None, 0, None)
    assert rc == csd.CSD_OK


# --------------------------------------------------------------------------- gate / memory modes
def test_modes_strict_gate_only_memory_only():
    """No memory = strict matching; lambda = 0 = gate only; tau <= 0 = memory only; tau > 1 = strict."""
    w = Workload(CONFIGS[2], V=3000, B=16)
    cfg = w.cfg
    prior = _prior_from_pairs(w, 5, n=256)
    for tau, lam, use_ocm in [(0.25, 3, False), (0.6, 0, True), (0.0, 3, True), (-1.0, 3, True), (1.0001, 0, True),
                              (1.0, 0, True), (0.25, 2 ** 32 - 1, True)]:
        orc = O.CSDOracle()
        orc.ocm_update(*prior)
        ocm = csd.new_ocm(4096)
        csd.csd_ocm_update(ocm, torch.tensor([(d << 20) | t for d, t in prior[0]], dtype=torch.int64, device="cuda"),
                           torch.tensor(prior[1], dtype=torch.int32, device="cuda"))
        for step in range(6):
            z, draft = w.step(step)
            bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), tau, lam, ocm if use_ocm else None)
            torch.cuda.synchronize()
            res = orc.verify_step(z, draft, tau=np.float32(tau), lam=lam, use_ocm=use_ocm)
            compare_step(res, bf, "tau=%g lam=%d ocm=%s step %d" % (tau, lam, use_ocm, step))
        compare_table(ocm, orc)


def test_deferred_updates_through_rejection_log():
    """flags = 0 leaves the memory untouched; replaying rej_log through csd_ocm_update gives the fused result."""
    w = Workload(CONFIGS[4], V=2048, B=64)
    cfg = w.cfg
    ocm_a, ocm_b = csd.new_ocm(1 << 14), csd.new_ocm(1 << 14)
    orc = O.CSDOracle()
    for step in range(30):
        z, draft = w.step(step)
        zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
        bfa = csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm_a, csd.CSD_APPLY_UPDATES)
        before = ocm_b.clone()
        bfb = csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm_b, 0)
        torch.cuda.synchronize()
        assert torch.equal(before, ocm_b)
        csd.csd_ocm_update(ocm_b, bfb.rej_log.view(-1))
        torch.cuda.synchronize()
        res = orc.verify_step(z, draft, tau=np.float32(cfg.tau), lam=cfg.lam)
        compare_step(res, bfa, "fused step %d" % step)
        compare_step(res, bfb, "deferred step %d" % step)
    compare_table(ocm_a, orc)
    compare_table(ocm_b, orc)


def test_in_kernel_updates_equal_replayed_log_at_full_batch():
    """The hand-over of the step log to the workgroup that applies it, at the contention workload's batch
    (256 sequences, 16 workgroups in the finish kernel): over 150 steps, a memory updated inside csd_verify
    and one updated by replaying each step's rej_log through csd_ocm_update stay identical, and so do all
    outputs (a log entry that the applying workgroup read too early would lose a count)."""
    w = Workload(CONFIGS[4], V=4096 + 6)
    cfg = w.cfg
    ocm_a, ocm_b = csd.new_ocm(1 << 14), csd.new_ocm(1 << 14)
    bfa = bfb = None
    inputs = []
    for step in range(12):                              # twelve distinct steps, cycled: the counts keep growing
        z, draft = w.step(step, threads=8)
        inputs.append((to_device_logits(z), torch.from_numpy(draft).cuda()))
    for step in range(150):
        zt, dt = inputs[step % len(inputs)]
        bfa = csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm_a, csd.CSD_APPLY_UPDATES, buffers=bfa)
        bfb = csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm_b, 0, buffers=bfb)
        csd.csd_ocm_update(ocm_b, bfb.rej_log.view(-1), status=bfb.status)
        torch.cuda.synchronize()
        for name in ("accept_len", "next_token", "argmax", "pos_flags", "rej_log"):
            assert torch.equal(getattr(bfa, name), getattr(bfb, name)), "step %d %s" % (step, name)
        if step % 10 == 0 or step == 149:
            assert decode_ocm(ocm_a) == decode_ocm(ocm_b), "memories differ at step %d" % step
    st = bfa.status.cpu().numpy().view(np.uint32)
    assert st[csd.CSD_STATUS_RESCUED] > 1000 and sum(decode_ocm(ocm_a).values()) == st[csd.CSD_STATUS_COUNTED]
    assert torch.equal(bfa.status, bfb.status)


@pytest.mark.parametrize("B,k", [(256, 4), (64, 63), (7, 3)])
def test_every_position_of_a_step_diverges_on_one_pair(B, k):
    """The most skewed step there is: every draft position of every sequence holds the same (draft, target) pair,
    with a ratio that passes the gate.  A sequence workgroup sends its equal pairs to the memory as one add of their
    number (up to 4 x 63 lanes merging in its LDS table), so B*k increments reach one slot from at most B/4 adds.
    Step 1 counts one divergence per sequence and stops there; once the pair is frequent every position is rescued
    and counted.  Every step against the oracle, counts included; a second pair on one position checks that the
    merge keeps pairs apart."""
    V = 5003
    rng = np.random.default_rng(B * 64 + k)
    z = (rng.standard_normal((B, k + 1, V)) * 0.5).astype(np.float32)
    z[:, :, 11] = 9.0                                   # target token 11 on every row
    z[:, :k, 7] = 8.5                                   # draft token 7: ratio exp(-0.5) = 0.61 passes tau = 0.3
    z[0, 0, 13] = 8.8                                   # one position drafts token 13 instead
    draft = np.full((B, k), 7, dtype=np.int32)
    draft[0, 0] = 13
    zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
    ocm = csd.new_ocm(1 << 8)
    orc = O.CSDOracle()
    bf = None
    for step in range(5):
        bf = csd.csd_verify(zt, dt, 0.3, 2, ocm, buffers=bf)
        torch.cuda.synchronize()
        res = orc.verify_step(z, draft, tau=np.float32(0.3), lam=2)
        compare_step(res, bf, "B=%d k=%d step %d" % (B, k, step))
        compare_table(ocm, orc, "B=%d k=%d step %d" % (B, k, step))
    T = decode_ocm(ocm)
    assert set(T) == {(7, 11), (13, 11)} and T[(7, 11)] > 2 * B * k and bf.accept_len.cpu().tolist() == [k] * B


@pytest.mark.parametrize("B", [300, 700, 2200])
def test_large_batches_update_paths(B):
    """B*k of 1200 and 2800 (several merge batches inside the finish kernel) and 8800 (beyond what the
    finish kernel applies itself: the separate update launch), on the skewed pair stream."""
    w = Workload(CONFIGS[4], V=1030, B=B)
    cfg = w.cfg
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    bf = None
    for step in range(5):
        z, draft = w.step(step)
        bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), cfg.tau, cfg.lam, ocm, buffers=bf)
        torch.cuda.synchronize()
        res = orc.verify_step(z, draft, tau=np.float32(cfg.tau), lam=cfg.lam)
        compare_step(res, bf, "B=%d step %d" % (B, step))
        compare_table(ocm, orc, "B=%d step %d" % (B, step))
    assert int(bf.status[csd.CSD_STATUS_COUNTED]) == sum(orc.T.values())


def test_bad_draft_ids_are_divergences_never_counted():
    rng = np.random.default_rng(4)
    B, k, V = 8, 4, 1000
    z = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
    am = z[:, :k].argmax(axis=-1).astype(np.int32)
    draft = am.copy()
    draft[0, 1] = V
    draft[1, 0] = -1
    draft[2, 3] = 2 ** 31 - 1
    draft[3, 2] = -2 ** 31
    draft[4, 0] = (am[4, 0] + 1) % V          # ordinary divergence first: the bad id behind it is not processed
    draft[4, 1] = V + 5
    # tau = 0: the ordinary divergence of sequence 4 is rescued, so the bad id behind it is reached (5 in all);
    # tau = 0.999: it is not rescued and the scan stops before the bad id (4 in all)
    for tau, n_bad in [(0.0, 5), (0.999, 4)]:
        ocm = csd.new_ocm(256)
        orc = O.CSDOracle()
        bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), tau, 0, ocm)
        torch.cuda.synchronize()
        res = orc.verify_step(z, draft, tau=np.float32(tau), lam=0)
        compare_step(res, bf, "bad ids")
        compare_table(ocm, orc)
        assert int(bf.status[csd.CSD_STATUS_BAD_DRAFT]) == orc.bad_draft == n_bad


# --------------------------------------------------------------------------- the memory on its own
def test_ocm_update_duplicates_weights_lookup():
    rng = np.random.default_rng(5)
    n = 200000
    d = rng.zipf(1.3, size=n) % 5000
    t = (d + 1 + rng.integers(0, 50, size=n)) % 5000
    keep = d != t
    d, t = d[keep], t[keep]
    wts = rng.integers(0, 4, size=d.size).astype(np.int32)          # zeros are skipped
    ocm = csd.new_ocm(1 << 16)
    orc = O.CSDOracle(capacity=1 << 16)
    keys = torch.from_numpy(((d.astype(np.int64) << 20) | t.astype(np.int64))).cuda()
    status = torch.zeros(csd.CSD_STATUS_WORDS, dtype=torch.int32, device="cuda")
    csd.csd_ocm_update(ocm, keys, torch.from_numpy(wts).cuda(), status)
    csd.csd_ocm_update(ocm, keys[:1000], None, status)
    orc.ocm_update(zip(d.tolist(), t.tolist()), wts.tolist())
    orc.ocm_update(zip(d[:1000].tolist(), t[:1000].tolist()))
    compare_table(ocm, orc)
    assert int(status[0]) == 0
    q = torch.cat([keys[:500], torch.tensor([(7 << 20) | 7, csd.CSD_OCM_EMPTY, (4999 << 20) | 4998], dtype=torch.int64,
                                            device="cuda")])
    got = csd.csd_ocm_lookup(ocm, q).cpu().tolist()
    want = [orc.T.get((int(x) >> 20, int(x) & 0xFFFFF), 0) for x in q.cpu().tolist()]
    want[-2] = 0
    assert got == want


def test_ocm_hot_key_contention_and_saturation():
    """Hundreds of thousands of increments onto a handful of keys; then saturation at 2^24 - 1."""
    n = 1 << 20
    rng = np.random.default_rng(6)
    d = rng.integers(0, 4, size=n)
    t = d + 10
    keys = torch.from_numpy((d.astype(np.int64) << 20) | t.astype(np.int64)).cuda()
    ocm = csd.new_ocm(64)
    csd.csd_ocm_update(ocm, keys)
    got = decode_ocm(ocm)
    assert got == {(i, i + 10): int((d == i).sum()) for i in range(4)}
    big = torch.full((40,), 2 ** 31 - 1, dtype=torch.int32, device="cuda")
    csd.csd_ocm_update(ocm, keys[:40], big)
    got = decode_ocm(ocm)
    assert all(got[(int(a), int(a) + 10)] == csd.CSD_OCM_COUNT_MAX for a in set(d[:40].tolist()))
    csd.csd_ocm_update(ocm, keys[:40])
    assert decode_ocm(ocm) == got


def test_ocm_full_table_drops_are_reported():
    ocm = csd.new_ocm(8)
    status = torch.zeros(csd.CSD_STATUS_WORDS, dtype=torch.int32, device="cuda")
    orc = O.CSDOracle(capacity=8)
    for j in range(12):                      # one new key per call: which insert is dropped is then well defined
        key = torch.tensor([((j + 1) << 20) | (j + 100)], dtype=torch.int64, device="cuda")
        wt = torch.tensor([j + 1], dtype=torch.int32, device="cuda")
        csd.csd_ocm_update(ocm, key, wt, status)
        orc.ocm_update([(j + 1, j + 100)], [j + 1])
    compare_table(ocm, orc)
    assert int(status[csd.CSD_STATUS_DROPPED]) == orc.dropped == 9 + 10 + 11 + 12
    # existing keys are still updated and found in a full table; absent keys read 0
    keys = torch.tensor([(3 << 20) | 102, (12 << 20) | 111], dtype=torch.int64, device="cuda")
    csd.csd_ocm_update(ocm, keys[:1], None, status)
    assert csd.csd_ocm_lookup(ocm, keys).cpu().tolist() == [4, 0]
    csd.csd_ocm_reset(ocm)
    assert decode_ocm(ocm) == {}


def test_ocm_merge_export_rehash_roundtrip():
    """Life cycle of the memory: export as a list, reload the list, grow by merging into a larger table,
    fold two memories calibrated separately."""
    rng = np.random.default_rng(12)
    def random_memory(n, seed):
        r = np.random.default_rng(seed)
        d = r.integers(0, 3000, size=n)
        t = (d + 1 + r.integers(0, 40, size=n)) % 3000
        keep = d != t
        d, t = d[keep], t[keep]
        wts = r.integers(1, 1000, size=d.size).astype(np.int32)
        orc = O.CSDOracle()
        orc.ocm_update(zip(d.tolist(), t.tolist()), wts.tolist())
        ocm = csd.new_ocm(1 << 15)
        csd.csd_ocm_update(ocm, torch.from_numpy((d.astype(np.int64) << 20) | t.astype(np.int64)).cuda(),
                           torch.from_numpy(wts).cuda())
        return orc, ocm
    orc_a, ocm_a = random_memory(9000, 1)
    orc_b, ocm_b = random_memory(7000, 2)
    compare_table(ocm_a, orc_a, "a")
    # export: the same pairs and counts as the oracle's dict, any order
    keys, counts, n = csd.csd_ocm_export(ocm_a)
    n = int(n.item())
    assert n == len(orc_a.T)
    got = {(int(x) >> 20, int(x) & 0xFFFFF): int(c) for x, c in zip(keys[:n].cpu().tolist(), counts[:n].cpu().tolist())}
    assert got == orc_a.ocm_export()
    # count-only call, and a list shorter than the table
    _, _, n0 = csd.csd_ocm_export(ocm_a, max_entries=0)
    assert int(n0.item()) == n
    k5, c5, n5 = csd.csd_ocm_export(ocm_a, max_entries=5)
    assert int(n5.item()) == n
    assert all(got[(int(x) >> 20, int(x) & 0xFFFFF)] == int(c) for x, c in zip(k5.cpu().tolist(), c5.cpu().tolist()))
    # the exported list reloads into an empty table of another size
    ocm_c = csd.new_ocm(1 << 14)
    csd.csd_ocm_update(ocm_c, keys[:n], counts[:n])
    compare_table(ocm_c, orc_a, "reloaded")
    # growth: a larger empty table takes the old one
    big = csd.new_ocm(1 << 17)
    status = torch.zeros(csd.CSD_STATUS_WORDS, dtype=torch.int32, device="cuda")
    csd.csd_ocm_merge(big, ocm_a, status)
    compare_table(big, orc_a, "grown")
    # folding a second memory in: counts of common pairs add
    csd.csd_ocm_merge(big, ocm_b, status)
    orc_a.ocm_merge(orc_b)
    compare_table(big, orc_a, "folded")
    assert len(set(orc_b.T) & set(orc_a.T)) > 0 and int(status[csd.CSD_STATUS_DROPPED]) == 0
    # saturation carries through a merge
    sat = csd.new_ocm(16)
    csd.csd_ocm_update(sat, torch.tensor([(5 << 20) | 6], dtype=torch.int64, device="cuda"),
                       torch.tensor([csd.CSD_OCM_COUNT_MAX - 3], dtype=torch.int32, device="cuda"))
    sat2 = sat.clone()
    csd.csd_ocm_merge(sat, sat2)
    assert decode_ocm(sat) == {(5, 6): csd.CSD_OCM_COUNT_MAX}


def test_exported_list_reloads_by_its_device_side_length():
    """csd_ocm_export leaves the list's length on the device; csd_ocm_update takes it from there (n_dev), so a
    memory is copied, grown or folded without the host ever learning the length - eagerly, and replayed from a
    captured graph while the source memory keeps changing between replays."""
    rng = np.random.default_rng(77)
    orc = O.CSDOracle()
    src = csd.new_ocm(1 << 13)

    def grow_source(n):
        d = rng.integers(0, 2000, size=n)
        t = (d + 1 + rng.integers(0, 30, size=n)) % 2000
        keep = d != t
        d, t = d[keep], t[keep]
        wts = rng.integers(1, 50, size=d.size).astype(np.int32)
        orc.ocm_update(zip(d.tolist(), t.tolist()), wts.tolist())
        csd.csd_ocm_update(src, torch.from_numpy((d.astype(np.int64) << 20) | t.astype(np.int64)).cuda(), torch.from_numpy(wts).cuda())

    grow_source(3000)
    cap = src.numel()
    bufs = (torch.empty(cap, dtype=torch.int64, device="cuda"), torch.empty(cap, dtype=torch.int32, device="cuda"),
            torch.empty(1, dtype=torch.int64, device="cuda"))
    # eager: export, then reload into a larger table; the host never reads n
    dst = csd.new_ocm(1 << 15)
    keys, counts, n = csd.csd_ocm_export(src, out=bufs)
    csd.csd_ocm_update(dst, keys, counts, n_dev=n)
    torch.cuda.synchronize()
    compare_table(dst, orc, "reloaded by device-side length")
    # the device-side length never reaches past the arrays handed in
    few = csd.new_ocm(1 << 10)
    csd.csd_ocm_update(few, keys[:100], counts[:100], n_dev=n)
    assert len(decode_ocm(few)) == 100
    zero = torch.zeros(1, dtype=torch.int64, device="cuda")
    csd.csd_ocm_update(few, keys, counts, n_dev=zero)
    assert len(decode_ocm(few)) == 100
    # captured: reset the copy, export the source, reload - replayed while the source grows
    copy = csd.new_ocm(1 << 14)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up outside the capture
        csd.csd_ocm_reset(copy)
        csd.csd_ocm_export(src, out=bufs)
        csd.csd_ocm_update(copy, bufs[0], bufs[1], n_dev=bufs[2])
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        csd.csd_ocm_reset(copy)
        csd.csd_ocm_export(src, out=bufs)
        csd.csd_ocm_update(copy, bufs[0], bufs[1], n_dev=bufs[2])
    for rep in range(4):
        g.replay()
        torch.cuda.synchronize()
        compare_table(copy, orc, "graph replay %d" % rep)
        grow_source(500)                                # eager work between the replays: the list gets longer
    assert len(orc.T) > 3000


def test_two_streams_share_one_memory():
    """Concurrent verification calls on one table (each with its own buffers and stream): counts stay
    exact.  With a threshold no count can reach, no lookup can change an outcome, so the result is the
    oracle's whatever the interleaving."""
    lam = 2 ** 32 - 1
    wa, wb = Workload(CONFIGS[4], V=4000, B=48), Workload(CONFIGS[4], V=4000, B=48, seed=5)
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    steps = 25
    ins = []
    for step in range(steps):
        za, da = wa.step(step)
        zb, db = wb.step(step)
        ins.append((za, da, zb, db, to_device_logits(za), torch.from_numpy(da).cuda(), to_device_logits(zb),
                    torch.from_numpy(db).cuda()))
    torch.cuda.synchronize()
    bfa = bfb = None
    outs = []
    for za, da, zb, db, zta, dta, ztb, dtb in ins:                  # both streams run ahead without host syncs
        with torch.cuda.stream(sa):
            bfa = csd.csd_verify(zta, dta, 0.3, lam, ocm, buffers=bfa)
            outs.append(bfa.accept_len.clone())
        with torch.cuda.stream(sb):
            bfb = csd.csd_verify(ztb, dtb, 0.3, lam, ocm, buffers=bfb)
            outs.append(bfb.accept_len.clone())
    torch.cuda.synchronize()
    j = 0
    for za, da, zb, db, *_ in ins:
        for z, d in ((za, da), (zb, db)):
            res = orc.verify_step(z, d, tau=np.float32(0.3), lam=lam)
            np.testing.assert_array_equal(outs[j].cpu().numpy(), res.accept_len)
            j += 1
    compare_table(ocm, orc, "two streams")


def test_ablation_ordering_on_one_memory():
    """Per sequence, on the same frozen memory: strict <= full method <= min(memory only, gate only);
    the acceptance counter of the status block equals the sum of the accept lengths."""
    w = Workload(CONFIGS[2], V=6000, B=64)
    cfg = w.cfg
    prior = _prior_from_pairs(w, cfg.lam, n=600)
    ocm = csd.new_ocm(1 << 13)
    csd.csd_ocm_update(ocm, torch.tensor([(d << 20) | t for d, t in prior[0]], dtype=torch.int64, device="cuda"),
                       torch.tensor(prior[1], dtype=torch.int32, device="cuda"))
    seen_rescue = False
    for step in range(8):
        z, draft = w.step(step)
        zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
        def run(tau, lam, table):
            bf = csd.csd_verify(zt, dt, tau, lam, table, flags=0)
            torch.cuda.synchronize()
            assert int(bf.status[csd.CSD_STATUS_ACCEPTED]) == int(bf.accept_len.sum())
            return bf.accept_len.cpu().numpy().copy()
        strict = run(cfg.tau, cfg.lam, None)
        full = run(cfg.tau, cfg.lam, ocm)
        mem_only = run(0.0, cfg.lam, ocm)
        gate_only = run(cfg.tau, 0, ocm)
        assert np.all(strict <= full) and np.all(full <= np.minimum(mem_only, gate_only))
        seen_rescue |= bool(np.any(full > strict))
    assert seen_rescue


def test_verify_on_a_side_stream():
    w = Workload(CONFIGS[1], V=5000)
    cfg = w.cfg
    z, draft = w.step(0)
    s = torch.cuda.Stream()
    zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        ocm = csd.new_ocm(1 << 12)
        bf = csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm)
    s.synchronize()
    orc = O.CSDOracle()
    compare_step(orc.verify_step(z, draft, tau=np.float32(cfg.tau), lam=cfg.lam), bf, "side stream")
    compare_table(ocm, orc)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_partials_combine_to_the_row_statistics(dtype):
    """csd_row_partials alone: combining the documented records on the host (fp64) gives the oracle's
    m, t*, S - also when the rows are two vocabulary shards merged with an index offset."""
    rng = np.random.default_rng(31)
    rows, V = 37, 48008
    z = (rng.standard_normal((rows, V)) * 3).astype(np.float32)
    z[np.arange(rows), rng.integers(0, V, rows)] += 9.0
    if dtype == "bf16":
        z = f32_to_bf16_bits(z).reshape(rows, V)
    m, t, S = O.row_stats(z)
    L = float(np.float32(1.4426950408889634))

    def combine(recs, offsets):
        mm = max(float(r[0]) for r in recs)
        idx = min(int(r[3]) + off for r, off in zip(recs, offsets) if float(r[0]) == mm)
        tot = sum(float(r[2]) * 2.0 ** (float(r[1]) - mm * L) for r in recs if float(r[2]) != 0.0)
        return mm, idx, tot

    def records(part_row):
        f = part_row.view(np.float32)
        return [(f[j, 0], f[j, 1], f[j, 2], part_row[j, 3]) for j in range(part_row.shape[0])]

    part = csd.csd_row_partials(to_device_logits(z))
    torch.cuda.synchronize()
    part = part.cpu().numpy()
    assert part.shape[1] == csd.csd_row_partials_per_row(rows, V, 0 if dtype == "f32" else 1)
    for r in range(rows):
        mm, idx, tot = combine(records(part[r]), [0] * part.shape[1])
        assert mm == m[r] and idx == t[r]
        assert tot == pytest.approx(S[r], rel=1e-5)

    # two shards of the vocabulary, reduced separately, merged with the shard base added to idx
    half = 24000
    pa = csd.csd_row_partials(to_device_logits(np.ascontiguousarray(z[:, :half]))).cpu().numpy()
    pb = csd.csd_row_partials(to_device_logits(np.ascontiguousarray(z[:, half:]))).cpu().numpy()
    for r in range(rows):
        recs = records(pa[r]) + records(pb[r])
        offs = [0] * pa.shape[1] + [half] * pb.shape[1]
        mm, idx, tot = combine(recs, offs)
        assert mm == m[r] and idx == t[r]
        assert tot == pytest.approx(S[r], rel=1e-5)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_verify_from_vocabulary_shards(dtype):
    """The vocabulary cut into three uneven shards, each reduced on its own (row partials + the logits of the
    draft tokens it owns), then one csd_verify_shards call: same step as the oracle on the whole rows."""
    cfg = CONFIGS[2] if dtype == "bf16" else CONFIGS[3]
    w = Workload(cfg, V=30008, B=24, n_pairs=200)
    cfg = w.cfg
    cuts = [0, 8199, 21003, cfg.V]                     # ragged shard widths: padded row pitches
    orc = O.CSDOracle()
    ocm = csd.new_ocm(1 << 12)
    prior = _prior_from_pairs(w, cfg.lam, n=100)
    orc.ocm_update(*prior)
    csd.csd_ocm_update(ocm, torch.tensor([(d << 20) | t for d, t in prior[0]], dtype=torch.int64, device="cuda"),
                       torch.tensor(prior[1], dtype=torch.int32, device="cuda"))
    bf = None
    for step in range(6):
        z, draft = w.step(step)
        dt = torch.from_numpy(draft).cuda()
        zd = torch.full((cfg.B, cfg.k), float("nan"), dtype=torch.float32, device="cuda")
        parts = []
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            shard = to_device_logits(np.ascontiguousarray(z[..., lo:hi]))
            parts.append(csd.csd_row_partials(shard))
            csd.csd_shard_draft_logits(shard, lo, dt, zd)
        bf = csd.csd_verify_shards(parts, cuts[:-1], zd, dt, cfg.V, cfg.tau, cfg.lam, ocm, buffers=bf)
        torch.cuda.synchronize()
        res = orc.verify_step(z, draft, tau=np.float32(cfg.tau), lam=cfg.lam)
        compare_step(res, bf, "shards step %d" % step)
        compare_table(ocm, orc, "shards step %d" % step)
    assert int(bf.status[csd.CSD_STATUS_RESCUED]) > 0


def test_workspace_needs_no_initialisation_and_is_reusable_across_shapes():
    """One workspace, full of garbage at first, serves calls of different shapes back to back."""
    rng = np.random.default_rng(41)
    shapes = [(5, 3, 9000, "bf16"), (2, 7, 40000, "f32"), (9, 1, 3000, "bf16"), (5, 3, 9000, "bf16")]
    need = max(csd.csd_verify_workspace_bytes(B, k, V, 0 if dt == "f32" else 1) for B, k, V, dt in shapes)
    ws = torch.full((need,), 0xAB, dtype=torch.uint8, device="cuda")      # garbage
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    for rep in range(3):
        for B, k, V, dt in shapes:
            z = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
            if dt == "bf16":
                z = f32_to_bf16_bits(z).reshape(B, k + 1, V)
            am = np.stack([O.row_stats(z)[1]])[0][:, :k]
            draft = np.where(rng.random((B, k)) < 0.5, am, rng.integers(0, 64, size=(B, k))).astype(np.int32)
            bf = csd.VerifyBuffers.allocate(B, k, V, 0 if dt == "f32" else 1)
            bf.workspace = ws
            csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), 0.05, 1, ocm, buffers=bf)
            torch.cuda.synchronize()
            res = orc.verify_step(z, draft, tau=np.float32(0.05), lam=1)
            compare_step(res, bf, "shape %r rep %d" % ((B, k, V, dt), rep))
    compare_table(ocm, orc)


def test_step_replayed_from_a_captured_graph():
    """A verification step allocates nothing and records only kernel launches, so it can be captured in a
    graph; several replays, with new inputs copied into the captured buffers and eager work in between,
    each match the oracle (memory updates included)."""
    w = Workload(CONFIGS[1], V=12000, B=8)
    cfg = w.cfg
    z0, d0 = w.step(0)
    zt = to_device_logits(z0)
    dt = torch.from_numpy(d0).cuda()
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    bf = csd.VerifyBuffers.allocate(cfg.B, cfg.k, cfg.V, csd.CSD_DTYPE_BF16)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture, then undo its updates
        csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm, buffers=bf)
        csd.csd_ocm_reset(ocm)
        bf.status.zero_()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        csd.csd_verify(zt, dt, cfg.tau, cfg.lam, ocm, buffers=bf)
    for step in range(5):
        z, d = w.step(step)
        zt.copy_(to_device_logits(z))
        dt.copy_(torch.from_numpy(d).cuda())
        g.replay()
        torch.cuda.synchronize()
        res = orc.verify_step(z, d, tau=np.float32(cfg.tau), lam=cfg.lam)
        compare_step(res, bf, "graph replay %d" % step)
        compare_table(ocm, orc, "graph replay %d" % step)
        assert int(csd.csd_ocm_lookup(ocm, torch.tensor([(1 << 20) | 2], dtype=torch.int64, device="cuda"))[0]) >= 0   # eager work between replays


def test_prepared_calls_run_the_same_step():
    """prepare_verify checks and marshals the arguments once; launch() then only makes the C call.  A stream run
    through one prepared call, its logits and draft tokens refilled in place, matches the oracle step by step -
    on the caller's workspace and on the library's static scratch."""
    w = Workload(CONFIGS[1], V=9001, B=6)
    cfg = w.cfg
    z0, d0 = w.step(0)
    zt, dt = to_device_logits(z0), torch.from_numpy(d0).cuda()
    for static in (False, True):
        ocm = csd.new_ocm(1 << 12)
        orc = O.CSDOracle()
        call = csd.prepare_verify(zt, dt, cfg.tau, cfg.lam, ocm, static_scratch=static)
        for step in range(8):
            z, d = w.step(step)
            zt.copy_(to_device_logits(z))
            dt.copy_(torch.from_numpy(d).cuda())
            bf = call.launch()
            torch.cuda.synchronize()
            compare_step(orc.verify_step(z, d, tau=np.float32(cfg.tau), lam=cfg.lam), bf, "prepared step %d" % step)
        compare_table(ocm, orc, "prepared, static=%s" % static)
    with pytest.raises(ValueError):
        csd.prepare_verify(zt, dt[:, :-1].contiguous(), cfg.tau, cfg.lam, ocm)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_largest_vocabulary_and_smallest_table(dtype):
    """V = 2^20 (the largest the packed pair allows), with the top token at the very end and a tie across
    the row; a memory of one slot (every second pair is dropped and reported)."""
    V = csd.CSD_MAX_V
    rng = np.random.default_rng(17)
    z = (rng.standard_normal((2, 2, V)) * 2).astype(np.float32)
    z[0, 0, V - 1] = 15.0
    z[0, 0, 3] = 15.0                                   # tie between token 3 and the last token
    z[0, 1, V - 1] = 14.0
    z[1, 0, V - 2] = 16.0
    z[1, 1, 12345] = 16.0
    if dtype == "bf16":
        z = f32_to_bf16_bits(z).reshape(z.shape)
    draft = np.array([[V - 1], [V - 2]], dtype=np.int32)
    ocm = csd.new_ocm(1)
    orc = O.CSDOracle(capacity=1)
    bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), 0.3, 0, ocm)
    torch.cuda.synchronize()
    res = orc.verify_step(z, draft, tau=np.float32(0.3), lam=0)
    compare_step(res, bf, "V=2^20")
    assert bf.argmax.cpu().tolist() == [[3, V - 1], [V - 2, 12345]]
    assert decode_ocm(ocm) == {(V - 1, 3): 1} == orc.T          # the pair of sequence 0; sequence 1 matched
    # a second pair finds the single slot taken: dropped, and said so
    draft2 = np.array([[5], [7]], dtype=np.int32)
    bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft2).cuda(), 0.3, 0, ocm, buffers=bf)
    torch.cuda.synchronize()
    assert decode_ocm(ocm) == {(V - 1, 3): 1} and int(bf.status[csd.CSD_STATUS_DROPPED]) == 2
