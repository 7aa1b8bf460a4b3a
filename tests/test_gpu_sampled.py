"""GPU parity of csd_verify_sampled (verification at a sampling temperature) against the fp64 oracle."""
import numpy as np
import pytest
import torch

from gen import CONFIGS, f32_to_bf16_bits
from gen.workload import SampledWorkload
from oracle import csd_oracle as O
from oracle import csd_oracle_sampled as OS
from paper_2604_13634_amd import binding as csd
from parity_util import (DrawStats, check_sampled_step, compare_table, decode_ocm, run_sampled_stream, settle_uniforms,
                         to_device_logits)

pytestmark = pytest.mark.gpu


def _prior(w, lam, n):
    pairs = [(int(d), int(t)) for t, d in zip(w.pair_target[:n], w.pair_draft[:n])]
    return pairs, [lam] * len(pairs)


@pytest.mark.parametrize("ci,V,T,steps", [(0, 3000, 1.0, 60), (1, 4099, 0.6, 40), (2, 8200, 1.0, 25), (3, 3001, 0.8, 20),
                                          (4, 2048 + 6, 1.0, 25), (1, 5000, 2.5, 20), (2, 4000, 0.3, 20)])
def test_streams_reduced_vocab(ci, V, T, steps):
    """The five configurations' batch, k, thresholds, pair skew and storage type on a reduced, ragged
    vocabulary, memory evolving from empty."""
    cfg = CONFIGS[ci]
    w = SampledWorkload(cfg, V=V, n_pairs=min(cfg.n_pairs, 256), B=min(cfg.B, 64))
    orc, ocm, rescued, counted, rejected = run_sampled_stream(w, range(steps), T)
    assert rejected > steps and counted > 0


@pytest.mark.parametrize("ci", [1, 2])
def test_full_size_step_with_prior(ci):
    """Full-size shapes of configurations 1 and 2, one or two steps, memory pre-loaded so that rescues occur."""
    w = SampledWorkload(CONFIGS[ci])
    prior = _prior(w, w.cfg.lam, min(512, w.cfg.n_pairs))
    orc, ocm, rescued, counted, rejected = run_sampled_stream(w, range(2 if ci == 1 else 1), 1.0, prior=prior,
                                                              check_table_every=1, threads=16)
    assert rejected > 0


@pytest.mark.parametrize("ci", [3, 4])
def test_full_size_step_of_the_large_configurations(ci):
    """Configurations 3 and 4 at full size (config 4 is the shape bench.py --path sampled times), one step."""
    w = SampledWorkload(CONFIGS[ci])
    prior = _prior(w, w.cfg.lam, min(512, w.cfg.n_pairs))
    orc, ocm, rescued, counted, rejected = run_sampled_stream(w, range(1), 1.0, prior=prior, check_table_every=1,
                                                              threads=16)
    assert rejected > 0 and counted > 0


def _one_step(zp, zq, draft, T, ua, ud, tau=0.3, lam=0, stats=None):
    ua, ud = settle_uniforms(zp, zq, draft, T, ua, ud, seed=1)
    orc = O.CSDOracle()
    ocm = csd.new_ocm(1 << 10)
    bf = csd.csd_verify_sampled(to_device_logits(zp), to_device_logits(zq), torch.from_numpy(draft).cuda(), T,
                                torch.from_numpy(ua.astype(np.float32)).cuda(), torch.from_numpy(ud.astype(np.float32)).cuda(),
                                tau, lam, ocm)
    torch.cuda.synchronize()
    res = check_sampled_step(orc, zp, zq, draft, T, ua, ud, np.float32(tau), lam, bf, "V=%d T=%g" % (zp.shape[-1], T), stats)
    compare_table(ocm, orc)
    assert int(bf.status[csd.CSD_STATUS_BAD_DRAFT]) == orc.bad_draft
    return bf, res


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1, 2, 3, 5, 8, 9, 17, 255, 1023, 1025, 2049, 4097, 8193, 40000, 70001])
def test_ragged_vocab_sizes(dtype, V):
    rng = np.random.default_rng(V)
    B, k = 3, 3
    zp = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
    zq = (zp[:, :k] + rng.standard_normal((B, k, V)).astype(np.float32) * 1.5).astype(np.float32)
    if dtype == "bf16":
        zp, zq = f32_to_bf16_bits(zp).reshape(zp.shape), f32_to_bf16_bits(zq).reshape(zq.shape)
    draft = rng.integers(0, V, (B, k)).astype(np.int32)
    bf, res = _one_step(zp, zq, draft, 0.9, rng.random((B, k), dtype=np.float32), rng.random((B, k + 1), dtype=np.float32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_diffuse_residuals_draws_near_boundaries(dtype):
    """Residuals spread over tens of thousands of tokens (two unrelated flat-ish models at a high temperature): a
    token holds about 1e-5 of the mass, so most draws land within the tolerance of a boundary of the running sum.
    None is dropped: each must be one of the tokens the oracle's running sum allows, and what follows is compared
    on that branch.  Uniforms at the very ends of [0, 1) and exact segment starts are among the draws."""
    rng = np.random.default_rng(61)
    B, k, V = 12, 4, 131072 + 37
    stats = DrawStats()
    for T in (2.0, 5.0):
        zp = (rng.standard_normal((B, k + 1, V)) * 1.2).astype(np.float32)
        zq = (rng.standard_normal((B, k, V)) * 1.2).astype(np.float32)
        if dtype == "bf16":
            zp, zq = f32_to_bf16_bits(zp).reshape(zp.shape), f32_to_bf16_bits(zq).reshape(zq.shape)
        draft = rng.integers(0, V, (B, k)).astype(np.int32)
        ua = np.ones((B, k), np.float32) * 0.999           # alpha is about 1 or well below: most positions are rejected
        ud = rng.random((B, k + 1), dtype=np.float32)
        ud[0, :] = 0.0
        ud[1, :] = np.float32(1.0) - np.float32(2.0 ** -24)
        ud[2, :] = np.float32(0.5)
        ud[3, :] = np.float32(0.25)
        bf, res = _one_step(zp, zq, draft, T, ua, ud, tau=0.2, lam=0, stats=stats)
        assert int(res.rejected.sum()) > B * k // 4
    print("diffuse residuals (%s): %d draws, %d within tolerance of a boundary, %d resolved to the other neighbour" % (
        dtype, stats.draws, stats.near_boundary, stats.other_neighbour))
    assert stats.near_boundary > stats.draws // 4


def test_peaked_rows_many_rejections_and_temperatures():
    """Rows with a handful of heavy tokens (residual mass on few tokens): most draws have a wide margin, so
    rejections are really exercised; several temperatures."""
    rng = np.random.default_rng(5)
    B, k, V = 16, 5, 30011
    total_rej = 0
    for T in (0.25, 0.7, 1.0, 1.6, 4.0):
        zp = (rng.standard_normal((B, k + 1, V)) * 1.5).astype(np.float32)
        zq = (rng.standard_normal((B, k, V)) * 1.5).astype(np.float32)
        heavy = rng.integers(0, V, (B, k + 1, 6))
        np.put_along_axis(zp, heavy, (12 + rng.random((B, k + 1, 6)) * 4).astype(np.float32), axis=-1)
        np.put_along_axis(zq, heavy[:, :k, ::-1].copy(), (12 + rng.random((B, k, 6)) * 4).astype(np.float32), axis=-1)
        draft = heavy[:, :k, rng.integers(0, 6)].astype(np.int32)
        bf, res = _one_step(zp, zq, draft, T, rng.random((B, k), dtype=np.float32), rng.random((B, k + 1), dtype=np.float32),
                            tau=0.2, lam=0)
        total_rej += int(res.rejected.sum())
    assert total_rej > 40


def test_masked_vocabulary_bad_ids_and_equal_models():
    rng = np.random.default_rng(8)
    B, k, V = 6, 4, 9000
    zp = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
    zq = (zp[:, :k] + rng.standard_normal((B, k, V)).astype(np.float32)).astype(np.float32)
    zp[0, :, rng.random(V) < 0.6] = -np.inf                     # masked vocabulary in the target
    zq[1, :, rng.random(V) < 0.6] = -np.inf                     # ... and in the draft model
    zq[2] = zp[2, :k]                                           # equal models: every token accepted
    draft = rng.integers(0, V, (B, k)).astype(np.int32)
    draft[0, 0] = int(np.argmax(zp[0, 0]))                      # a finite entry of the masked row
    draft[1, :] = np.argmax(zq[1], axis=-1)                     # the draft model can only draft what it has not masked
    draft[3, 1] = V                                             # ids outside the vocabulary
    draft[4, 0] = -7
    ua = rng.random((B, k), dtype=np.float32)
    ua[2] = 1.0
    bf, res = _one_step(zp, zq, draft, 1.0, ua, rng.random((B, k + 1), dtype=np.float32))
    assert int(res.accept_len[2]) == k and int(bf.status[csd.CSD_STATUS_BAD_DRAFT]) >= 1


def test_no_draft_tokens_is_a_bonus_draw_and_empty_batch_is_a_noop():
    rng = np.random.default_rng(9)
    zp = (rng.standard_normal((5, 1, 7000)) * 3).astype(np.float32)
    zq = np.zeros((5, 0, 7000), np.float32)
    bf, res = _one_step(zp, zq, np.zeros((5, 0), np.int32), 0.8, np.zeros((5, 0), np.float32),
                        rng.random((5, 1), dtype=np.float32))
    np.testing.assert_array_equal(bf.next_token.cpu().numpy(), res.bonus_token)
    rc = csd.load_library().csd_verify_sampled(None, None, 0, 100, 100, None, 0, 2, 100, 1.0, None, None, 0.3, 2, None, 0, 0,
                                               None, None, None, None, None, None, None, None, None, None, None, None, 0, None)
    assert rc == csd.CSD_OK


def test_small_temperature_agrees_with_the_greedy_entry_point():
    """T -> 0 with a clear top token in every target row and a draft model certain of its token:
    csd_verify_sampled and csd_verify give the same accept lengths, emitted tokens, flags and memory."""
    rng = np.random.default_rng(2)
    B, k, V, T = 16, 5, 6000, 0.02
    ocm_g, ocm_s = csd.new_ocm(1 << 12), csd.new_ocm(1 << 12)
    pool = rng.integers(0, V, 40)                                  # few tokens, so that pairs recur and get rescued
    rescued = 0
    for step in range(30):
        zp = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
        top = pool[rng.integers(0, 40, (B, k + 1))]
        np.put_along_axis(zp, top[..., None], zp.max(-1, keepdims=True) + 3.0, axis=-1)
        draft = np.where(rng.random((B, k)) < 0.5, top[:, :k], pool[rng.integers(0, 40, (B, k))]).astype(np.int32)
        zd = zp[:, :k]                                             # a view: a divergent draft token sits 1.0 below the top
        off = np.where(draft == top[:, :k], 0.0, 1.0).astype(np.float32)
        np.put_along_axis(zd, draft[..., None].astype(np.int64), (zd.max(-1) - off)[..., None], axis=-1)
        zq = np.zeros((B, k, V), np.float32)
        np.put_along_axis(zq, draft[..., None].astype(np.int64), 30.0, axis=-1)
        zt, dt = to_device_logits(zp), torch.from_numpy(draft).cuda()
        g = csd.csd_verify(zt, dt, 0.3, 2, ocm_g)
        s = csd.csd_verify_sampled(zt, to_device_logits(zq), dt, T,
                                   torch.from_numpy((rng.random((B, k)) * 0.9 + 0.05).astype(np.float32)).cuda(),
                                   torch.from_numpy((rng.random((B, k + 1)) * 0.9 + 0.05).astype(np.float32)).cuda(),
                                   0.3, 2, ocm_s)
        torch.cuda.synchronize()
        assert torch.equal(g.accept_len, s.accept_len) and torch.equal(g.next_token, s.next_token)
        assert torch.equal(g.pos_flags, s.pos_flags)
        rescued += int(s.status[csd.CSD_STATUS_RESCUED])
    assert rescued > 5
    assert decode_ocm(ocm_g) == decode_ocm(ocm_s) and len(decode_ocm(ocm_g)) > 10


@pytest.mark.parametrize("B,k,V", [(2200, 4, 520), (3, 31, 1500), (2, 63, 900), (300, 7, 1030), (2, 8, 700001), (5, 3, 300000)])
def test_large_batches_and_long_drafts(B, k, V):
    """More than 8192 draft positions (the separate update launch), k up to the limit (one lane per row in
    the sequence kernels), several merge batches of the in-kernel update; huge vocabularies under a small batch
    (more records per row than one round of loads takes, more segments per lane than the draw waves keep in
    registers)."""
    rng = np.random.default_rng(B + k)
    ocm = csd.new_ocm(1 << 13)
    orc = O.CSDOracle()
    bf = None
    heavy_n = 5
    for step in range(3):
        zp = (rng.standard_normal((B, k + 1, V)) * 1.5).astype(np.float32)
        zq = (rng.standard_normal((B, k, V)) * 1.5).astype(np.float32)
        heavy = rng.integers(0, 40, (B, k + 1, heavy_n))            # few tokens carry the mass: pairs recur
        np.put_along_axis(zp, heavy, (10 + rng.random((B, k + 1, heavy_n)) * 3).astype(np.float32), axis=-1)
        np.put_along_axis(zq, heavy[:, :k, ::-1].copy(), (10 + rng.random((B, k, heavy_n)) * 3).astype(np.float32), axis=-1)
        draft = heavy[:, :k, 0].astype(np.int32)
        ua, ud = settle_uniforms(zp, zq, draft, 1.0, rng.random((B, k), dtype=np.float32),
                                 rng.random((B, k + 1), dtype=np.float32), seed=step)
        bf = csd.csd_verify_sampled(to_device_logits(zp), to_device_logits(zq), torch.from_numpy(draft).cuda(), 1.0,
                                    torch.from_numpy(ua).cuda(), torch.from_numpy(ud).cuda(), 0.05, 1, ocm, buffers=bf)
        torch.cuda.synchronize()
        check_sampled_step(orc, zp, zq, draft, 1.0, ua, ud, np.float32(0.05), 1, bf, "B=%d k=%d step %d" % (B, k, step))
        compare_table(ocm, orc, "B=%d k=%d step %d" % (B, k, step))
    assert int(bf.status[csd.CSD_STATUS_COUNTED]) == sum(orc.T.values()) > 0


def test_prior_calibration_run_counts_without_rescuing():
    """Phase 1 of the memory: standard speculative sampling (here at T = 0.6) with the frequency threshold out
    of reach - nothing is rescued, every first divergence of a sequence is counted; the table it leaves is then
    the prior of a run with the method's thresholds."""
    w = SampledWorkload(CONFIGS[1], V=5003, B=32, n_pairs=64)
    cfg = w.cfg
    orc, ocm, rescued, counted, rejected = run_sampled_stream(w, range(25), 0.6, lam=2 ** 32 - 1, capacity=1 << 12)
    assert rescued == 0 and counted > 100
    # every sequence stops at its first failed acceptance test, so it counts at most one pair per step
    assert counted <= 25 * cfg.B
    before = dict(orc.T)
    orc2, ocm2, rescued2, _, _ = run_sampled_stream(w, range(25, 40), 0.6, lam=2, capacity=1 << 12,
                                                    prior=(list(before.keys()), list(before.values())))
    assert rescued2 > 0


def test_sampled_step_replayed_from_a_captured_graph():
    """The sampled step's three launches allocate nothing either: captured once, replayed with new logits, draft
    tokens and uniforms copied into the captured tensors and eager work in between; each replay matches the
    oracle, memory included.  (The replays run under one per-call number: the announcements and records of one
    replay must not pass for the next.)"""
    ws = SampledWorkload(CONFIGS[1], V=9001, B=12, n_pairs=16)
    cfg = ws.cfg
    T = 0.8

    def inputs(step):
        zp, zq, d, ua, ud = ws.sampled_step(step)
        ua, ud = settle_uniforms(zp, zq, d, T, ua, ud, seed=step)
        return zp, zq, d, ua, ud

    zp, zq, d, ua, ud = inputs(0)
    dev = [to_device_logits(zp), to_device_logits(zq), torch.from_numpy(d).cuda(), torch.from_numpy(ua).cuda(),
           torch.from_numpy(ud).cuda()]
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    bf = csd.SampledBuffers.allocate(cfg.B, cfg.k, cfg.V, csd.CSD_DTYPE_BF16)

    def call():
        return csd.csd_verify_sampled(dev[0], dev[1], dev[2], T, dev[3], dev[4], cfg.tau, 1, ocm, buffers=bf)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture, then undo its updates
        call()
        csd.csd_ocm_reset(ocm)
        bf.status.zero_()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    rejected = 0
    for step in range(6):
        zp, zq, d, ua, ud = inputs(step)
        for t, h in zip(dev, (to_device_logits(zp), to_device_logits(zq), torch.from_numpy(d).cuda(), torch.from_numpy(ua).cuda(),
                              torch.from_numpy(ud).cuda())):
            t.copy_(h)
        g.replay()
        torch.cuda.synchronize()
        check_sampled_step(orc, zp, zq, d, T, ua, ud, np.float32(cfg.tau), 1, bf, "sampled graph replay %d" % step)
        compare_table(ocm, orc, "sampled graph replay %d" % step)
        rejected += int((bf.tstar.cpu().numpy() >= 0).sum())
        assert len(decode_ocm(ocm)) >= 0               # eager work between replays
    assert rejected > 0 and int(bf.status[csd.CSD_STATUS_STALLED]) == 0
