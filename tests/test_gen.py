"""The synthetic workload generator: determinism, structure, threshold margin, mixture."""
import math

import numpy as np
import pytest

from gen import CONFIGS, Workload, bf16_bits_to_f32, f32_to_bf16_bits
from gen.workload import BRANCH_MATCH, BRANCH_SYNONYM, BRANCH_UNIFORM, MARGIN


def test_bf16_rounding_is_nearest_even_and_roundtrips():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625, 0.0, -0.0, 1e-20, 21.4375], dtype=np.float32)
    h = f32_to_bf16_bits(x)
    back = bf16_bits_to_f32(h)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert back[1] == 1.0 and back[2] == 1.015625
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    np.testing.assert_array_equal(f32_to_bf16_bits(back), h)
    assert np.signbit(back[6]) and back[6] == 0.0


@pytest.mark.parametrize("ci", [0, 1, 3])
def test_deterministic_and_thread_independent(ci):
    w = Workload(CONFIGS[ci], V=2048, B=3)
    z1, d1 = w.step(5)
    z2, d2 = w.step(5, threads=4)
    np.testing.assert_array_equal(z1, z2)
    np.testing.assert_array_equal(d1, d2)
    z3, d3 = w.step(6)
    assert not np.array_equal(z1, z3)
    w2 = Workload(CONFIGS[ci], V=2048, B=3, seed=1)
    assert not np.array_equal(w2.step(5)[0], z1)


def test_full_config_shapes():
    for c in CONFIGS:
        assert c.rows == c.B * (c.k + 1)
    assert [c.bytes_per_step for c in CONFIGS] == [640000, 12312576, 77791232, 350355456, 655360000]
    w = Workload(CONFIGS[0])
    z, d = w.step(0)
    assert z.shape == (1, 5, 32000) and z.dtype == np.float32 and d.shape == (1, 4)
    assert len(w.pair_target) == 512 and np.all(w.pair_target != w.pair_draft)
    assert len({(int(a), int(b)) for a, b in zip(w.pair_target, w.pair_draft)}) == 512


@pytest.mark.parametrize("ci", [0, 1, 2, 3, 4])
def test_structure_margin_and_mixture(ci):
    cfg = CONFIGS[ci]
    w = Workload(cfg, V=1024, B=16, n_pairs=min(cfg.n_pairs, 256))
    cfg = w.cfg
    pairs = {(int(t), int(d)) for t, d in zip(w.pair_target, w.pair_draft)}
    counts = np.zeros(3)
    for step in range(12):
        z, draft, meta = w.step(step, return_meta=True)
        zf = w.logits_as_f32(z).astype(np.float64)
        assert np.all(np.isfinite(zf))
        top = zf.max(axis=-1)
        am = zf.argmax(axis=-1)
        assert np.all((draft >= 0) & (draft < cfg.V))
        for b in range(cfg.B):
            for i in range(cfg.k):
                br = meta[b, i]
                counts[br] += 1
                d = draft[b, i]
                ratio = math.exp(zf[b, i, d] - top[b, i])
                assert abs(ratio - cfg.tau) >= MARGIN
                if br == BRANCH_SYNONYM:
                    # draft and (unless a storage tie moved it) target come from the pair map
                    assert any(dd == d for _, dd in pairs)
                    assert ratio > math.exp(-3.2)
                elif br == BRANCH_UNIFORM and not cfg.two_peak:
                    assert ratio < math.exp(-7.0)
                elif br == BRANCH_MATCH and not cfg.two_peak:
                    assert am[b, i] == d
        # the planted top stands 8 above the noise (up to storage rounding)
        srt = np.sort(zf, axis=-1)
        gap = srt[..., -1] - srt[..., -3]
        assert np.all(gap > 7.5)
    frac = counts / counts.sum()
    n = counts.sum()
    for f, p in zip(frac, cfg.mix):
        assert abs(f - p) < 4.0 * math.sqrt(p * (1 - p) / n) + 1e-9


def test_two_peak_rows_have_exact_ties_sometimes():
    w = Workload(CONFIGS[3], V=512, B=32)
    ties = 0
    total = 0
    for step in range(6):
        z, _ = w.step(step)
        srt = np.sort(z.astype(np.float64), axis=-1)
        ties += int(np.sum(srt[..., -1] == srt[..., -2]))
        total += srt.shape[0] * srt.shape[1]
        assert np.all(srt[..., -1] - srt[..., -2] <= 1.0 + 1e-6)
    assert 0 < ties < 0.15 * total


def test_zipf_head_is_heavy():
    w = Workload(CONFIGS[4], V=4096, B=64)
    seen = {}
    for step in range(10):
        z, draft, meta = w.step(step, return_meta=True)
        for b in range(w.cfg.B):
            for i in range(w.cfg.k):
                if meta[b, i] == BRANCH_SYNONYM:
                    seen[int(draft[b, i])] = seen.get(int(draft[b, i]), 0) + 1
    top = max(seen.values())
    assert top > 0.3 * sum(seen.values())          # Zipf(1.5): rank 1 carries about 40 %


def test_sampled_workload_is_seeded_and_shaped():
    """Draft-model rows and uniforms of the sampling-temperature workload: deterministic by seed and step,
    target rows identical to the greedy workload's, the drafted token on top of its draft row, the target's
    top token planted below it, uniforms in [0, 1)."""
    from gen.workload import SampledWorkload
    for ci in (0, 1):
        w = SampledWorkload(CONFIGS[ci], V=3001, B=3)
        cfg = w.cfg
        zp, zq, d, ua, ud = w.sampled_step(5)
        zp2, zq2, d2, ua2, ud2 = SampledWorkload(CONFIGS[ci], V=3001, B=3).sampled_step(5)
        for a, b in ((zp, zp2), (zq, zq2), (d, d2), (ua, ua2), (ud, ud2)):
            assert np.array_equal(a, b)
        z_greedy, d_greedy = Workload(CONFIGS[ci], V=3001, B=3).step(5)
        assert np.array_equal(zp, z_greedy) and np.array_equal(d, d_greedy)
        assert zp.shape == (cfg.B, cfg.k + 1, cfg.V) and zq.shape == (cfg.B, cfg.k, cfg.V)
        assert ua.shape == (cfg.B, cfg.k) and ud.shape == (cfg.B, cfg.k + 1) and ua.dtype == np.float32
        assert (ua >= 0).all() and (ua < 1).all() and (ud >= 0).all() and (ud < 1).all()
        qf, pf = w.logits_as_f32(zq), w.logits_as_f32(zp)
        assert np.array_equal(qf.argmax(-1), d)                          # the draft model is sure of what it drafted
        top = pf[:, :cfg.k].argmax(-1)
        differs = top != d
        second = np.take_along_axis(qf, top[..., None], -1)[..., 0]
        assert np.all(second[differs] > qf.max(-1)[differs] - 3.2)       # the target's choice sits within 3 below
        assert not np.array_equal(w.sampled_step(6)[1], zq)
