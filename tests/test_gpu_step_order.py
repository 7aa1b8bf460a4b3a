"""GPU parity of csd_verify's second grid order (needs an MI355X).

A large step streams the bonus rows last: the loop, the barrier of the sequence workgroups and the updates run on
the draft positions' rows while the bonus rows are still being streamed, and one more set of workgroups takes the
bonus rows' statistics and the emitted token of sequences that kept every draft token.  The library picks that
order from the shape (from about 96 MB of bonus rows: the full-size steps of the largest configuration in
test_gpu_parity.py take it by themselves).  A test hook of the library (csd_test_set_step_order, not part of csd.h)
forces it on any shape with a draft position, so that the same element-by-element comparisons with the fp64 oracle
run on small and ragged shapes, on every update path and on the failure path, in seconds."""
import ctypes

import numpy as np
import pytest
import torch

import test_gpu_parity as P
from gen import CONFIGS, Workload
from oracle import csd_oracle as O
from paper_2604_13634_amd import binding as csd
from parity_util import compare_step, compare_table, to_device_logits

pytestmark = pytest.mark.gpu

ORDER_BY_SHAPE, ORDER_PLAIN, ORDER_BONUS_LAST = 0, 1, 2


def _set_order(order):
    lib = csd.load_library()
    lib.csd_test_set_step_order.restype = None
    lib.csd_test_set_step_order.argtypes = [ctypes.c_int]
    lib.csd_test_set_step_order(order)


@pytest.fixture
def bonus_rows_last():
    _set_order(ORDER_BONUS_LAST)
    try:
        yield
    finally:
        _set_order(ORDER_BY_SHAPE)


@pytest.mark.parametrize("ci,V,steps", [(1, 4099, 200), (2, 8200, 80), (3, 3001, 60), (4, 2048 + 6, 80)])
def test_streams_with_an_evolving_memory(bonus_rows_last, ci, V, steps):
    P.test_long_streams_reduced_vocab(ci, V, steps)


def test_config0_stream(bonus_rows_last):
    """One sequence workgroup (no barrier between workgroups), one workgroup for the bonus row."""
    w = Workload(CONFIGS[0])
    orc, ocm, rescued, counted = P.run_stream(w, range(300), check_table_every=50)
    assert counted > 100


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1, 5, 8, 17, 1025, 8193, 16389, 65537, 131109])
def test_ragged_vocab_sizes(bonus_rows_last, dtype, V):
    P.test_ragged_vocab_sizes(dtype, V)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ties_and_masked_rows(bonus_rows_last, dtype):
    P.test_ties_resolve_to_lowest_id_everywhere(dtype)
    P.test_masked_vocab_and_extreme_ranges(dtype)
    P.test_row_stride_larger_than_vocab(dtype)


@pytest.mark.parametrize("dtype,B,k,V", [("f32", 1, 4, 1 << 20), ("bf16", 300, 3, 5000)])
def test_huge_vocabulary_and_a_batch_past_the_barrier(bonus_rows_last, dtype, B, k, V):
    P.test_few_sequences_over_huge_vocabularies_and_batches_past_the_barrier(dtype, B, k, V)


def test_k_limits_modes_and_logs(bonus_rows_last):
    P.test_many_rows_and_k_limits()
    P.test_modes_strict_gate_only_memory_only()
    P.test_deferred_updates_through_rejection_log()
    P.test_bad_draft_ids_are_divergences_never_counted()


def test_waits_that_run_out(bonus_rows_last):
    """Every wait of the order runs out (records, the sequence word, the barrier): reported once per sequence and once
    per sequence workgroup as in the plain order, nothing accepted, memory untouched, next call fine."""
    P.test_waits_that_run_out_are_reported_and_leave_everything_usable()


def test_replay_from_a_captured_graph_and_static_scratch(bonus_rows_last):
    P.test_step_replayed_from_a_captured_graph()
    P.test_workspace_needs_no_initialisation_and_is_reusable_across_shapes()
    P.test_prepared_calls_run_the_same_step()


def test_every_sequence_keeps_all_its_draft_tokens(bonus_rows_last):
    """accept_len = k everywhere: every emitted token comes from the workgroups that take the bonus rows."""
    rng = np.random.default_rng(5)
    B, k, V = 37, 5, 10007
    z = rng.standard_normal((B, k + 1, V)).astype(np.float32)
    top = rng.integers(0, V, size=(B, k + 1))
    for b in range(B):
        for r in range(k + 1):
            z[b, r, top[b, r]] = 9.0
    draft = top[:, :k].astype(np.int32)
    ocm = csd.new_ocm(1 << 10)
    orc = O.CSDOracle()
    bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), 0.3, 2, ocm)
    torch.cuda.synchronize()
    res = orc.verify_step(z, draft, tau=np.float32(0.3), lam=2)
    compare_step(res, bf, "all accepted")
    assert bf.accept_len.cpu().tolist() == [k] * B and bf.next_token.cpu().tolist() == top[:, k].tolist()
    compare_table(ocm, orc, "all accepted")


def test_both_orders_agree_on_a_full_size_step():
    """The largest configuration's shape, one step, both orders forced in turn: identical outputs and memories."""
    w = Workload(CONFIGS[4])
    z, draft = w.step(0, threads=16)
    zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
    outs = []
    for order in (ORDER_PLAIN, ORDER_BONUS_LAST):
        _set_order(order)
        try:
            ocm = csd.new_ocm(w.cfg.capacity)
            pairs, weights = P._prior_from_pairs(w, w.cfg.lam)
            keys = torch.tensor([(d << 20) | t for d, t in pairs], dtype=torch.int64, device="cuda")
            csd.csd_ocm_update(ocm, keys, torch.tensor(weights, dtype=torch.int32, device="cuda"))
            bf = csd.csd_verify(zt, dt, w.cfg.tau, w.cfg.lam, ocm)
            torch.cuda.synchronize()
        finally:
            _set_order(ORDER_BY_SHAPE)
        outs.append((bf, P.decode_ocm(ocm)))
    (b0, t0), (b1, t1) = outs
    for name in ("accept_len", "next_token", "argmax", "pos_flags", "rej_log", "row_max", "row_sumexp", "ratio", "p_draft"):
        assert torch.equal(getattr(b0, name), getattr(b1, name)), name
    assert t0 == t1 and int(b0.status[csd.CSD_STATUS_RESCUED]) > 0


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_in_both_orders(seed):
    """Random small shapes (batches that are no multiple of four, k from 0 to 12, vocabularies from a handful of
    tokens to tens of thousands, both storage types, a few ids outside the vocabulary), four steps on the same
    inputs with a threshold of 1 so that pairs counted in one step are rescued in the next: every step and every
    memory against the oracle, in the plain order and with the bonus rows last."""
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 41))
    k = int(rng.integers(0, 13))
    V = int(rng.choice([3, 17, 260, 2049, 9001, 33000]))
    bf16 = bool(rng.integers(0, 2))
    z = (rng.standard_normal((B, k + 1, V)) * 2).astype(np.float32)
    top = z.argmax(axis=-1)
    m = z.max(axis=-1)
    draft = np.zeros((B, k), dtype=np.int32)
    for b in range(B):
        for i in range(k):
            u = rng.random()
            if u < 0.5 or V < 4:
                draft[b, i] = top[b, i]
            elif u < 0.9:                               # a planted neighbour: ratio 0.61 (passes 0.2) or 0.08 (does not)
                d = (int(top[b, i]) + 1 + int(rng.integers(0, 2))) % V
                z[b, i, d] = m[b, i] - (0.5 if u < 0.75 else 2.5)
                draft[b, i] = d
            elif u < 0.97:
                draft[b, i] = int(rng.integers(0, V))
            else:
                draft[b, i] = -1 if rng.random() < 0.5 else V + 3
    if bf16:
        z = P.f32_to_bf16_bits(z).reshape(B, k + 1, V)
    zt, dt = to_device_logits(z), torch.from_numpy(draft).cuda()
    for order in (ORDER_PLAIN, ORDER_BONUS_LAST):
        _set_order(order)
        try:
            ocm = csd.new_ocm(1 << 10)
            orc = O.CSDOracle()
            bf = None
            for step in range(4):
                bf = csd.csd_verify(zt, dt, 0.2, 1, ocm, buffers=bf)
                torch.cuda.synchronize()
                res = orc.verify_step(z, draft, tau=np.float32(0.2), lam=1)
                what = "seed %d B=%d k=%d V=%d %s order %d step %d" % (seed, B, k, V, "bf16" if bf16 else "f32", order, step)
                compare_step(res, bf, what)
                compare_table(ocm, orc, what)
            assert int(bf.status[csd.CSD_STATUS_STALLED]) == 0
        finally:
            _set_order(ORDER_BY_SHAPE)


def test_orders_alternate_on_one_workspace():
    """The same buffers and workspace, the grid order switched from call to call: what one order leaves behind (records,
    sequence words, the barrier's control head) never passes for the other's; every step against the oracle."""
    w = Workload(CONFIGS[2], V=6007, B=21)
    cfg = w.cfg
    ocm = csd.new_ocm(1 << 12)
    orc = O.CSDOracle()
    bf = None
    try:
        for step in range(8):
            _set_order(ORDER_BONUS_LAST if step % 2 else ORDER_PLAIN)
            z, draft = w.step(step)
            bf = csd.csd_verify(to_device_logits(z), torch.from_numpy(draft).cuda(), cfg.tau, 1, ocm, buffers=bf)
            torch.cuda.synchronize()
            res = orc.verify_step(z, draft, tau=np.float32(cfg.tau), lam=1)
            compare_step(res, bf, "alternating orders, step %d" % step)
            compare_table(ocm, orc, "alternating orders, step %d" % step)
    finally:
        _set_order(ORDER_BY_SHAPE)
    assert int(bf.status[csd.CSD_STATUS_STALLED]) == 0 and int(bf.status[csd.CSD_STATUS_RESCUED]) > 0
