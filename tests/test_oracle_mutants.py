"""The pins must bite: plausible mistakes planted in a copy of the oracle (on the CPU) each fail a pin.

A mutant is the oracle's source text with one edit, loaded as a throw-away module; the pin tests of
test_oracle_verify / test_oracle_rows are then run against it and at least one must fail.
"""
import os
import sys
import types

import pytest

import test_oracle_rows as rows_pins
import test_oracle_verify as verify_pins
from oracle import csd_oracle as O

_SRC = open(O.__file__.replace(".pyc", ".py")).read()
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

MUTANTS = [
    ("lookup_after_update", "snapshot.get((d, ts), 0) >= lam", "snapshot.get((d, ts), 0) + 1 >= lam"),
    ("exclusive_frequency_threshold", "snapshot.get((d, ts), 0) >= lam", "snapshot.get((d, ts), 0) > lam"),
    ("count_only_final_rejections", "pending.append((d, ts))                       # UpdateMemory: every processed divergence",
     "pending.append((d, ts)) if not (is_freq and ratio[b, i] >= tau) else None"),
    ("reversed_pair", "pending.append((d, ts))", "pending.append((ts, d))"),
    ("inverted_ratio", "math.exp(logit(z[b, i], d) - m[b, i])", "math.exp(m[b, i] - logit(z[b, i], d))"),
    ("gate_on_probability_not_ratio", "is_safe = ratio[b, i] >= tau", "is_safe = p_draft[b, i] >= tau"),
    ("rescue_needs_only_frequency", "if is_freq and is_safe:", "if is_freq:"),
    ("rescue_needs_only_gate", "if is_freq and is_safe:", "if is_safe:"),
    ("keep_scanning_after_stop", "                    flags[b, i] = f\n                    break",
     "                    flags[b, i] = f\n                    continue"),
    ("next_token_off_by_one", "next_token[b] = t[b, n]", "next_token[b] = t[b, min(n + 1, k)]"),
    ("immediate_updates_across_batch", "            log.append(pending)\n",
     "            log.append(pending)\n            self.ocm_update(pending) if apply_updates and use_ocm else None\n"
     "            pending = []\n            log[-1] = list(log[-1])\n"),
]

VERIFY_PINS = [
    lambda: verify_pins.test_worked_example(GOLDEN),
    lambda: verify_pins.test_matches_literal_algorithm1_single_sequence(6, 4, 2, 0.3),
    lambda: verify_pins.test_matches_literal_algorithm1_single_sequence(16, 5, 0, 0.6),
    verify_pins.test_tau_above_every_ratio_is_strict_matching,
    verify_pins.test_accept_len_bounded_by_strict_plus_rescues_and_flag_accounting,
    lambda: verify_pins.test_counts_equal_bruteforce_recount_of_logged_rejections(8, 5, 4),
    verify_pins.test_first_possible_rescue_is_occurrence_lambda_plus_one,
    verify_pins.test_pair_is_ordered_draft_then_target,
    verify_pins.test_positions_after_the_stop_are_neither_tested_nor_counted,
    verify_pins.test_batch_snapshot_lookups_precede_all_updates_of_the_step,
    rows_pins.test_eq3_ratio_identity_and_temperature_invariance,
]


def _load_mutant(old, new):
    assert _SRC.count(old) >= 1, "mutation site not found: " + old
    mod = types.ModuleType("csd_oracle_mutant")
    mod.__file__ = O.__file__
    sys.modules["csd_oracle_mutant"] = mod          # dataclasses look their module up by name
    exec(compile(_SRC.replace(old, new, 1), "csd_oracle_mutant", "exec"), mod.__dict__)
    return mod


def _failures(monkeypatch, mod):
    monkeypatch.setattr(verify_pins, "O", mod)
    monkeypatch.setattr(rows_pins, "O", mod)
    failed = 0
    for pin in VERIFY_PINS:
        try:
            pin()
        except (AssertionError, KeyError, IndexError):
            failed += 1
    return failed


def test_unmutated_copy_passes_every_pin(monkeypatch):
    assert _failures(monkeypatch, _load_mutant("snapshot = self.T", "snapshot = self.T ")) == 0


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, old, new):
    assert _failures(monkeypatch, _load_mutant(old, new)) >= 1, name


def test_planted_mistakes_in_row_statistics_are_caught(tmp_path, monkeypatch):
    """Edits to the C loops (last-max argmax, missing max subtraction) fail the row pins."""
    import ctypes
    import subprocess

    src = open(os.path.join(os.path.dirname(O.__file__), "csd_oracle_rows.c")).read()
    for old, new, pins in [
        ("if (x > m) {", "if (x >= m) {", [rows_pins.test_closed_form_two_equal_peaks,
                                            rows_pins.test_bf16_ties_resolve_to_lowest_id]),
        ("S += exp(widen(z, dtype, v) - m);", "S += exp(widen(z, dtype, v));",
         [rows_pins.test_closed_form_single_spike]),
        ("for (int64_t v = 0; v < V; ++v) {\n        S +=", "for (int64_t v = 1; v < V; ++v) {\n        S +=",
         [rows_pins.test_closed_form_constant_row]),
    ]:
        assert src.count(old) == 1
        c = tmp_path / "mut.c"
        so = tmp_path / ("mut%d.so" % abs(hash(new)))
        c.write_text(src.replace(old, new))
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
        lib = ctypes.CDLL(str(so))
        lib.csd_oracle_logit.restype = ctypes.c_double
        lib.csd_oracle_logit.argtypes = O._load().csd_oracle_logit.argtypes
        lib.csd_oracle_rows.restype = None
        lib.csd_oracle_rows.argtypes = O._load().csd_oracle_rows.argtypes
        monkeypatch.setattr(O, "_lib", lib)
        for pin in pins:
            with pytest.raises(AssertionError):
                pin()
        monkeypatch.undo()


# --------------------------------------------------------------------------- the sampling-temperature oracle
import test_oracle_sampled as sampled_pins
from oracle import csd_oracle_sampled as OS

_SRC_S = open(OS.__file__.replace(".pyc", ".py")).read()

MUTANTS_SAMPLED = [
    ("inverted_acceptance_ratio", "min(1.0, p[d] / q[d])", "min(1.0, q[d] / p[d])"),
    ("exclusive_acceptance_test", "if r <= res.alpha[b, i]:", "if r < res.alpha[b, i]:"),
    ("residual_sign", "w = np.maximum(0.0, p - q)", "w = np.maximum(0.0, q - p)"),
    ("residual_not_clamped", "w = np.maximum(0.0, p - q)", "w = np.abs(p - q)"),
    ("residual_is_target", "w = np.maximum(0.0, p - q)", "w = p"),
    ("inverse_cdf_boundary_rule", 'side="right"', 'side="left"'),
    ("gate_on_tempered_probabilities", "res.ratio[b, i] = np.exp(z[d] - z[t])", "res.ratio[b, i] = p[d] / p[t]"),
    ("inverted_gate_ratio", "res.ratio[b, i] = np.exp(z[d] - z[t])", "res.ratio[b, i] = np.exp(z[t] - z[d])"),
    ("temperature_ignored", "e = np.exp((z64 - m) / T)", "e = np.exp(z64 - m)"),
    ("lookup_after_update", "snapshot.get((d, ts), 0) >= lam", "snapshot.get((d, ts), 0) + 1 >= lam"),
    ("reversed_pair", "pending.append((d, ts))", "pending.append((ts, d))"),
    ("count_only_final_rejections", "            pending.append((d, ts))\n", "            pending.append((d, ts)) if not (is_freq and is_safe) else None\n"),
    ("bonus_from_wrong_row", "pk = softmax_T(widen(zp[b, k]), T)", "pk = softmax_T(widen(zp[b, k - 1]), T)"),
    ("emits_draft_token_on_stop", "                res.next_token[b] = ts\n", "                res.next_token[b] = d\n"),
    ("rescue_needs_only_gate", "if is_freq and is_safe:", "if is_safe:"),
    ("keeps_going_after_stop", "                res.next_token[b] = ts\n                stopped = True\n                break",
     "                res.next_token[b] = ts\n                stopped = True\n                continue"),
    ("invalid_id_emits_the_bonus_draw", "                res.next_token[b] = int(np.argmax(widen(zp[b, i])))\n                stopped = True\n",
     "                res.next_token[b] = int(np.argmax(widen(zp[b, i])))\n                stopped = False\n"),
    ("invalid_id_emits_argmax_of_the_wrong_row", "res.next_token[b] = int(np.argmax(widen(zp[b, i])))",
     "res.next_token[b] = int(np.argmax(widen(zp[b, 0])))"),
    ("invalid_id_is_skipped_not_a_stop", "                res.next_token[b] = int(np.argmax(widen(zp[b, i])))\n                stopped = True\n                break",
     "                res.next_token[b] = int(np.argmax(widen(zp[b, i])))\n                stopped = True\n                continue"),
    ("empty_residual_reports_token_zero", "                t = int(np.argmax(z))                 # no residual mass: the target's own choice",
     "                t = 0"),
]

SAMPLED_PINS = [
    sampled_pins.test_worked_example,
    sampled_pins.test_inverse_cdf_against_a_plain_loop_and_its_edges,
    lambda: sampled_pins.test_emitted_token_follows_the_target_distribution(5, 1.0, 0),
    lambda: sampled_pins.test_emitted_token_follows_the_target_distribution(7, 0.6, 1),
    sampled_pins.test_bonus_token_follows_p_of_the_last_row,
    sampled_pins.test_small_temperature_reduces_to_the_greedy_oracle,
    sampled_pins.test_gate_uses_raw_logits_whatever_the_temperature,
    sampled_pins.test_counts_equal_bruteforce_recount_and_snapshot_rule,
    sampled_pins.test_equal_models_accept_everything,
    sampled_pins.test_invalid_draft_id_ends_the_loop_uncounted,
    sampled_pins.test_residual_without_mass_reports_the_target_argmax,
]


def _load_sampled_mutant(old, new):
    assert _SRC_S.count(old) >= 1, "mutation site not found: " + old
    mod = types.ModuleType("oracle.csd_oracle_sampled_mutant")
    mod.__file__ = OS.__file__
    mod.__package__ = "oracle"
    sys.modules["oracle.csd_oracle_sampled_mutant"] = mod
    exec(compile(_SRC_S.replace(old, new, 1), "csd_oracle_sampled_mutant", "exec"), mod.__dict__)
    return mod


def _sampled_failures(monkeypatch, mod):
    monkeypatch.setattr(sampled_pins, "OS", mod)
    failed = 0
    for pin in SAMPLED_PINS:
        try:
            pin()
        except (AssertionError, KeyError, IndexError, TypeError):
            failed += 1
    return failed


def test_unmutated_sampled_copy_passes_every_pin(monkeypatch):
    assert _sampled_failures(monkeypatch, _load_sampled_mutant("snapshot = orc.T", "snapshot = orc.T ")) == 0


@pytest.mark.parametrize("name,old,new", MUTANTS_SAMPLED, ids=[m[0] for m in MUTANTS_SAMPLED])
def test_planted_mistake_in_sampled_oracle_is_caught(monkeypatch, name, old, new):
    assert _sampled_failures(monkeypatch, _load_sampled_mutant(old, new)) >= 1, name
