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
