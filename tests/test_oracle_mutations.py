"""The pins must bite: each plausible mistake, planted into the oracle on the CPU,
has to make at least one of the pin tests fail.

Every case replaces one oracle function by a wrong variant (a dropped tie rule,
a sign kept in the key, a sample instead of a population variance, a reversed
summation order, a residual that is not zeroed, ...) and then runs the pin
tests that are supposed to guard that function.  The case passes if one of them
raises AssertionError.
"""

import numpy as np
import pytest

from oracle import artopk_oracle as orc
from tests import test_oracle_pins as pins

_MASK = np.uint32(0x7FFFFFFF)


def _fails(monkeypatch, name, wrong, guards):
    monkeypatch.setattr(orc, name, wrong)
    caught = []
    for guard in guards:
        try:
            guard()
        except AssertionError:
            caught.append(guard.__name__)
        except Exception:       # a mutant may also crash a pin: that counts as caught
            caught.append(guard.__name__)
    return caught


# ---- wrong Top-k variants ---------------------------------------------------
def _topk_ties_to_highest_index(acc, k):
    key = orc.magnitude_keys(acc).astype(np.int64)
    order = np.lexsort((-np.arange(key.size), -key))     # ties: the highest index first
    return np.sort(order[:k]).astype(np.int32)


def _topk_by_signed_value(acc, k):
    order = np.argsort(-np.asarray(acc, dtype=np.float64), kind="stable")   # largest values, not magnitudes
    return np.sort(order[:k]).astype(np.int32)


def _topk_unsorted_output(acc, k):
    key = orc.magnitude_keys(acc)
    order = np.argsort(_MASK - key, kind="stable")
    return order[:k].astype(np.int32)                     # magnitude order instead of ascending index


def _topk_one_short(acc, k):
    good = _GOOD["topk_indices"](acc, k)
    return good[:-1] if k > 1 else good


_TOPK_GUARDS = [pins.test_topk_brute_force_rank, pins.test_topk_subset_enumeration,
                pins.test_topk_distinct_equals_argpartition, pins.test_topk_invariants_and_certificate,
                pins.test_hand_worked_trace_star]

_GOOD = {"topk_indices": orc.topk_indices}


@pytest.mark.parametrize("wrong", [_topk_ties_to_highest_index, _topk_by_signed_value, _topk_unsorted_output,
                                   _topk_one_short])
def test_wrong_topk_is_caught(monkeypatch, wrong):
    assert _fails(monkeypatch, "topk_indices", wrong, _TOPK_GUARDS)


def test_key_that_keeps_the_sign_is_caught(monkeypatch):
    wrong = lambda x: np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)   # noqa: E731
    assert _fails(monkeypatch, "magnitude_keys", wrong,
                  [pins.test_magnitude_key_special_values, pins.test_topk_brute_force_rank])


# ---- wrong variance / leader -------------------------------------------------
def test_sample_variance_is_caught(monkeypatch):
    wrong = lambda x: float(np.var(np.asarray(x, dtype=np.float64), ddof=1))      # noqa: E731
    assert _fails(monkeypatch, "variance", wrong, [pins.test_variance_library_and_closed_forms])


def test_mean_of_squares_instead_of_variance_is_caught(monkeypatch):
    wrong = lambda x: float(np.mean(np.asarray(x, dtype=np.float64) ** 2))        # noqa: E731
    assert _fails(monkeypatch, "variance", wrong, [pins.test_variance_library_and_closed_forms])


def test_last_maximum_as_leader_is_caught(monkeypatch):
    wrong = lambda v: int(len(v) - 1 - np.argmax(np.asarray(v)[::-1]))            # noqa: E731
    assert _fails(monkeypatch, "leader_var", wrong, [pins.test_leader_rules])


def test_zero_based_round_robin_off_by_one_is_caught(monkeypatch):
    wrong = lambda step, w: (step - 1) % w                                        # noqa: E731
    assert _fails(monkeypatch, "leader_star", wrong, [pins.test_leader_rules, pins.test_hand_worked_trace_star])


# ---- wrong sum / error feedback / residual ------------------------------------
def test_reversed_summation_order_is_caught(monkeypatch):
    def wrong(vals):
        s = vals[-1].copy()
        for r in range(vals.shape[0] - 2, -1, -1):
            s = s + vals[r]
        return s
    assert _fails(monkeypatch, "ordered_sum", wrong, [pins.test_ordered_sum_is_left_to_right])


def test_pairwise_library_sum_is_caught(monkeypatch):
    wrong = lambda vals: np.sum(vals.astype(np.float64), axis=0).astype(np.float32)   # noqa: E731
    assert _fails(monkeypatch, "ordered_sum", wrong, [pins.test_ordered_sum_is_left_to_right])


def test_error_feedback_with_the_wrong_sign_is_caught(monkeypatch):
    wrong = lambda g, r: np.asarray(g, np.float32) - np.asarray(r, np.float32)    # noqa: E731
    assert _fails(monkeypatch, "ef_add", wrong,
                  [pins.test_ef_add_is_single_fp32_add, pins.test_hand_worked_trace_star,
                   pins.test_step_invariants_multi_step])


def test_error_feedback_rounded_from_double_is_caught(monkeypatch):
    # adding in float64 and rounding once differs from the single float32 add only through what the
    # operands are converted from; here the mistake is to scale the residual on the way
    wrong = lambda g, r: (np.asarray(g, np.float64) + 0.5 * np.asarray(r, np.float64)).astype(np.float32)  # noqa: E731
    assert _fails(monkeypatch, "ef_add", wrong,
                  [pins.test_ef_add_is_single_fp32_add, pins.test_step_invariants_multi_step])


def test_residual_that_keeps_the_sent_values_is_caught(monkeypatch):
    wrong = lambda acc, idx: np.array(acc, dtype=np.float32, copy=True)           # noqa: E731
    assert _fails(monkeypatch, "residual_rewrite", wrong,
                  [pins.test_step_invariants_multi_step, pins.test_hand_worked_trace_star])


def test_residual_with_negative_zero_is_caught(monkeypatch):
    def wrong(acc, idx):
        r = np.array(acc, dtype=np.float32, copy=True)
        r[idx] = np.float32(-0.0)
        return r
    assert _fails(monkeypatch, "residual_rewrite", wrong,
                  [pins.test_step_invariants_multi_step, pins.test_hand_worked_trace_star])


def test_update_that_accumulates_instead_of_overwriting_is_caught(monkeypatch):
    def wrong(n, idx, summed):
        u = np.zeros(n, dtype=np.float32)
        u[idx] = summed
        u[(np.asarray(idx)[:1] + 1) % n] += np.float32(1.0)    # something lands off the indices
        return u
    assert _fails(monkeypatch, "scatter_update", wrong,
                  [pins.test_step_invariants_multi_step, pins.test_hand_worked_trace_star,
                   pins.test_step_k_equals_n_is_dense_ordered_allreduce])


def test_gather_from_the_leader_only_is_caught(monkeypatch):
    wrong = lambda accs, idx: np.stack([accs[0][idx] for _ in accs]).astype(np.float32)   # noqa: E731
    assert _fails(monkeypatch, "gather", wrong,
                  [pins.test_hand_worked_trace_star, pins.test_step_invariants_multi_step,
                   pins.test_step_k_equals_n_is_dense_ordered_allreduce])


# ---- wrong widening of 16-bit gradients ---------------------------------------
def test_bfloat16_widened_into_the_lower_half_is_caught(monkeypatch):
    wrong = lambda b, kind: np.ascontiguousarray(b, np.uint16).astype(np.uint32).view(np.float32)   # noqa: E731
    assert _fails(monkeypatch, "widen_gradient", wrong, [pins.test_widen_bf16_known_values_and_round_trip])


def test_float16_with_flushed_subnormals_is_caught(monkeypatch):
    def wrong(b, kind):
        x = np.ascontiguousarray(b, np.uint16).view(np.float16).astype(np.float32)
        x[np.abs(x) < 2.0 ** -14] = 0.0
        return x
    assert _fails(monkeypatch, "widen_gradient", wrong, [pins.test_widen_f16_all_bit_patterns_against_field_decoding])
