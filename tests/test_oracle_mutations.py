"""Do the pins bite?  Each case plants one plausible mistake in the CPU oracle
(a wrong direction, a dropped accumulation, a missing term, a shifted index,
an unstable grouping ...) and checks that at least one pin of
test_oracle_pins.py fails on it.  CPU only; the mistakes live in the oracle's
Python namespace for the duration of one test and never reach a GPU."""
import importlib.util
import os

import numpy as np
import pytest

import oracle as orc
from oracle import rtp_oracle as impl

_spec = importlib.util.spec_from_file_location("_pins", os.path.join(os.path.dirname(__file__), "test_oracle_pins.py"))
pins = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(pins)


def plant(monkeypatch, name, fn):
    """Replace a function where the oracle's own code and the pins both look it up."""
    monkeypatch.setattr(impl, name, fn)
    monkeypatch.setattr(orc, name, fn)


def some_pin_fails(*calls):
    for call in calls:
        try:
            call()
        except (AssertionError, ValueError, IndexError, KeyError):
            return True
    return False


def test_pins_pass_unmutated():
    assert not some_pin_fails(lambda: pins.test_schedule_invariants_exhaustive(5),
                              lambda: pins.test_rotated_equals_plain_bit_for_bit(4),
                              lambda: pins.test_gradient_accumulates_onto_arriving_content(),
                              lambda: pins.test_moe_dispatch_against_a_stable_sort(4),
                              lambda: pins.test_moe_rotated_matches_the_token_by_token_definition(2, False))


def test_wrong_forward_direction_is_caught(monkeypatch):
    plant(monkeypatch, "fwd_shard", lambda r, t, n: (r + t) % n)
    assert some_pin_fails(lambda: pins.test_schedule_invariants_exhaustive(5))
    assert some_pin_fails(lambda: pins.test_rotated_equals_plain_bit_for_bit(4))


def test_backward_starting_on_the_wrong_shard_is_caught(monkeypatch):
    plant(monkeypatch, "bwd_shard", lambda r, s, n: (r + s) % n)
    assert some_pin_fails(lambda: pins.test_schedule_invariants_exhaustive(5))
    assert some_pin_fails(lambda: pins.test_rotated_equals_plain_bit_for_bit(4))


def test_shifted_shard_boundaries_are_caught(monkeypatch):
    def shifted(k, O, n):
        o = O // n
        return min(k * o + 1, O), min((k + 1) * o + 1, O)
    plant(monkeypatch, "shard_rows", shifted)
    assert some_pin_fails(lambda: pins.test_rotated_equals_plain_bit_for_bit(3),
                          lambda: pins.test_input_partition_sums_to_plain(3))


def test_overwriting_instead_of_accumulating_is_caught(monkeypatch):
    real = impl.gemm_tn
    plant(monkeypatch, "gemm_tn", lambda A, B, C, accumulate=False: real(A, B, C, accumulate=False))
    assert some_pin_fails(lambda: pins.test_gradient_accumulates_onto_arriving_content())
    assert some_pin_fails(lambda: pins.test_full_ring_reduces_gradients(3))


def test_transposed_operand_is_caught(monkeypatch):
    real = impl.gemm_nn
    def wrong(A, B, C, accumulate=False):
        # uses B^T where B is square, garbage-free otherwise: a transposed-operand slip
        return real(A, np.ascontiguousarray(B.T), C, accumulate) if B.shape[0] == B.shape[1] else real(A, B, C, accumulate)
    plant(monkeypatch, "gemm_nn", wrong)
    assert some_pin_fails(lambda: pins.test_linear_gradients_by_finite_differences(),
                          lambda: pins.test_plain_vs_library_matmul(5, 5, 5),
                          lambda: pins.test_gemm_views_and_accumulate())


def test_gradient_shard_left_behind_is_caught(monkeypatch):
    real = impl._Ring.rotate
    monkeypatch.setattr(impl._Ring, "rotate", lambda self, incoming, with_grad: real(self, incoming, False))
    assert some_pin_fails(lambda: pins.test_rotated_equals_plain_bit_for_bit(4))
    assert some_pin_fails(lambda: pins.test_mlp_rotated_matches_plain_and_fd(orc.GELU_ERF))


def test_missing_term_in_an_activation_derivative_is_caught(monkeypatch):
    real = impl.act_grad
    def wrong(x, kind):
        g = real(x, kind)
        if kind == orc.GELU_ERF:      # drop the x * pdf(x) term: what is left is the normal cdf
            x = np.asarray(x, dtype=np.float64)
            g = g - x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
        return g
    plant(monkeypatch, "act_grad", wrong)
    assert some_pin_fails(lambda: pins.test_activation_derivative_by_central_difference(orc.GELU_ERF))
    assert some_pin_fails(lambda: pins.test_mlp_rotated_matches_plain_and_fd(orc.GELU_ERF))


def test_wrong_sign_in_the_gate_derivative_is_caught(monkeypatch):
    real = impl.act_grad
    plant(monkeypatch, "act_grad", lambda x, kind: -real(x, kind) if kind == orc.SILU else real(x, kind))
    assert some_pin_fails(lambda: pins.test_swiglu_rotated_matches_plain_and_fd())
    assert some_pin_fails(lambda: pins.test_moe_gradients_by_finite_differences(True))


def test_unstable_expert_grouping_is_caught(monkeypatch):
    real = impl.moe_dispatch
    def reversed_groups(route, n, align=1):
        counts, begin, perm = real(route, n, align)
        for e in range(n):
            seg = perm[begin[e]:begin[e] + counts[e]]
            perm[begin[e]:begin[e] + counts[e]] = seg[::-1]
        return counts, begin, perm
    plant(monkeypatch, "moe_dispatch", reversed_groups)
    assert some_pin_fails(lambda: pins.test_moe_dispatch_against_a_stable_sort(4))


def test_expert_run_on_the_wrong_tokens_is_caught(monkeypatch):
    real = impl.moe_dispatch
    def rotated_groups(route, n, align=1):
        return real([(int(e) + 1) % n for e in route], n, align)
    plant(monkeypatch, "moe_dispatch", rotated_groups)
    assert some_pin_fails(lambda: pins.test_moe_rotated_matches_the_token_by_token_definition(5, False))
    assert some_pin_fails(lambda: pins.test_moe_special_cases())


def test_dropped_bias_is_caught(monkeypatch):
    real = impl.plain_linear_fwd
    plant(monkeypatch, "plain_linear_fwd", lambda X, W, b=None: real(X, W, None))
    assert some_pin_fails(lambda: pins.test_bias_plain_vs_brute_force())


def test_wrong_memory_row_is_caught(monkeypatch):
    real = impl.param_bytes
    plant(monkeypatch, "param_bytes", lambda tech, W, G, n: real(tech, W, G, n) + (W // n if n > 1 else 1))
    assert some_pin_fails(lambda: pins.test_table1_closed_forms(1000, 2000, 4),
                          lambda: pins.test_table1_large_config_numbers())


def test_bias_piece_added_at_every_step_is_caught(monkeypatch):
    # every shard carrying the whole first piece: entries of b added N times or never
    real = impl.bias_pieces
    plant(monkeypatch, "bias_pieces", lambda O, n: [real(O, n)[0]] * n)
    assert some_pin_fails(lambda: pins.test_input_partition_bias_spread_over_the_shards(3, 7))
    assert some_pin_fails(lambda: pins.test_mlp_with_biases_rotated_matches_plain_numpy_and_fd(orc.GELU_ERF))
