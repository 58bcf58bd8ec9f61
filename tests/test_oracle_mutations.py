"""The pins must have teeth: plant one plausible mistake at a time in a copy of the oracle (on the CPU) and check
that at least one pin fails.  A pin suite that passes a mutated oracle would not be pinning that part."""
import inspect
import types

import pytest

from oracle import dmoe_oracle as orc
from tests import test_oracle_indices as ti
from tests import test_oracle_values as tv
from tests import test_oracle_capacity as tc

MUTATIONS = {
    "gelu_forgets_sqrt2": ("return 0.5 * v * (1.0 + _erf(v / math.sqrt(2.0)))", "return 0.5 * v * (1.0 + _erf(v))"),
    "gelu_grad_drops_density_term": (" + v * np.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)", ""),
    "logits_accumulate_backwards": ("for i in range(d):\n        acc +=", "for i in reversed(range(d)):\n        acc +="),
    "logits_forget_bias": ("acc += np.asarray(bias, dtype=np.float32)[None, :]", "pass"),
    "topk_ties_go_to_highest": ("best = np.argmax(work, axis=1)", "best = work.shape[1] - 1 - np.argmax(work[:, ::-1], axis=1)"),
    "softmax_without_normalisation": ("return e / e.sum(axis=1, keepdims=True)", "return e"),
    "renormalisation_skipped": ("w = w / w.sum(axis=1, keepdims=True)", "w = w"),
    "padding_adds_a_block_to_exact_multiples": ("padded = ((n.astype(np.int64) + block - 1) // block) * block",
                                                "padded = (n.astype(np.int64) // block + 1) * block"),
    "groups_in_descending_token_order": ("S_e = np.flatnonzero(flat == e)         # ascending f",
                                         "S_e = np.flatnonzero(flat == e)[::-1]"),
    "transpose_offsets_point_at_rows": ("block_offsets_t.append(number[r, c])", "block_offsets_t.append(r)"),
    "row_indices_hold_columns": ("row_indices.append(r)", "row_indices.append(c)"),
    "mask_puts_every_expert_in_column_zero": ("m[r0:r1, e * hb:(e + 1) * hb] = 1", "m[r0:r1, 0:hb] = 1"),
    "forward_forgets_confidence": ("np.add.at(y, tok, w_flat[S_e, None] * O_e)", "np.add.at(y, tok, O_e)"),
    "forward_uses_wrong_expert_slice_of_w2": ("W2_e = widen_bf16(w2_bits[e * h:(e + 1) * h, :])\n        X_e = x[tok]",
                                              "W2_e = widen_bf16(w2_bits[0:h, :])\n        X_e = x[tok]"),
    "dw2_from_preactivation": ("dw2[e * h:(e + 1) * h, :] = A_e.T @ dO_e", "dw2[e * h:(e + 1) * h, :] = H_e.T @ dO_e"),
    "dw1_without_activation_derivative": ("dH_e = dA_e * activation_pair(activation)[1](H_e)", "dH_e = dA_e"),
    "tanh_gelu_wrong_cubic_coefficient": ("return 0.5 * v * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))",
                                          "return 0.5 * v * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (v + 0.44715 * v ** 3)))"),
    "tanh_gelu_grad_forgets_inner_derivative": (" * (1.0 + 3.0 * 0.044715 * v * v)", ""),
    "backward_uses_exact_derivative_for_tanh_form": ("dH_e = dA_e * activation_pair(activation)[1](H_e)", "dH_e = dA_e * gelu_grad(H_e)"),
    "dx_forgets_router_term": ("dx += dlogits @ wr.T", "pass"),
    "dweights_sign": ("dwt[S_e] = np.einsum(\"ij,ij->i\", dy[tok], O_e)", "dwt[S_e] = -np.einsum(\"ij,ij->i\", dy[tok], O_e)"),
    "renormalisation_gradient_drops_mean": ("dsel = (dwt - (dwt * w).sum(axis=1, keepdims=True)) / Z", "dsel = dwt / Z"),
    "softmax_jacobian_drops_projection": ("dlogits = p * (dp - (dp * p).sum(axis=1, keepdims=True))", "dlogits = p * dp"),
    "capacity_keeps_the_last_assignments": ("for f in range(flat.size):\n            e = flat[f]\n            keep[f]",
                                            "for f in reversed(range(flat.size)):\n            e = flat[f]\n            keep[f]"),
    "capacity_off_by_one": ("keep[f] = taken[e] < capacity", "keep[f] = taken[e] <= capacity"),
    "capacity_equation_ignores_the_factor": ("num_tokens * top_k / num_experts * capacity_factor", "num_tokens * top_k / num_experts"),
    "pad_to_capacity_pads_to_the_load": ("padded = np.full(num_experts, ((capacity + block - 1) // block) * block, dtype=np.int64)",
                                         "padded = -(-n.astype(np.int64) // block) * block"),
    "dropped_assignments_are_computed_anyway": ("expert_idx = np.where(np.asarray(keep_mask, dtype=bool), expert_idx, -1)",
                                                "expert_idx = expert_idx"),
    "dw_router_transposed_operand": ("dw_router = x.T @ dlogits", "dw_router = (dlogits.T @ x).T * 0 + x.T @ dlogits[::-1]"),
}


def _pins():
    return [
        lambda: ti.test_logits_accumulate_in_ascending_index_order_in_float32(),
        lambda: ti.test_topk_ties_go_to_lowest_expert_and_are_distinct(),
        lambda: ti.test_routing_against_float64_stable_sort(2, 8, 1, 1.2),
        lambda: ti.test_permutation_invariants("block_pm1"),
        lambda: ti.test_permutation_invariants("exact_blocks"),
        lambda: ti.test_permutation_against_stable_argsort(),
        lambda: ti.test_topology_hand_worked_example(),
        lambda: ti.test_encode_mask_against_scipy_on_arbitrary_masks(),
        lambda: ti.test_topology_generic_equals_closed_form_and_invariants([5, 1, 0, 2, 0, 0, 7], 3),
        lambda: tv.test_forward_equals_dense_masked_brute_force(tv.CASES[1]),
        lambda: tv.test_single_expert_is_the_textbook_mlp(),
        lambda: tv.test_gelu_values_and_derivative(),
        lambda: tv.test_tanh_gelu_values_and_derivative(),
        lambda: tv.test_tanh_form_forward_and_backward_equal_torch_autograd(),
        lambda: tv.test_backward_equals_torch_autograd_on_dense_formulation(tv.CASES[1]),
        lambda: tv.test_backward_equals_torch_autograd_on_dense_formulation(tv.CASES[2]),
        lambda: tv.test_top1_with_normalised_weight_gives_router_no_gradient(),
        lambda: tc.test_capacity_equation_values(),
        lambda: tc.test_keep_mask_and_permutation_invariants(tc.CASES[1]),
        lambda: tc.test_forward_equals_gated_dense_brute_force(tc.CASES[0]),
        lambda: tc.test_backward_equals_torch_autograd_on_gated_dense_formulation(tc.CASES[1]),
    ]


def _pins_pass() -> bool:
    for pin in _pins():
        try:
            pin()
        except AssertionError:
            return False
        except Exception:
            return False          # a mutated oracle that crashes a pin is caught as well
    return True


def test_the_unmutated_oracle_passes_the_pin_suite():
    assert _pins_pass()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_a_planted_mistake_fails_at_least_one_pin(name, monkeypatch):
    old, new = MUTATIONS[name]
    source = inspect.getsource(orc)
    assert source.count(old) == 1, "mutation %r does not apply cleanly" % name
    mutant = types.ModuleType("mutant_oracle")
    mutant.__dict__["__name__"] = "mutant_oracle"
    exec(compile(source.replace(old, new), "mutant_oracle.py", "exec"), mutant.__dict__)
    for attr, val in list(mutant.__dict__.items()):
        if callable(val) and hasattr(orc, attr) and getattr(val, "__module__", None) == "mutant_oracle":
            monkeypatch.setattr(orc, attr, val)
    assert not _pins_pass(), "no pin noticed the mutation %r" % name
