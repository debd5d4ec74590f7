"""The pins must be able to fail: every plausible mistake planted in the oracle (on the CPU,
by patching one of its functions) has to be caught by at least one pin of
test_oracle_pins.py.  Also checks that the product package never touches the oracle."""
import math
import os
import re

import numpy as np
import pytest

from oracle import loki_oracle as O
from tests import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# the pins that exercise Algorithm 1 / Eq. 1 (cheap ones; the PCA pin is not needed here)
BATTERY = [
    pins.test_hand_worked_example,
    pins.test_dense_matches_torch_sdpa,
    pins.test_dense_closed_forms,
    pins.test_rotation_invariance_identity,
    lambda: pins.test_full_k_equals_dense(5),
    pins.test_full_d_equals_exact_topk,
    pins.test_scores_use_first_d_columns_only,
    pins.test_topk_brute_force_all_k,
    pins.test_topk_ties_lowest_position_wins,
    pins.test_topk_is_by_signed_value,
    pins.test_selected_attention_closed_forms,
    pins.test_softmax_runs_over_selected_rows_only,
    pins.test_permutation_symmetry,
    pins.test_value_space_is_not_rotated,
    pins.test_batch_matches_single_head_and_gqa_mapping,
    pins.test_group_mode_reduces_to_per_head_when_G_is_1,
    pins.test_group_mode_selects_on_group_max,
    pins.test_bf16_rounding_matches_torch,
    pins.test_rank_at_closed_form,
    pins.test_layer_rank_and_width_closed_forms,
    pins.test_cost_model_prints_2p6x,
    pins.test_step_without_options_is_the_batch_function,
    pins.test_step_ragged_ignores_rows_past_each_sequence_and_pads_indices,
    pins.test_step_keeping_one_row_returns_that_value_row,
    pins.test_step_append_writes_the_rotated_rounded_key_then_attends,
    pins.test_step_with_several_new_tokens_is_sequential_decoding,
    pins.test_pca_attention_pins,
    pins.test_jaccard_closed_forms,
]


def battery_fails() -> bool:
    for t in BATTERY:
        try:
            t()
        except AssertionError:
            return True
        except Exception:
            return True  # a mutation that makes a pin crash is caught as well
    return False


def test_battery_passes_on_the_real_oracle():
    assert not battery_fails()


def _softmax_no_max(z):
    e = np.exp(np.asarray(z, dtype=np.float64))
    return e / e.sum()


MUTATIONS = {
    # rotation
    "query rotated by P^T": ("rotate_query", lambda q, P: np.asarray(q, float) @ np.asarray(P, float).T),
    "keys rotated by P^T": ("rotate_keys", lambda K, P: np.asarray(K, float) @ np.asarray(P, float).T),
    "query not rotated": ("rotate_query", lambda q, P: np.asarray(q, float)),
    # approximate scores
    "scores use d+1 columns": ("approx_scores", lambda qh, Kh, d: np.asarray(Kh, float)[:, :d + 1] @ np.asarray(qh, float)[:d + 1]),
    "scores use d-1 columns": ("approx_scores", lambda qh, Kh, d: np.asarray(Kh, float)[:, :max(d - 1, 0)] @ np.asarray(qh, float)[:max(d - 1, 0)]),
    "scores use the LAST d columns": ("approx_scores", lambda qh, Kh, d: np.asarray(Kh, float)[:, -d:] @ np.asarray(qh, float)[-d:]),
    "scores negated": ("approx_scores", lambda qh, Kh, d: -(np.asarray(Kh, float)[:, :d] @ np.asarray(qh, float)[:d])),
    # top-k
    "top-k by magnitude": ("topk_indices", lambda a, k: np.sort(np.argsort(-np.abs(np.asarray(a, float)), kind="stable")[:k])),
    "top-k picks the smallest": ("topk_indices", lambda a, k: np.sort(np.argsort(np.asarray(a, float), kind="stable")[:k])),
    "ties go to the highest position": ("topk_indices", lambda a, k: np.sort((len(a) - 1 - np.argsort(-np.asarray(a, float)[::-1], kind="stable"))[:k])),
    "top-k returns k-1 plus a repeat": ("topk_indices", lambda a, k: np.sort(np.concatenate([np.argsort(-np.asarray(a, float), kind="stable")[:max(k - 1, 1)], np.argsort(-np.asarray(a, float), kind="stable")[:1]])[:k])),
    # exact attention on the selected rows
    "no 1/sqrt(D) scale": ("attend_selected", lambda qh, Kh, V, idx: O.softmax(np.asarray(Kh, float)[idx] @ np.asarray(qh, float)) @ np.asarray(V, float)[idx]),
    "scale 1/D": ("attend_selected", lambda qh, Kh, V, idx: O.softmax(np.asarray(Kh, float)[idx] @ np.asarray(qh, float) / len(qh)) @ np.asarray(V, float)[idx]),
    "softmax over all rows, output over selected": ("attend_selected", lambda qh, Kh, V, idx: O.softmax(np.asarray(Kh, float) @ np.asarray(qh, float) / math.sqrt(len(qh)))[idx] @ np.asarray(V, float)[idx]),
    "exact stage uses only the first half of the columns": ("attend_selected", lambda qh, Kh, V, idx: O.softmax(np.asarray(Kh, float)[idx][:, :len(qh) // 2] @ np.asarray(qh, float)[:len(qh) // 2] / math.sqrt(len(qh))) @ np.asarray(V, float)[idx]),
    "unnormalised weights": ("attend_selected", lambda qh, Kh, V, idx: np.exp(np.asarray(Kh, float)[idx] @ np.asarray(qh, float) / math.sqrt(len(qh))) @ np.asarray(V, float)[idx]),
    # dense
    "dense without scale": ("dense_attention", lambda q, K, V: O.softmax(np.asarray(K, float) @ np.asarray(q, float)) @ np.asarray(V, float)),
    "dense uses K for the output": ("dense_attention", lambda q, K, V: O.softmax(np.asarray(K, float) @ np.asarray(q, float) / math.sqrt(len(q))) @ np.asarray(K, float)),
    # helpers
    "bf16 truncation instead of rounding": ("to_bf16", lambda x: (np.asarray(x, np.float64).astype(np.float32).view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32).astype(np.float64)),
    "rank_at off by one": ("rank_at", lambda ev, v: max(1, _real_rank_at(ev, v) - 1)),
    "layer rank is the largest head's instead of the mean": ("layer_rank_at", lambda ev, v: float(max(_real_rank_at(e, v) for e in np.asarray(ev, float)))),
    "layer width rounds down to the multiple": ("layer_width", lambda ev, v, multiple=1: min(int(math.ceil(O.layer_rank_at(ev, v))) // multiple * multiple, np.asarray(ev).shape[-1])),
    "layer width rounds the mean to nearest": ("layer_width", lambda ev, v, multiple=1: min(-(-int(math.floor(O.layer_rank_at(ev, v))) // multiple) * multiple, np.asarray(ev).shape[-1])),
    "PCAAttn scaled by sqrt(d)": ("pca_attention", lambda q, P, Khat, V, d: O.softmax(O.approx_scores(O.rotate_query(q, P), Khat, d) / math.sqrt(d)) @ np.asarray(V, float)),
    "PCAAttn over the d LAST columns": ("pca_attention", lambda q, P, Khat, V, d: O.softmax((np.asarray(Khat, float)[:, -d:] @ O.rotate_query(q, P)[-d:]) / math.sqrt(len(q))) @ np.asarray(V, float)),
    "Jaccard over the smaller set": ("jaccard", lambda a, b: len(set(a) & set(b)) / max(1, min(len(set(a)), len(set(b))))),
    "speed-up formula without the factor 1/2": ("theoretical_speedup", lambda D, S, d, k, exact=True: 1.0 / (d / D + k / S)),
}
_real_rank_at = O.rank_at


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, monkeypatch):
    attr, fn = MUTATIONS[name]
    monkeypatch.setattr(O, attr, fn)
    assert battery_fails(), f"no pin noticed: {name}"


def test_group_mode_mutation_is_caught(monkeypatch):
    """Group selection by the MEAN instead of the maximum of the group's scores."""
    real = O.loki_decode_batch
    src = real.__code__

    def mean_mode(q, P, Khat, V, d, k, select_mode=0, units=None):
        if select_mode == 0:
            return real(q, P, Khat, V, d, k, 0, units)
        real_max = np.max
        try:
            np.max = lambda a, axis=None: np.mean(a, axis=axis)  # only np.max(np.stack(a), axis=0) is hit
            return real(q, P, Khat, V, d, k, select_mode, units)
        finally:
            np.max = real_max

    monkeypatch.setattr(O, "loki_decode_batch", mean_mode)
    assert battery_fails()
    del src


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2406_02542_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "loki_oracle" not in text, f
    # and the oracle does not import the product
    otext = open(os.path.join(ROOT, "oracle", "loki_oracle.py")).read()
    assert "paper_2406_02542_amd" not in otext


def _step_mutant(**change):
    real = O.loki_decode_step

    def mutant(q, P, Khat, V, d, k_max, select_mode=0, seq_lens=None, ks=None, k_new=None, v_new=None,
               storage="f32", units=None, queries_per_seq=1):
        if change.get("later_tokens_visible") and queries_per_seq > 1 and k_new is not None:
            return _chunk_all_visible(real, q, P, Khat, V, d, k_max, select_mode, seq_lens, ks, k_new,
                                      v_new, storage, queries_per_seq)
        if change.get("ignore_lens"):
            seq_lens = None if ks is None else np.maximum(np.asarray(ks), np.asarray(seq_lens))
        if change.get("append_row_off_by_one") and k_new is not None and seq_lens is not None:
            seq2 = np.asarray(seq_lens) - 1
            out = real(q, P, Khat, V, d, k_max, select_mode, np.maximum(seq2, np.asarray(ks) if ks is not None else 1), ks, k_new, v_new, storage, units, queries_per_seq)
            return out
        if change.get("no_rounding"):
            storage = "f32"
        return real(q, P, Khat, V, d, k_max, select_mode, seq_lens, ks, k_new, v_new, storage, units,
                    queries_per_seq)
    return mutant


def _chunk_all_visible(real, q, P, Khat, V, d, k_max, mode, seq_lens, ks, k_new, v_new, storage, m):
    """Mistake: appends the chunk at the right rows but lets every token attend over all of it."""
    _, _, _, K1, V1 = real(q, P, Khat, V, d, k_max, mode, seq_lens, ks, k_new, v_new, storage, None, m)
    full = np.repeat(np.asarray(seq_lens).reshape(-1, m).max(axis=1), m) if m > 1 else seq_lens
    out, idx, sc, _, _ = real(q, P, K1, V1, d, k_max, mode, full, ks, None, None, storage, None, m)
    return out, idx, sc, K1, V1


@pytest.mark.parametrize("change", ["ignore_lens", "append_row_off_by_one", "no_rounding", "later_tokens_visible"])
def test_planted_mistake_in_the_step_is_caught(change, monkeypatch):
    monkeypatch.setattr(O, "loki_decode_step", _step_mutant(**{change: True}))
    assert battery_fails(), f"no pin noticed: {change}"
