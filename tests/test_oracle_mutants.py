"""The pins of tests/test_oracle_pins.py are meant to catch a plausible mistake anywhere in the oracle.
This file checks that claim on the CPU: each case plants one mistake in the oracle (a wrong index, a
dropped term, a strict instead of an inclusive comparison, the wrong head mapping, the wrong rounding)
and expects at least one of the listed pins to fail; with the mistake removed the same pins pass."""
import math

import numpy as np
import pytest

import test_oracle_pins as P
from oracle import vlcache_oracle as O


def _strict_mask(m, tau):
    i = np.arange(tau)[:, None]
    j = np.arange(m)[None, :]
    return j < (m - tau + i)                          # a window row no longer sees itself


def _mask_without_offset(m, tau):
    i = np.arange(tau)[:, None]
    j = np.arange(m)[None, :]
    return j <= i                                     # window row i treated as prompt position i


def _logits_interleaved_heads(q_win, k, scale):
    q = np.asarray(q_win, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    Hq, Hkv = q.shape[0], kk.shape[0]
    s = np.empty((Hq, q.shape[1], kk.shape[1]))
    for h in range(Hq):
        s[h] = q[h] @ kk[h % Hkv].T                   # query head h reads KV head h mod Hkv
    return s * float(scale)


def _logits_without_scale(q_win, k, scale):
    return _ORIG["logits"](q_win, k, 1.0)


def _region_size_short(m, tau):
    return tau * (m - tau) + tau * (tau - 1) // 2


def _k_min_floor(m):
    return max(1, m // 100)


def _recent_count_ceil(k, num, den):
    return -(-(int(k) * int(num)) // int(den))


def _topk_ties_to_higher(psi, k, n_recent=0):
    psi = np.asarray(psi, dtype=np.float64)
    m = psi.shape[0]
    r = min(n_recent, k)
    head = psi[: m - r]
    order = (m - r - 1) - np.argsort(-head[::-1], kind="stable")
    return np.sort(np.concatenate([order[: k - r], np.arange(m - r, m)])).astype(np.int64)


def _topk_ignores_recent(psi, k, n_recent=0):
    return _ORIG["topk"](psi, k, 0)


def _score_mean_over_rows(q_win, k, scale):
    psi_kv, psi_h, M, Z = _ORIG["score"](q_win, k, scale)
    tau = np.asarray(q_win).shape[1]
    return psi_kv / tau, psi_h / tau, M, Z


def _sparsity_strict(q_win, k, scale, p=0.01, want_margin=False):
    s = O.logits(q_win, k, scale)
    tau, m = s.shape[1], s.shape[2]
    valid = O.causal_valid(m, tau)[None]
    M = np.where(valid, s, -np.inf).max(axis=2)
    keep = valid & ((s - M[:, :, None]) > math.log(p))
    nnz = keep.sum(axis=(1, 2)).astype(np.int64)
    gamma = 1.0 - nnz / float(O.region_size(m, tau))
    if not want_margin:
        return nnz, gamma
    return nnz, gamma, np.where(valid, np.abs(s - M[:, :, None] - math.log(p)), np.inf), keep


def _allocate_ties_to_higher_layer(nnz_lh, m, alpha_num, alpha_den):
    nn = [int(sum(int(x) for x in row)) for row in np.asarray(nnz_lh)]
    L, N = len(nn), sum(nn)
    B_tot = (alpha_num * L * m) // alpha_den
    quota = [(n * B_tot) // N for n in nn] if N else [B_tot // L] * L
    rem = [(n * B_tot) % N for n in nn] if N else [0] * L
    for l in sorted(range(L), key=lambda l: (-rem[l], -l))[: B_tot - sum(quota)]:
        quota[l] += 1
    kk = np.array([min(max(q, O.k_min(m)), m) for q in quota], dtype=np.int64)
    return kk, kk / float(m)


def _allocate_without_lower_clip(nnz_lh, m, alpha_num, alpha_den):
    kk, _ = _ORIG["allocate"](nnz_lh, m, alpha_num, alpha_den)
    nn = np.asarray(nnz_lh).sum(axis=1).astype(object)
    B_tot = (alpha_num * len(nn) * m) // alpha_den
    raw = np.array([int(n * B_tot // max(1, int(nn.sum()))) for n in nn], dtype=np.int64)
    kk = np.where(kk == O.k_min(m), np.maximum(raw, 1), kk)
    return kk, kk / float(m)


def _decode_without_scale(q, kc, vc, scale):
    return _ORIG["decode_attn"](q, kc, vc, 1.0)


def _window_attention_wrong_value_head(q_win, k, v, scale):
    A, _, M, Z = O.post_vision_attention(q_win, k, scale)
    vv = np.asarray(v, dtype=np.float64)
    Hq, Hkv = A.shape[0], vv.shape[0]
    return np.stack([A[h] @ vv[h % Hkv] for h in range(Hq)]), M, Z


def _quantize_truncating(x):
    x = np.asarray(x, dtype=np.float64)
    amax = np.abs(x).max(axis=-1)
    scale = np.where(amax > 0, (amax.astype(np.float32) / np.float32(448.0)).astype(np.float32), np.float32(1.0))
    y = (x.astype(np.float32) / scale[..., None]).astype(np.float32).astype(np.float64)
    vals = O.e4m3_values()
    finite = np.where(np.isfinite(vals), vals, np.inf)
    code = np.zeros(x.shape, dtype=np.uint8)
    for idx in np.ndindex(x.shape):
        t = y[idx]
        cand = np.where((np.sign(finite) == np.sign(t)) | (finite == 0), np.abs(finite), np.inf)
        ok = cand <= abs(t)                           # toward zero instead of to nearest even
        code[idx] = int(np.argmax(np.where(ok, cand, -1.0)))
    return code, scale.astype(np.float32)


def _decode_query_attention_mean(q_next, k, scale):
    g = np.asarray(q_next).shape[0] // np.asarray(k).shape[0]
    return _ORIG["decode_query_attention"](q_next, k, scale) / g


def _cache_hit_rate_over_kept(psi_star, kept, k):
    hits, _ = _ORIG["cache_hit_rate"](psi_star, kept, k)
    return hits, hits / float(max(1, len(np.asarray(kept))))


def _compact_descending(k, v, idx):
    return np.asarray(k)[idx[::-1]].copy(), np.asarray(v)[idx[::-1]].copy()


def _score_from_stats_ignores_sum(q_win, k, scale, M, Z):
    return _ORIG["score_from_stats"](q_win, k, scale, M, np.ones_like(np.asarray(Z, dtype=np.float64)))


def _e4m3_values_bias_8():
    return _ORIG["e4m3_values"]() / 2.0


def _allocate_float_without_clip(gamma_lh, alpha):
    g = np.asarray(gamma_lh, dtype=np.float64).mean(axis=1)
    return (1.0 - g) / (1.0 - g).sum() * alpha * g.shape[0]


def _decode_layer_attends_before_appending(self, l, q, k_new, v_new, scale):
    out = np.empty(np.asarray(q).shape, dtype=np.float64)
    for b in range(self.B):
        out[b] = O.decode_attn(q[b], self.kc[b][l], self.vc[b][l], scale)       # the new token is not attended
        if k_new is not None:
            for h in range(self.Hkv):
                self.kc[b][l][h] = np.concatenate([self.kc[b][l][h], np.asarray(k_new)[b, h][None]], axis=0)
                self.vc[b][l][h] = np.concatenate([self.vc[b][l][h], np.asarray(v_new)[b, h][None]], axis=0)
    return out


def _post_vision_attention_unmasked_max(q_win, k, scale):
    s = O.logits(q_win, k, scale)
    tau, m = s.shape[1], s.shape[2]
    valid = O.causal_valid(m, tau)[None]
    M = s.max(axis=2)                                   # the row maximum taken over masked keys too
    e = np.where(valid, np.exp(s - M[:, :, None]), 0.0)
    Z = e.sum(axis=2)
    return e / Z[:, :, None], s, M, Z


_ORIG = {n: getattr(O, n) for n in ("logits", "topk", "score", "allocate", "decode_attn", "decode_query_attention",
                                    "cache_hit_rate", "score_from_stats", "e4m3_values")}

MUTANTS = [
    ("causal_valid", _strict_mask, ["test_region_size_formula_vs_count", "test_equal_logits_give_harmonic_scores_golden",
                                   "test_window_attention_special_cases"]),
    ("causal_valid", _mask_without_offset, ["test_region_size_formula_vs_count", "test_scores_vs_torch_softmax_and_sdpa"]),
    ("logits", _logits_interleaved_heads, ["test_gqa_head_mapping_is_consecutive", "test_scores_vs_torch_softmax_and_sdpa"]),
    ("logits", _logits_without_scale, ["test_scores_vs_torch_softmax_and_sdpa", "test_window_attention_equals_library_sdpa_with_the_causal_mask"]),
    ("region_size", _region_size_short, ["test_region_size_formula_vs_count"]),
    ("k_min", _k_min_floor, ["test_k_min", "test_alloc_integer_worked_examples"]),
    ("recent_count", _recent_count_ceil, ["test_recent_window_as_a_fraction_of_the_budget"]),
    ("topk", _topk_ties_to_higher, ["test_topk_equals_full_sort", "test_cache_hit_rate_definition"]),
    ("topk", _topk_ignores_recent, ["test_topk_recent_window", "test_recent_window_as_a_fraction_of_the_budget"]),
    ("score", _score_mean_over_rows, ["test_rows_sum_to_one_and_mass_is_tau", "test_equal_logits_give_harmonic_scores_golden"]),
    ("sparsity", _sparsity_strict, ["test_threshold_boundary_is_inclusive", "test_two_level_logits_count"]),
    ("allocate", _allocate_ties_to_higher_layer, ["test_alloc_integer_worked_examples", "test_alloc_golden_float"]),
    ("allocate", _allocate_without_lower_clip, ["test_alloc_integer_worked_examples", "test_alloc_invariants_random"]),
    ("decode_attn", _decode_without_scale, ["test_decode_is_textbook_attention"]),
    ("window_attention", _window_attention_wrong_value_head, ["test_window_attention_equals_library_sdpa_with_the_causal_mask"]),
    ("quantize_e4m3_rows", _quantize_truncating, ["test_e4m3_table_and_row_quantiser"]),
    ("decode_query_attention", _decode_query_attention_mean, ["test_decode_query_attention_is_a_library_softmax_summed_over_the_group"]),
    ("cache_hit_rate", _cache_hit_rate_over_kept, ["test_cache_hit_rate_definition"]),
    ("compact", _compact_descending, ["test_compact_is_a_gather", "test_compressed_cache_keeps_topk_rows"]),
    ("score_from_stats", _score_from_stats_ignores_sum, ["test_score_from_stats_equals_scores_and_follows_its_statistics"]),
    ("e4m3_values", _e4m3_values_bias_8, ["test_e4m3_table_and_row_quantiser"]),
    ("allocate_float", _allocate_float_without_clip, ["test_alloc_golden_float", "test_alloc_invariants_random"]),
    ("post_vision_attention", _post_vision_attention_unmasked_max, ["test_window_attention_equals_library_sdpa_with_the_causal_mask",
                                                                    "test_window_attention_special_cases"]),
]


def test_a_decode_step_that_attends_before_appending_fails_a_pin(monkeypatch):
    pins = ["test_full_budget_decode_equals_uncompressed_and_is_permutation_invariant"]
    assert _failures(pins) == []
    monkeypatch.setattr(O.CompressedCache, "decode_layer", _decode_layer_attends_before_appending)
    assert _failures(pins)


def _failures(names):
    failed = []
    for n in names:
        try:
            getattr(P, n)()
        except (AssertionError, ValueError, IndexError, ZeroDivisionError):
            failed.append(n)
    return failed


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("attr,mutant,pins", MUTANTS, ids=[f"{a}:{f.__name__.lstrip('_')}" for a, f, _ in MUTANTS])
def test_a_planted_mistake_fails_a_pin(monkeypatch, attr, mutant, pins):
    assert _failures(pins) == [], "the pins must pass on the oracle as it stands"
    monkeypatch.setattr(O, attr, mutant)
    assert _failures(pins), f"no pin noticed the mistake planted in {attr}"
