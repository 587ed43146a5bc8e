"""Mutation check of the oracle's pins (CPU only).

Every entry below plants one plausible mistake -- a dropped term, a wrong sign or index, an
off-by-one, a swapped operand, a flipped tie rule -- into a private copy of the oracle's source,
and the pins of test_oracle_pins.py are then run against that copy.  A mutant that no pin
rejects means the pins do not fix that part of the arithmetic, which fails this test.  The
mutants never leave this process and the real oracle module is not modified."""
import itertools
import os
import types

import pytest

import test_oracle_pins as pins
from oracle import dynsplit_oracle as O

SRC_PATH = os.path.abspath(O.__file__)

# (name, exact text in the oracle source, replacement)
MUTANTS = [
    ("widen_shift", "<< np.uint32(16)", "<< np.uint32(15)"),
    ("candidate_position_shifted", "pos.append(t)", "pos.append(t + 1)"),
    ("candidate_class_off", "cls.append(c)", "cls.append(c + 1)"),
    ("sample_lower_edge", "if t < R or t > L - 1 - W:", "if t <= R or t > L - 1 - W:"),
    ("sample_upper_edge", "if t < R or t > L - 1 - W:", "if t < R or t > L - W:"),
    ("sample_takes_last_not_first", "if seen[c] < M:\n            samp[c, seen[c]] = t",
     "if True:\n            samp[c, seen[c] % M] = t"),
    ("retained_region_one_longer", "o_lo, o_hi = max(0, t - R + 1), t", "o_lo, o_hi = max(0, t - R), t"),
    ("retained_region_excludes_delimiter", "o_lo, o_hi = max(0, t - R + 1), t", "o_lo, o_hi = max(0, t - R + 1), t - 1"),
    ("discarded_region_one_shorter", "d_lo, d_hi = 0, max(0, t - R)", "d_lo, d_hi = 0, max(0, t - R - 1)"),
    ("discarded_sign", "- alpha_imp * float(A[d_lo", "+ alpha_imp * float(A[d_lo"),
    ("alpha_dropped", "- alpha_imp * float(A[d_lo", "- float(A[d_lo"),
    ("window_starts_at_delimiter", "qpos = t + 1 + w", "qpos = t + w"),
    ("gqa_head_mapping", "Kh = K[h // G]\n        for w in range(W):", "Kh = K[h % Hkv]\n        for w in range(W):"),
    ("causal_excludes_self", "z = (Kh[: qpos + 1] @ qwin[w, h]) * scale", "z = (Kh[: qpos] @ qwin[w, h]) * scale"),
    ("importance_scale_dropped", "z = (Kh[: qpos + 1] @ qwin[w, h]) * scale", "z = (Kh[: qpos + 1] @ qwin[w, h])"),
    ("importance_mean_over_heads_only", "return acc / (Hq * W)", "return acc / Hq"),
    ("weight_affine_map_dropped", "w = (mean[c] + alpha_imp) / (1.0 + alpha_imp)", "w = mean[c]"),
    ("weight_round_down", "wq[c] = int(math.floor(x + 0.5))", "wq[c] = int(math.floor(x))"),
    ("weight_no_clamp", "w = min(1.0, max(0.0, w))", "w = w"),
    ("score_weight_term_unscaled", "return a_num * wq_e * dd +", "return a_num * wq_e +"),
    ("score_alpha_complement", "(a_den - a_num) * 10 * (dd - abs(e - s_e))", "a_den * 10 * (dd - abs(e - s_e))"),
    ("score_distance_signed", "(dd - abs(e - s_e))", "(dd - (e - s_e))"),
    ("score_distance_sign_flipped", "(dd - abs(e - s_e))", "(dd + abs(e - s_e))"),
    ("boundary_at_delimiter_not_after", "wq_at = {int(t) + 1:", "wq_at = {int(t):"),
    ("tie_goes_to_larger_e", "if best_score is None or sc > best_score:", "if best_score is None or sc >= best_score:"),
    ("window_upper_edge", "lo, hi = s_e - delta, min(L, s_e + delta)", "lo, hi = s_e - delta, min(L, s_e + delta - 1)"),
    ("window_lower_edge", "lo, hi = s_e - delta, min(L, s_e + delta)", "lo, hi = s_e - delta + 1, min(L, s_e + delta)"),
    ("final_chunk_test", "if s_e >= L:\n            e_star = L", "if s_e > L:\n            e_star = L"),
    ("empty_window_cut", "e_star = s_e if best_e is None else best_e", "e_star = hi if best_e is None else best_e"),
    ("slot_count_rounding", "base.append(base[-1] + (ln + b - 1) // b)", "base.append(base[-1] + ln // b + 1)"),
    ("slot_span_block_lookup", 'i = int(np.searchsorted(slot_base, g, side="right")) - 1',
     'i = int(np.searchsorted(slot_base, g, side="left")) - 1'),
    ("slot_span_no_tail_clip", "ln = min(b, int(block_start[i + 1]) - start)", "ln = b"),
    ("summary_min_max_swapped", "xmin[h, i] = seg.min(axis=0)\n            xmax[h, i] = seg.max(axis=0)",
     "xmin[h, i] = seg.max(axis=0)\n            xmax[h, i] = seg.min(axis=0)"),
    ("summary_drops_last_token", "seg = X[h, int(block_start[i]): int(block_start[i + 1])]",
     "seg = X[h, int(block_start[i]): max(int(block_start[i]) + 1, int(block_start[i + 1]) - 1)]"),
    ("block_score_takes_min", "s[h] = np.maximum(", "s[h] = np.minimum("),
    ("block_score_ignores_kmin", "q[h][None, :] * kmin[hk]).sum(axis=1)", "q[h][None, :] * kmax[hk]).sum(axis=1)"),
    ("block_score_gqa_mapping", "hk = h // G\n        s[h] =", "hk = h % Hkv\n        s[h] ="),
    ("topk_ascending", "key=lambda g: (-slot_score[g], g)", "key=lambda g: (slot_score[g], g)"),
    ("topk_tie_to_higher_slot", "key=lambda g: (-slot_score[g], g)", "key=lambda g: (-slot_score[g], -g)"),
    ("topk_one_short", "take = order[: min(k, n_slots)]", "take = order[: max(min(k, n_slots) - 1, 0)]"),
    ("attention_scale_dropped", "z = (K[tokens] @ q) * scale", "z = (K[tokens] @ q)"),
    ("attention_values_are_keys", "o = (p[:, None] * V[tokens]).sum(axis=0) / den", "o = (p[:, None] * K[tokens]).sum(axis=0) / den"),
    ("attention_not_normalised", "o = (p[:, None] * V[tokens]).sum(axis=0) / den", "o = (p[:, None] * V[tokens]).sum(axis=0)"),
    ("dense_scale_dropped", "z[t] = float(np.dot(q, K[t])) * scale", "z[t] = float(np.dot(q, K[t]))"),
    ("dense_values_are_keys", "o += (w[t] / den) * V[t]", "o += (w[t] / den) * K[t]"),
    ("dense_not_normalised", "o += (w[t] / den) * V[t]", "o += w[t] * V[t]"),
    ("dense_lse_forgets_max", "return o, zmax + math.log(den)", "return o, math.log(den)"),
    ("dense_skips_last_token", "for t in range(L):\n        o +=", "for t in range(L - 1):\n        o +="),
    ("append_ignores_search_range", "if int(block_start[i]) + C + delta > L_old:", "if int(block_start[i]) + C > L_old:"),
    ("append_finality_edge", "if int(block_start[i]) + C + delta > L_old:", "if int(block_start[i]) + C + delta >= L_old:"),
    ("append_restarts_one_chunk_late", "s0 = int(block_start_old[i0]) if i0 < len(block_start_old) - 1 else L_old",
     "s0 = int(block_start_old[min(i0 + 1, len(block_start_old) - 1)])"),
    ("append_keeps_one_chunk_too_many", "keep = [int(x) for x in block_start_old[:i0]]",
     "keep = [int(x) for x in block_start_old[:i0 + 1]]"),
    ("mean_divides_by_len_plus_one", "out[h, i] = acc / (e - s)", "out[h, i] = acc / (e - s + 1)"),
    ("mean_is_a_sum", "out[h, i] = acc / (e - s)", "out[h, i] = acc"),
    ("mean_skips_first_token", "for t in range(s, e):\n                acc += X[h, t]", "for t in range(s + 1, e):\n                acc += X[h, t]"),
    ("mean_score_gqa_mapping", "s[h, i] = float(np.dot(q[h], kmean[h // G, i]))", "s[h, i] = float(np.dot(q[h], kmean[h % Hkv, i]))"),
    ("layers_unweighted_by_rows", "acc += delimiter_importance(qwin, K, t, R, alpha_imp, scale) * (Hq * W)", "acc += delimiter_importance(qwin, K, t, R, alpha_imp, scale) * W"),
    ("layers_sum_not_mean", "    return acc / n_rows\n", "    return acc\n"),
    ("group_score_takes_min", "if score[hk * G + g, i] > best:", "if score[hk * G + g, i] < best:"),
    ("group_score_skips_last_head", "for g in range(1, G):\n                if score[hk * G + g, i]", "for g in range(1, G - 1):\n                if score[hk * G + g, i]"),
    ("group_score_interleaved_heads", "best = score[hk * G, i]\n            for g in range(1, G):\n                if score[hk * G + g, i] > best:\n                    best = score[hk * G + g, i]",
     "best = score[hk, i]\n            for g in range(1, G):\n                if score[hk + g * (Hq // G), i] > best:\n                    best = score[hk + g * (Hq // G), i]"),
    ("reuse_ignores_selection", "if x >= 0 and x in chosen and", "if x >= 0 and"),
    ("reuse_stale_edge", "(stale_from is None or x < stale_from)", "(stale_from is None or x <= stale_from)"),
    ("reuse_max_over_heads", "r = min((len(pos) for pos in reusable), default=0)", "r = max((len(pos) for pos in reusable), default=0)"),
    ("reuse_keeps_last_r", "keep = reusable[h][:r]", "keep = reusable[h][len(reusable[h]) - r:]"),
    ("reuse_no_truncation", "keep = reusable[h][:r]", "keep = reusable[h]"),
    ("reuse_loads_descending_positions", "row[free[i]] = x\n            plan.append((free[i], x))",
     "row[free[-1 - i]] = x\n            plan.append((free[-1 - i], x))"),
    ("reuse_reloads_kept_slots", "need = [int(x) for x in sel[h] if int(x) not in kept_slots]", "need = [int(x) for x in sel[h]][: k - r]"),
    ("reuse_apply_gqa_mapping", "X[h // G, start:start + ln]", "X[h % (X.shape[0]), start:start + ln]"),
    ("reuse_apply_no_zero_fill", "buf[h, p * b:(p + 1) * b] = 0\n", "pass\n"),
    ("lse_forgets_max", "return o, float(m + math.log(den))", "return o, float(math.log(den))"),
]


def _mutant_module(old: str, new: str) -> types.ModuleType:
    src = open(SRC_PATH).read()
    assert src.count(old) == 1, "mutation site must be unique: %r (%d matches)" % (old, src.count(old))
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = SRC_PATH
    exec(compile(src.replace(old, new), SRC_PATH, "exec"), mod.__dict__)
    return mod


def _pin_calls():
    """Every pin of test_oracle_pins with its parametrisations expanded, as zero-argument callables."""
    calls = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        axes = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                names = [n.strip() for n in mark.args[0].split(",")]
                vals = [v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,) for v in mark.args[1]]
                axes.append((names, vals))
        for combo in itertools.product(*[vals for _, vals in axes]) if axes else [()]:
            kw = {}
            for (names, _), v in zip(axes, combo):
                kw.update(dict(zip(names, v)))
            calls.append((name, kw, fn))
    return calls


def _killed_by(mutant) -> list:
    real = pins.O
    pins.O = mutant
    killers = []
    try:
        for name, kw, fn in _pin_calls():
            try:
                fn(**kw)
            except Exception:            # assertion or a crash inside the mutant: either way rejected
                killers.append(name)
    finally:
        pins.O = real
    return killers


def test_the_unmutated_oracle_passes_every_pin():
    assert _killed_by(_mutant_module("import math", "import math")) == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_rejected_by_a_pin(name, old, new):
    killers = _killed_by(_mutant_module(old, new))
    assert killers, "no pin rejects the mutant %r" % name
