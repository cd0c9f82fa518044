"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's source
(a dropped term, a wrong sign or index, a swapped weight) and requires the named pin to fail on
it.  Everything runs on the CPU; the real oracle is untouched."""
import os
import sys
import types

import pytest

from tests import test_oracle_attn as TA
from tests import test_oracle_compress as TC
from tests import test_oracle_loop as TL
from tests import test_oracle_prefill as TP

_SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "keepkv_oracle.py")

# (name, text in the oracle, replacement, test module, pin, arguments of the pin)
MUTANTS = [
    ("attention ignores the votes", "z = logit + np.log(p)[None, :]", "z = logit + 0.0 * np.log(p)[None, :]",
     TA, "test_votes_equal_physical_duplication", (0,)),
    ("log-sum-exp without its maximum", "lse = m + np.log(den)", "lse = np.log(den)", TA,
     "test_unit_votes_is_textbook_softmax", (0,)),
    ("group-mean logit replaced by the first head's", "return o, lse, logit.mean(axis=0)", "return o, lse, logit[0]", TC,
     "test_gqa_lossless_for_the_group_mean_query", ()),
    ("EMA weights swapped", "np.logaddexp(math.log(alpha) + log_S[:length], math.log1p(-alpha) + x)",
     "np.logaddexp(math.log1p(-alpha) + log_S[:length], math.log(alpha) + x)", TA, "test_ema_closed_form", (0.9,)),
    ("no bias correction", "out[seen] = log_S[seen] - np.log(-np.expm1(n[seen] * math.log(alpha)))",
     "out[seen] = log_S[seen]", TA, "test_ema_constant_input_is_unbiased_and_alpha_zero_tracks_last", ()),
    ("window weights off by one", "coef = math.log1p(-alpha) + (W - 1 - j) * math.log(alpha)",
     "coef = math.log1p(-alpha) + (W - j) * math.log(alpha)", TA, "test_window_score_equals_one_update_per_query",
     (0.5, -1)),
    ("causal window off by one", "(i <= first_pos + j)", "(i < first_pos + j)", TA,
     "test_window_score_equals_one_update_per_query", (0.5, 15)),
    ("selection ignores the votes", "key = np.log(np.asarray(votes[:length], dtype=np.float64)) + log_s_hat(",
     "key = 0.0 * np.log(np.asarray(votes[:length], dtype=np.float64)) + log_s_hat(", TC,
     "test_select_votes_weight_the_mass", ()),
    ("ties go to the higher index", "order = cand[np.lexsort((cand, -key[cand]))]",
     "order = cand[np.lexsort((-cand, -key[cand]))]", TC, "test_select_brute_force_with_ties", (0,)),
    ("similarity not normalised by the retained key", "* rn_e[:, None]) * rn_c[None, :]", "* rn_e[:, None])", TC,
     "test_match_brute_force_cosine", (False,)),
    ("threshold not strict", "target = np.where(sim > threshold, best, -1)", "target = np.where(sim >= threshold, best, -1)",
     TC, "test_match_ties_go_to_lowest_retained_position_and_threshold_is_strict", ()),
    ("last maximiser instead of the first", "best = U.argmax(axis=1)",
     "best = U.shape[1] - 1 - U[:, ::-1].argmax(axis=1)", TC,
     "test_match_ties_go_to_lowest_retained_position_and_threshold_is_strict", ()),
    ("merged key not rescaled", "out.k[r] = kbar * (L / ell_bar)", "out.k[r] = kbar", TC,
     "test_theorem2_single_step_lossless", (0,)),
    ("merge weights without votes", "w = p * np.exp(Eg - m)", "w = np.exp(Eg - m)", TC,
     "test_theorem2_single_step_lossless", (0,)),
    ("merged score without the vote-weighted mean", "L = m + math.log(W / P)", "L = m + math.log(W)", TC,
     "test_mass_conservation_with_ema_scores", (0.9, 3)),
    ("merged votes not summed", "out.votes[r] = int(np.asarray(votes)[g].sum())", "out.votes[r] = int(votes[c])", TC,
     "test_theorem2_single_step_lossless", (0,)),
    ("merged score stored without the bias factor",
     "out.log_S[r] = L + math.log(-math.expm1(n_r * math.log(alpha)))", "out.log_S[r] = L", TC,
     "test_mass_conservation_with_ema_scores", (0.9, 3)),
    ("votes of unmatched evicted slots not counted", "out.dropped = int(np.asarray(votes)[evict_idx[target < 0]].sum())",
     "out.dropped = 0", TL, "test_tiny_loop_conserves_votes", (0.8,)),
    ("merged values averaged without weights", "out.v[r] = wn @ v[g]", "out.v[r] = v[g].mean(axis=0)", TC,
     "test_theorem2_single_step_lossless", (0,)),
    ("prefill: a slot may match itself or later keys", "row = U[i, :i]", "row = U[i, :i + 1]", TP,
     "test_nearest_earlier_key_brute_force", (0,)),
    ("prefill: threshold not strict", "if row[j] > threshold:", "if row[j] >= threshold:", TP,
     "test_nearest_earlier_key_brute_force", (0,)),
    ("prefill: last maximiser instead of the first", "j = int(row.argmax())                              # first maximiser",
     "j = int(row.shape[0] - 1 - row[::-1].argmax())", TP, "test_nearest_earlier_key_brute_force", (0,)),
    ("prefill: chains collapse transitively", "absorbed[i] = j >= 0 and not absorbed[j]", "absorbed[i] = j >= 0", TP,
     "test_groups_on_hand_made_forests", ()),
    ("prefill: absorbed slots point at the wrong receiver", "return root_idx, absorbed_idx, pos[near[absorbed_idx]]",
     "return root_idx, absorbed_idx, np.zeros_like(absorbed_idx)", TP, "test_groups_on_hand_made_forests", ()),
    ("prefill: survivors not compacted to the new length", "            cache.len[b, h] = nk\n            trace.append((near, roots))",
     "            trace.append((near, roots))", TP, "test_exact_duplicates_collapse_with_zero_error_at_any_query", ()),
]


def _load(text, replacement):
    src = open(_SRC).read()
    assert src.count(text) == 1, f"mutation site not found exactly once: {text!r}"
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = _SRC
    sys.modules["oracle_mutant"] = mod                       # dataclasses look their module up by name
    try:
        exec(compile(src.replace(text, replacement), _SRC, "exec"), mod.__dict__)
    finally:
        del sys.modules["oracle_mutant"]
    return mod


@pytest.mark.parametrize("name,text,replacement,module,pin,args", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, text, replacement, module, pin, args):
    getattr(module, pin)(*args)                              # the pin passes on the real oracle
    monkeypatch.setattr(module, "O", _load(text, replacement))
    with pytest.raises(AssertionError):
        getattr(module, pin)(*args)
