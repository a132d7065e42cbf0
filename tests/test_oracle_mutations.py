"""Do the oracle's pins notice a mistake?  Each case plants one plausible error in a copy of the
oracle's source (a swapped gate, a dropped term, a transposed operand, a forgotten mask, a wrong
normaliser ...), loads that copy as a module of its own, and runs the pin tests of
tests/test_oracle_pins.py against it.  Every planted error must make at least one pin fail; the
unchanged source must pass them all.  Everything here runs on the CPU; the HIP path is not involved."""
import os
import types

import pytest

try:
    from tests import test_oracle_pins as pins
except ImportError:                       # pytest started with tests/ itself on the path
    import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "nmt_oracle.py")).read()

# (what is planted, text in the oracle, replacement)
MUTATIONS = [
    ("cell: input and forget gate swapped", "c_new = f * c_prev + i * g", "c_new = i * c_prev + f * g"),
    ("cell: tanh of the cell state dropped", "h_new = o * np.tanh(c_new)", "h_new = o * c_new"),
    ("cell: gate blocks g and o swapped",
     "g = np.tanh(pre[:, 2 * h:3 * h])\n    o = sigmoid(pre[:, 3 * h:4 * h])",
     "g = np.tanh(pre[:, 3 * h:4 * h])\n    o = sigmoid(pre[:, 2 * h:3 * h])"),
    ("cell: weight columns taken as [h; x]", "xh = np.concatenate([x, h_prev], axis=1)", "xh = np.concatenate([h_prev, x], axis=1)"),
    ("cell: bias dropped", "pre = _op(xh) @ _op(W).T + b", "pre = _op(xh) @ _op(W).T"),
    ("mask: padded step emits its state", "y = m * h_new", "y = h"),
    ("mask: padded step updates the state", "h = m * h_new + (1 - m) * h_prev", "h = h_new"),
    ("mask: padded step updates the cell", "c = m * c_new + (1 - m) * c_prev", "c = c_new"),
    ("encoder: reverse direction runs forwards", "order = range(T - 1, -1, -1) if reverse else range(T)", "order = range(T)"),
    ("attention: W_a transposed", "q = _op(Ht) @ _op(W_a).T", "q = _op(Ht) @ _op(W_a)"),
    ("attention: padding takes part in the softmax", "valid = src_mask.T > 0  ", "valid = src_mask.T > -1 "),
    ("attention: [H_t; C_s] instead of [C_s; H_t]", "Cst = np.concatenate([Cs, Ht], axis=1)", "Cst = np.concatenate([Ht, Cs], axis=1)"),
    ("attention: tanh of Eq. 7 dropped", "Ho = np.tanh(_op(Cst) @ _op(W_c).T)", "Ho = _op(Cst) @ _op(W_c).T"),
    ("output: bias dropped", "u = _op(Ho) @ _op(W_o).T + B_o", "u = _op(Ho) @ _op(W_o).T"),
    ("output: smoothing term dropped", "row = (1.0 - eps) * nll + eps * (lse - z.mean(axis=1))", "row = (1.0 - eps) * nll"),
    ("step: decoder input not shifted",
     "dec_in = np.concatenate([np.full((B, 1), bos_id, tgt_ids.dtype), tgt_ids[:, :T - 1]], axis=1)", "dec_in = tgt_ids"),
    ("step: loss averaged over all slots", "loss = float((nll_all * tgt_mask).sum() / n_tok)", "loss = float((nll_all * tgt_mask).sum() / (B * T))"),
    ("step: decoder starts from zero states", "h = [enc_fin[l][0] for l in range(L)]", "h = [np.zeros((B, H), F64) for l in range(L)]"),
    ("step: input feed sees H_o before dropout", "Ho_prev = Ho_d", "Ho_prev = Ho"),
    ("step: no input feeding at all", "x = np.concatenate([Xt[j], Ho_prev], axis=1)", "x = np.concatenate([Xt[j], 0.0 * Ho_prev], axis=1)"),
    ("backward: cell-state path dropped", "dc = dc_new + dh_new * o * (1.0 - tc * tc)", "dc = dh_new * o * (1.0 - tc * tc)"),
    ("backward: forget gate sees the new cell", "df = dc * c_prev", "df = dc * c_new"),
    ("backward: bias gradient averaged", "db = dpre.sum(axis=0)", "db = dpre.mean(axis=0)"),
    ("backward: weight gradient transposed operand", "dW = _op(dpre).T @ _op(xh)", "dW = _op(dpre).T @ _op(xh)[:, ::-1]"),
    ("backward: masked step drops the state gradient", "dh_prev = dh_prev + (1 - m) * dh_state", "dh_prev = dh_prev + 0.0"),
    ("backward: softmax Jacobian without the mean term", "ds = a * (da - (a * da).sum(axis=1, keepdims=True))", "ds = a * da"),
    ("backward: H_s gradient through the scores dropped", 'dHs += np.einsum("bi,bh->ibh", ds, q)', "dHs += 0.0"),
    ("backward: W_a transposed in dH_t", "dHt += _op(dq) @ _op(W_a)", "dHt += _op(dq) @ _op(W_a).T"),
    ("backward: second consumer of H_t forgotten", "dCs, dHt = dCst[:, :H], dCst[:, H:].copy()", "dCs, dHt = dCst[:, :H], 0.0 * dCst[:, H:]"),
    ("backward: smoothed target taken as one-hot", "dz[np.arange(z.shape[0]), labels] -= 1.0 - eps", "dz[np.arange(z.shape[0]), labels] -= 1.0"),
    ("backward: input-feed gradient dropped", "dHo = (dHo + dHo_feed) * D_ho[j]", "dHo = dHo * D_ho[j]"),
    ("backward: dropout forgotten between decoder layers", "dy = dx * D_dec[l - 1][j] if l > 0 else dx", "dy = dx"),
    ("backward: repeated target ids overwrite",
     'np.add.at(g["E_tgt"], dec_in.T.reshape(-1), dXt.reshape(-1, E))', 'g["E_tgt"][dec_in.T.reshape(-1)] += dXt.reshape(-1, E)'),
    ("backward: decoder initial-state gradient not sent to the encoder",
     'dY, dW, db, _, _ = lstm_backward(dY, dh[l], dc[l], enc_sv[l], p[f"enc.l{l}.W"])',
     'dY, dW, db, _, _ = lstm_backward(dY, 0.0 * dh[l], dc[l], enc_sv[l], p[f"enc.l{l}.W"])'),
    ("dropout: wrong scale", "/ (1.0 - float(np.float32(p)))", "/ 1.0"),
    ("dropout: keeps with probability p", "(u >= thresh)", "(u < thresh)"),
    ("beam: ties go to the higher flat index", "order = np.lexsort((np.arange(cand.size), -cand))", "order = np.lexsort((-np.arange(cand.size), -cand))"),
    ("beam: finished hypotheses are not length-normalised", "finished.append((cand[f] / length_penalty(len(seq), alpha), len(finished), seq))", "finished.append((cand[f], len(finished), seq))"),
    ("beam: states of the survivors not reordered", "h = [hh[parents] for hh in h]", "h = [hh[:len(parents)] for hh in h]"),
    ("search: length penalty base", "return ((5.0 + length) / 6.0) ** alpha", "return ((5.0 + length) / 5.0) ** alpha"),
    ("greedy: highest index wins", "tok = z.argmax(axis=1)", "tok = z.shape[1] - 1 - z[:, ::-1].argmax(axis=1)"),
]

# the pins, cheapest first; parametrised ones are called with their arguments
FAST_PINS = [
    (pins.test_lstm_zero_weights_gives_zero_state, ()),
    (pins.test_lstm_bias_only_geometric_series, ()),
    (pins.test_lstm_saturated_gates_carry_the_cell, ()),
    (pins.test_gate_order_distinguishes_i_f_g_o, ()),
    (pins.test_lstm_layer_matches_torch_lstm, (False,)),
    (pins.test_lstm_layer_matches_torch_lstm, (True,)),
    (pins.test_padded_batch_equals_single_sentences, ()),
    (pins.test_attention_rows_sum_to_one_and_vanish_on_padding, ()),
    (pins.test_zero_output_layer_gives_log_vocab, ()),
    (pins.test_output_layer_matches_torch_log_softmax, ()),
    (pins.test_full_model_matches_torch_autograd_restatement, (4, 1)),
    (pins.test_full_model_matches_torch_autograd_restatement, (8, 3)),
    (pins.test_dropout_mask_values_rate_and_indexing, ()),
    (pins.test_no_regularisation_is_the_plain_step, ()),
    (pins.test_regularised_model_matches_torch_autograd_restatement, (4, 1)),
    (pins.test_regularised_model_matches_torch_autograd_restatement, (8, 3)),
    (pins.test_label_smoothed_output_layer_matches_torch_and_closed_forms, ()),
    (pins.test_greedy_decode_is_the_training_forward_with_its_own_output_fed_back, ()),
    (pins.test_greedy_decode_end_token_and_length_cap, ()),
    (pins.test_ties_go_to_the_lower_token_and_the_lower_slot, ()),
    (pins.test_beam_of_one_is_greedy_and_length_penalty_closed_form, ()),
    (pins.test_wide_beam_finds_the_best_sequence_by_brute_force, ()),
    (pins.test_intermediates_are_consistent, ()),
    (pins.test_tiny_config_loss_is_near_log_vocab_and_sgd_descends, ()),
]
SLOW_PINS = [
    (pins.test_finite_differences_every_tensor, (4, 1, False)),
    (pins.test_finite_differences_with_dropout_and_label_smoothing, (4, 1)),
    (pins.test_finite_differences_every_tensor, (6, 2, False)),
    (pins.test_finite_differences_with_dropout_and_label_smoothing, (6, 2)),
]


def load(source):
    mod = types.ModuleType("nmt_oracle_under_test")
    mod.__file__ = os.path.join(ROOT, "oracle", "nmt_oracle.py")
    exec(compile(source, mod.__file__, "exec"), mod.__dict__)
    return mod


def first_failing_pin(module, monkeypatch):
    """Name of the first pin that fails against `module`, or None."""
    monkeypatch.setattr(pins, "O", module)
    for fn, args in FAST_PINS + SLOW_PINS:
        try:
            fn(*args)
        except Exception:                     # an assertion, or the planted error breaking a shape
            return fn.__name__
    return None


def test_the_unchanged_oracle_passes_every_pin_used_here(monkeypatch):
    assert first_failing_pin(load(SOURCE), monkeypatch) is None


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_error_fails_a_pin(what, old, new, monkeypatch):
    assert SOURCE.count(old) == 1, f"the text to replace must occur exactly once: {old!r}"
    killer = first_failing_pin(load(SOURCE.replace(old, new)), monkeypatch)
    assert killer is not None, f"no pin notices: {what}"
