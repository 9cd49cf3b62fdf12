"""Do the pins bite?  Each case plants one plausible mistake in the oracle -- a wrong sign, a dropped factor, a swapped
axis, an off-by-one -- by editing the source text of one oracle function in memory, and checks that at least one of the
named pins then fails.  Everything here runs on the CPU; the files on disk are never touched."""
import inspect
import textwrap

import pytest

from oracle import accounting, attention, hadamard, kvcache, layout, quantizer
from tests import test_oracle_attention as pa
from tests import test_oracle_layout as pl
from tests import test_oracle_quantizer as pq


def _planted(monkeypatch, module, name, old, new, count=1):
    """Replace `old` by `new` in the source of module.name and install the result for the duration of the test."""
    src = textwrap.dedent(inspect.getsource(getattr(module, name)))
    assert src.count(old) >= count, (name, old)
    namespace = dict(vars(module))
    exec(compile(src.replace(old, new), "<planted mistake in %s.%s>" % (module.__name__, name), "exec"), namespace)
    monkeypatch.setattr(module, name, namespace[name])


def _some_pin_fails(pins):
    failed = []
    for pin in pins:
        fn, args = (pin, ()) if callable(pin) else (pin[0], pin[1:])
        try:
            fn(*args)
        except Exception as e:  # an assertion, or a shape error the mistake provokes
            failed.append((fn.__name__, type(e).__name__))
    assert failed, "no pin noticed the planted mistake"
    return failed


CASES = [
    # (module, function, old text, new text, pins that should notice)
    ("dequantize sign of the zero-point", quantizer, "dequantize", "+ z[..., None]", "- z[..., None]",
     [pa.test_bits_to_16_converges_to_textbook_attention, (pq.test_eq1_round_trip_bound_and_levels, 2)]),
    ("Eq. 1 scale over 2^b instead of 2^b - 1", quantizer, "quantize_real", "2 ** bits - 1", "2 ** bits",
     [(pq.test_eq1_round_trip_bound_and_levels, 2), pq.test_eq1_literal_small_case]),
    ("Hadamard matrix left unnormalised", hadamard, "orthonormal", "/ np.sqrt(", "/ (",
     [pq.test_rotation_is_orthogonal_and_self_inverse, pa.test_rotation_invariance_without_quantization]),
    ("one softmax over all 256 logits instead of one per half", kvcache, "feature_map",
     "np.concatenate([softmax_rows(x @ W[0]), softmax_rows(x @ W[1])], axis=-1)",
     "softmax_rows(np.concatenate([x @ W[0], x @ W[1]], axis=-1))",
     [pa.test_zero_weights_closed_form, pa.test_states_are_additive_over_groups]),
    ("states built from the raw rotated values instead of the dequantized ones", kvcache, "build_cache",
     'out["S"] = phi_k.T @ out["V_hat"]', 'out["S"] = phi_k.T @ Vr[:n_quant].astype(np.float64)',
     [pa.test_recurrent_states_equal_quadratic_form_and_literal_eq5]),
    ("key error with the wrong sign", kvcache, "build_cache",
     'K_err = K[:n_quant].astype(np.float64) - out["K_hat"]', 'K_err = out["K_hat"] - K[:n_quant].astype(np.float64)',
     [pa.test_recurrent_states_equal_quadratic_form_and_literal_eq5]),
    ("keys quantized per token instead of per channel", kvcache, "build_cache",
     "ck, sk, zk = _quantize_rows(K[t0:t1].T, bits, mode)",
     "ck, sk, zk = _quantize_rows(K[t0:t1], bits, mode); ck, sk, zk = ck.T, sk[:d], zk[:d]",
     [pa.test_partial_tail_group_uses_valid_tokens_only, pa.test_tiny_case_brute_force]),
    ("values quantized without the rotation", kvcache, "build_cache", "Vr = hadamard.fwht_spec32(V)", "Vr = V",
     [pa.test_the_three_arithmetic_modes_describe_the_same_cache]),
    ("16-bit state rounded at the end only, whatever the stated points", kvcache, "build_cache",
     "cuts = sorted({int(c) for c in state_rounding if 0 < int(c) < n_quant} | {n_quant})", "cuts = [n_quant]",
     [pa.test_sixteen_bit_state_storage_rounds_at_the_stated_points]),
    ("16-bit state: the sum restarts at every rounding point", kvcache, "build_cache",
     'S = S + phi_k[prev:cut].T @ out["V_hat"][prev:cut]', 'S = phi_k[prev:cut].T @ out["V_hat"][prev:cut]',
     [pa.test_sixteen_bit_state_storage_rounds_at_the_stated_points]),
    ("window flushed one append early", kvcache, "window_split", "(n - 1) % G + 1", "n % G",
     [pa.test_window_split_is_the_lazy_block_flush]),
    ("correction added without the e^-M factor", attention, "decode", "if literal_alg1:", "if True:",
     [pa.test_recurrent_states_equal_quadratic_form_and_literal_eq5]),
    ("scores scaled by 1/d instead of 1/sqrt(d)", attention, "decode", "/ np.sqrt(float(d))", "/ float(d)",
     [pa.test_bits_to_16_converges_to_textbook_attention, pa.test_tiny_case_brute_force]),
    ("the fp16 window left out of the attention", attention, "_operands",
     'np.concatenate([cache["K_hat"], cache["k_res"].astype(np.float64)], axis=0)',
     'np.concatenate([cache["K_hat"], cache["k_res"][:0].astype(np.float64)], axis=0)',
     [pa.test_bits_to_16_converges_to_textbook_attention]),
    ("sliding value window: the window is one token short", attention, "_operands", "first = max(0, n - R)",
     "first = max(0, n - R + 1)", [pa.test_sliding_value_window_uniform_attention_closed_form]),
    ("sliding value window: values leave with the keys after all", attention, "_operands", "first = max(0, n - R)",
     "first = nq", [pa.test_sliding_value_window_uniform_attention_closed_form]),
    ("sliding value window: window values taken unrotated-window order (from the start of the sequence)", attention,
     "_operands", 'vals[first:] = cache["v_rot"][first:]', 'vals[first:] = cache["v_rot"][:n - first]',
     [pa.test_sliding_value_window_uniform_attention_closed_form]),
    ("block merge weighted by exp(M - m) instead of exp(m - M)", attention, "decode_blocks", "w = np.exp(m - M)",
     "w = np.exp(M - m)", [(pa.test_block_merge_equals_single_softmax, False)]),
    ("C_d taken from S instead of P", attention, "correction_terms", 'float(phi_q @ cache["P"])',
     'float((phi_q @ cache["S"]).sum())', [pa.test_zero_weights_closed_form]),
    # the functions the GPU is held to bit for bit
    ("spec32: the odd thresholds lose their tie rule", quantizer, "quantize_spec32", "(t >= thr)",
     "(t > thr)", [pq.test_spec32_ties_literal, (pq.test_spec32_is_eq1_against_stored_scale, 2), (pq.test_spec32_is_eq1_against_stored_scale, 4)]),
    ("spec32: the tie rule on the wrong thresholds", quantizer, "quantize_spec32", "if k % 2 else",
     "if k % 2 == 0 else", [pq.test_spec32_ties_literal]),
    ("spec32: codes taken against the unrounded scale", quantizer, "quantize_spec32",
     "s = s16.astype(f32)[..., None]", "s = (d32 / f32(L)).astype(f32)[..., None]",
     [(pq.test_spec32_is_eq1_against_stored_scale, 2), (pq.test_spec32_is_eq1_against_stored_scale, 4)]),
    ("spec32: a negative zero kept as zero-point", quantizer, "quantize_spec32",
     "mn = np.where(mn == 0, f32(0.0), mn).astype(f32)", "mn = mn.astype(f32)",
     [pq.test_spec32_negative_zero_is_canonical]),
    ("spec32: scale over 2^N levels", quantizer, "quantize_spec32", "d32 / f32(L)", "d32 / f32(L + 1)",
     [(pq.test_spec32_is_eq1_against_stored_scale, 2), (pq.test_spec32_vs_exact16_mismatch_rate_is_tiny, 4)]),
    ("exact16: codes against the unrounded zero-point", quantizer, "quantize_exact16",
     "codes = np.rint((x - z16.astype(np.float64)[..., None]) / safe[..., None])",
     "codes = np.rint((x - mn[..., None]) / (((mx - mn) / levels)[..., None] + 1e-300))",
     [(pq.test_spec32_is_eq1_against_stored_scale, 2), (pq.test_spec32_vs_exact16_mismatch_rate_is_tiny, 2),
      pq.test_constant_group_is_all_zero_codes]),
    ("fast transform: difference taken the other way round", hadamard, "fwht_spec32", "t = (a - b)", "t = (b - a)",
     [pq.test_fwht_spec32_equals_dense_product]),
    ("fast transform: the last stage left out", hadamard, "fwht_spec32", "while h < d:", "while h < d // 2:",
     [pq.test_fwht_spec32_equals_dense_product]),
    ("fast transform: scale of the wrong dimension", hadamard, "fwht_spec32", "x * INV_SQRT_128_F32",
     "x * np.float32(0.125)", [pq.test_fwht_spec32_equals_dense_product]),
    ("Sylvester matrix from i | j instead of i & j", hadamard, "sylvester", "i[:, None] & i[None, :]",
     "i[:, None] | i[None, :]", [(pq.test_sylvester_is_hadamard, 4), pq.test_fwht_spec32_equals_dense_product]),
    ("average bits: the window counted at the quantized width", accounting, "average_bits", "n_w * d * 16.0",
     "n_w * d * bits_per_element_quantized(bits, group)", [pq.test_average_bits_match_table1]),
    ("average bits: P left out of the states", accounting, "average_bits", "(D * d + D)", "(D * d)",
     [pq.test_average_bits_match_table1]),
    ("average bits: scale and zero-point at 8 bits", accounting, "bits_per_element_quantized", "2.0 * 16.0",
     "2.0 * 8.0", [pq.test_average_bits_match_table1]),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_a_planted_mistake_is_noticed(monkeypatch, case):
    _, module, name, old, new, pins = case
    _planted(monkeypatch, module, name, old, new)
    _some_pin_fails(pins)


def test_the_unplanted_oracle_passes_the_same_pins():
    """The harness itself must not be what fails: with nothing planted every pin named above passes."""
    for case in CASES:
        for pin in case[5]:
            fn, args = (pin, ()) if callable(pin) else (pin[0], pin[1:])
            fn(*args)


LAYOUT_CASES = [
    ("tile: odd and even codes of a word exchanged", "_position_maps", "p = 2 * (k % 8) + (k % 16) // 8",
     "p = 2 * (k % 8) + 1 - (k % 16) // 8", [pl.test_tiles_are_bijections_and_match_the_definition, pl.test_literal_corners]),
    ("tile: the words of odd blocks before those of even blocks", "_position_maps", "2 * (n % 2) + w",
     "2 * (1 - n % 2) + w", [pl.test_literal_corners]),
    ("tile: quarters of the contraction axis 8 rows apart instead of 16", "_position_maps", "j + 16 * g", "j + 8 * g",
     [pl.test_tiles_are_bijections_and_match_the_definition]),
    ("value tile: positions hold the tokens in plain order", "_value_token_of_position",
     "return 16 * (k % 8) + 4 * ((k // 16) % 4) + 2 * (k // 64) + (k // 8) % 2", "return k",
     [pl.test_tiles_are_bijections_and_match_the_definition]),
    ("value tile: rows are tokens instead of channels", "_v_index_maps",
     "word[tok[None, :], np.arange(128)[:, None]] = word_rk", "word[np.arange(128)[:, None], tok[None, :]] = word_rk",
     [pl.test_tiles_are_bijections_and_match_the_definition]),
    ("record: value scales and zero-points in plain token order", "pack_records",
     "rec[:, 2176:2304][:, _SZ_WORD] = ", "rec[:, 2176:2304] = ", [pl.test_record_fields_sit_where_the_header_says]),
    ("value window: token and channel exchanged inside a block", "pack_value_window",
     "full.reshape(R // 4, 4, 128).transpose(0, 2, 1)", "full.reshape(R // 4, 128, 4)",
     [pl.test_value_window_order]),
    ("state tiles: channel half before feature block", "pack_state_tiles",
     "tile = (f // 64 * 2 + c // 64) * 16 + (f % 64) // 4", "tile = (c // 64 * 4 + f // 64) * 16 + (f % 64) // 4",
     [pl.test_state_tiles_are_a_bijection]),
    ("4-bit record: the low plane of the key tile before the high plane", "pack_records4",
     "rec[:, 0:1024] = pack_k_tile(k_codes // 4)\n    rec[:, 1024:2048] = pack_k_tile(k_codes % 4)",
     "rec[:, 0:1024] = pack_k_tile(k_codes % 4)\n    rec[:, 1024:2048] = pack_k_tile(k_codes // 4)",
     [pl.test_four_bit_literal_corners]),
    ("4-bit record: the value planes hold the key tile's order", "pack_records4",
     "rec[:, 2048:3072] = pack_v_tile(v_codes // 4)", "rec[:, 2048:3072] = pack_k_tile(v_codes // 4)",
     [pl.test_four_bit_literal_corners, pl.test_four_bit_record_is_two_planes_per_tile]),
    ("4-bit record: the planes are the digits in base 2 and 8", "pack_records4",
     "rec[:, 0:1024] = pack_k_tile(k_codes // 4)\n    rec[:, 1024:2048] = pack_k_tile(k_codes % 4)",
     "rec[:, 0:1024] = pack_k_tile(k_codes // 8 * 2 + k_codes % 2)\n    rec[:, 1024:2048] = pack_k_tile(k_codes // 2 % 4)",
     [pl.test_four_bit_literal_corners]),
    ("4-bit record: the key zero-points before the key scales", "pack_records4", "rec[:, 4096:4160] = _halves_to_words(k_scale)\n    rec[:, 4160:4224] = _halves_to_words(k_zero)",
     "rec[:, 4096:4160] = _halves_to_words(k_zero)\n    rec[:, 4160:4224] = _halves_to_words(k_scale)", [pl.test_four_bit_record_is_two_planes_per_tile]),
]


@pytest.mark.parametrize("case", LAYOUT_CASES, ids=[c[0] for c in LAYOUT_CASES])
def test_a_planted_layout_mistake_is_noticed(monkeypatch, case):
    _, name, old, new, pins = case
    _planted(monkeypatch, layout, name, old, new)
    if name in ("_position_maps", "_value_token_of_position", "_v_index_maps"):  # tabulated when the module is loaded
        word, shift = layout._k_index_maps()
        monkeypatch.setattr(layout, "_K_WORD", word)
        monkeypatch.setattr(layout, "_K_SHIFT", shift)
        word, shift = layout._v_index_maps()
        monkeypatch.setattr(layout, "_V_WORD", word)
        monkeypatch.setattr(layout, "_V_SHIFT", shift)
    _some_pin_fails(pins)


def test_a_wrong_symbol_table_is_noticed(monkeypatch):
    """The bit pairs of codes 0 and 1 exchanged (pack side), and of codes 2 and 3 (unpack side)."""
    import numpy as np
    monkeypatch.setattr(layout, "SYMBOL_OF_CODE", np.array([0b10, 0b11, 0b00, 0b01], dtype=np.uint32))
    _some_pin_fails([pl.test_literal_corners])
    monkeypatch.undo()
    monkeypatch.setattr(layout, "CODE_OF_SYMBOL", np.array([3, 2, 1, 0], dtype=np.uint8))
    _some_pin_fails([pl.test_tiles_are_bijections_and_match_the_definition])


def test_layout_and_accounting_mistakes_are_noticed(monkeypatch):
    # the record order: key and value tiles exchanged
    src = inspect.getsource(layout)
    assert "pack_records" in src and "average_bits" in inspect.getsource(accounting)
    calls = [pl.test_record_fields_sit_where_the_header_says]
    real = layout.pack_records

    def swapped(k_codes, v_codes, *rest):
        return real(v_codes, k_codes, *rest)  # key and value tiles exchanged

    monkeypatch.setattr(layout, "pack_records", swapped)
    _some_pin_fails(calls)
    monkeypatch.setattr(layout, "pack_records", real)
    # the 2.46 / 2.71 bit figures: scale and zero-point counted at 8 bits instead of 16
    real_bits = accounting.average_bits
    monkeypatch.setattr(accounting, "average_bits", lambda *a, **k: real_bits(*a, **k) - 0.125)
    _some_pin_fails([pq.test_average_bits_match_table1])
