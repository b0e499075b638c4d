"""The pins must be able to fail: plausible slips (a wrong divisor, basis, index, sign, axis, order of two steps) are
planted in a COPY of the oracle's source, one at a time, and the pin named beside each must then fail.  The copies
live only inside this test; the oracle itself is never changed.  CPU only."""
import inspect
import sys
import types

import pytest

import oracle.eigen_attention as attention_oracle
import oracle.eviction as eviction_oracle
import oracle.quant_cache as quant_oracle
import test_oracle_eviction as eviction_pins
import test_oracle_pins as attention_pins
import test_oracle_quant as quant_pins


def mutant(mod, old: str, new: str):
    """A module built from mod's source with the one occurrence of `old` replaced by `new`."""
    src = inspect.getsource(mod)
    assert src.count(old) == 1, f"the text to replace must occur exactly once in {mod.__name__}"
    name = mod.__name__ + "_with_a_planted_mistake"
    m = types.ModuleType(name)
    m.__package__ = "oracle"
    m.__file__ = mod.__file__
    sys.modules[name] = m                      # dataclasses look their module up while the class is built
    try:
        exec(compile(src.replace(old, new), mod.__file__, "exec"), m.__dict__)
    finally:
        del sys.modules[name]
    return m


def pin_fails(pins, alias: str, planted, pin_name: str) -> bool:
    """Runs one pin (all its parameter sets) with the pins' oracle alias pointing at the planted copy."""
    fn = getattr(pins, pin_name)
    marks = [mk for mk in getattr(fn, "pytestmark", []) if mk.name == "parametrize"]
    arg_sets = [a if isinstance(a, tuple) else (a,) for a in marks[0].args[1]] if marks else [()]
    saved = getattr(pins, alias)
    setattr(pins, alias, planted)
    try:
        for args in arg_sets:
            try:
                fn(*args)
            except Exception:                  # an assertion, or shapes that no longer fit
                return True
        return False
    finally:
        setattr(pins, alias, saved)


ATTENTION = [
    ("decode divides by sqrt(r) instead of sqrt(d_h)",
     "s = (K @ q_r[b, i]) / math.sqrt(d_head)", "s = (K @ q_r[b, i]) / math.sqrt(K.shape[1])",
     "test_rank_space_equals_projected_back_form"),
    ("prefill divides by sqrt(r)",
     "s = (K[:pos + 1] @ q_r[b, j, i]) / math.sqrt(d_head)", "s = (K[:pos + 1] @ q_r[b, j, i]) / math.sqrt(K.shape[1])",
     "test_rank_space_equals_projected_back_form"),
    ("prefill without the causal mask",
     "                pos = L - n + j\n                s = (K[:pos + 1] @ q_r",
     "                pos = L - 1\n                s = (K[:pos + 1] @ q_r",
     "test_full_rank_equals_standard_attention_prefill"),
    ("query head i uses kv head i mod H_kv",
     "    return i // (n_heads // n_kv_heads)", "    return i % n_kv_heads", "test_fold_weights_elementwise"),
    ("W^Q folded with the value basis",
     "Wq_f.append(Wq_i @ Uk[g])", "Wq_f.append(Wq_i @ Uv[g])", "test_fold_weights_elementwise"),
    ("W^O folded with the key basis",
     "Wo_f.append(Uv[g].T @ Wo_i)", "Wo_f.append(Uk[g].T @ Wo_i)", "test_fold_weights_elementwise"),
    ("W^K' built from W^Q (the slip in the paper's algorithm box, against Eq. 8)",
     "Wk_f.append(Wk_g @ Uk[g])", "Wk_f.append(Wq[:, g * d_h:(g + 1) * d_h] @ Uk[g])", "test_fold_weights_elementwise"),
    ("W^V folded with the key basis",
     "Wv_f.append(Wv_g @ Uv[g])", "Wv_f.append(Wv_g @ Uk[g])", "test_fold_weights_elementwise"),
    ("W^O_i taken as a block of columns, transposed",
     "Wo_i = Wo[i * d_h:(i + 1) * d_h, :]", "Wo_i = Wo[:, i * d_h:(i + 1) * d_h].T",
     "test_full_rank_equals_standard_attention_decode"),
    ("the generation step attends before it appends (the new token does not see itself)",
     "    for b in range(x.shape[0]):\n        cache.append(b, k[b:b + 1], v[b:b + 1])\n"
     "    o = decode_attention(q, cache, d_head, counter, alibi_slopes=alibi_slopes)",
     "    o = decode_attention(q, cache, d_head, counter, alibi_slopes=alibi_slopes)\n"
     "    for b in range(x.shape[0]):\n        cache.append(b, k[b:b + 1], v[b:b + 1])",
     "test_full_rank_equals_standard_attention_decode"),
    ("the generation step drops the ALiBi slopes it was given",
     "    o = decode_attention(q, cache, d_head, counter, alibi_slopes=alibi_slopes)",
     "    o = decode_attention(q, cache, d_head, counter)",
     "test_alibi_step_full_rank_equals_the_textbook_block_with_the_bias_written_out"),
    ("every head goes through W^O'_0",
     "        y += o[:, i, :] @ Wo_f[i]", "        y += o[:, i, :] @ Wo_f[0]", "test_brute_force_projection_and_out_proj"),
    ("values taken in reversed token order",
     "            out[b, i] = p @ V\n", "            out[b, i] = p @ V[::-1]\n", "test_special_cases"),
    ("rotary: sign slip in the first component",
     "    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * sn", "    out[..., 0::2] = x[..., 0::2] * c + x[..., 1::2] * sn",
     "test_rope_rotation_against_its_definition_and_textbook_properties"),
    ("rotary: frequency exponent j/d instead of 2j/d",
     "theta = np.asarray(base, F64) ** (-np.arange(0, d, 2, dtype=F64) / d)",
     "theta = np.asarray(base, F64) ** (-np.arange(0, d // 2, dtype=F64) / d)",
     "test_rope_rotation_against_its_definition_and_textbook_properties"),
    ("rotary decode: the query one position too far",
     "            q_pos = rope_rotate(q[b, i], n - 1, base)\n            s = (K_pos @ q_pos) / math.sqrt(d_head)\n"
     "            out[b, i] = softmax(s) @ cache.V[b][g]",
     "            q_pos = rope_rotate(q[b, i], n, base)\n            s = (K_pos @ q_pos) / math.sqrt(d_head)\n"
     "            out[b, i] = softmax(s) @ cache.V[b][g]",
     "test_rope_variant_full_rank_equals_standard_rope_attention"),
    ("rotary decode: the rank-r key rotated first and brought back to d_h channels afterwards",
     "            K_pos = rope_rotate(K_up, np.arange(n), base)\n            q_pos",
     "            K_pos = rope_rotate(cache.K[b][g], np.arange(n), base) @ Uk.T\n            q_pos",
     "test_rope_variant_full_rank_equals_standard_rope_attention"),
    ("ALiBi bias with the wrong sign",
     "    return -float(slope) * (pos_q - np.arange(n_keys, dtype=F64))",
     "    return float(slope) * (pos_q - np.arange(n_keys, dtype=F64))",
     "test_alibi_bias_definition_limits_and_shift_invariance"),
    ("cache size without the values",
     "    return batch * n * n_kv_heads * (r_k + r_v) * n_layers * bytes_per_el",
     "    return batch * n * n_kv_heads * r_k * n_layers * bytes_per_el", "test_intro_memory_example"),
]

QUANT = [
    ("truncation instead of rounding",
     "    q = np.rint((x32 - z32) / safe)", "    q = np.floor((x32 - z32) / safe)",
     "test_rounding_is_to_nearest_not_truncation"),
    ("seventeen levels", "LEVELS = 15 ", "LEVELS = 16 ", "test_values_on_the_grid_round_trip_exactly"),
    ("key groups of 32 tokens", "GROUP_TOKENS = 64", "GROUP_TOKENS = 32", "test_key_groups_are_64_tokens_long"),
    ("a chunked prefill never quantises the chunks it has finished",
     "[V[:, :c1]], [c0], d_head,", "[V[:, :c1]], [0], d_head,", "test_prefill_attention_over_a_partly_quantised_cache"),
    ("the prefill over a partly quantised cache drops the causal mask (every query sees the whole cache)",
     "    return ea_oracle.prefill_attention(q_r, cache, d_head, alibi_slopes=alibi_slopes)",
     "    return np.stack([ea_oracle.decode_attention(np.asarray(q_r)[:, j], cache, d_head) for j in range(n)], axis=1)",
     "test_prefill_attention_over_a_partly_quantised_cache"),
    ("the rotary prefill over a partly quantised cache attends the unquantised cache",
     "    rope_prefill_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits)\n",
     "    rope_prefill_views = [(np.asarray(K_list[b], np.float64), np.asarray(V_list[b], np.float64))\n",
     "test_rotary_prefill_over_a_partly_quantised_cache"),
    ("the rotary prefill over a partly quantised cache ignores the base it is given",
     "    return ea_oracle.prefill_attention_rope(q, cache, Uk, d_head, base)",
     "    return ea_oracle.prefill_attention_rope(q, cache, Uk, d_head)",
     "test_rotary_prefill_over_a_partly_quantised_cache"),
    ("the prefill over a partly quantised cache drops the ALiBi slopes it was given",
     "    return ea_oracle.prefill_attention(q_r, cache, d_head, alibi_slopes=alibi_slopes)",
     "    return ea_oracle.prefill_attention(q_r, cache, d_head)",
     "test_prefill_attention_over_a_partly_quantised_cache"),
    ("the key quantiser ignores the group length it is given",
     "    Kg = K.astype(np.float32).reshape(n // group_tokens, group_tokens, r)",
     "    Kg = K.astype(np.float32).reshape(n // GROUP_TOKENS, GROUP_TOKENS, r)", "test_key_groups_of_128_tokens"),
    ("the view of a partly quantised cache ignores the group length",
     "            Kq[h, :n_quant] = dequantize_keys(*quantize_keys(K[h, :n_quant], group_tokens, bits))",
     "            Kq[h, :n_quant] = dequantize_keys(*quantize_keys(K[h, :n_quant], GROUP_TOKENS, bits))",
     "test_key_groups_of_128_tokens"),
    ("three-bit codes take sixteen levels",
     "    return LEVELS if bits == 4 else 7", "    return LEVELS", "test_three_bit_codes"),
    ("the values of a partly quantised cache stay at four bits when three are asked for",
     "            Vq[h, :n_quant] = dequantize_values(*quantize_values(V[h, :n_quant], bits))",
     "            Vq[h, :n_quant] = dequantize_values(*quantize_values(V[h, :n_quant]))", "test_three_bit_codes"),
    ("the rotary form over a quantised cache stays at four bits when three are asked for",
     "    rope_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits) for b in range(len(K_list))]",
     "    rope_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens) for b in range(len(K_list))]",
     "test_three_bit_codes_in_the_rotary_and_the_prefill_form"),
    ("the prefill over a quantised cache stays at four bits when three are asked for",
     "    prefill_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens, bits)",
     "    prefill_views = [quantized_view(K_list[b], V_list[b], int(n_quant[b]), group_tokens)",
     "test_three_bit_codes_in_the_rotary_and_the_prefill_form"),
    ("a prompt prefilled in chunks quantises its finished chunks at four bits when three are asked for",
     "                                                 group_tokens, bits)[0]",
     "                                                 group_tokens)[0]",
     "test_three_bit_codes_in_the_rotary_and_the_prefill_form"),
    ("zero point at the group's maximum",
     "    return step.astype(np.float16), lo.astype(np.float16)", "    return step.astype(np.float16), hi.astype(np.float16)",
     "test_values_on_the_grid_round_trip_exactly"),
    ("values quantised per channel",
     "    scale, zero = _scale_zero(V32.min(axis=1), V32.max(axis=1), _levels(bits))\n"
     "    return _codes(V32, scale[:, None], zero[:, None], _levels(bits)), scale, zero",
     "    scale, zero = _scale_zero(V32.min(axis=0), V32.max(axis=0), _levels(bits))\n"
     "    return _codes(V32, scale[None, :], zero[None, :], _levels(bits)), scale, zero",
     "test_values_on_the_grid_round_trip_exactly"),
    ("keys quantised per token",
     "    scale, zero = _scale_zero(Kg.min(axis=1), Kg.max(axis=1), _levels(bits))\n"
     "    codes = _codes(Kg, scale[:, None, :], zero[:, None, :], _levels(bits)).reshape(n, r)",
     "    scale, zero = _scale_zero(Kg.min(axis=2), Kg.max(axis=2), _levels(bits))\n"
     "    codes = _codes(Kg, scale[:, :, None], zero[:, :, None], _levels(bits)).reshape(n, r)",
     "test_key_groups_are_64_tokens_long"),
    ("value dequantisation with the zero inside the scale",
     "    return scale.astype(np.float64)[:, None] * codes.astype(np.float64) + zero.astype(np.float64)[:, None]",
     "    return scale.astype(np.float64)[:, None] * (codes.astype(np.float64) + zero.astype(np.float64)[:, None])",
     "test_constant_group_is_exact_and_has_code_zero"),
    ("metadata counted per scalar instead of per group",
     "    return n_elements * (bits + meta_bits_per_group / group) / 8.0",
     "    return n_elements * (bits + meta_bits_per_group) / 8.0",
     "test_cache_size_accounting_reproduces_the_papers_quantisation_table"),
    ("the 16-bit tail quantised as well",
     "        if n_quant:\n            Kq[h, :n_quant]",
     "        if n_quant:\n            n_quant = K.shape[1] // GROUP_TOKENS * GROUP_TOKENS\n            Kq[h, :n_quant]",
     "test_attention_over_a_quantised_cache"),
]

EVICTION = [
    ("heads summed into the wrong kv head",
     "            m[i // G] += probs[b * H + i]", "            m[i % cache.n_kv_heads] += probs[b * H + i]",
     "test_heads_of_different_kv_heads_do_not_mix"),
    ("every sequence gets the first sequence's probabilities",
     "            m[i // G] += probs[b * H + i]", "            m[i // G] += probs[i]",
     "test_mass_rows_sum_to_the_group_size_and_match_brute_force"),
    ("the recent window is not protected",
     "    return int(np.argmin(acc[:n - n_recent]))", "    return int(np.argmin(acc))", "test_h2o_selection_rule"),
    ("the heaviest token is evicted",
     "    return int(np.argmin(acc[:n - n_recent]))", "    return int(np.argmax(acc[:n - n_recent]))",
     "test_h2o_selection_rule"),
    ("rotary, after pruning: a key is rotated to its slot index, not to its position",
     "K_rot = ea_oracle.rope_rotate(K_up, pk, base)", "K_rot = ea_oracle.rope_rotate(K_up, np.arange(n), base)",
     "test_a_kept_token_scores_as_in_the_sequence_it_was_kept_from"),
    ("rotary, after pruning: the query is rotated to the last slot index",
     "q_rot = ea_oracle.rope_rotate(q[b, i], int(pos_q[b]), base)", "q_rot = ea_oracle.rope_rotate(q[b, i], n - 1, base)",
     "test_a_kept_token_scores_as_in_the_sequence_it_was_kept_from"),
    ("rotary, after pruning: the query turns the other way",
     "q_rot = ea_oracle.rope_rotate(q[b, i], int(pos_q[b]), base)", "q_rot = ea_oracle.rope_rotate(q[b, i], -int(pos_q[b]), base)",
     "test_rope_positions_against_the_complex_form_slot_order_and_a_common_shift"),
    ("rotary, after pruning: scores divided by sqrt(r_k)",
     "p = ea_oracle.softmax((K_rot @ q_rot) / np.sqrt(d_head))", "p = ea_oracle.softmax((K_rot @ q_rot) / np.sqrt(Uk.shape[1]))",
     "test_rope_positions_against_the_complex_form_slot_order_and_a_common_shift"),
    ("rotary, after pruning: keys brought back to d_h channels with rows of the basis instead of its transpose",
     "K_up = cache.K[b][g] @ Uk.T ", "K_up = cache.K[b][g] @ Uk[:cache.K[b][g].shape[1], :] ",
     "test_rope_positions_reduce_to_the_plain_rotary_form_when_nothing_was_dropped"),
    ("rotary, after pruning: the mass of a kv head sums the wrong heads",
     "            per_kv_head[i // G] += probs[b * H + i]", "            per_kv_head[i % cache.n_kv_heads] += probs[b * H + i]",
     "test_a_kept_token_scores_as_in_the_sequence_it_was_kept_from"),
]


@pytest.mark.parametrize("what,old,new,pin", ATTENTION, ids=[m[0] for m in ATTENTION])
def test_attention_oracle_pins_catch(what, old, new, pin):
    assert pin_fails(attention_pins, "ora", mutant(attention_oracle, old, new), pin), f"{pin} did not notice: {what}"


@pytest.mark.parametrize("what,old,new,pin", QUANT, ids=[m[0] for m in QUANT])
def test_quantiser_oracle_pins_catch(what, old, new, pin):
    assert pin_fails(quant_pins, "oq", mutant(quant_oracle, old, new), pin), f"{pin} did not notice: {what}"


@pytest.mark.parametrize("what,old,new,pin", EVICTION, ids=[m[0] for m in EVICTION])
def test_eviction_oracle_pins_catch(what, old, new, pin):
    assert pin_fails(eviction_pins, "oe", mutant(eviction_oracle, old, new), pin), f"{pin} did not notice: {what}"


def test_the_unplanted_copy_passes():
    """The machinery itself: a copy with nothing changed passes the same pins."""
    same = mutant(attention_oracle, "F64 = np.float64", "F64 = np.float64")
    for pin in sorted({m[3] for m in ATTENTION}):
        assert not pin_fails(attention_pins, "ora", same, pin), pin
