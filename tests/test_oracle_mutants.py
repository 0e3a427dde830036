"""Do the pins pin?  Each case plants one plausible mistake in a copy of the oracle's source (a wrong sign, a
dropped normalization, a transposed index, a different rounding or tie rule, a constant off by one) and runs the
pin tests of test_oracle_pins.py against the mutated copy: at least one pin must fail.  A mistake that no pin
notices means the oracle is not pinned there.  CPU only; nothing here touches the HIP path."""
import importlib
import os
import types

import pytest

import test_oracle_pins as pins

ORACLE_SRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", "oracle", "polykv_oracle.py")

# (what is planted, text in the oracle, replacement, pins that are expected to notice -- run first)
MUTANTS = [
    ("butterfly with the wrong sign", "z[..., 1, :] = a - b", "z[..., 1, :] = b - a",
     ["test_fwht_equals_dense_sylvester_matrix"]),
    ("butterfly stage skipped", "        h *= 2\n    return y", "        h *= 4\n    return y",
     ["test_fwht_equals_dense_sylvester_matrix"]),
    ("forward rotation not normalized", "    return fwht(v) / math.sqrt(d)\n", "    return fwht(v)\n",
     ["test_v_codec_statistics_on_gaussian_input", "test_v_decode_inverts_rotation_exactly_when_no_quantization_error"]),
    ("dequantization divides by d (the printed text taken literally)", "v = fwht(c[idx]) / math.sqrt(d)",
     "v = fwht(c[idx]) / d",
     ["test_v_decode_inverts_rotation_exactly_when_no_quantization_error", "test_end_to_end_pool_roundtrip_and_linearity_of_rotation"]),
    ("a tie goes to the upper centroid", "idx += (v_rot > tk).astype(np.uint8)", "idx += (v_rot >= tk).astype(np.uint8)",
     ["test_v_encode_single_spike_and_constant_vectors", "test_v_quantize_is_bruteforce_nearest_centroid"]),
    ("thresholds are not the midpoints", "        t = 0.5 * (c[:-1] + c[1:])\n        edges", "        t = 0.45 * (c[:-1] + c[1:])\n        edges",
     ["test_codebook_rounds_to_paper_values", "test_codebook_fixed_point_by_numerical_integration"]),
    ("centroids are cell midpoints, not conditional means", "new[k] = (_phi(a) - _phi(b)) / (_Phi(b) - _Phi(a))",
     "new[k] = 0.5 * (max(a, -3.0) + min(b, 3.0))",
     ["test_codebook_rounds_to_paper_values", "test_codebook_fixed_point_by_numerical_integration"]),
    ("key scale is absmax / 128", "s16 = np.minimum((amax / np.float32(127.0)).astype(np.float32), np.float32(FP16_MAX))",
     "s16 = np.minimum((amax / np.float32(128.0)).astype(np.float32), np.float32(FP16_MAX))",
     ["test_q8_error_bound_and_extremes", "test_q8_special_blocks_and_scale_invariance"]),
    ("key codes formed with the unrounded scale", "    s32 = s16.astype(np.float32)\n    with np.errstate(divide=\"ignore\"):\n        inv = np.where(s32 > 0, np.float32(1.0) / s32, np.float32(0.0)).astype(np.float32)\n    pre",
     "    s32 = (amax / np.float32(127.0)).astype(np.float32)\n    with np.errstate(divide=\"ignore\"):\n        inv = np.where(s32 > 0, np.float32(1.0) / s32, np.float32(0.0)).astype(np.float32)\n    pre",
     ["test_q8_codes_are_bruteforce_nearest_multiples_of_stored_scale"]),
    ("bit stream packed most significant bit first", "    return np.packbits(stream, axis=-1, bitorder=\"little\")",
     "    return np.packbits(stream, axis=-1, bitorder=\"big\")", ["test_pack_layout_hand_computed"]),
    ("code bits in the stream most significant first", "stream = ((idx[..., :, None] >> np.arange(bits, dtype=np.uint8)) & 1).astype(np.uint8)",
     "stream = ((idx[..., :, None] >> np.arange(bits, dtype=np.uint8)[::-1]) & 1).astype(np.uint8)",
     ["test_pack_layout_hand_computed"]),
    ("attention scale 1/d", "        scale = 1.0 / math.sqrt(d)\n    out = np.zeros_like(Q)", "        scale = 1.0 / d\n    out = np.zeros_like(Q)",
     ["test_attend_matches_pure_python_bruteforce_with_gqa_and_tails", "test_attend_special_cases_and_agent_count_invariance"]),
    ("softmax without the normalization", "    p /= np.sum(p)\n", "    p = p\n",
     ["test_attend_matches_pure_python_bruteforce_with_gqa_and_tails", "test_attend_special_cases_and_agent_count_invariance"]),
    ("query head h reads KV head h mod H", "                kv = h // G\n", "                kv = h % H\n",
     ["test_attend_matches_pure_python_bruteforce_with_gqa_and_tails"]),
    ("causal tail off by one", "seen = max(0, t_a - (nq - 1 - i)) if tail_causal else t_a", "seen = max(0, t_a - (nq - i)) if tail_causal else t_a",
     ["test_causal_tail_attention_equals_dense_masked_attention"]),
    ("value scale is the norm, not the root mean square", "    rms = np.sqrt(np.mean(v * v, axis=-1))", "    rms = np.sqrt(np.sum(v * v, axis=-1))",
     ["test_scaled_values_closed_forms", "test_scaled_values_match_turboquant_on_unit_vectors"]),
    ("scaled thresholds divided by the scale", "idx += (v_rot > tk * g).astype(np.uint8)", "idx += (v_rot * g > tk).astype(np.uint8)",
     ["test_scaled_values_are_the_unscaled_codec_on_the_normalized_vector", "test_scaled_values_closed_forms"]),
    ("sign diagonal from bit 1 of the generator's output", "-1.0 if z & 1 else 1.0", "-1.0 if z & 2 else 1.0",
     ["test_sign_diagonal_generator_matches_published_splitmix64_vectors", "test_sign_diagonal_rotation_is_orthonormal_and_equals_the_dense_matrix"]),
    ("generator multiplier mistyped", "0xBF58476D1CE4E5B9", "0xBF58476D1CE4E5B7",
     ["test_sign_diagonal_generator_matches_published_splitmix64_vectors"]),
    ("sign diagonal applied after the transform in the forward rotation", "    return fwht(v) / math.sqrt(d)\n", "    return fwht(np.asarray(V, dtype=np.float64)) * (1.0 if signs is None else signs) / math.sqrt(d)\n",
     ["test_sign_diagonal_rotation_is_orthonormal_and_equals_the_dense_matrix"]),
    ("stored bytes without the block scales", "    packed = k_codes + k_scales + v_codes + v_scales", "    packed = k_codes + v_codes + v_scales",
     ["test_compression_accounting_matches_paper"]),
    ("int8 value scale is absmax / 128", "s16 = np.minimum((amax / np.float32(127.0)).astype(np.float32), np.float32(V_SCALE_MAX))",
     "s16 = np.minimum((amax / np.float32(128.0)).astype(np.float32), np.float32(V_SCALE_MAX))",
     ["test_int8_values_error_bound_extremes_and_bruteforce"]),
    ("int8 value codes truncated instead of rounded", "    q = np.clip(np.rint(pre), -128, 127).astype(np.int8)\n    return q, s16, pre",
     "    q = np.clip(np.trunc(pre), -128, 127).astype(np.int8)\n    return q, s16, pre",
     ["test_int8_values_error_bound_extremes_and_bruteforce"]),
    ("scaled values decoded without their scale", "    return v_decode(idx, signs, bits) * np.asarray(g16).astype(np.float64)[..., None]",
     "    return v_decode(idx, signs, bits)", ["test_scaled_values_scale_invariance_and_distortion", "test_scaled_values_pool_roundtrip_and_bytes"]),
    ("a zero scale stores the code above zero", "np.uint8((1 << bits) // 2 - 1)", "np.uint8((1 << bits) // 2)",
     ["test_scaled_values_closed_forms"]),
    ("b-bit codebook with 2b levels", "_CODEBOOKS[bits] = lloyd_max_gaussian(1 << bits)", "_CODEBOOKS[bits] = lloyd_max_gaussian(2 * bits)",
     ["test_codebooks_of_2_3_4_bits_match_the_published_table_and_the_bound"]),
    ("per-tensor key scale taken per head", "        per_layer = [k_encode(K[l], block=None) for l in range(K.shape[0])]",
     "        per_layer = [k_encode(K[l, :1], block=None) for l in range(K.shape[0])]",
     ["test_per_tensor_key_scale_pool_form_and_the_papers_ratio"]),
    ("unpacking reads the code bits most significant first", "    return (stream << np.arange(bits, dtype=np.uint8)).sum(axis=-1).astype(np.uint8)",
     "    return (stream << np.arange(bits, dtype=np.uint8)[::-1]).sum(axis=-1).astype(np.uint8)",
     ["test_pack_unpack_exhaustive_one_group"]),
    ("value scale not capped", "    return np.minimum(rms, V_SCALE_MAX).astype(np.float16), rms", "    return rms.astype(np.float16), rms",
     ["test_scaled_values_closed_forms"]),
    ("key dequantization with the scale of the neighbouring block", "    return (q * s[..., None]).reshape(codes.shape)",
     "    return (q * np.roll(s, 1, axis=-1)[..., None]).reshape(codes.shape)",
     ["test_q8_error_bound_and_extremes", "test_end_to_end_pool_roundtrip_and_linearity_of_rotation"]),
]


def _load_mutant(old: str, new: str):
    src = open(ORACLE_SRC).read()
    assert src.count(old) >= 1, "the oracle no longer contains %r: update this mutant" % old
    mod = types.ModuleType("polykv_oracle_mutant")
    mod.__file__ = ORACLE_SRC
    exec(compile(src.replace(old, new, 1), ORACLE_SRC, "exec"), mod.__dict__)
    return mod


def _calls(fn):
    """The test function's invocations: one per parameter set of its (single) parametrize mark."""
    for mark in getattr(fn, "pytestmark", []):
        if mark.name == "parametrize":
            names, values = mark.args[0], mark.args[1]
            return [lambda v=v: fn(**{names: v}) for v in values]
    return [fn]


def _first_failing_pin(expected):
    every = [n for n in dir(pins) if n.startswith("test_")]
    for name in list(expected) + [n for n in every if n not in expected]:
        for call in _calls(getattr(pins, name)):
            try:
                call()
            except Exception:  # an assertion, or the mutant breaking down altogether
                return name
    return None


@pytest.mark.parametrize("what,old,new,expected", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(what, old, new, expected, monkeypatch):
    mutant = _load_mutant(old, new)
    monkeypatch.setattr(pins, "O", mutant)
    killer = _first_failing_pin(expected)
    assert killer is not None, "no pin notices: " + what


def test_the_unmutated_oracle_passes_the_same_harness(monkeypatch):
    monkeypatch.setattr(pins, "O", importlib.import_module("oracle.polykv_oracle"))
    assert _first_failing_pin([]) is None
