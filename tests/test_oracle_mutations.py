"""Do the pins bite?  Each case plants one plausible mistake in a copy of the
oracle's C source (on the CPU, in a temporary directory), builds it, runs the
pin tests against the mutant, and requires at least one of them to fail."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "fcdp_oracle.c")

SCALED = "int fcdp_oracle_reduce_scaled("

MUTATIONS = {
    "reduce_starts_from_plus_zero": ("            acc = ((const float *)partials[0])[e0 + k];",
                                     "            acc = 0.0f + ((const float *)partials[0])[e0 + k];"),
    "reduce_reverse_rank_order": ("        for (int32_t g = 1; g < G; ++g) {\n            float v;",
                                  "        for (int32_t gg = 1; gg < G; ++gg) {\n            int32_t g = G - gg; if (g == 0) g = 0;\n            float v;"),
    "reduce_drops_last_rank": ("        for (int32_t g = 1; g < G; ++g) {\n            float v;",
                               "        for (int32_t g = 1; g < G - (G > 2); ++g) {\n            float v;"),
    "reduce_ignores_offset": ("                v = ((const float *)partials[g])[e0 + k];",
                              "                v = ((const float *)partials[g])[k];"),
    "bf16_round_half_up": ("    u += 0x7fffu + lsb;", "    u += 0x8000u; (void)lsb;"),
    "bf16_truncates": ("    u += 0x7fffu + lsb;", "    (void)lsb;"),
    "bf16_nan_becomes_inf": ("    if ((u & 0x7fffffffu) > 0x7f800000u)\n        return (uint16_t)((u >> 16) | 0x0040u);",
                             ""),
    "bf16_widening_wrong_shift": ("static float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }",
                                  "static float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 15); }"),
    "layout_pads_to_q_not_Gq": ("    int64_t Q = (int64_t)G * (int64_t)q;\n    int64_t N_pad = ((N + Q - 1) / Q) * Q;\n    *N_out = N;",
                                "    int64_t Q = (int64_t)q;\n    int64_t N_pad = ((N + Q - 1) / Q) * Q;\n    N_pad = ((N_pad + G - 1) / G) * G;\n    *N_out = N;"),
    "flatten_leaves_padding": ("    for (int64_t i = N; i < N_pad; ++i)\n        for (int32_t b = 0; b < esz; ++b)\n            f[i * esz + b] = 0;",
                               "    (void)N_pad;"),
    "materialize_shard_index_off": ("            int64_t k = i % S;\n            if (r >= G) return ORACLE_EINVAL;",
                                    "            int64_t k = (i + (r > 0)) % S;\n            if (r >= G) return ORACLE_EINVAL;"),
    "materialize_from_flat_skips_offset": ("            put_elem(dst, j, f, off_t + j, esz);\n        off_t += n[t];\n    }\n    return ORACLE_OK;\n}\n\n/*\n * Cache store",
                                           "            put_elem(dst, j, f, off_t + j, esz);\n        off_t += n[t] - (t == 0 && n[t] > 0);\n    }\n    return ORACLE_OK;\n}\n\n/*\n * Cache store"),
    "cache_store_reversed_shards": ("            put_elem(h, (int64_t)r * S + k, (const unsigned char *)shards[r],",
                                    "            put_elem(h, (int64_t)(G - 1 - r) * S + k, (const unsigned char *)shards[r],"),
    "segments_wrong_upper_bound": ("            int64_t hi_r = ((int64_t)r + 1) * S;", "            int64_t hi_r = ((int64_t)r + 1) * S - 1;"),
    "pack_no_zero_tail": ("    for (int64_t i = c; i < Np; ++i)\n        for (int32_t b = 0; b < esz; ++b) p[i * esz + b] = 0;",
                          "    (void)Np;"),
    "unpack_writes_frozen_too": ("        if (trainable[t]) {\n            for (int64_t j = 0; j < n[t]; ++j)\n                put_elem(f, off_t + j, p, c + j, esz);\n            c += n[t];\n        }",
                                 "        if (trainable[t] || t == 0) {\n            for (int64_t j = 0; j < n[t]; ++j)\n                put_elem(f, off_t + j, p, c + j, esz);\n            c += n[t];\n        }"),
    # edits of the scaled reduction: (old, new, text after which to look)
    "scaled_forgets_scale": ("        acc = acc * scale;\n", "", SCALED),
    "scaled_divides_by_reciprocal": ("        acc = acc * scale;", "        acc = acc / (1.0f / scale);", SCALED),
    "scaled_scales_the_terms": [
        ("            acc = ((const float *)partials[0])[e0 + k];",
         "            acc = ((const float *)partials[0])[e0 + k] * scale;", SCALED),
        ("            acc = acc + v;", "            acc = acc + v * scale;", SCALED),
        ("        acc = acc * scale;\n", "", SCALED)],
    "scaled_rounds_to_bf16_before_scaling": (
        "        acc = acc * scale;",
        "        if (out_dtype == 0) acc = bf16_to_f32(fcdp_oracle_bf16_rne(acc));\n        acc = acc * scale;", SCALED),
    "split_uses_wrong_stride": ("            put_elem(s, k, f, (int64_t)r * S + k, esz);", "            put_elem(s, k, f, (int64_t)r * S + (k + (r > 0)) % S, esz);"),
}

# pin tests run against every mutant (name, args)
CHECKS = [
    (pins.test_brute_force_tiny_layers, [(G, seed) for G in (1, 3, 4) for seed in (0, 1, 2, 4)]),
    (pins.test_layout_invariants, [(G, seed) for G in (2, 8) for seed in (0, 3)]),
    (pins.test_materialize_never_reads_padding, [()]),
    (pins.test_baseline_config_sizes, [()]),
    (pins.test_paper_model_sizes_and_cache_bytes, [()]),
    (pins.test_reduce_matches_float32_loop, [(3,), (8,)]),
    (pins.test_reduce_order_and_start_value, [()]),
    (pins.test_reduce_bf16_inputs, [()]),
    (pins.test_reduce_shards_concatenate_to_full_sum, [()]),
    (pins.test_scaled_reduce_special_cases, [()]),
    (pins.test_scaled_reduce_hand_worked_cases, [()]),
    (pins.test_bf16_rne_hand_worked_cases, [()]),
    (pins.test_bf16_rne_vs_torch_all_boundaries, [()]),
    (pins.test_pack_unpack_invariants, [(3,), (8,)]),
    (pins.test_segment_counts_and_straddles, [()]),
]


def _pins_fail():
    for fn, arglist in CHECKS:
        for args in arglist:
            try:
                fn(*args)
            except (AssertionError, ValueError, IndexError):
                return fn.__name__
    return None


def test_pins_pass_on_the_real_oracle():
    assert _pins_fail() is None


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path):
    edits = MUTATIONS[name]
    if not isinstance(edits, list):
        edits = [edits]
    text = open(SRC).read()
    for edit in edits:
        old, new = edit[0], edit[1]
        start = text.index(edit[2]) if len(edit) > 2 else 0
        assert text.count(old, start) >= 1, \
            "mutation site not found: the oracle changed, update this test"
        text = text[:start] + text[start:].replace(old, new, 1)
    src = tmp_path / "mutant.c"
    src.write_text(text)
    so = tmp_path / "mutant.so"
    subprocess.check_call(["gcc", *[f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")], "-w",
                           "-o", str(so), str(src)])
    real = oracle.lib()
    mutant = ctypes.CDLL(str(so))
    mutant.fcdp_oracle_segments.restype = ctypes.c_int64
    mutant.fcdp_oracle_bf16_rne.restype = ctypes.c_uint16
    mutant.fcdp_oracle_bf16_rne.argtypes = [ctypes.c_float]
    oracle._lib = mutant
    try:
        caught = _pins_fail()
    finally:
        oracle._lib = real
    assert caught is not None, "no pin noticed the planted mistake '%s'" % name
