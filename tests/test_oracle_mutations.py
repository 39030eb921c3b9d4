"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source
(a transposed index, a dropped offset, an inclusive scan, a reversed loop, a wrong sign or bias),
builds it on the CPU and checks that at least one pin test fails against it."""
import ctypes
import os
import subprocess

import pytest

import oracle
import tests.test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "bls_oracle.c")

MUTATIONS = {
    "counts transposed": ("sendcounts[s * P + d] += 1;", "sendcounts[d * P + s] += 1;"),
    "send displacements inclusive": ("{ sdispls[s * P + d] = run; run += sendcounts[s * P + d]; }",
                                     "{ run += sendcounts[s * P + d]; sdispls[s * P + d] = run; }"),
    "recv displacements not accumulated": ("{ rdispls[d * P + s] = run; run += recvcounts[d * P + s]; }",
                                           "{ rdispls[d * P + s] = run; run += 0; }"),
    "placement not stable": ("for (l = offsets[g]; l < offsets[g + 1]; ++l) {\n                int64_t idx = indices[l], r, rank;",
                             "for (l = offsets[g + 1] - 1; l >= offsets[g]; --l) {\n                int64_t idx = indices[l], r, rank;"),
    "local row not rebased": ("r = idx - (int64_t)d * rps;", "r = idx;"),
    "plain sum wrong sign": ("a32 += x;", "a32 -= x;"),
    "plain sum drops first term": ("for (l = offsets[g]; l < offsets[g + 1]; ++l) {\n                    float x",
                                   "for (l = offsets[g] + 1; l < offsets[g + 1]; ++l) {\n                    float x"),
    "pool ignores shard base": ("float x = elem(tables[t], dtype, D, shard_first + ridx[j], c);",
                                "float x = elem(tables[t], dtype, D, ridx[j], c);"),
    "weights not carried": ("rweights[rbase[d] + rdispls[d * P + s] + rank] = weights[l];",
                            "rweights[rbase[d] + rdispls[d * P + s] + rank] = weights[offsets[g]];"),
    "weighted term fused into double": ("float term = weights[l] * x;\n                        a64", "float term = (float)((double)weights[l] * 1.0000001 * x);\n                        a64"),
    "pool weight of the neighbour": ("float term = rweights[j] * x; acc += term;", "float term = rweights[segoff[sg]] * x; acc += term;"),
    "mean divides by length + 1": ("a32 /= (float)(offsets[g + 1] - offsets[g]);", "a32 /= (float)(offsets[g + 1] - offsets[g] + 1);"),
    "unpack mean uses the wrong bag": ("int64_t g = (int64_t)t * B + f + b_loc, len", "int64_t g = (int64_t)t * B + b_loc, len"),
    "pool column transposed": ("y[c] = acc;", "y[D - 1 - c] = acc;"),
    "pack drops mini-batch offset": ("Y + ybase + ((int64_t)tl * B + f + b_loc) * D, sizeof(float) * D);",
                                     "Y + ybase + ((int64_t)tl * B + b_loc) * D, sizeof(float) * D);"),
    "exchange block sizes from the other side": ("prcount[s * P + d] = pcount[d * P + s];", "prcount[s * P + d] = pcount[s * P + d];"),
    "unpack keeps only the last partial": ("for (c = 0; c < D; ++c) o[c] += r[c];", "for (c = 0; c < D; ++c) o[c] = r[c];"),
    "unpack reads local table index t": ("R + rbase + blk + ((int64_t)loc[t] * n + b_loc) * D;",
                                         "R + rbase + blk + ((int64_t)(part_kind ? loc[t] : 0) * n + b_loc) * D;"),
    "half exponent bias": ("bits = sign | ((e + 127 - 15) << 23) | (m << 13);", "bits = sign | ((e + 127 - 16) << 23) | (m << 13);"),
    "row-quantised scale and bias swapped": ("memcpy(&scale, p + D, 4);\n        memcpy(&bias, p + D + 4, 4);",
                                             "memcpy(&bias, p + D, 4);\n        memcpy(&scale, p + D + 4, 4);"),
    "row-quantised stride not padded": ("return ((int64_t)D + 8 + 15) / 16 * 16;", "return (int64_t)D + 8;"),
    "row-quantised codes read as signed": ("(dtype == 2 ? (float)p[c] :", "(dtype == 2 ? (float)(int8_t)p[c] :"),
    "row-quantised decoding rounded once": ("prod = (dtype == 2 ? (float)p[c] : e4m3_to_float(p[c])) * scale;\n        return prod + bias;",
                                            "return (float)((double)(dtype == 2 ? (float)p[c] : e4m3_to_float(p[c])) * (double)scale + (double)bias);"),
    "layer weight read transposed": ("double w = (double)W[(int64_t)n * K + k], xv = x[m * K + k];",
                                     "double w = (double)W[(int64_t)k * N + n], xv = x[m * K + k];"),
    "layer bias dropped": ("double acc = bias ? (double)bias[n] : 0.0;", "double acc = 0.0;"),
    "relu lets negatives through": ("if (act == 1) v = acc > 0.0 ? acc : 0.0;", "if (act == 1) v = acc;"),
    "sigmoid of the wrong sign": ("v = 1.0 / (1.0 + exp(-acc));", "v = 1.0 / (1.0 + exp(acc));"),
    "interaction pairs ordered by j": ("for (i = 1; i <= T; ++i)\n            for (j = 0; j < i; ++j) {\n                const float *ei",
                                       "for (j = 0; j < T; ++j)\n            for (i = j + 1; i <= T; ++i) {\n                const float *ei"),
    "interaction keeps the diagonal": ("for (j = 0; j < i; ++j) {\n                const float *ei", "for (j = 1; j <= i; ++j) {\n                const float *ei"),
    "interaction pairs the wrong embedding": ("(double)emb[(b * T + (j - 1)) * D + c]", "(double)emb[(b * T + j) * D + c]"),
    "e4m3 exponent bias": ("uint32_t bits = ((uint32_t)(e + 120) << 23) | ((uint32_t)m << 20);", "uint32_t bits = ((uint32_t)(e + 119) << 23) | ((uint32_t)m << 20);"),
    "e4m3 subnormals flushed": ("if (e == 0) mag = (float)m * 0.001953125f;", "if (e == 0) mag = 0.0f;"),
    "e4m3 sign dropped": ("return (v & 0x80u) ? -mag : mag;", "return mag;"),
    "single-bag sum accumulated in double": ("for (j = 0; j < n; ++j) { a32 += rows_nd[j * D + c]; a64 += (double)rows_nd[j * D + c]; }\n        if (out32) out32[c] = a32;",
                                             "for (j = 0; j < n; ++j) { a32 += rows_nd[j * D + c]; a64 += (double)rows_nd[j * D + c]; }\n        if (out32) out32[c] = (float)a64;"),
    "single-bag sum in reverse order": ("for (j = 0; j < n; ++j) { a32 += rows_nd[j * D + c];", "for (j = n - 1; j >= 0; --j) { a32 += rows_nd[j * D + c];"),
    "single-bag sum drops the last row": ("for (j = 0; j < n; ++j) { a32 += rows_nd[j * D + c];", "for (j = 0; j + 1 < n; ++j) { a32 += rows_nd[j * D + c];"),
    "single-bag sum reads the neighbouring column": ("{ a32 += rows_nd[j * D + c]; a64 += (double)rows_nd[j * D + c]; }",
                                                     "{ a32 += rows_nd[j * D + (c + 1) % D]; a64 += (double)rows_nd[j * D + (c + 1) % D]; }"),
    "tolerance mass over one lookup too many": ("double a = 0.0;\n                for (l = offsets[g]; l < offsets[g + 1]; ++l) {\n                    double x",
                                                "double a = 0.0;\n                for (l = offsets[g]; l < offsets[g + 1] + (g + 1 < (int64_t)T * B); ++l) {\n                    double x"),
    "tolerance mass over the next bag too": ("double a = 0.0;\n                for (l = offsets[g]; l < offsets[g + 1]; ++l) {\n                    double x",
                                             "double a = 0.0;\n                for (l = offsets[g]; l < offsets[g + 1 < (int64_t)T * B ? g + 2 : g + 1]; ++l) {\n                    double x"),
    "tolerance mass without the absolute value": ("a += x < 0 ? -x : x;", "a += x;"),
    "tolerance mass doubled": ("mass[((int64_t)b * T + t) * D + c] = a;", "mass[((int64_t)b * T + t) * D + c] = 2.0 * a;"),
    "half subnormals flushed": ("if (m == 0) bits = sign;\n        else {", "if (m >= 0) bits = sign;\n        else {"),
}

PINS = [
    lambda: pins.test_plan_matches_brute_force(pins.TINY[1], 3),
    lambda: pins.test_plan_matches_brute_force(pins.TINY[2], 3),
    lambda: pins.test_pipeline_out_matches_brute_force_and_plain(pins.TINY[1]),
    lambda: pins.test_pipeline_out_matches_brute_force_and_plain(pins.TINY[2]),
    lambda: pins.test_pooling_one_is_a_row_copy_and_integer_tables(),
    lambda: pins.test_pack_exchange_unpack_addresses(pins.TINY[1]),
    lambda: pins.test_pack_exchange_unpack_addresses(pins.TINY[2]),
    lambda: pins.test_against_torch_embedding_bag(5, "small"),
    lambda: pins.test_half_conversion_all_bit_patterns(),
    lambda: pins.test_weighted_and_mean_match_brute_force(pins.TINY[1]),
    lambda: pins.test_weighted_and_mean_match_brute_force(pins.TINY[2]),
    lambda: pins.test_weighted_and_mean_against_torch(3),
    lambda: pins.test_weights_exact_cases(),
    lambda: pins.test_rowq_worked_example(),
    lambda: pins.test_rowq_stride_and_padding(),
    lambda: pins.test_rowq_decoding_rounds_twice_in_fp32(),
    lambda: pins.test_rowq_pipeline_against_decoded_fp32_tables(1),
    lambda: pins.test_e4m3_decoder_all_codes(),
    lambda: pins.test_f8rq_worked_example_and_decoded_tables(),
    lambda: pins.test_mlp_layer_brute_force_and_closed_forms(),
    lambda: pins.test_mlp_layer_against_torch_linear(2),
    lambda: pins.test_interact_brute_force_order_and_torch(),
    lambda: pins.test_bag_sum_is_the_ordered_fp32_sum(70),
    lambda: pins.test_bag_sum_signed_zero_and_exact_cases(),
    lambda: pins.test_absmass_is_the_sum_of_magnitudes(pins.TINY[1], "fp32"),
    lambda: pins.test_absmass_bounds_the_plain_sums_tightly(),
]


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, f"pattern for '{name}' no longer in the oracle source"
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new, 1))
    lib = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-ffp-contract=off", "-std=c99", "-shared", "-fPIC", "-o", str(lib), str(mutated), "-lm"])
    monkeypatch.setattr(oracle, "_lib", ctypes.CDLL(str(lib)))
    caught = 0
    for pin in PINS:
        try:
            pin()
        except (AssertionError, oracle.OracleError):
            caught += 1
    assert caught >= 1, f"no pin noticed: {name}"


def test_pins_pass_on_the_real_oracle():
    for pin in PINS:
        pin()
