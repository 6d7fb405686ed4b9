"""Plant one mistake at a time in a COPY of the oracle's C source (on the CPU, in a temp
directory) and check that the pins notice: a plausible slip anywhere in the oracle -- a
wrong sign, a dropped term, a swapped index, a wrong constant -- must fail at least one
pin.  The committed oracle itself is never modified."""
import os
import subprocess

import pytest

import oracle
from oracle_pins import ALL_PINS

SRC = os.path.join(os.path.dirname(oracle.__file__), "brq_oracle.c")

# (name, text in brq_oracle.c, replacement)
MUTANTS = [
    ("butterfly_diff_sign", "v[i + h] = a - b;", "v[i + h] = b - a;"),
    ("butterfly_descending", "for (int64_t h = 1; h < B; h *= 2)\n        for (int64_t i = 0; i < B; ++i)",
     "for (int64_t h = B / 2; h >= 1; h /= 2)\n        for (int64_t i = 0; i < B; ++i)"),
    ("butterfly_missing_last_stage", "for (int64_t h = 1; h < B; h *= 2)\n        for (int64_t i = 0; i < B; ++i)",
     "for (int64_t h = 1; h < B / 2; h *= 2)\n        for (int64_t i = 0; i < B; ++i)"),
    ("no_normalisation", "float out = v[i] * c;", "float out = v[i];"),
    ("norm_is_1_over_B", "return (float)(1.0 / sqrt((double)B));", "return (float)(1.0 / (double)B);"),
    ("hadamard_or_instead_of_and", "popcount_u32((uint32_t)i & (uint32_t)j)", "popcount_u32((uint32_t)i | (uint32_t)j)"),
    ("sylvester_wrong_corner", "out[(i + n) * B + (j + n)] = -h;", "out[(i + n) * B + (j + n)] = h;"),
    ("dense_transposed_block", "x[r * K + b * B + i] * (double)oracle_hadamard_entry((int)B, (int)i, (int)j)",
     "x[r * K + b * B + j] * (double)oracle_hadamard_entry((int)B, (int)i, (int)j)"),
    ("e2m1_bias_0", "ldexp(1.0 + 0.5 * m, E - 1)", "ldexp(1.0 + 0.5 * m, E)"),
    ("e2m1_no_subnormal", ": 0.5 * m;", ": 0.0;"),
    ("scale_emax_3", "e = (ex - 1) - 2;", "e = (ex - 1) - 3;"),
    ("scale_ceil", "e = (ex - 1) - 2;", "e = ex - 2;"),
    ("scale_bias_128", "return (uint8_t)(e + 127);", "return (uint8_t)(e + 128);"),
    ("ties_to_odd", "(d == bestd && (c & 1) == 0)", "(d == bestd && (c & 1) == 1)"),
    ("ties_down", "(d == bestd && (c & 1) == 0)", "0"),
    ("negative_zero_kept", "if (best == 0) return 0;", ""),
    ("sign_dropped", "(signbit(y) ? 8 : 0)", "0"),
    ("nibbles_swapped", "(uint8_t)(lo | (hi << 4))", "(uint8_t)(hi | (lo << 4))"),
    ("group_of_16", "for (int i = 0; i < 32; ++i) {\n        float a = fabsf(y[i]);", "for (int i = 0; i < 16; ++i) {\n        float a = fabsf(y[i]);"),
    ("amax_without_abs", "float a = fabsf(y[i]);", "float a = y[i];"),
    ("dequant_nibbles_swapped", "(k & 1) ? (byte >> 4) : (byte & 0xF)", "(k & 1) ? (byte & 0xF) : (byte >> 4)"),
    ("dequant_scale_per_16", "scales[r * (K / 32) + k / 32]", "scales[r * (K / 32) + (k / 16) % (K / 32)]"),
    ("gemm_w_row_pitch", "double p = ad[k] * wd[n * K + k];", "double p = ad[k] * wd[n * (K - 32) + k];"),
    ("bf16_truncates", "u += 0x7FFFu + lsb;", ""),
    ("bf16_half_up", "u += 0x7FFFu + lsb;", "u += 0x8000u;"),
    ("sign_test_inverted", "if (signs && signs[b * B + i] < 0) e = -e;", "if (signs && signs[b * B + i] > 0) e = -e;"),
    ("sign_index_within_block_only", "if (signs && signs[b * B + i] < 0) e = -e;", "if (signs && signs[i] < 0) e = -e;"),
    ("signs_ignored", "if (signs && signs[b * B + i] < 0) e = -e;", ""),
    ("fused_drops_signs", "int rc = oracle_block_rotate_signed(x, xdt, M, K, ldx, B, signs, y, ORACLE_F32, K);",
     "int rc = oracle_block_rotate_signed(x, xdt, M, K, ldx, B, NULL, y, ORACLE_F32, K);"),
    ("swiglu_exp_sign", "return g / (1.0 + exp(-g)) * u;", "return g / (1.0 + exp(g)) * u;"),
    ("swiglu_forgets_up", "return g / (1.0 + exp(-g)) * u;", "return g / (1.0 + exp(-g));"),
    ("swiglu_is_sigmoid_only", "return g / (1.0 + exp(-g)) * u;", "return 1.0 / (1.0 + exp(-g)) * u;"),
    ("swiglu_denominator_without_one", "return g / (1.0 + exp(-g)) * u;", "return g / exp(-g) * u;"),
    ("swiglu_gate_and_up_swapped", "return (float)oracle_swiglu_f64((double)g, (double)u);", "return (float)oracle_swiglu_f64((double)u, (double)g);"),
    ("swiglu_bf16_through_fp32", "q = ldexp(rint(ldexp(a, -quantum)), quantum);", "q = ldexp(rint(ldexp((double)(float)a, -quantum)), quantum);"),
    ("swiglu_bf16_seven_bits", "int quantum = ex - 8;", "int quantum = ex - 7;"),
    ("swiglu_bf16_no_subnormal_quantum", "if (quantum < -133) quantum = -133;", ""),
    ("swiglu_bf16_sign_lost", "(signbit(x) ? 0x8000u : 0u)", "0u"),
    ("swiglu_up_read_with_gate_pitch", "(double)load_elem(up, dt, r * ldu + k));\n            if (hdt == ORACLE_BF16)",
     "(double)load_elem(up, dt, r * ldg + k));\n            if (hdt == ORACLE_BF16)"),
    ("swiglu_fused_skips_bf16", "        if (hdt == ORACLE_BF16) {\n            rc = oracle_swiglu(gate, up, dt, M, K, ldg, ldu, hb, ORACLE_BF16, K);",
     "        if (0) {\n            rc = oracle_swiglu(gate, up, dt, M, K, ldg, ldu, hb, ORACLE_BF16, K);"),
    ("swiglu_fused_never_rotates", "        if (B == 1)\n            rc = signs ?", "        if (B >= 1)\n            rc = signs ?"),
    ("swiglu_fused_drops_signs", "rc = oracle_rotate_quantize_fused_signed(h, ORACLE_F32, M, K, K, B, signs, codes, scales);",
     "rc = oracle_rotate_quantize_fused_signed(h, ORACLE_F32, M, K, K, B, NULL, codes, scales);"),
    ("matrot_transposed", "double rv = (double)Rb[i * 32 + j];", "double rv = (double)Rb[j * 32 + i];"),
    ("matrot_always_first_block", "const float *Rb = R + (nR == 1 ? 0 : b) * 1024;", "const float *Rb = R;"),
    ("matrot_block_pitch", "const float *Rb = R + (nR == 1 ? 0 : b) * 1024;", "const float *Rb = R + (nR == 1 ? 0 : b) * 32;"),
    ("matrot_bound_without_abs", "mag += fabs(xv) * fabs(rv);", "mag += xv * rv;"),
    ("matrot_fused_skips_rotation", "for (int64_t i = 0; i < M * K; ++i) yf[i] = (float)y[i];",
     "for (int64_t i = 0; i < M * K; ++i) yf[i] = load_elem(x, xdt, (i / K) * ldx + i % K);"),
    ("encode_nibbles_swapped", "(uint8_t)((hi << 4) | lo);", "(uint8_t)((lo << 4) | hi);"),
    ("encode_scale_per_row", "uint8_t sb = scales[r * (K / 32) + j / 16];", "uint8_t sb = scales[r * (K / 32)];"),
    ("stats_not_strict", "if (a > thresholds[t]) count[t] += 1;", "if (a >= thresholds[t]) count[t] += 1;"),
    ("stats_amax_signed", "float a = fabsf(v[j]);\n                    if (a > am) am = a;", "float a = v[j];\n                    if (a > am) am = a;"),
    ("stats_loss_ignores_scale", "oracle_e2m1_value(code) * oracle_e8m0_value(sb);", "oracle_e2m1_value(code);"),
    ("stats_loss_not_squared", "loss += d * d;", "loss += fabs(d);"),
    ("stats_never_rotates", "    if (B == 1) {\n        for (int64_t r = 0; r < M; ++r)\n            for (int64_t k = 0; k < K; ++k) y[r * K + k]", "    if (B >= 1) {\n        for (int64_t r = 0; r < M; ++r)\n            for (int64_t k = 0; k < K; ++k) y[r * K + k]"),
    ("stats_nibbles_swapped", "int code = (j & 1) ? (codes16[j / 2] >> 4) : (codes16[j / 2] & 0xF);", "int code = (j & 1) ? (codes16[j / 2] & 0xF) : (codes16[j / 2] >> 4);"),
    ("summary_bin_not_strict", "if (amax[i] > edges[e]) bin += 1;", "if (amax[i] >= edges[e]) bin += 1;"),
    ("summary_outlier_not_strict", "int outl = r > outlier;", "int outl = r >= outlier;"),
    ("summary_classifies_by_own_scale", "float r = ref ? ref[i] : amax[i];\n        int outl", "float r = amax[i];\n        int outl"),
    ("summary_grew_not_strict", "if (ref && amax[i] > r) counts[2 + outl] += 1;", "if (ref && amax[i] >= r) counts[2 + outl] += 1;"),
    ("summary_loss_classes_swapped", "if (sqerr) sums[outl] += (double)sqerr[i];", "if (sqerr) sums[1 - outl] += (double)sqerr[i];"),
    ("summary_scale_sum_unsplit", "sums[2 + outl] += (double)amax[i];", "sums[2] += (double)amax[i];"),
    ("bfp4_scale_max_4", "const float s = oracle_round_to_f16(am / 6.0f);", "const float s = oracle_round_to_f16(am / 4.0f);"),
    ("bfp4_scale_not_rounded", "const float s = oracle_round_to_f16(am / 6.0f);", "const float s = am / 6.0f;"),
    ("bfp4_dequant_without_scale", "oracle_e2m1_value(code) * (double)s;", "oracle_e2m1_value(code);"),
    ("f16_truncates", "b += 0xFFFu + lsb; /* keep 10 mantissa bits */", "/* keep 10 mantissa bits */"),
    ("f16_no_saturation", "if (a >= 65520.0f) a = 65504.0f;", "if (0) a = 65504.0f;"),
    ("fused_skips_rotation", "if (rc == ORACLE_OK) rc = oracle_mxfp4_quantize(y, ORACLE_F32, M, K, K, codes, scales);",
     "rc = oracle_mxfp4_quantize(x, xdt, M, K, ldx, codes, scales);"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation site for %s not found exactly once" % name
    c = tmp_path / "mutant.c"
    c.write_text(src.replace(old, new))
    so = tmp_path / ("mutant_%s.so" % name)
    subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-w",
                           "-o", str(so), str(c), "-lm"])
    mutant = oracle.Oracle(str(so))
    failed = []
    for pin in ALL_PINS:
        try:
            pin(mutant)
        except Exception:  # a pin may also trip over a crash-free but malformed result
            failed.append(pin.__name__)
    assert failed, "no pin notices the planted mistake '%s'" % name
