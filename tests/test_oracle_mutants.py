"""How strong are the oracle's pins?  Each case plants one plausible mistake in a copy of the oracle's C
source (on the CPU; the GPU path is not involved), builds it, swaps it in behind the oracle's Python
wrapper and runs the pin tests: at least one pin must fail for every planted mistake.  A mutant that
survived would mean the pins leave that part of the oracle unchecked."""
import ctypes as C
import inspect
import os
import subprocess

import pytest

from oracle import q8_oracle as O
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(O.__file__), "q8_oracle.c")

MUTANTS = [
    ("ties_toward_zero", "if (fabsf(frac) >= 0.5f) t +=", "if (fabsf(frac) > 0.5f) t +="),
    ("ties_to_even", "    float t = truncf(p);\n    float frac = p - t;\n    if (fabsf(frac) >= 0.5f) t += (p < 0.0f) ? -1.0f : 1.0f;\n    return t;",
     "    return rintf(p);"),
    ("add_half_then_truncate", "    float t = truncf(p);\n    float frac = p - t;\n    if (fabsf(frac) >= 0.5f) t += (p < 0.0f) ? -1.0f : 1.0f;\n    return t;",
     "    return truncf(p + ((p < 0.0f) ? -0.5f : 0.5f));"),
    ("no_clamp", "        r = fminf(fmaxf(r, -m), m); /* Clamp(x,a,b) = min(max(x,a),b) */", "        (void)m;"),
    ("clamp_at_128", "        r = fminf(fmaxf(r, -m), m); /* Clamp(x,a,b) = min(max(x,a),b) */", "        r = fminf(fmaxf(r, -m - 1.0f), m);"),
    ("scale_inverted", "float s = (amax == 0.0f) ? 1.0f : m / amax;", "float s = (amax == 0.0f) ? 1.0f : amax / m;"),
    ("scale_from_128", "static double top_value(int bits) { return ldexp(1.0, bits - 1) - 1.0; }", "static double top_value(int bits) { return ldexp(1.0, bits - 1); }"),
    ("absmax_of_signed", "        float v = fabsf(x[i]);\n        if (v > a) a = v;", "        float v = x[i];\n        if (v > a) a = v;"),
    ("bias_without_weight_scale", "        float sb = sx * sw[j / per];", "        float sb = sx;"),
    ("bias_truncated", "        double r = (double)round_half_away(p);", "        double r = (double)truncf(p);"),
    ("gemm_transposed_weight", "(int64_t)wq[n * K + k];", "(int64_t)wq[(k * N + n) % (N * K)];"),
    ("gemm_drops_bias", "            int64_t s = bq ? (int64_t)bq[n] : 0;", "            int64_t s = 0; (void)bq;"),
    ("gemm_skips_last_k", "            for (int64_t k = 0; k < K; ++k)\n                s += (int64_t)xq[m * K + k]", "            for (int64_t k = 0; k < K - 1; ++k)\n                s += (int64_t)xq[m * K + k]"),
    ("gemm_int8_as_unsigned", "s += (int64_t)xq[m * K + k] *", "s += (int64_t)(uint8_t)xq[m * K + k] *"),
    ("dequant_by_sx_only", "            double s = (double)sx * (double)sw[n / per];", "            double s = (double)sx; (void)per;"),
    ("dequant_multiplies", "(float)((double)acc[m * N + n] / s);", "(float)((double)acc[m * N + n] * s);"),
    ("gelu_wrong_tail", "erfc(-d / sqrt(2.0))", "erfc(d / sqrt(2.0))"),
    ("gelu_tanh_form", "out[i] = (float)(0.5 * d * erfc(-d / sqrt(2.0)));", "out[i] = (float)(0.5 * d * (1.0 + tanh(0.7978845608028654 * (d + 0.044715 * d * d * d))));"),
    ("embedding_wrong_row", "int8_t q = table[id * H + h];", "int8_t q = table[((id + 1) % V) * H + h];"),
    ("embedding_multiplies_scale", "(float)((double)q / (double)scale);", "(float)((double)q * (double)scale);"),
    ("sum3_one_scale_for_all", "(double)pos[b * H + h] / (double)sp)", "(double)pos[b * H + h] / (double)sw_)"),
    ("fake_quantize_multiplies", "        xq[i] = r / scale;", "        xq[i] = r * scale;"),
    ("fake_quantize_no_rounding", "        float r = round_half_away(p);\n        r = fminf(fmaxf(r, -m), m);\n        xq[i] = r / scale;",
     "        float r = fminf(fmaxf(p, -m), m);\n        xq[i] = r / scale;"),
    ("ema_weights_swapped", "    float keep = decay * ema_prev;\n    float w = 1.0f - decay;\n    float take = w * amax;",
     "    float keep = decay * amax;\n    float w = 1.0f - decay;\n    float take = w * ema_prev;"),
    ("ema_ignores_first_batch", "    if (!initialized) {\n        *ema_out = amax;", "    if (!initialized) {\n        *ema_out = 0.0f;"),
    ("ste_scales_gradient", "grad_x[i] = grad_xq[i] * 1.0f;", "grad_x[i] = grad_xq[i] * 0.5f;"),
    ("layernorm_unbiased_variance", "double rstd = 1.0 / sqrt(ss / (double)H + eps);", "double rstd = 1.0 / sqrt(ss / (double)(H - 1) + eps);"),
    ("layernorm_no_mean", "double mean = sum / (double)H, ss = 0.0;", "double mean = 0.0 * sum, ss = 0.0;"),
    ("layernorm_drops_residual", "float x = pr ? pa[h] + pr[h] : pa[h];\n            y[m * H + h]", "float x = pa[h];\n            y[m * H + h]"),
    ("attention_no_scale", "s[j] = scale * dot + (mask", "s[j] = dot + (mask"),
    ("attention_keys_are_queries", "const float *k = qkv + (b * S + j) * ld + HD + h * d;", "const float *k = qkv + (b * S + j) * ld + h * d;"),
    ("attention_values_are_keys", "o += s[j] * (double)qkv[(b * S + j) * ld + 2 * HD + h * d + c];", "o += s[j] * (double)qkv[(b * S + j) * ld + HD + h * d + c];"),
    ("attention_mask_by_query", "(double)mask[b * S + j] : 0.0);", "(double)mask[b * S + i] : 0.0);"),
    ("attention_not_normalised", "(float)(o / den);", "(float)(o);"),
    ("attention_head_offset_dropped", "const float *q = qkv + (b * S + i) * ld + h * d;", "const float *q = qkv + (b * S + i) * ld;"),
    ("attention_mask_of_sequence_0", "(double)mask[b * S + j] : 0.0);", "(double)mask[j] : 0.0);"),
    ("layernorm_beta_scaled", "* (double)gamma[h] + (double)beta[h]);", "* (double)gamma[h] + (double)beta[h] * (double)gamma[h]);"),
]


def _pin_functions():
    return [(n, f) for n, f in inspect.getmembers(pins, inspect.isfunction) if n.startswith("test_")]


def _run_pins(golden_dir):
    """Names of the pins that fail (assertion or oracle error) with the library currently swapped in."""
    failed = []
    for name, fn in _pin_functions():
        params = list(inspect.signature(fn).parameters)
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [{}]
        for m in marks:                                   # expand @pytest.mark.parametrize by hand
            keys = [k.strip() for k in m.args[0].split(",")]
            cases = [dict(c, **dict(zip(keys, v if isinstance(v, (tuple, list)) else (v,)))) for c in cases for v in m.args[1]]
        for case in cases:
            kw = dict(case)
            if "golden_dir" in params:
                kw["golden_dir"] = golden_dir
            try:
                fn(**kw)
            except KeyboardInterrupt:
                raise
            except BaseException:                         # noqa: BLE001 -- assertion, oracle error or pytest.fail: caught
                failed.append(name)
                break
    return failed


def test_the_unmutated_oracle_passes_every_pin(golden_dir):
    assert _run_pins(golden_dir) == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, golden_dir, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site of {name} not found: the oracle changed, update this list"
    mutated = tmp_path / "q8_oracle_mutant.c"
    mutated.write_text(src.replace(old, new, 1))
    so = tmp_path / "libq8_oracle_mutant.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
                    "-o", str(so), str(mutated), "-lm"], check=True)
    good = O.lib()
    try:
        O._lib = C.CDLL(str(so))
        failed = _run_pins(golden_dir)
    finally:
        O._lib = good
    assert failed, f"no pin notices the planted mistake '{name}'"
