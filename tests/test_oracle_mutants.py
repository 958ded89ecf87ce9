"""Do the pins bite?  Plant one plausible mistake at a time in a COPY of the oracle's C source
(a dropped term, a wrong sign or index, a swapped operand, a different norm), compile it on the CPU,
run the pin tests against the mutant and require that at least one fails.  CPU only.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins
import test_oracle_topk_pins as topk_pins

MUTANTS = [
    # (id, old text, new text)
    ("compensate_minus", "u[j] = mi + werr[base + j];", "u[j] = mi - werr[base + j];"),
    ("error_negated", "werr[base + j] = u[j] - c[j];", "werr[base + j] = c[j] - u[j];"),
    ("drop_gradient_term", "float mi = bm + bg;", "float mi = bm;"),
    ("drop_momentum_term", "float mi = bm + bg;", "float mi = bg;"),
    ("swap_m_g", "float bm = beta * m[base + j];", "float bm = beta * g[base + j];"),
    ("beta_on_wrong_term", "float bg = one_minus_beta * g[base + j];", "float bg = beta * g[base + j];"),
    ("msb_first", "(uint32_t)1u << (j & 31);", "(uint32_t)1u << (31 - (j & 31));"),
    ("zero_is_negative", "int positive = (u[j] >= 0.0f);", "int positive = (u[j] > 0.0f);"),
    ("scale_not_rooted", "float s = (float)sqrt(mean_sq);", "float s = (float)mean_sq;"),
    ("scale_l1", "S += (long double)u[j] * (long double)u[j];", "S += fabsl((long double)u[j]) * 1e-2L;"),
    ("scale_sum_not_mean", "double mean_sq = (double)S / (double)L;", "double mean_sq = (double)S;"),
    ("scale_float_accum", "long double S = 0.0L;", "float S = 0.0f;"),
    ("decode_flipped", "& 1u) ? scale : -scale;", "& 1u) ? -scale : scale;"),
    ("no_average", "float avg = acc * inv_n;", "float avg = acc;"),
    ("server_error_minus", "ubar[j] = avg + serr[base + j];", "ubar[j] = avg - serr[base + j];"),
    ("server_error_not_fed_back", "serr[base + j] = ubar[j] - c[j];", "serr[base + j] = 0.0f;"),
    ("server_reads_worker0", "const int64_t wbase = (int64_t)i * d + base;", "const int64_t wbase = base;"),
    ("server_scale_transposed", "scales[(int64_t)i * C + k],\n", "scales[(int64_t)k * n + i],\n"),
    ("worker_scale_transposed", "&scales[(int64_t)i * C + k], c);", "&scales[(int64_t)k * n + i], c);"),
    ("gather_one_worker", "for (int32_t i = 0; i < n; ++i)\n            m[(int64_t)i * d + j] = mj;",
     "for (int32_t i = 0; i < 1; ++i)\n            m[(int64_t)i * d + j] = mj;"),
    ("no_sqrt_of_v", "float root = sqrtf(v[j]);", "float root = v[j];"),
    ("ascent", "x[j] = x[j] - step;\n    }\n    return 0;\n}\n\n/*\n * APGSqueeze",
     "x[j] = x[j] + step;\n    }\n    return 0;\n}\n\n/*\n * APGSqueeze"),
    ("apply_no_lr", "float step = lr * ratio;\n        x[j] = x[j] - step;\n    }\n    return 0;\n}\n\n/*\n * APGSqueeze",
     "float step = ratio;\n        x[j] = x[j] - step;\n    }\n    return 0;\n}\n\n/*\n * APGSqueeze"),
    ("apg_ascent", "x[j] = x[j] - delta_x;", "x[j] = x[j] + delta_x;"),
    ("apply_scale_of_chunk0", "sscales[k], sdense ? sdense + base : NULL,", "sscales[0], sdense ? sdense + base : NULL,"),
    ("adam_v_uses_g_not_gsq", "float v_inc = omb2 * gsq;", "float v_inc = omb2 * gbar;"),
    ("adam_no_bias_correction_m", "float mhat = m_new / bc1;", "float mhat = m_new;"),
    ("adam_no_bias_correction_v", "float vhat = v_new / bc2;", "float vhat = v_new;"),
    ("adam_t_off_by_one", "pow((double)beta2, (double)t)", "pow((double)beta2, (double)(t - 1) + 1e-9)"),
    ("adam_eps_inside_sqrt", "float root = sqrtf(vhat);", "float root = sqrtf(vhat + 1e-6f);"),
    ("adam_sum_not_mean", "float gbar = acc * inv_n;", "float gbar = acc;"),
    ("apg_compensate_minus", "u[j] = g[base + j] + werr[base + j];", "u[j] = g[base + j] - werr[base + j];"),
    ("apg_momentum_not_decayed", "float keep = beta * m[(int64_t)i * d + j];", "float keep = m[(int64_t)i * d + j];"),
    ("apg_beta_on_gradient", "float inc = one_minus_beta * ghat;", "float inc = beta * ghat;"),
    ("apg_step_uses_gradient", "float direction = m[j] / precond;", "float direction = ghat / precond;"),
    ("apg_no_sqrt_of_v", "float root_v = sqrtf(v[j]);", "float root_v = v[j];"),
    ("apg_one_worker", "for (int32_t i = 0; i < n; ++i) {\n            float keep", "for (int32_t i = 0; i < 1; ++i) {\n            float keep"),
    ("f16_bias_off_by_one", "const int bias = (1 << (exp_bits - 1)) - 1;", "const int bias = (1 << (exp_bits - 1));"),
    ("g16_subnormal_as_normal", "value = ldexp((double)f, 1 - bias - frac_bits);", "value = ldexp((double)((1 << frac_bits) + f), e - bias - frac_bits);"),
    ("g16_sign_dropped", "out[j] = (float)(negative ? -value : value);", "out[j] = (float)value;"),
    ("topk_smallest_kept", "if (ma > mb) return -1;\n    if (ma < mb) return 1;", "if (ma > mb) return 1;\n    if (ma < mb) return -1;"),
    ("topk_signed_not_magnitude", "const float ma = fabsf(topk_sort_values[a]), mb = fabsf(topk_sort_values[b]);",
     "const float ma = topk_sort_values[a], mb = topk_sort_values[b];"),
    ("topk_ties_higher_index_first", "    return (a < b) ? -1 : (a > b);\n}\n\nstatic int topk_by_index",
     "    return (a > b) ? -1 : (a < b);\n}\n\nstatic int topk_by_index"),
    ("topk_wire_not_index_ordered", "qsort(order, (size_t)K, sizeof(uint32_t), topk_by_index);", ""),
    ("topk_error_keeps_sent_part", "werr[base + j] = u[j] - sent[j];", "werr[base + j] = u[j];"),
    ("topk_server_error_keeps_sent_part", "serr[base + j] = ubar[j] - sent[j];", "serr[base + j] = ubar[j];"),
    ("topk_compensate_minus", "u[j] = local_m + werr[base + j];", "u[j] = local_m - werr[base + j];"),
    ("topk_drop_gradient", "float local_m = keep_m + new_g;", "float local_m = keep_m;"),
    ("topk_server_no_mean", "float mean = ubar[j] * inv_n;", "float mean = ubar[j];"),
    ("topk_server_last_worker_only", "ubar[j] = ubar[j] + dense[j];", "ubar[j] = dense[j];"),
    ("topk_server_error_minus", "ubar[j] = mean + serr[base + j];", "ubar[j] = mean - serr[base + j];"),
    ("topk_server_chunk0_lists", "const int64_t in = ((int64_t)i * C + k) * K;", "const int64_t in = ((int64_t)i * C) * K;"),
    ("topk_gather_one_worker", "for (int32_t i = 0; i < n; ++i)\n            m[(int64_t)i * d + j] = gathered;",
     "for (int32_t i = 0; i < 1; ++i)\n            m[(int64_t)i * d + j] = gathered;"),
    ("topk_apply_no_sqrt", "float root_of_v = sqrtf(v[j]);", "float root_of_v = v[j];"),
    ("topk_apply_ascent", "x[j] = x[j] - move;", "x[j] = x[j] + move;"),
    ("freeze_keeps_errors", "memset(serr, 0, (size_t)d * sizeof(float));", ""),
]


def _pin_calls():
    calls = []
    for module in (pins, topk_pins):
        for name in sorted(dir(module)):
            fn = getattr(module, name)
            if not (name.startswith("test_") and callable(fn)):
                continue
            calls.extend(_expand(name, fn))
    return calls


def _expand(name, fn):
    """One call per parametrize value (single-argument parametrisations only)."""
    marks = [mk for mk in getattr(fn, "pytestmark", []) if mk.name == "parametrize"]
    if not marks:
        return [(name, fn, ())]
    return [(name, fn, (val,)) for val in marks[0].args[1]]


def _first_failure():
    for name, fn, args in _pin_calls():
        try:
            fn(*args)
        except AssertionError:
            return name
        except Exception:          # a mutant may also break a pin with a ValueError etc.
            return name
    return None


def test_unmutated_oracle_passes_every_pin():
    assert _first_failure() is None


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda mt: mt[0])
def test_pins_catch_planted_mistake(mutant, tmp_path, monkeypatch):
    mid, old, new = mutant
    src = open(os.path.join(os.path.dirname(oracle.__file__), "apms_oracle.c")).read()
    assert src.count(old) == 1, "mutation site for %s must be unique (found %d)" % (mid, src.count(old))
    c_path = tmp_path / "mutant.c"
    so_path = tmp_path / "mutant.so"
    c_path.write_text(src.replace(old, new))
    flags = [f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.check_call(["gcc", *flags, "-w", "-o", str(so_path), str(c_path), "-lm"])
    good = oracle._load()
    bad = ctypes.CDLL(str(so_path))
    for fname in ("apms_oracle_compress", "apms_oracle_server_reduce", "apms_oracle_apply",
                  "apms_oracle_warmup_step", "apms_oracle_freeze", "apms_oracle_widen_g16",
                  "apms_oracle_apply_gradient", "apms_oracle_topk_compress", "apms_oracle_topk_server_reduce",
                  "apms_oracle_topk_apply"):
        getattr(bad, fname).argtypes = getattr(good, fname).argtypes
        getattr(bad, fname).restype = getattr(good, fname).restype
    monkeypatch.setattr(oracle, "_lib", bad)
    caught_by = _first_failure()
    assert caught_by is not None, "no pin notices mutant '%s'" % mid
