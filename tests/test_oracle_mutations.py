"""Do the oracle's pins notice a plausible mistake?  Each case plants one in a copy of the
oracle's C source (a dropped term, a wrong sign or index, a transposed operand, a wrong rounding),
builds that copy, and runs the pin tests against it in a child process: they must fail.  The
unmodified source goes through the same route first and must pass, so a failure is the mutation's.
CPU only; nothing here touches the GPU path.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_SRC = os.path.join(_ROOT, "oracle", "pg_oracle.c")
_PINS = ["tests/test_oracle_codec.py", "tests/test_oracle_ops.py", "tests/test_oracle_chain.py"]

# (name, text in the oracle's source, what a mistaken author might have written instead)
MUTATIONS = [
    ("gelu_sign", "erfc(-a / sqrt(2.0))", "erfc(a / sqrt(2.0))"),
    ("gelu_no_sqrt", "erfc(-a / sqrt(2.0))", "erfc(-a / 2.0)"),
    ("gelu_no_half", "return 0.5 * a * erfc", "return a * erfc"),
    ("gelu_tanh_form", "return 0.5 * a * erfc(-a / sqrt(2.0));",
     "return 0.5 * a * (1.0 + tanh(0.7978845608028654 * (a + 0.044715 * a * a * a)));"),
    ("rms_no_eps", "sqrt(ss / (double)cols + eps)", "sqrt(ss / (double)cols)"),
    ("rms_sum_not_mean", "sqrt(ss / (double)cols + eps)", "sqrt(ss + eps)"),
    ("rms_eps_inside_sum", "sqrt(ss / (double)cols + eps)", "sqrt((ss + eps) / (double)cols)"),
    ("rms_gain_index", "* scale * ld(dtype, g, i)", "* scale * ld(dtype, g, 0)"),
    ("rms_gain_dropped", "* scale * ld(dtype, g, i)", "* scale"),
    ("rms_row_stride", "double v = ld(dtype, x, r * cols + i);", "double v = ld(dtype, x, i);"),
    ("gemv_transposed", "ld(dtype, W, j * cols + i)", "ld(dtype, W, i * n_out + j)"),
    ("gemv_first_row_only", "ld(dtype, h, r * cols + i)", "ld(dtype, h, i)"),
    ("gemv_out_transposed", "st(dtype, out, r * n_out + j, acc)", "st(dtype, out, j * rows + r, acc)"),
    ("gemv_fp32_accumulate", "double acc = 0.0;\n        for (i = 0; i < cols; i++) acc +=",
     "float acc = 0.0f;\n        for (i = 0; i < cols; i++) acc +="),
    ("add_no_broadcast", "ld(dtype, a, i) + ld(dtype, b, i % m)", "ld(dtype, a, i) + ld(dtype, b, 0)"),
    ("add_is_sub", "ld(dtype, a, i) + ld(dtype, b, i % m)", "ld(dtype, a, i) - ld(dtype, b, i % m)"),
    ("mul_is_add", "ld(dtype, a, i) * ld(dtype, b, i % m)", "ld(dtype, a, i) + ld(dtype, b, i % m)"),
    ("mul_broadcast_block", "ld(dtype, a, i) * ld(dtype, b, i % m)", "ld(dtype, a, i) * ld(dtype, b, (i / m) % m)"),
    ("sbr_channel_index", "int64_t c = (i / inner) % channels;", "int64_t c = i % channels;"),
    ("sbr_no_relu", "st(dtype, out, i, v > 0.0 ? v : 0.0);", "st(dtype, out, i, v);"),
    ("sbr_bias_before_scale", "ld(dtype, x, i) * ld(dtype, s, c) + ld(dtype, b, c)",
     "(ld(dtype, x, i) + ld(dtype, b, c)) * ld(dtype, s, c)"),
    ("sbr_scale_bias_swapped", "ld(dtype, x, i) * ld(dtype, s, c) + ld(dtype, b, c)",
     "ld(dtype, x, i) * ld(dtype, b, c) + ld(dtype, s, c)"),
    ("bf16_truncates", "r = nearbyint(x / q) * q;", "r = trunc(x / q) * q;"),
    ("bf16_ties_away", "r = nearbyint(x / q) * q;", "r = round(x / q) * q;"),
    ("bf16_via_fp32", "else ((uint16_t *)p)[i] = orc_bf16_from_f64(v);",
     "else ((uint16_t *)p)[i] = orc_bf16_from_f64((double)(float)v);"),
    ("bf16_subnormal_quantum", "if (e < -126) e = -126;", ""),
    ("bf16_quantum_off_by_one", "q = ldexp(1.0, e - 7);", "q = ldexp(1.0, e - 8);"),
    ("bf16_load_low_half", "uint32_t u = (uint32_t)bits << 16;", "uint32_t u = (uint32_t)bits;"),
    ("chain_ext_as_weight", "case ORC_EXT: return ext[k->in_index[j]];", "case ORC_EXT: return weights[k->in_index[j]];"),
    ("chain_operands_swapped", "const void *b = operand(k, 1, ext, weights, ints);",
     "const void *b = operand(k, 2, ext, weights, ints);"),
    ("chain_skips_last_kernel", "for (i = k_begin; i < k_end; i++) {", "for (i = k_begin; i < k_end - 1; i++) {"),
    ("chain_ignores_begin", "for (i = k_begin; i < k_end; i++) {", "for (i = 0; i < k_end; i++) {"),
    ("select_last_of_equal", "c < cost[3 * s + best]", "c <= cost[3 * s + best]"),
    ("select_max", "c < cost[3 * s + best]", "c > cost[3 * s + best]"),
    ("select_takes_infinite", "if (!isfinite(c)) continue;", "if (isnan(c)) continue;"),
    ("select_first_segment_only", "double c = cost[3 * s + m];", "double c = cost[m];"),
    ("bf16_loses_negative_zero", "return signbit(x) ? 0x8000u : 0x0000u;", "return 0x0000u;"),
    ("bf16_nan_becomes_inf", "if (isnan(x)) return 0x7FC0u;", "if (isnan(x)) return 0x7F80u;"),
    ("rms_sum_not_squares", "ss += v * v;", "ss += fabs(v);"),
    ("rms_no_sqrt", "scale = 1.0 / sqrt(ss / (double)cols + eps);", "scale = 1.0 / (ss / (double)cols + eps);"),
    ("rms_output_from_row_0", "st(dtype, out, r * cols + i, ld(dtype, x, r * cols + i) * scale",
     "st(dtype, out, r * cols + i, ld(dtype, x, i) * scale"),
    ("sbr_channel_from_inner", "int64_t c = (i / inner) % channels;", "int64_t c = (i % inner) % channels;"),
    ("sbr_abs_not_relu", "st(dtype, out, i, v > 0.0 ? v : 0.0);", "st(dtype, out, i, v > 0.0 ? v : -v);"),
    ("select_nothing_available_is_eager", "if (best < 0) return -(s + 1);", "if (best < 0) best = 0;"),
    ("chain_ignores_op_errors", "if (rc != 0) return -(i + 1);", "(void)rc;"),
    ("chain_int_as_ext", "case ORC_INT: return ints[k->in_index[j]];", "case ORC_INT: return ext[k->in_index[j]];"),
]


def _build(source: str, out_so: str, src_path: str) -> None:
    with open(src_path, "w") as f:
        f.write(source)
    subprocess.run(["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-w",
                    "-I", os.path.join(_ROOT, "oracle"), "-shared", "-fPIC", "-o", out_so, src_path, "-lm"],
                   check=True)


def _pins_pass(so: str) -> bool:
    env = dict(os.environ, PG_ORACLE_SO_OVERRIDE=so, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + _PINS,
                       cwd=_ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)
    return r.returncode == 0


@pytest.fixture(scope="module")
def source():
    with open(_SRC) as f:
        return f.read()


@pytest.fixture(scope="module")
def verdicts(source, tmp_path_factory):
    """name -> did the pins pass?  All copies are built and checked here, a few at a time."""
    d = tmp_path_factory.mktemp("mutants")
    jobs = [("unmodified", source)] + [(name, source.replace(old, new)) for name, old, new in MUTATIONS]

    def one(job):
        name, text = job
        so = str(d / (name + ".so"))
        _build(text, so, str(d / (name + ".c")))
        return name, _pins_pass(so)

    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(pool.map(one, jobs))


def test_every_mutation_site_exists_once(source):
    for name, old, new in MUTATIONS:
        assert source.count(old) == 1, f"{name}: the text to replace occurs {source.count(old)} times"
        assert old != new


def test_unmodified_copy_passes_through_the_same_route(verdicts):
    assert verdicts["unmodified"]


@pytest.mark.parametrize("name", [m[0] for m in MUTATIONS])
def test_pins_catch(verdicts, name):
    assert not verdicts[name], f"no pin noticed the planted mistake '{name}'"
