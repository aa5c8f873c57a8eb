"""Do the pins have teeth?  Each case below plants one plausible mistake in a copy of the CPU
checker's source (a wrong rounding rule, constant, sign, index or operand), builds it, and runs
the pin suites (tests/test_oracle_quant.py, tests/test_oracle_attn.py) against that build in a
child process: they must fail.  The unmodified source, built the same way, must pass.  Nothing
here touches the GPU or the GPU library; the mistakes exist only in temporary files."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvq_oracle.c")

# (name, text in the source, what a mistaken author might have written instead)
MUTANTS = [
    ("int8_rounds_half_up",
     "r = rint(x / (double)s); /* default rounding mode: to nearest, ties to even */",
     "r = floor(x / (double)s + 0.5);"),
    ("int8_allows_minus_128",
     "if (r < -127.0) r = -127.0;", "if (r < -128.0) r = -128.0;"),
    ("int8_scale_divides_by_128",
     "oracle_scale(m, 127.0)", "oracle_scale(m, 128.0)"),
    ("int8_write_swaps_k_and_v",
     "const uint16_t* src = kv ? v : k;", "const uint16_t* src = kv ? k : v;"),
    ("int8_write_ignores_the_token_offset_for_scales",
     "scales[(((size_t)blk * 2 + kv) * H + h) * bs + off] = s;\n          uint8_t* dst = cache + tile_index(blk, kv, h, H, bs, D) + (size_t)off * D;",
     "scales[(((size_t)blk * 2 + kv) * H + h) * bs] = s;\n          uint8_t* dst = cache + tile_index(blk, kv, h, H, bs, D) + (size_t)off * D;"),
    ("int8_dequant_reads_the_code_unsigned",
     "return (double)(int8_t)c * s;", "return (double)c * s;"),
    ("int4_nibbles_swapped_on_read",
     "int nib = (d & 1) ? (byte >> 4) : (byte & 15);", "int nib = (d & 1) ? (byte & 15) : (byte >> 4);"),
    ("int4_scale_divides_by_8",
     "oracle_scale(m, 7.0)", "oracle_scale(m, 8.0)"),
    ("int4_group_scale_taken_over_64_channels",
     "#define ORACLE_INT4_GROUP 32", "#define ORACLE_INT4_GROUP 64"),
    ("int4_group_dequant_uses_the_first_group_scale",
     "(double)scales[token * (D / ORACLE_INT4_GROUP) + d / ORACLE_INT4_GROUP]",
     "(double)scales[token * (D / ORACLE_INT4_GROUP)]"),
    ("int4_group_codes_written_to_the_first_group",
     "dst[g * (ORACLE_INT4_GROUP / 2) + j] = (uint8_t)((lo & 15) | ((hi & 15) << 4));",
     "dst[j] = (uint8_t)((lo & 15) | ((hi & 15) << 4));"),
    ("fp8_ties_go_to_the_odd_code",
     "(err == best_err && (c & 1) == 0)", "(err == best_err && (c & 1) == 1)"),
    ("fp8_exponent_bias_8",
     "mag = ldexp(1.0 + (double)m / 8.0, e - 7);", "mag = ldexp(1.0 + (double)m / 8.0, e - 8);"),
    ("fp8_subnormals_one_binade_low",
     "mag = ldexp((double)m / 8.0, -6);", "mag = ldexp((double)m / 8.0, -7);"),
    ("fp8_overflow_becomes_nan",
     "if (a >= 448.0) return (uint8_t)(sign | 0x7E);", "if (a >= 448.0) return (uint8_t)(sign | 0x7F);"),
    ("fp8_scale_divides_by_240",
     "oracle_scale(m, 448.0)", "oracle_scale(m, 240.0)"),
    ("fp8_block_keeps_a_stale_scale_on_a_fresh_block",
     "float s_prev = (o_min > 0) ? *sp : 0.0f;", "float s_prev = *sp;"),
    ("fp8_block_scale_is_not_a_running_max",
     "float s_new = (s_prev > s_cand) ? s_prev : s_cand;", "float s_new = s_cand;"),
    ("fp8_block_rescale_upside_down",
     "val * (double)s_prev / (double)s_new", "val * (double)s_new / (double)s_prev"),
    ("attention_query_does_not_see_itself",
     "const int32_t n = L - q_len + j + 1;", "const int32_t n = L - q_len + j;"),
    ("attention_heads_interleaved_instead_of_grouped",
     "const int h = hq / G;", "const int h = hq % num_kv_heads;"),
    ("attention_without_the_softmax_scale",
     "z[p] = sm_scale * dot;", "z[p] = dot;"),
    ("attention_sums_k_rows_instead_of_v_rows",
     "orow[d] += w * vd[(size_t)p * D + d];", "orow[d] += w * kd[(size_t)p * D + d];"),
    ("attention_denominator_misses_the_last_position",
     "for (int32_t p = 0; p < n; ++p) {\n          z[p] = exp(z[p] - zmax);\n          denom += z[p];\n        }",
     "for (int32_t p = 0; p < n; ++p) {\n          z[p] = exp(z[p] - zmax);\n          if (p + 1 < n) denom += z[p];\n        }"),
    ("table_walk_uses_the_wrong_offset",
     "int off = p % block_size;", "int off = (p + 1) % block_size;"),
]


def build(source_text, workdir, name):
    c_path = os.path.join(workdir, name + ".c")
    so_path = os.path.join(workdir, name + ".so")
    with open(c_path, "w") as f:
        f.write(source_text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                           "-ffp-contract=off", "-w", "-o", so_path, c_path, "-lm"])
    return so_path


def run_pins(so_path):
    env = dict(os.environ, KVQ_ORACLE_SO=so_path, OMP_NUM_THREADS="1")
    return subprocess.run(
        [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
         os.path.join(ROOT, "tests", "test_oracle_quant.py"),
         os.path.join(ROOT, "tests", "test_oracle_attn.py")],
        cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Builds the control and every mutant and runs the pins on each, a few at a time."""
    from concurrent.futures import ThreadPoolExecutor
    workdir = str(tmp_path_factory.mktemp("mutants"))
    text = open(SRC).read()
    jobs = {"control": text}
    for name, right, wrong in MUTANTS:
        assert right in text, "the checker's source no longer contains the text '%s' alters" % name
        jobs[name] = text.replace(right, wrong, 1)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as pool:
        done = pool.map(lambda kv: (kv[0], run_pins(build(kv[1], workdir, kv[0]))), jobs.items())
        return dict(done)


def test_the_unmodified_source_passes_through_the_same_harness(outcomes):
    r = outcomes["control"]
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_a_planted_mistake_is_noticed(outcomes, name):
    r = outcomes[name]
    assert r.returncode != 0, "no pin failed for the planted mistake '%s'" % name
    assert " failed" in r.stdout or " error" in r.stdout, r.stdout[-2000:]
