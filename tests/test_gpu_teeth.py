"""Would the GPU parity tests notice?  The same comparisons as test_gpu_write.py and
test_gpu_attn.py, but with the expected values taken from a build of the CPU checker with one
planted mistake (in a temporary copy of its C source): each must now fail.  The GPU library is
untouched and runs exactly as in the real tests; the mistakes live on the CPU side only."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2605_29639_amd import workloads as W
from helpers import gpu_fill, oracle_fill
from test_oracle_mutants import MUTANTS, SRC

BY_NAME = {m[0]: m for m in MUTANTS}


@pytest.fixture(scope="module")
def mutant(tmp_path_factory):
    workdir = str(tmp_path_factory.mktemp("gpu_teeth"))
    text = open(SRC).read()

    def build(name):
        _, right, wrong = BY_NAME[name]
        assert right in text
        c_path, so_path = os.path.join(workdir, name + ".c"), os.path.join(workdir, name + ".so")
        with open(c_path, "w") as f:
            f.write(text.replace(right, wrong, 1))
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-w", "-o", so_path, c_path, "-lm"])
        return so_path
    return build


@pytest.mark.parametrize("name,mode", [
    ("int8_rounds_half_up", W.MODE_INT8),
    ("int8_scale_divides_by_128", W.MODE_INT8),
    ("int8_write_swaps_k_and_v", W.MODE_INT8),
    ("int4_scale_divides_by_8", W.MODE_INT4),
    ("fp8_ties_go_to_the_odd_code", W.MODE_FP8),
    ("fp8_scale_divides_by_240", W.MODE_FP8),
    ("fp8_block_scale_is_not_a_running_max", W.MODE_FP8),
])
def test_write_parity_fails_against_a_wrong_checker(mutant, name, mode):
    """Prompt-sized writes with rows full of rounding ties, then single-token appends."""
    import test_gpu_write as T
    so = mutant(name)
    with oracle.use_library(so):
        with pytest.raises(AssertionError):
            T.test_prefill_of_several_sequences_in_one_call(mode, 16, 128, 2)
            if mode == W.MODE_FP8:
                T.test_fp8_token_by_token_append_with_rescale(16, 128)
    T.test_prefill_of_several_sequences_in_one_call(mode, 16, 128, 2)   # and passes with the real one


@pytest.mark.parametrize("name", [
    "attention_query_does_not_see_itself",
    "attention_heads_interleaved_instead_of_grouped",
    "attention_without_the_softmax_scale",
    "attention_sums_k_rows_instead_of_v_rows",
    "attention_denominator_misses_the_last_position",
    "int8_dequant_reads_the_code_unsigned",
    "table_walk_uses_the_wrong_offset",
])
def test_attention_parity_fails_against_a_wrong_checker(mutant, name):
    import test_gpu_attn as T
    so = mutant(name)
    with oracle.use_library(so):
        with pytest.raises(AssertionError):
            T.check(W.tiny(W.MODE_INT8), chunks=(0, 64))
    T.check(W.tiny(W.MODE_INT8), chunks=(0, 64))
