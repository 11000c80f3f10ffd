"""The pins have teeth: plant one plausible mistake at a time in a temporary copy of the oracle's
source (on the CPU, never in the GPU path), rebuild it, and check that the pin suite rejects it.

Each mutant is a text substitution that must apply exactly once; the checks re-run are the
exact rational brute force, the bijection check, the slice check and the implementation I/II
agreement from the other oracle test files.
"""
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import reference as R
from oracle import build as oracle_build
from tests import test_oracle_method as TM
from tests import test_oracle_selector as TS

MUTANTS = [
    ("residual sign", "r[i * n + j] = v[i * n + j] - vprime[i * n + j]", "r[i * n + j] = vprime[i * n + j] - v[i * n + j]"),
    ("mean not divided by n", "vbar[j] = sum / real(pb.W)", "vbar[j] = sum"),
    ("first worker counted twice", "for (uint32_t i = 1; i < pb.W; ++i) sum", "for (uint32_t i = 0; i < pb.W; ++i) sum"),
    ("classical instead of Nesterov update", "p[i * n + j] = eta * fused_mul_add(beta, mij, gij)", "p[i * n + j] = eta * mij"),
    ("momentum without decay", "mij = fused_mul_add(beta, mij, gij)", "mij = mij + gij"),
    ("model moved the wrong way", "x[i * pb.ld + j] - pprime[i * n + j];\n      e[", "x[i * pb.ld + j] + pprime[i * n + j];\n      e["),
    ("residual accumulated with wrong sign", "e[i * pb.ld + j] = e[i * pb.ld + j] - r[i * n + j]", "e[i * pb.ld + j] = e[i * pb.ld + j] + r[i * n + j]"),
    ("reset forgets to remove the old residual", "(x[i * pb.ld + j] - ehalf[i * n + j]) + eprime[i * n + j]", "x[i * pb.ld + j] + eprime[i * n + j]"),
    ("reset corrects the model on the unchosen blocks only", "if (chosen[(pb.col0 + j) / pb.block])\n        x[", "if (!chosen[(pb.col0 + j) / pb.block])\n        x["),
    ("reset sends the unchosen blocks through (x - e) + e' too", "if (chosen[(pb.col0 + j) / pb.block])\n        x[", "if (true)\n        x["),
    ("reset keeps the old residual", "e[i * pb.ld + j] = r[i * n + j];", "e[i * pb.ld + j] = ehalf[i * n + j];"),
    ("reset reuses the step's blocks", "select_blocks(pb.seed, 1, t, B, blocks_kept(B, R_reset), nullptr, chosen.data());\n  std::vector<real> ehalf", "select_blocks(pb.seed, 0, t, B, blocks_kept(B, R_reset), nullptr, chosen.data());\n  std::vector<real> ehalf"),
    ("compressor keeps the complement", "cv[j] = chosen[b] ? v[j] : real(0)", "cv[j] = chosen[b] ? real(0) : v[j]"),
    ("block id ignores the slice offset", "const uint64_t b = (pb.col0 + j) / pb.block;", "const uint64_t b = j / pb.block;"),
    ("B/R rounded down", "return R == 0 ? 0 : ceil_div(B, R);", "return R == 0 ? 0 : B / R;"),
    ("feistel round without the swap", "left = right;\n      right = new_right;", "right = new_right;"),
    ("inverse rounds in forward order", "for (int round = kFeistelRounds - 1; round >= 0; --round)", "for (int round = 0; round < kFeistelRounds; ++round)"),
    ("implementation II averages nothing", "x[i * pb.ld + j] = xprime[i * n + j];", "x[i * pb.ld + j] = xhalf[i * n + j];"),
]


def _suite():
    """A fast subset of the pins; raises AssertionError if the loaded oracle is wrong."""
    for case in [(2, 12, 4, 2, 2, 2, 4), (4, 11, 3, 2, 1, 3, 6), (4, 10, 4, 3, 2, 1, 3)]:
        TM.test_algorithm3_matches_exact_rational_arithmetic(*case)
    TM.test_non_power_of_two_worker_count_against_exact_arithmetic()
    TM.test_a_block_slice_evolves_exactly_as_in_the_full_run()
    TM.test_implementations_one_and_two_give_the_same_models(4, 2, 3, 0.9)
    TM.test_error_reset_touches_only_the_blocks_it_chose_and_follows_the_written_formula_there()
    TS.test_permutation_is_bijection_and_inverse_matches(17)
    TS.test_permutation_is_bijection_and_inverse_matches(257)
    TS.test_exactly_k_distinct_blocks_and_mask_agrees(7, 100)
    TS.test_exactly_k_distinct_blocks_and_mask_agrees(1672, 32)


def test_the_unmutated_oracle_passes_the_subset():
    _suite()


_CHILD = """
import sys
sys.path.insert(0, {root!r})
from oracle import reference as R
R._LIB = R.load({so!r})
from tests import test_oracle_mutants as T
try:
    T._suite()
except (AssertionError, ValueError):
    sys.exit(3)
sys.exit(0)
"""


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    """The suite runs in a child process under a time limit: a mutant whose permutation is no
    longer a bijection may never finish its cycle walk, and not terminating counts as caught."""
    src = open(oracle_build.SOURCE).read()
    assert src.count(old) == 1, f"mutant '{name}' must apply exactly once ({src.count(old)})"
    cpp = tmp_path / "mutant.cpp"
    so = tmp_path / "mutant.so"
    cpp.write_text(src.replace(old, new))
    subprocess.run(["g++", "-std=c++17", "-O1", "-ffp-contract=off", "-shared", "-fPIC", str(cpp), "-o", str(so)],
                   check=True)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        rc = subprocess.run([sys.executable, "-c", _CHILD.format(root=root, so=str(so))], timeout=30).returncode
    except subprocess.TimeoutExpired:
        rc = 3
    assert rc == 3, f"mutant '{name}' survived the pins (exit {rc})"
