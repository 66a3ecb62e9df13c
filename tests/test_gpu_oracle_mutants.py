"""The GPU parity tests compare two independent implementations, and notice when one of them is
wrong: with a mistake planted in a COPY of the ORACLE (CPU side; the HIP library is untouched
and nothing faulty runs on the GPU), the small parity tests must fail in a child process, and
with the unmodified copy they must pass."""
import os
import subprocess
import sys

import pytest

from test_oracle_mutants import ROOT, SRC, build_copy, nth_replace

pytestmark = pytest.mark.gpu

SMALL = ["tests/test_gpu_parity.py::test_tiny_config_attention",
         "tests/test_gpu_parity.py::test_tiny_config_accept_and_append",
         "tests/test_gpu_parity.py::test_ragged_lengths_span_tiles_and_tails"]

MUTANTS = [
    ("attention: a new token sees the token after it",
     "mask[n] = (unsigned char)(n <= L + j);", "mask[n] = (unsigned char)(n <= L + j + 1);"),
    ("attention: values are read from the key arena",
     "val[(size_t)n * D + d] = widen(v_cache[off], dtype);", "val[(size_t)n * D + d] = widen(k_cache[off], dtype);"),
    ("accept: the token after the accepted drafts is not counted", "tau = m + 1;", "tau = m;"),
    ("append: the last accepted row is not appended",
     "for (int j = 0; j < accepted[i]; ++j) {", "for (int j = 0; j < accepted[i] - 1; ++j) {"),
]


def run_small(lib):
    env = dict(os.environ, EMS_ORACLE_LIBRARY=lib)
    cmd = [sys.executable, "-u", "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "--timeout", "120",
           "--timeout-method", "thread"] + SMALL
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=400)


def test_small_parity_tests_pass_against_the_unmodified_copy(tmp_path):
    res = run_small(build_copy(tmp_path, open(SRC).read(), "copy"))
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_parity_fails_when_the_oracle_is_wrong(tmp_path, what, old, new):
    res = run_small(build_copy(tmp_path, nth_replace(open(SRC).read(), old, new, 0), "mutant"))
    assert res.returncode == 1 and " failed" in res.stdout, res.stdout[-2000:]
