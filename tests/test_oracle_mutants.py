"""Do the pins bite?  Each case plants ONE plausible mistake (a dropped term, a shifted index,
a swapped operand, a lost +1) in a COPY of the oracle's C source, builds that copy with the
oracle's own compiler line, and runs the oracle's pin tests against it in a child process:
at least one pin must fail.  The unmodified copy must pass, so that it is the planted mistake
that is noticed and not the harness.  Everything here runs on the CPU and touches neither the
oracle's own library nor the HIP path; every mutant keeps all memory accesses in bounds."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ems_oracle.c")

ATT, ACC, TREE, PAD = ("tests/test_oracle_attention.py", "tests/test_oracle_accept_append.py",
                       "tests/test_oracle_tree.py", "tests/test_oracle_padded.py")

# (what goes wrong, pin file that must notice, text, replacement, which occurrence of the text)
MUTANTS = [
    ("a new token does not see itself", ATT,
     "mask[n] = (unsigned char)(n <= L + j);", "mask[n] = (unsigned char)(n < L + j);", 0),
    ("a new token sees the token after it", ATT,
     "mask[n] = (unsigned char)(n <= L + j);", "mask[n] = (unsigned char)(n <= L + j + 1);", 0),
    ("the softmax scale is dropped", ATT, "S[n] = (double)scale * dot;", "S[n] = dot;", 0),
    ("values are read from the key arena", ATT,
     "val[(size_t)n * D + d] = widen(v_cache[off], dtype);", "val[(size_t)n * D + d] = widen(k_cache[off], dtype);", 0),
    ("new values are read from the new keys", ATT,
     "val[(size_t)n * D + d] = widen(v_new[off], dtype);", "val[(size_t)n * D + d] = widen(k_new[off], dtype);", 0),
    ("the softmax is not normalised", ATT, "out[qoff + d] = acc / Z;", "out[qoff + d] = acc;", 0),
    ("the sample's start location is ignored", ATT,
     "int64_t off = (s + n) * row_stride + (int64_t)h * head_stride + d;",
     "int64_t off = (int64_t)n * row_stride + (int64_t)h * head_stride + d;", 0),
    ("new rows are taken from the wrong head", ATT,
     "int64_t off = ((int64_t)(cu[i] + n - L) * H + h) * D + d;",
     "int64_t off = ((int64_t)(cu[i] + n - L) * H + (H - 1 - h)) * D + d;", 0),
    ("the query is dotted with the key reversed", ATT,
     "dot += widen(q[qoff + d], dtype) * key[(size_t)n * D + d];",
     "dot += widen(q[qoff + d], dtype) * key[(size_t)n * D + (D - 1 - d)];", 0),
    ("the maximum is added instead of subtracted", ATT,
     "p[n] = mask[n] ? exp(S[n] - m) : 0.0;", "p[n] = mask[n] ? exp(S[n] + m) : 0.0;", 0),
    ("a draft is compared with its own row's input", ACC,
     "x[cu[i] + m] == input_ids[cu[i] + m + 1]", "x[cu[i] + m] == input_ids[cu[i] + m]", 0),
    ("the token after the accepted drafts is not counted", ACC, "tau = m + 1;", "tau = m;", 0),
    ("the highest index wins arg-max ties", ACC,
     "if (y > best) { best = y; arg = v; }", "if (y >= best) { best = y; arg = v; }", 0),
    ("the running sum does not run", ACC,
     "accepted_cu[i + 1] = accepted_cu[i] + tau;", "accepted_cu[i + 1] = tau;", 0),
    ("the input tokens are emitted instead of the target's", ACC,
     "out_tokens[accepted_cu[i] + j] = x[cu[i] + j];", "out_tokens[accepted_cu[i] + j] = input_ids[cu[i] + j];", 0),
    ("the last accepted row is not appended", ACC,
     "for (int j = 0; j < accepted[i]; ++j) {", "for (int j = 0; j < accepted[i] - 1; ++j) {", 0),
    ("appended values are the keys", ACC, "v_cache[dst] = v_new[src];", "v_cache[dst] = k_new[src];", 0),
    ("the new length lags by one", ACC,
     "kv_len_out[i] = kv_len[i] + accepted[i];", "kv_len_out[i] = kv_len[i] + accepted[i] - 1;", 0),
    ("concatenation gives every slot of a sample that sample's first token", ACC,
     "packed_ids[t] = padded_ids[(size_t)i * k_max + (t - first)];",
     "packed_ids[t] = padded_ids[(size_t)i * k_max];", 0),
    ("the highest index wins arg-max ties in fp32 logits", ACC,
     "if (y > best) { best = y; arg = v; }", "if (y >= best) { best = y; arg = v; }", 1),
    ("a sample's first packed row is given to the sample before it", ACC,
     "if (r >= first && r < first + rows_per_sample[i]) {", "if (r >= first && r <= first + rows_per_sample[i]) {", 0),
    ("write-through leaves out the last new row", ACC,
     "for (int j = 0; j < k; ++j)\n            for (int h = 0; h < H; ++h)", "for (int j = 0; j < k - 1; ++j)\n            for (int h = 0; h < H; ++h)", 0),
    ("bf16 is widened as if it were fp16", ATT, "if (dtype == ORACLE_BF16) {", "if (dtype == 7) {", 0),
    ("fp16 subnormals lose their scale", ACC, "int expo = (bits >> 10) & 0x1f;", "int expo = ((bits >> 10) & 0x1f) | 1;", 0),
    ("tree: a row sees only its parent, not all ancestors", TREE,
     "for (int u = j; u >= 0; u = parent[cu[i] + u]) mask[L + u] = 1;",
     "mask[L + j] = 1; if (j > 0) mask[L + parent[cu[i] + j]] = 1;", 0),
    ("tree: a row sees every earlier row", TREE,
     "for (int u = j; u >= 0; u = parent[cu[i] + u]) mask[L + u] = 1;",
     "for (int u = j; u >= 0; --u) mask[L + u] = 1;", 0),
    ("tree: any row with the right token is accepted, child or not", TREE,
     "if (parent[cu[i] + c] == u && input_ids[cu[i] + c] == x[cu[i] + u]) next = c;",
     "if (input_ids[cu[i] + c] == x[cu[i] + u]) next = c;", 0),
    ("tree: the accepted rows are reported as a chain", TREE,
     "accepted_rows[accepted_cu[i] + tau] = cu[i] + u;", "accepted_rows[accepted_cu[i] + tau] = cu[i] + tau;", 0),
    ("tree: the gathered append copies consecutive rows", TREE,
     "const int64_t src_row = accepted_rows[accepted_cu[i] + j];",
     "const int64_t src_row = accepted_rows[accepted_cu[i]] + j;", 0),
    ("padded: padding keys are visible", PAD,
     "if (n < l_pad) mask[n] = key_mask[(int64_t)i * cap + n] != 0;", "if (n < l_pad) mask[n] = 1;", 0),
    # (dropping "n - l_pad < k_valid[i]" from that line is NOT a mistake the pins could see: for a
    #  real row j < k_valid[i] it is implied by n - l_pad <= j, and padding rows are don't-care)
    ("padded: a new token does not see itself", PAD,
     "else mask[n] = (n - l_pad <= j) && (n - l_pad < k_valid[i]);",
     "else mask[n] = (n - l_pad < j) && (n - l_pad < k_valid[i]);", 0),
    ("padded: padding rows are appended after the real ones of the NEXT sample's count", PAD,
     "key_mask[dst_row] = (uint8_t)(j < accepted[i]);", "key_mask[dst_row] = (uint8_t)(j < accepted[(i + 1) % B]);", 0),
    ("padded: every appended row is marked real", PAD,
     "key_mask[dst_row] = (uint8_t)(j < accepted[i]);", "key_mask[dst_row] = 1;", 0),
]


def nth_replace(text, old, new, occurrence):
    pos = -1
    for _ in range(occurrence + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, "the oracle no longer contains: " + old
    return text[:pos] + new + text[pos + len(old):]


def build_copy(tmp_path, text, name):
    src = tmp_path / (name + ".c")
    lib = tmp_path / (name + ".so")
    src.write_text(text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), str(src), "-lm"])
    return str(lib)


def run_pins(lib, files):
    env = dict(os.environ, EMS_ORACLE_LIBRARY=lib, OMP_NUM_THREADS="4")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + list(files)
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_the_unmodified_copy_passes_every_pin(tmp_path):
    res = run_pins(build_copy(tmp_path, open(SRC).read(), "copy"), [ATT, ACC, TREE, PAD])
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("what,pins,old,new,occurrence", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_noticed(tmp_path, what, pins, old, new, occurrence):
    lib = build_copy(tmp_path, nth_replace(open(SRC).read(), old, new, occurrence), "mutant")
    res = run_pins(lib, [pins])
    assert res.returncode != 0, "no pin in %s notices that %s" % (pins, what)
    assert " failed" in res.stdout or " error" in res.stdout, res.stdout[-2000:]
