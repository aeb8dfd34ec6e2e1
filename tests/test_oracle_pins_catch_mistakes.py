"""The pins of the oracle, tried on oracles with a planted mistake (CPU only).

Every case below edits one expression of a copy of `oracle/tf_oracle.c` -- a dropped term, a wrong
sign, a swapped operand, a wrong index -- builds it, and runs the pin tests of that part against the
copy (the front end loads the library named by TF_ORACLE_LIB). The pins must fail on every one of
them, and pass on an unedited copy built the same way."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "tf_oracle.c")

# (name, pin file, text in tf_oracle.c, replacement, occurrences)
MISTAKES = [
    ("attention: causal alignment off by one", "test_oracle_attention.py",
     "n_all - G + 1 + g", "n_all - G + g", 1),
    ("attention: softmax scale dropped", "test_oracle_attention.py",
     "z[t] = scale * acc;", "z[t] = acc;", 1),
    ("attention: weights not normalised", "test_oracle_attention.py",
     "double w = z[t] / denom;", "double w = z[t];", 1),
    ("attention: values taken from K", "test_oracle_attention.py",
     "o[j] += w * bf16_to_f64(Vbh[t * d + j]);", "o[j] += w * bf16_to_f64(Kbh[t * d + j]);", 1),
    ("attention: LSE without the maximum", "test_oracle_attention.py",
     "= m + log(denom);", "= log(denom);", 1),
    ("chunk mean: sum instead of mean", "test_oracle_retrieval.py",
     "out[m * d + j] = s / (double)c;", "out[m * d + j] = s;", 1),
    ("chunk mean: strided instead of contiguous chunks", "test_oracle_retrieval.py",
     "s += bf16_to_f64(Kbh[(m * c + i) * d + j]);", "s += bf16_to_f64(Kbh[(m + i * M) * d + j]);", 1),
    ("retrieval: ascending instead of descending", "test_oracle_retrieval.py",
     "if (x->s > y->s) return -1;\n    if (x->s < y->s) return 1;",
     "if (x->s > y->s) return 1;\n    if (x->s < y->s) return -1;", 1),
    ("retrieval: ties toward the higher index", "test_oracle_retrieval.py",
     "return (x->i > y->i) - (x->i < y->i);", "return (x->i < y->i) - (x->i > y->i);", 1),
    ("gather: V rows copied from K", "test_oracle_retrieval.py",
     "memcpy(Vr + dst, V + src,", "memcpy(Vr + dst, K + src,", 1),
    ("gather: chunk-major destination transposed", "test_oracle_retrieval.py",
     "(int64_t)bh * R_cap + (int64_t)j * c + i", "(int64_t)bh * R_cap + (int64_t)i * k + j", 1),
    ("accept: p and q swapped in the test", "test_oracle_accept.py",
     "* q[x[n]];\n                double rhs = p[x[n]];", "* p[x[n]];\n                double rhs = q[x[n]];", 1),
    ("accept: residual sign", "test_oracle_accept.py",
     "r[v] = p[v] - q[v] > 0.0 ? p[v] - q[v] : 0.0;", "r[v] = q[v] - p[v] > 0.0 ? q[v] - p[v] : 0.0;", 1),
    ("accept: bonus token from the first row", "test_oracle_accept.py",
     "softmax_T(tl + (int64_t)gamma * V, V, T, p);", "softmax_T(tl, V, T, p);", 1),
    ("accept: temperature dropped", "test_oracle_accept.py",
     "(double)logits[v] / T", "(double)logits[v]", 2),
    ("accept: greedy test against the draft's arg-max", "test_oracle_accept.py",
     "if (x[n] != argmax_first(tl + (int64_t)n * V, V)) break;",
     "if (x[n] != argmax_first(dl + (int64_t)n * V, V)) break;", 1),
    ("accept: zero-probability token accepted", "test_oracle_accept.py",
     "if (!(lhs < rhs)) { rejected = 1; break; }", "if (!(lhs <= rhs)) { rejected = 1; break; }", 1),
]


def _build(text, path):
    src = path + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", path, src, "-lm"])


def _run_pins(pin_file, lib):
    env = dict(os.environ, TF_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pin_file), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)


def test_unedited_copy_passes_its_pins(tmp_path):
    lib = str(tmp_path / "same.so")
    _build(open(SRC).read(), lib)
    res = _run_pins("test_oracle_attention.py", lib)
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("name,pin_file,old,new,count", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_pins_fail_on_a_planted_mistake(tmp_path, name, pin_file, old, new, count):
    text = open(SRC).read()
    assert text.count(old) == count, f"{name}: the oracle's text changed, update this case"
    lib = str(tmp_path / "mistake.so")
    _build(text.replace(old, new), lib)
    res = _run_pins(pin_file, lib)
    assert res.returncode == 1 and " failed" in res.stdout, \
        f"{name}: the pins in {pin_file} did not notice\n{res.stdout[-1500:]}"


# The oracle's functions that are written in Python on top of the C routines (the widened rows:
# gather-free drafting, grouped heads, token trees, cache append, bf16 table, ragged accept,
# Algorithm 1): (name, pin file, file under oracle/, text, replacement)
PY_MISTAKES = [
    ("indexed: first recent row dropped", "test_oracle_cache_update.py", "tf_oracle.py",
     "rows.append(np.arange(min(int(rb[b]), int(kv[b])), int(kv[b])))",
     "rows.append(np.arange(min(int(rb[b]) + 1, int(kv[b])), int(kv[b])))"),
    ("indexed: negative chunk entries not skipped", "test_oracle_cache_update.py", "tf_oracle.py",
     "for m in idx[b, h].tolist() if m >= 0 and (m + 1) * c <= kv_len_all]",
     "for m in idx[b, h].tolist() if (m + 1) * c <= kv_len_all]"),
    ("append: rows written backwards", "test_oracle_cache_update.py", "tf_oracle.py",
     "t = int(pos[b]) + i", "t = int(pos[b]) - i"),
    ("append: V rows taken from Knew", "test_oracle_cache_update.py", "tf_oracle.py",
     "V[b, :, t] = Vnew[b, :, i]", "V[b, :, t] = Knew[b, :, i]"),
    ("grouped heads: interleaved instead of blocked head mapping", "test_oracle_attention.py", "tf_oracle.py",
     "Kr = np.ascontiguousarray(np.repeat(K, q_group, axis=1))",
     "Kr = np.ascontiguousarray(np.tile(K, (1, q_group, 1, 1)))"),
    ("tree: mask bits read in reverse", "test_oracle_tree.py", "tf_oracle.py",
     "if (mask[g] >> j) & 1 and n - G + j >= 0]", "if (mask[g] >> (G - 1 - j)) & 1 and n - G + j >= 0]"),
    ("tree: first speculated token visible to everyone", "test_oracle_tree.py", "tf_oracle.py",
     "ctx = np.arange(max(n - G, 0))", "ctx = np.arange(max(n - G + 1, 0))"),
    ("bf16 rounding: one bit too coarse", "test_oracle_retrieval.py", "tf_oracle.py",
     "return np.ldexp(np.rint(m * 256.0), e - 8)", "return np.ldexp(np.rint(m * 128.0), e - 7)"),
    ("bf16 table: exact mean rounded once instead of the fp32 mean", "test_oracle_retrieval.py", "tf_oracle.py",
     "return round_to_bf16(chunk_mean_fp32(K, c).astype(np.float64))", "return round_to_bf16(chunk_mean(K, c))"),
    ("bf16 table: fp32 additions not in token order", "test_oracle_retrieval.py", "tf_oracle.py",
     "for i in range(c):                          # one rounded", "for i in range(c - 1, -1, -1):               # one rounded"),
    ("ragged accept: every sequence takes the full draft length", "test_oracle_accept.py", "tf_oracle.py",
     "g = int(min(max(int(n_draft[b]), 0), G - 1))", "g = G - 1"),
    ("Algorithm 1: verification against the small model's distribution", "test_oracle_loop.py", "triforce_loop.py",
     "p_hat_all = retrieval_table[N:N + n]", "p_hat_all = draft_table[N:N + n]"),
    ("Algorithm 1: bonus token not counted", "test_oracle_loop.py", "triforce_loop.py",
     "N += n2 + 1", "N += max(n2, 1)"),
    ("Algorithm 1: first-level accept against the target table", "test_oracle_loop.py", "triforce_loop.py",
     "p_hat = retrieval_table[base:base + gamma1 + 1]", "p_hat = target_table[base:base + gamma1 + 1]"),
]


def _scratch_root(tmp_path):
    """A root that holds a copy of oracle/ (to be edited) and links to the rest of the tree."""
    shutil.copytree(os.path.join(ROOT, "oracle"), tmp_path / "oracle",
                    ignore=shutil.ignore_patterns("__pycache__", "*.tmp"))
    for d in ("tests", "paper_2404_11912_amd", "include"):
        os.symlink(os.path.join(ROOT, d), tmp_path / d)


def _run_pins_in(root, pin_file):
    env = {k: v for k, v in os.environ.items() if k != "TF_ORACLE_LIB"}
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join("tests", pin_file), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=root, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)


def test_unedited_copy_of_the_python_part_passes_its_pins(tmp_path):
    _scratch_root(tmp_path)
    res = _run_pins_in(tmp_path, "test_oracle_tree.py")
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("name,pin_file,rel,old,new", PY_MISTAKES, ids=[m[0] for m in PY_MISTAKES])
def test_pins_fail_on_a_planted_mistake_in_the_python_part(tmp_path, name, pin_file, rel, old, new):
    _scratch_root(tmp_path)
    path = tmp_path / "oracle" / rel
    text = path.read_text()
    assert text.count(old) == 1, f"{name}: the oracle's text changed, update this case"
    path.write_text(text.replace(old, new))
    res = _run_pins_in(tmp_path, pin_file)
    assert res.returncode == 1 and " failed" in res.stdout, \
        f"{name}: the pins in {pin_file} did not notice\n{res.stdout[-1500:]}"
