"""The pins must notice plausible mistakes: each case plants one in a copy of the
oracle's C source (on the CPU), builds it, and expects the pin suite to fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "nexus_oracle.c")

MUTATIONS = [
    ("softmax scale uses head_dim instead of its root", "1.0 / sqrt((double)hd)", "1.0 / (double)hd"),
    ("kv head chosen by modulo", "int kvh = hq / G;", "int kvh = hq % m->n_kv_heads;"),
    ("rope sign flipped", "(float)(a * c - bb * s)", "(float)(a * c + bb * s)"),
    ("rope frequency exponent halved", "-2.0 * (double)j / (double)hd", "-1.0 * (double)j / (double)hd"),
    ("rope pairs adjacent elements", "bb = v[j + half];", "bb = v[j ^ 1];"),
    ("causal bound excludes the token itself", "n = pos + 1;", "n = pos > 0 ? pos : 1;"),
    ("rmsnorm forgets eps", "+ (double)eps)", ")"),
    ("rmsnorm divides by sum not mean", "ss / (double)d", "ss"),
    ("linear reads W transposed", "const float *wr = W + (size_t)o * n_in;", "const float *wr = W + (size_t)(o % n_in) * n_in;"),
    ("page slot uses division twice", "*slot = pos % page_size;", "*slot = pos / page_size % page_size;"),
    ("V is rotated too", "oracle_rope(row + qd, Hkv, hd, tok_pos[t], m->rope_theta);",
     "oracle_rope(row + qd, 2 * Hkv, hd, tok_pos[t], m->rope_theta);"),
    ("silu without the gate factor", "z / (1.0 + exp(-z)) * up", "1.0 / (1.0 + exp(-z)) * up"),
    ("gate and up swapped", "double z = gu[(size_t)t * 2 * F + f], up = gu[(size_t)t * 2 * F + F + f];",
     "double up = gu[(size_t)t * 2 * F + f], z = gu[(size_t)t * 2 * F + F + f];"),
    ("second residual dropped", "(float)((double)x1[i] + (double)y[i])", "(float)((double)y[i])"),
    ("first residual dropped", "(float)((double)x[i] + (double)x1[i])", "(float)((double)x1[i])"),
    ("ffn norm uses the attention gain", "oracle_rmsnorm(x1, w->ffn_norm_g", "oracle_rmsnorm(x1, w->attn_norm_g"),
    ("keys cached before rotation", "oracle_rope(row + qd, Hkv, hd, tok_pos[t], m->rope_theta);", ""),
    ("bias dropped", "if (b) acc += (double)b[o];", ""),
    ("row subset: keys projected with the query rows", "w->w_qkv + (size_t)qd * d, w->b_qkv ? w->b_qkv + qd : NULL", "w->w_qkv, w->b_qkv ? w->b_qkv + qd : NULL"),
    ("row subset: bias of the keys taken from the queries", "w->b_qkv ? w->b_qkv + qd : NULL", "w->b_qkv"),
    ("row subset: position of the i-th batch row instead of the listed row", "int t = rows[i];", "int t = i;"),
    ("row subset: queries not rotated", "oracle_rope(q + (size_t)i * qd, Hq, hd, pos[t], m->rope_theta);", ""),
    ("row subset: residual taken from the first rows", "memcpy(xs + (size_t)i * d, x + (size_t)rows[i] * d", "memcpy(xs + (size_t)i * d, x + (size_t)i * d"),
    ("prefill-prioritised constraint uses alpha", "(double)beta * t_d_min", "(double)alpha * t_d_min"),
]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch(tmp_path, what, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site not found: {old!r}"
    mutated = src.replace(old, new)
    c = tmp_path / "mut.c"
    so = tmp_path / "libmut.so"
    c.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"],
                   check=True)
    env = dict(os.environ, NEXUS_ORACLE_LIB_OVERRIDE=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], env=env, cwd=ROOT,
                       capture_output=True, text=True)
    assert r.returncode != 0, f"pins did not notice: {what}"
