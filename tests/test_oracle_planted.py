"""Planted mistakes in the transformer oracle: every plausible slip below is written into a copy of
oracle/sd_oracle.c, compiled, and the oracle's own pins are run against the broken copy in a fresh process.
At least one pin must fail each time - otherwise the pins would not tell a right oracle from a wrong one."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sd_oracle.c")

# name -> (list of (old, new) replacements, pin files to run - the ones expected to notice, fastest first)
FWD = ["tests/test_oracle_forward.py"]
ACC = ["tests/test_oracle_accept.py", "tests/test_oracle_sd.py"]
BF = ["tests/test_oracle_bf16.py"]
MISTAKES = {
    "residual is |p - q| instead of max(0, p - q)": ([("w[x] = r > 0.0 ? r : 0.0;", "w[x] = r > 0.0 ? r : -r;")], ACC),
    "acceptance ratio inverted": ([("float ratio = p[cand[i]] / qc;", "float ratio = qc / p[cand[i]];")], ACC),
    "acceptance ratio squared": ([("float ratio = p[cand[i]] / qc;", "float ratio = p[cand[i]] / qc * (p[cand[i]] / qc);")], ACC),
    "next token drawn from the previous row": ([("orc_softmax_T(logits + (size_t)n_acc * V, V, T, p);",
                                                 "orc_softmax_T(logits + (size_t)(n_acc > 0 ? n_acc - 1 : 0) * V, V, T, p);")], ACC),
    "temperature multiplies instead of divides": ([("- mx) / T)", "- mx) * T)")], ACC),
    "a row does not see its own key": ([("t <= pos; t++", "t < pos + (pos == 0); t++")], FWD),
    "rotary embedding turns the other way": ([("x[i] = a * c - b * s;", "x[i] = a * c + b * s;"),
                                              ("x[i + half] = b * c + a * s;", "x[i + half] = b * c - a * s;")], FWD),
    "rotary frequency uses i / hd instead of 2 i / hd": ([("pow(base, -2.0 * i / hd)", "pow(base, -1.0 * i / hd)")], FWD),
    "scores scaled by 1 / head_dim": ([("1.0 / sqrt((double)hd)", "1.0 / (double)hd")], FWD),
    "epsilon added outside the square root": ([("1.0 / sqrt(ss / d + eps)", "1.0 / (sqrt(ss / d) + eps)")], FWD),
    "SiLU on the up projection instead of the gate": ([("double g = tmp[i];\n                a[i] = round_act(g / (1.0 + exp(-g)) * tmp2[i], dt);",
                                                        "double g = tmp2[i];\n                a[i] = round_act(g / (1.0 + exp(-g)) * tmp[i], dt);")], FWD),
    "feed-forward output not added to the residual": ([("matvec(m->wdown[l], dt, d, F, a, y);\n            for (int i = 0; i < d; i++) hr[i] += y[i];",
                                                        "matvec(m->wdown[l], dt, d, F, a, y);\n            for (int i = 0; i < d; i++) hr[i] = y[i];")], FWD),
    # the bf16 contract's rounding points, the synthetic-cache loader and adapters with bf16 factors
    "lo term of a two-term activation dropped": ([("return (double)hi + (double)lo;", "return (double)hi;")], BF),
    "attention output not rounded": ([("ob[hh * hd + i] = round_act(acc / z, dt);", "ob[hh * hd + i] = acc / z;")], BF),
    "rotated query not rounded": ([("qb[(size_t)r * HD + i] = round_act(tmp[i], dt);", "qb[(size_t)r * HD + i] = tmp[i];")], BF),
    "key cache stored as two terms": ([("Kc[(size_t)pos * HD + i] = (float)round_storage(tmp[i], dt);",
                                        "Kc[(size_t)pos * HD + i] = (float)round_act(tmp[i], dt);")], BF),
    "value cache stored as two terms": ([("Vc[(size_t)pos * HD + i] = (float)round_storage(tmp[i], dt);",
                                          "Vc[(size_t)pos * HD + i] = (float)round_act(tmp[i], dt);")], BF),
    "SwiGLU product rounded to one term": ([("a[i] = round_act(g / (1.0 + exp(-g)) * tmp2[i], dt);",
                                             "a[i] = round_storage(g / (1.0 + exp(-g)) * tmp2[i], dt);")], BF),
    "final norm not rounded": ([("for (int i = 0; i < d; i++) a[i] = round_act(a[i], dt);\n        matvec(m->lm_head",
                                 "matvec(m->lm_head")], BF),
    "synthetic cache rows read as [dim][token]": ([("kd[i] = (float)weight_at(k, m->c.dtype, i);",
                                                    "kd[i] = (float)weight_at(k, m->c.dtype, (i % HD) * (size_t)len + i / HD);")], BF),
    "synthetic value rows loaded from the key rows": ([("vd[i] = (float)weight_at(v, m->c.dtype, i);",
                                                        "vd[i] = (float)weight_at(k, m->c.dtype, i);")], BF),
    "adapter's B factor read as [rank][out]": ([("b0 + (size_t)n * r + j)", "b0 + (size_t)j * N + n)")],
                                               BF + ["tests/test_oracle_lora.py"]),
    "adapter scale dropped": ([("y[n] += lo->scale * acc;", "y[n] += acc;")], BF + ["tests/test_oracle_lora.py"]),
}


@pytest.mark.parametrize("name", sorted(MISTAKES))
def test_planted_mistake_in_the_c_oracle_is_caught(name, tmp_path):
    edits, pins = MISTAKES[name]
    src = open(SRC).read()
    for old, new in edits:
        assert src.count(old) >= 1, f"the oracle no longer contains the text this mistake replaces: {old!r}"
        src = src.replace(old, new)
    c_file, lib = tmp_path / "broken.c", tmp_path / "libbroken.so"
    c_file.write_text(src)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), str(c_file), "-lm"])
    env = dict(os.environ, SD_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", *pins, "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, f"no pin notices: {name}\n{r.stdout[-1500:]}"
    assert " failed" in r.stdout


def test_unbroken_copy_passes_the_same_way(tmp_path):
    """The harness itself: an unchanged copy, built and loaded the same way, passes the pins."""
    lib = tmp_path / "libsame.so"
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), SRC, "-lm"])
    env = dict(os.environ, SD_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_accept.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-1500:]
