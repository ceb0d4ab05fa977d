"""Mutation check of the oracle's pins: every mistake planted into a COPY of the C oracle (a dropped
bias, a transposed weight, swapped block/slot arithmetic, a missing scale or normalisation, the
wrong K/V block layout, ...) must make tests/test_oracle_pins.py fail.  A pin set that lets one of
them through would not pin the oracle.  CPU only; the source tree is never modified: the altered
source is compiled in a temporary directory and loaded through APT_ORACLE_LIB."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "apt_oracle.c")

# (name, text in apt_oracle.c, replacement)
MUTATIONS = [
    ("drop b_V", "vj[c] = elem(b_V, (int64_t)h * hd + c, dt);", "vj[c] = 0.0;"),
    ("drop b_K", "kj[c] = elem(b_K, (int64_t)h * hd + c, dt);", "kj[c] = 0.0;"),
    ("transpose W_K", "wk[(int64_t)i * hd + c] = elem(W_K, (int64_t)i * d + (int64_t)h * hd + c, dt);",
     "wk[(int64_t)i * hd + c] = elem(W_K, ((int64_t)h * hd + c) * d + i, dt);"),
    ("transpose W_V", "wv[(int64_t)i * hd + c] = elem(W_V, (int64_t)i * d + (int64_t)h * hd + c, dt);",
     "wv[(int64_t)i * hd + c] = elem(W_V, ((int64_t)h * hd + c) * d + i, dt);"),
    ("slot from block index", "*slot = j % bs;", "*slot = (j / bs) % bs;"),
    ("block from slot index", "max_blocks + j / bs]", "max_blocks + j % bs]"),
    ("no softmax scale", "sc[j] = s->scale * dot;\n            if (sc[j] > mx) mx = sc[j];\n        }\n        /*",
     "sc[j] = dot;\n            if (sc[j] > mx) mx = sc[j];\n        }\n        /*"),
    ("no normalisation", "const double a = sc[j] / den;", "const double a = sc[j];"),
    ("K/V block token-major", "int64_t off = ((int64_t)h * bs + slot) * hd;",
     "int64_t off = ((int64_t)slot * s->n_heads + h) * hd;"),
    ("V through the K list", "apt_oracle_locate(block_tables, s->max_blocks, bs, r, 1, j, &bv, &slot);",
     "apt_oracle_locate(block_tables, s->max_blocks, bs, r, 0, j, &bv, &slot);"),
    ("sign of the exponent", "sc[j] = exp(sc[j] - mx);", "sc[j] = exp(mx - sc[j]);"),
    ("merge without weights", "ls += l[s] * w;", "ls += l[s];"),
    ("partial uses head 0's query",
     "dot += elem(q, ((int64_t)r * H + h) * hd + c, s->dtype) * k[(int64_t)j * hd + c];\n        sc[j] = s->scale * dot;\n"
     "        if (sc[j] > mx) mx = sc[j];\n    }\n    double l = 0.0;",
     "dot += elem(q, ((int64_t)r * H + 0) * hd + c, s->dtype) * k[(int64_t)j * hd + c];\n        sc[j] = s->scale * dot;\n"
     "        if (sc[j] > mx) mx = sc[j];\n    }\n    double l = 0.0;"),
    ("fp16 subnormals flushed", "if (e == 0) v = ldexp((double)m, -24);", "if (e == 0) v = 0.0;"),
]


def _pins_pass(lib_path):
    env = dict(os.environ, APT_ORACLE_LIB=lib_path)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode == 0


def _build(src_text, out_dir, tag):
    c = os.path.join(out_dir, f"oracle_{tag}.c")
    so = os.path.join(out_dir, f"liboracle_{tag}.so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", so, c, "-lm"], check=True)
    return so


def test_every_planted_mistake_fails_a_pin(tmp_path):
    orig = open(SRC).read()
    # the unaltered copy, loaded the same way, passes: a failure below is due to the mutation
    assert _pins_pass(_build(orig, str(tmp_path), "orig"))

    def run(i):
        name, a, b = MUTATIONS[i]
        if orig.count(a) != 1:
            return name, "anchor text not found exactly once in apt_oracle.c"
        so = _build(orig.replace(a, b), str(tmp_path), str(i))
        return name, "missed" if _pins_pass(so) else "caught"

    with ThreadPoolExecutor(4) as ex:
        results = list(ex.map(run, range(len(MUTATIONS))))
    bad = [(n, r) for n, r in results if r != "caught"]
    assert not bad, bad
