"""How strong the oracle's pins are: plausible mistakes are planted, one at a time, in a copy of the oracle (its C
source, or the Python module that chains the steps) on the CPU, in a temporary directory; the pin tests
(tests/test_oracle_*.py) are run against each copy in a child process.  Every planted mistake must make at least one
pin fail; the unmodified copies must pass."""
import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "turborag_oracle.c")

# (name, text in the source, what a mistaken author could have written instead); a pair of tuples where the mistake
# needs a second edit to stay inside its buffers: every planted mistake computes wrong values, none touches memory it
# does not own, so a failure is a pin's assertion and never a crash
MISTAKES = [
    ("rotation turns the other way", "y[a] = xa * c - xb * s;\n        y[b] = xb * c + xa * s;", "y[a] = xa * c + xb * s;\n        y[b] = xb * c - xa * s;"),
    ("cos and sin exchanged", "double c = cos(ang), s = sin(ang);", "double c = sin(ang), s = cos(ang);"),
    ("second element of the pair keeps its own sine term", "y[b] = xb * c + xa * s;", "y[b] = xb * c + xb * s;"),
    ("theta without the factor 2", "pow(base, -2.0 * (double)m / (double)d)", "pow(base, -1.0 * (double)m / (double)d)"),
    ("theta index starts at 1", "pow(base, -2.0 * (double)m / (double)d)", "pow(base, -2.0 * (double)(m + 1) / (double)d)"),
    ("half-split partner off by one", "2 * m + 1 : m + d / 2;", "2 * m + 1 : m + d / 2 - 1 + (m == 0);"),
    ("layout argument ignored", "int a = (layout == ORC_ROPE_INTERLEAVED) ? 2 * m : m;\n        int b = (layout == ORC_ROPE_INTERLEAVED) ? 2 * m + 1 : m + d / 2;",
     "int a = 2 * m;\n        int b = 2 * m + 1; (void)layout;"),
    ("reordered ids restart in every chunk", "pos[off + t] = (int32_t)((pos_mode == ORC_POS_REORDERED) ? off + t : t);", "pos[off + t] = (int32_t)t;"),
    ("composite ids run on", "pos[off + t] = (int32_t)((pos_mode == ORC_POS_REORDERED) ? off + t : t);", "pos[off + t] = (int32_t)(off + t);"),
    ("re-rotation offset one chunk late", "delta[i] = (pos_mode == ORC_POS_REORDERED) ? off : 0;", "delta[i] = (pos_mode == ORC_POS_REORDERED) ? off + len : 0;"),
    ("keys turned back instead of forward", "rope_vec(tmp, out_k + dn, d, (double)delta[i], theta, layout);", "rope_vec(tmp, out_k + dn, d, -(double)delta[i], theta, layout);"),
    ("rows of a chunk gathered one row late", "int64_t so = ((src0 + t) * n_kv + h) * (int64_t)d;", "int64_t so = ((src0 + (t + 1) % len) * n_kv + h) * (int64_t)d;"),
    ("values re-rotated like keys", "out_v[dn + e] = load_elem(v_store, so + e, dtype);", "out_v[dn + e] = load_elem(k_store, so + e, dtype);"),
    ("score scale dropped", "double scale = 1.0 / sqrt((double)d);", "double scale = 1.0;"),
    ("score scale 1/d", "double scale = 1.0 / sqrt((double)d);", "double scale = 1.0 / (double)d;"),
    ("softmax exponent without the row maximum", "scratch[j - lo] = exp(scratch[j - lo] - smax);", "scratch[j - lo] = exp(scratch[j - lo]); (void)smax;"),
    ("softmax relative to the first score, not the largest", "if (s > smax) smax = s;", "if (j == lo) smax = s;"),
    ("weights not normalised", "double w = scratch[j - lo] / denom;", "double w = scratch[j - lo];"),
    ("query token does not see itself", "0, n_doc + i, scratch", "0, n_doc + i - 1, scratch"),
    ("query token sees its successor", "0, n_doc + i, scratch", "0, (n_doc + i + 1 < kv_len ? n_doc + i + 1 : n_doc + i), scratch"),
    ("query heads dealt round-robin to KV heads", "attend_row(q_rot + ((int64_t)i * n_qh + h) * d, k, v, n_kv, h / g, d,", "attend_row(q_rot + ((int64_t)i * n_qh + h) * d, k, v, n_kv, h % n_kv, d,"),
    ("documents attend across chunks", ("cu[c], t, scratch", "double* scratch = (double*)malloc(sizeof(double) * (size_t)max_len);"),
     ("0, t, scratch", "double* scratch = (double*)malloc(sizeof(double) * (size_t)(cu[n_chunks] + 1)); (void)max_len;")),
    ("one-pass mask ignores the range start", "lo[t], t, scratch", "0, t, scratch"),
    ("bf16 by truncation", "double q = nearbyint(ldexp(x, -ulp_exp));", "double q = trunc(ldexp(x, -ulp_exp));"),
    ("bf16 with 7 significant bits", "int ulp_exp = (e - 1) - 7;", "int ulp_exp = (e - 1) - 6;"),
    ("bf16 read from the low half", "(uint32_t)((const uint16_t*)p)[i] << 16;", "(uint32_t)((const uint16_t*)p)[i] << 15;"),
]


# mistakes in the Python module: the chaining of the steps, the sequence plan, the projection
PY_MISTAKES = [
    ("query tokens' keys appended without rotation", "kq_rot = rope(k_q, q_pos, base, layout)", "kq_rot = widen(k_q)"),
    ("queries rotated at their index among the query tokens", "q_rot = rope(q, q_pos, base, layout)\n    res[\"out\"] = attn_prefix(",
     "q_rot = rope(q, np.arange(len(q_pos)), base, layout)\n    res[\"out\"] = attn_prefix("),
    ("values appended before the documents", "v_cache = np.concatenate([v_asm, widen(v_q)], axis=0)", "v_cache = np.concatenate([widen(v_q), v_asm], axis=0)"),
    ("offline queries not rotated", "q_rot = rope(q, lp, base, layout)", "q_rot = widen(q)"),
    ("offline keys rotated at packed positions", "k_rot = rope(k, lp, base, layout)", "k_rot = rope(k, np.arange(lp.size), base, layout)"),
    ("document tokens see the previous chunks", "lo[off:off + l] = off\n", "lo[off:off + l] = 0\n"),
    ("tail ids restart at zero", "pos[n_doc:] = tail_start + np.arange(n_tail)", "pos[n_doc:] = np.arange(n_tail)"),
    ("composite tail starts behind all documents", "tail_start = n_doc if pos_mode == POS_REORDERED else (max(chunk_lens) if chunk_lens else 0)", "tail_start = n_doc"),
    ("one-pass keys rotated, queries not", "q_rot = rope(q, pos, base, layout)", "q_rot = widen(q)"),
    ("projection with the weight not transposed", "np.matmul(widen(x), widen(w).T)", "np.matmul(widen(x), widen(w))"),
]


def _apply(text, name, old, new):
    olds, news = (old, new) if isinstance(old, tuple) else ((old,), (new,))
    for o, n in zip(olds, news):
        assert text.count(o) == 1, "the source text of mistake %r is not unique in the oracle: %d" % (name, text.count(o))
        text = text.replace(o, n)
    return text


def _build(src_text, path):
    with open(path + ".c", "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", path + ".so", path + ".c", "-lm"], check=True)
    return path + ".so"


def _pins_pass(where):
    """where: a compiled copy of the C source (.so), or a directory that holds a copy of the oracle package"""
    env = dict(os.environ, OMP_NUM_THREADS="2")
    env["TR_ORACLE_LIB" if where.endswith(".so") else "TR_ORACLE_PATH"] = where
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode in (0, 1), "the pin tests did not run to an ordinary end (exit %d):\n%s" % (r.returncode, r.stdout[-600:] + r.stderr[-600:])
    return r.returncode == 0, r.stdout[-600:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    src = open(SRC).read()
    libs = []
    for i, (name, old, new) in enumerate(MISTAKES):
        libs.append(_build(_apply(src, name, old, new), str(tmp_path / ("mistake%02d" % i))))
    control = _build(src, str(tmp_path / "control"))
    with ThreadPoolExecutor(4) as ex:
        results = list(ex.map(_pins_pass, libs + [control]))
    ok, tail = results[-1]
    assert ok, "the pins fail on an unmodified copy of the oracle:\n" + tail
    missed = [MISTAKES[i][0] for i, (passed, _) in enumerate(results[:-1]) if passed]
    assert not missed, "no pin notices: " + "; ".join(missed)


def _package_copy(tmp_path, name, old=None, new=None):
    d = tmp_path / name
    shutil.copytree(os.path.join(ROOT, "oracle"), str(d / "oracle"), ignore=shutil.ignore_patterns("__pycache__"))
    if old is not None:
        f = d / "oracle" / "__init__.py"
        f.write_text(_apply(f.read_text(), name, old, new))
    return str(d)


def test_every_mistake_planted_in_the_python_module_fails_a_pin(tmp_path):
    dirs = [_package_copy(tmp_path, "py%02d" % i, old, new) for i, (_, old, new) in enumerate(PY_MISTAKES)]
    control = _package_copy(tmp_path, "control")
    with ThreadPoolExecutor(4) as ex:
        results = list(ex.map(_pins_pass, dirs + [control]))
    ok, tail = results[-1]
    assert ok, "the pins fail on an unmodified copy of the oracle:\n" + tail
    missed = [PY_MISTAKES[i][0] for i, (passed, _) in enumerate(results[:-1]) if passed]
    assert not missed, "no pin notices: " + "; ".join(missed)
