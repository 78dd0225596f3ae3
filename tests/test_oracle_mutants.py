"""The pins must notice a mistake planted in the oracle.

Each case below is a copy of the oracle's C source with one plausible slip (a sign, an index,
an off-by-one, a dropped term, swapped operands), compiled on the CPU and run against
``tests/test_oracle_pins.py`` in a child process.  The pins have to fail for every one of them
and pass for the untouched source.  Nothing here touches the GPU or the HIP library.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "lshe_oracle.c")

# (name, text in the source, replacement); the text must occur exactly `count` times and the
# `which`-th occurrence (0-based) is replaced
MUTANTS = [
    ("hash: zero projection signs to 0", "if (p >= 0.0)", "if (p > 0.0)", 0),
    ("hash: bit order inside a word reversed", "1u << (j % 32);", "1u << (31 - j % 32);", 0),
    ("hash: R read transposed",
     "p += (double)x[i] * (double)R[(size_t)i * r + j];",
     "p += (double)x[i] * (double)R[(size_t)j * d + i];", 0),
    ("hash: sign flipped", "if (p >= 0.0)", "if (p < 0.0)", 0),
    ("score: only the first query head votes",
     "for (int g = 0; g < G; ++g)\n            for (int w = 0; w < W; ++w)",
     "for (int g = 0; g < 1; ++g)\n            for (int w = 0; w < W; ++w)", 0),
    ("score: AND instead of XOR", "uint32_t x = a ^ b;", "uint32_t x = a & b;", 0),
    ("score: top bit of a word not counted", "for (int k = 0; k < 32; ++k)", "for (int k = 0; k < 31; ++k)", 0),
    ("score: second code word ignored",
     "acc += hamming_word(codes[(size_t)s * W + w], cq[(size_t)g * W + w]);",
     "acc += hamming_word(codes[(size_t)s * W], cq[(size_t)g * W]);", 0),
    ("select: ties go to the highest slot", "if (score[s] > best_score) {", "if (score[s] >= best_score) {", 0),
    ("select: recent window one token short", "p > t - 1 - n_recent", "p > t - n_recent", 0),
    ("select: one sink too many", "if (p < n_sink ||", "if (p <= n_sink ||", 0),
    ("select: a filling cache overwrites slot 0", "return n_valid;\n    int best", "return 0;\n    int best", 0),
    ("select: smallest score evicted",
     "if (score[s] > best_score) {\n            best_score = score[s];",
     "if (best < 0 || score[s] < best_score) {\n            best_score = score[s];", 0),
    ("apply: position off by one", "slot_pos[e] = t;", "slot_pos[e] = t + 1;", 0),
    ("apply: key stored as value", "memcpy(V + (size_t)e * d, v_new,", "memcpy(V + (size_t)e * d, k_new,", 0),
    ("apply: query code stored in the table",
     "c + (size_t)G * W, t);\n    if (rc == 0 && do_attend && out)", "c, t);\n    if (rc == 0 && do_attend && out)", 0),
    ("attend: scaled by 1/d", "double inv = 1.0 / sqrt((double)d);", "double inv = 1.0 / (double)d;", 0),
    ("attend: weights not normalised", "double p = a[s] / den;", "double p = a[s];", 0),
    ("attend: keys summed instead of values",
     "o[i] += p * (double)V[(size_t)s * d + i];", "o[i] += p * (double)K[(size_t)s * d + i];", 0),
    ("attend: last slot left out",
     "for (int s = 0; s < n_valid; ++s) {\n            double dot = 0.0;",
     "for (int s = 0; s < n_valid - 1; ++s) {\n            double dot = 0.0;", 0),
    ("mass: the new key is not in the denominator",
     "for (int s = 0; s <= C; ++s)\n            den += exp(a[s] - mx);",
     "for (int s = 0; s < C; ++s)\n            den += exp(a[s] - mx);", 0),
    ("mass: probability of the new key reported", "mass[g] = exp(a[e] - mx) / den;",
     "mass[g] = exp(a[C] - mx) / den;", 0),
    ("mass: scaled by 1/d", "double inv = 1.0 / sqrt((double)d);", "double inv = 1.0 / (double)d;", 1),
    ("step: attention before the overwrite",
     "    int rc = lsheo_apply(K, V, codes, slot_pos, n_valid, C, d, W, e, k_new, v_new, c + (size_t)G * W, t);\n"
     "    if (rc == 0 && do_attend && out)\n        lsheo_attend(q, K, V, *n_valid, d, G, out, NULL);",
     "    if (do_attend && out)\n        lsheo_attend(q, K, V, *n_valid, d, G, out, NULL);\n"
     "    int rc = lsheo_apply(K, V, codes, slot_pos, n_valid, C, d, W, e, k_new, v_new, c + (size_t)G * W, t);", 0),
    ("prefill: query layout [N][G] instead of [G][N]",
     "Qp + ((size_t)g * N + t) * d", "Qp + ((size_t)t * G + g) * d", 0),
    ("prefill: victim logged one step late", "evict_log[t - C] = e;\n    }\n    free(q);",
     "evict_log[t - C] = t > C ? evict_log[t - C - 1] : e;\n    }\n    free(q);", 0),
    ("apply: a slot index of -1 is written", "if (e < 0 || e >= C || e > *n_valid)", "if (e >= C || e > *n_valid)", 0),
    ("l2: sum of absolute values", "s += (double)x[i] * (double)x[i];\n    return s;",
     "s += fabs((double)x[i]);\n    return s;", 0),
    ("l2: norm accumulated in single precision",
     "double s = 0.0;\n    for (int i = 0; i < d; ++i)\n        s += (double)x[i] * (double)x[i];\n    return s;",
     "float s = 0.0f;\n    for (int i = 0; i < d; ++i)\n        s = fmaf(x[i], x[i], s);\n    return s;", 0),
    ("l2: the new key's norm is not stored", "norm2[e] = lsheo_norm2(k_new, d);", "", 0),
    ("l2: smallest norm evicted",
     "if (norm2[s] > best_norm) {\n            best_norm = norm2[s];",
     "if (best < 0 || norm2[s] < best_norm) {\n            best_norm = norm2[s];", 0),
    ("l2: ties go to the highest slot", "if (norm2[s] > best_norm) {", "if (norm2[s] >= best_norm) {", 0),
    ("l2: recent tokens not protected",
     "if (p < n_sink || p > t - 1 - n_recent)\n            continue;\n        if (norm2[s] > best_norm) {",
     "if (p < n_sink)\n            continue;\n        if (norm2[s] > best_norm) {", 0),
    ("l2: a supplied victim is ignored", "int e = victim_in >= 0 ? victim_in\n                           :", "int e =", 0),
]


def _build(tmp, name, text):
    c = os.path.join(tmp, name + ".c")
    so = os.path.join(tmp, name + ".so")
    with open(c, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-w", "-o", so, c, "-lm"])
    return so


# The child process loads the library under test explicitly, before the pins import the oracle
# package (which would otherwise build and load the real one), then runs the pins.
_RUNNER = ("import sys; sys.path.insert(0, %r); import oracle; oracle.load(sys.argv[1]); import pytest; "
           "sys.exit(pytest.main([%r, '-x', '-q', '-p', 'no:cacheprovider']))"
           % (ROOT, os.path.join(HERE, "test_oracle_pins.py")))


def _pins_pass(so):
    env = dict(os.environ, OMP_NUM_THREADS="1")
    p = subprocess.run([sys.executable, "-c", _RUNNER, so], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=600)
    return p.returncode == 0, p.stdout[-1500:]


def _nth_replace(src, old, new, which):
    parts = src.split(old)
    assert len(parts) - 1 > which, "text to mutate not found: %r" % old
    return old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])


def test_pins_catch_every_planted_mistake(tmp_path):
    src = open(SRC).read()
    tmp = str(tmp_path)
    jobs = [("untouched", _build(tmp, "m_ref", src))]
    for i, (name, old, new, which) in enumerate(MUTANTS):
        jobs.append((name, _build(tmp, "m%02d" % i, _nth_replace(src, old, new, which))))
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda j: _pins_pass(j[1]), jobs))
    ok_ref, out_ref = results[0]
    assert ok_ref, "the pins fail on the untouched oracle:\n" + out_ref
    survivors = [name for (name, _), (ok, _) in zip(jobs[1:], results[1:]) if ok]
    assert not survivors, "no pin notices: " + "; ".join(survivors)
