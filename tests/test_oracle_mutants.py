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
     "c + (size_t)G * W, t);\n    if (do_attend && out)", "c, t);\n    if (do_attend && out)", 0),
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
     "    lsheo_apply(K, V, codes, slot_pos, n_valid, C, d, W, e, k_new, v_new, c + (size_t)G * W, t);\n"
     "    if (do_attend && out)\n        lsheo_attend(q, K, V, *n_valid, d, G, out, NULL);",
     "    if (do_attend && out)\n        lsheo_attend(q, K, V, *n_valid, d, G, out, NULL);\n"
     "    lsheo_apply(K, V, codes, slot_pos, n_valid, C, d, W, e, k_new, v_new, c + (size_t)G * W, t);", 0),
    ("prefill: query layout [N][G] instead of [G][N]",
     "Qp + ((size_t)g * N + t) * d", "Qp + ((size_t)t * G + g) * d", 0),
    ("prefill: victim logged one step late", "evict_log[t - C] = e;\n    }\n    free(q);",
     "evict_log[t - C] = t > C ? evict_log[t - C - 1] : e;\n    }\n    free(q);", 0),
    ("l2: sum of absolute values", "s = fmaf(x[i], x[i], s);", "s = s + fabsf(x[i]);", 0),
    ("l2: new key's code is the old slot's",
     "uint32_t c_new = float_bits(lsheo_norm2(k_new, d));",
     "uint32_t c_new = e >= 0 && e < *n_valid ? codes[e] : float_bits(lsheo_norm2(k_new, d));", 0),
]


def _build(tmp, name, text):
    c = os.path.join(tmp, name + ".c")
    so = os.path.join(tmp, name + ".so")
    with open(c, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-w", "-o", so, c, "-lm"])
    return so


def _pins_pass(so):
    env = dict(os.environ, LSHE_ORACLE_LIB=so, OMP_NUM_THREADS="1")
    p = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
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
