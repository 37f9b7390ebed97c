"""Do the pins bite?  Each case plants one plausible mistake (a dropped term, a wrong sign, index,
constant or operand order) in a temporary copy of the oracle's C source, builds it, and runs the pin
suite against that copy in a child process: the suite must FAIL.  CPU only; nothing here touches
the real oracle or the HIP path."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "itq3s_ref.c")

# (name, text in the oracle, replacement)
MUTATIONS = [
    ("butterfly: difference with the wrong sign", "a[i + step] = u - v;", "a[i + step] = v - u;"),
    ("butterfly: stages in descending order",
     "for (int step = 1; step < ITQ3S_REF_BLOCK; step <<= 1)\n        for (int i = 0; i < ITQ3S_REF_BLOCK; i++)",
     "for (int step = 128; step >= 1; step >>= 1)\n        for (int i = 0; i < ITQ3S_REF_BLOCK; i++)"),
    ("normalisation 1/8 instead of 1/16", "a[j] = a[j] * 0.0625;", "a[j] = a[j] * 0.125;"),
    ("mean over 255", "double mu = ref_pairwise_sum256(a) / 256.0;", "double mu = ref_pairwise_sum256(a) / 255.0;"),
    ("sample instead of population deviation", "sqrt(ref_pairwise_sum256(e2) / 256.0)", "sqrt(ref_pairwise_sum256(e2) / 255.0)"),
    ("deviation about zero instead of the mean", "double dev = a[j] - mu;", "double dev = a[j];"),
    ("zero-point with the wrong sign", "double z = 0.0 - r;", "double z = r;"),
    ("zero-point truncated instead of rounded", "floor(mu / d + 0.5)", "floor(mu / d)"),
    ("upper tie goes down", "a[j] >= t_hi ? 2", "a[j] > t_hi ? 2"),
    ("lower tie goes down", "a[j] < t_lo ? 0", "a[j] <= t_lo ? 0"),
    ("threshold with +z", "double t_hi = (0.5 - z) * d", "double t_hi = (0.5 + z) * d"),
    ("dequantize adds z", "v[e] = ((double)c - 1.0) - z;", "v[e] = ((double)c - 1.0) + z;"),
    ("dequantize forgets the code offset", "v[e] = ((double)c - 1.0) - z;", "v[e] = ((double)c) - z;"),
    ("dequantize scale off by 0.16 %", "out[e] = d * v[e] * 0.0625;", "out[e] = d * v[e] * 0.0626;"),
    ("storage: neighbouring fields swapped",
     "int lane = 16 * (e >> 6) + r, i = e & 63;\n    uint32_t lo = ", "int lane = 16 * (e >> 6) + r, i = (e & 63)^1;\n    uint32_t lo = "),
    ("matmul: activations reversed", "acc += x[k] * wrow[k];", "acc += x[k] * wrow[K-1-k];"),
    ("scale constant 0.798", "static const double ITQ3S_REF_T_STAR = 0.7979;", "static const double ITQ3S_REF_T_STAR = 0.798;"),
    ("fp16 rounding: ties away", "if (rem > 0x1000u || (rem == 0x1000u && (kept & 1u))) out++;", "if (rem >= 0x1000u) out++;"),
    ("scale word halves swapped", "(uint32_t)dbits | ((uint32_t)zbits << 16)", "(uint32_t)zbits | ((uint32_t)dbits << 16)"),
    ("n-point round trip: normalisation of n = 128", "case 128: return 0.08838834764831843;", "case 128: return 0.0883883476483;"),
    ("n-point round trip: reconstruction forgets z", "m[j] = (double)((int)c[j] - 1) - z;", "m[j] = (double)((int)c[j] - 1);"),
    ("sub-scales: deviation over 31", "double sigma_j = sqrt(ref_pairwise_sum32(e2 + 32 * j) / 32.0);", "double sigma_j = sqrt(ref_pairwise_sum32(e2 + 32 * j) / 31.0);"),
    ("sub-scales: threshold ignores the sub-scale", "double t_hi = (0.5 * s - z) * d, t_lo = (-0.5 * s - z) * d;", "double t_hi = (0.5 - z) * d, t_lo = (-0.5 * s - z) * d;"),
    ("sub-scales: zero-point scaled by the sub-scale", "v[e] = s * ((double)c - 1.0) - z;", "v[e] = s * (((double)c - 1.0) - z);"),
    ("sub-scales: halves of the storage word swapped", "(uint32_t)sb[2 * g] | ((uint32_t)sb[2 * g + 1] << 16)", "(uint32_t)sb[2 * g + 1] | ((uint32_t)sb[2 * g] << 16)"),
    ("sub-scales: relative to sigma instead of d", "double s64 = ITQ3S_REF_T_STAR * sigma_j / d;", "double s64 = sigma_j / sigma;"),
    ("n-point round trip: mean over n - 1", "double mu = ref_pairwise_sum_n(a, n) / (double)n;", "double mu = ref_pairwise_sum_n(a, n) / (double)(n - 1);"),
]


def run_pins_against(tmp_path, idx, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, "the oracle no longer contains: %r" % old
    src = os.path.join(str(tmp_path), "mut%d.c" % idx)
    with open(src, "w") as f:
        f.write(text.replace(old, new, 1))
    env = dict(os.environ, ITQ3S_REF_SRC=src, ITQ3S_REF_LIB=os.path.join(str(tmp_path), "libmut%d.so" % idx))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_sub_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode, r.stdout[-400:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda a: run_pins_against(tmp_path, a[0], a[1][1], a[1][2]), enumerate(MUTATIONS)))
    survivors = [MUTATIONS[i][0] for i, (rc, _) in enumerate(results) if rc == 0]
    broken = [(MUTATIONS[i][0], out) for i, (rc, out) in enumerate(results) if rc not in (0, 1)]
    assert not broken, "the pin suite did not run for: %r" % broken
    assert not survivors, "no pin noticed: %r" % survivors


def test_the_unmutated_copy_passes(tmp_path):
    """Control: the same procedure with no mistake planted passes, so a failure above is the mistake's."""
    rc, out = run_pins_against(tmp_path, 999, "static const double ITQ3S_REF_T_STAR = 0.7979;", "static const double ITQ3S_REF_T_STAR = 0.7979;")
    assert rc == 0, out


def test_summation_tree_is_a_reading_not_a_pin(tmp_path):
    """The neighbour-first tree of the block sums is this build's reading of an unspecified detail
    (any summation order satisfies the paper); a sequential sum passes every pin, and this test
    records that fact so that nobody mistakes the tree for something the paper fixes."""
    old = "static double ref_pairwise_sum256(const double *v)\n{"
    text = open(SRC).read()
    assert old in text
    rc, out = run_pins_against(tmp_path, 998, old, old + "\n    { double s_ = 0.0; for (int i_ = 0; i_ < 256; i_++) s_ += v[i_]; return s_; }")
    assert rc == 0, out
