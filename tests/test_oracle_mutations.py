"""The pins really pin: a mistake planted in a copy of the oracle's C source (on the CPU) must make at least
one pin test fail.  Each mutation is one plausible slip: a sign, an index, a dropped term, a wrong divisor."""
import ctypes
import os
import subprocess

import pytest

import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "tri_oracle.c")

MUTATIONS = [
    ("phase sign", "atan2(qim, qre) - atan2(kim, kre)", "atan2(kim, kre) - atan2(qim, qre)"),
    ("offset sign", "Delta + offsets[j]", "Delta - offsets[j]"),
    ("distance sign", "int64_t Delta = p_q - p_k;", "int64_t Delta = p_k - p_q;"),
    ("norm term unweighted", "s += (qabs - hypot(qre, qim)) * hypot(kre, kim);", "s += qabs * hypot(kre, kim);"),
    ("norm term dropped", "tri_oracle_s_norm(stats, key, dtype, first, d, pairs);\n        acc += S;",
     "0.0;\n        acc += S;"),
    ("sample sigma", "sigma[g] = sqrt(ss / (double)N);", "sigma[g] = sqrt(ss / (double)(N - 1));"),
    ("equal scores not recognised", "if (lo == hi) ss = 0.0;", ""),
    ("tie to the higher index", "if (a[j].score > a[i].score) tmp", "if (a[j].score >= a[i].score) tmp"),
    ("min instead of max", "if (g == 0 || z > best) best = z;", "if (g == 0 || z < best) best = z;"),
    ("frequency exponent", "-2.0 * (double)f / (double)d", "-1.0 * (double)f / (double)d"),
    ("sum instead of mean over offsets", "return acc / (double)n_off;", "return acc;"),
    ("imaginary part from the wrong element", "first + 2 * (int64_t)f + 1);", "first + 2 * (int64_t)f);"),
    ("centre modulus mean dropped", "sabs += hypot(re, im);", "sabs += fabs(re);"),
    ("un-rotation by the wrong sign", "double ki = -s * xr + c * xi;", "double ki = s * xr + c * xi;"),
    ("un-rotation not applied", "kd = ORACLE_F64;\n            first = 0;", "kd = ORACLE_F64;\n            first = 0;\n            for (int e = 0; e < d; ++e) tmp[e] = load_elem(K, dtype, n * row_stride + e);"),
    ("w/o R keeps the weighted term", "if (variant == 0 || variant == 2) S += tri_oracle_s_norm(", "if (variant != 1) S += tri_oracle_s_norm("),
    ("trig-only keeps the norm term", "if (variant == 3) S += tri_oracle_s_norm0(", "if (variant == 3 || variant == 1) S += tri_oracle_s_norm0("),
    ("unweighted norm uses the centre modulus", "s += qabs * hypot(kre, kim);", "s += hypot((double)stats[3 * f], (double)stats[3 * f + 1]) * hypot(kre, kim);"),
    ("MRL inverted", "out[i] = ab > 0.0 ? hypot(re, im) / ab : 0.0;", "out[i] = ab > 0.0 ? ab / hypot(re, im) : 0.0;"),
    ("band contribution from the centre modulus", "c[f] = (double)q[3 * f + 2] * (double)k[3 * f + 2];", "c[f] = hypot((double)q[3 * f], (double)q[3 * f + 1]) * (double)k[3 * f + 2];"),
    ("dominant bands: KV head of the wrong group", "kstats + ((int64_t)l * Hkv + h / G) * F * 3;", "kstats + ((int64_t)l * Hkv + h % Hkv) * F * 3;"),
    ("compaction source off by one", "(int64_t)idx[j] * src_stride_bytes", "(int64_t)(idx[j] + 1) * src_stride_bytes"),
]

PIN_TESTS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]


def run_pins(oracle_module):
    """Run every pin test against `oracle_module`; return the names of those that fail."""
    failed = []
    for fn in PIN_TESTS:
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [{}]
        for m in marks:
            names = [x.strip() for x in m.args[0].split(",")]
            cases = [dict(c, **dict(zip(names, v if isinstance(v, (tuple, list)) else (v,)))) for c in cases for v in m.args[1]]
        for kw in cases:
            try:
                fn(oracle_module, **kw)
            except Exception:   # an assertion, or a crash caused by the planted mistake
                failed.append(fn.__name__)
                break
    return failed


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(oracle, tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation target not found: %s" % old
    src = tmp_path / "mut.c"
    lib = tmp_path / "libmut.so"
    src.write_text(text.replace(old, new, 1))
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-o", str(lib), str(src), "-lm"])
    good = oracle._lib
    try:
        oracle._lib = None
        real_build, real_path = oracle.build, oracle._LIB
        oracle.build = lambda force=False: str(lib)
        oracle._LIB = str(lib)
        oracle.lib()
        failed = run_pins(oracle)
    finally:
        oracle.build, oracle._LIB, oracle._lib = real_build, real_path, good
    assert failed, "no pin noticed the planted mistake '%s'" % name


def test_unmutated_oracle_passes_all_pins(oracle):
    assert run_pins(oracle) == []
