"""The pins must notice plausible mistakes. Each case below plants ONE mistake in a copy of the
oracle's C source (CPU only, nothing here touches the HIP path), builds it, and runs the pin suite
against that build in a child process: the suite has to fail, and the planted line has to be one
the unmodified source really contains."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rtlynx_oracle.c")

MUTATIONS = [
    ("tie goes to the higher index", "(aj == ai && j < i)", "(aj == ai && j > i)"),
    ("sign bit takes part in the magnitude key", "unsigned ai = x[i] & 0x7FFFu;", "unsigned ai = x[i] & 0xFFFFu;"),
    ("three kept per group", "(uint8_t)(beaten < 2)", "(uint8_t)(beaten < 3)"),
    ("eps dropped from the kept norm", "den = den + eps;", "den = den;"),
    ("compensation inverted", "s[m * (K / 4) + g] = sqrtf(num / den);", "s[m * (K / 4) + g] = sqrtf(den / num);"),
    ("row scale without the square root", "s[m] = (float)sqrt(num / (den + (double)eps));", "s[m] = (float)(num / (den + (double)eps));"),
    ("nibble halves swapped", "unsigned nib = (unsigned)pos[0] | ((unsigned)pos[1] << 2);\n            meta[m * (K / 8) + g / 2] |= (uint8_t)(nib << (4 * (g & 1)));\n        }\n    }\n    return 0;\n}\n\n/* Inverse",
     "unsigned nib = (unsigned)pos[0] | ((unsigned)pos[1] << 2);\n            meta[m * (K / 8) + g / 2] |= (uint8_t)(nib << (4 * ((g & 1) ^ 1)));\n        }\n    }\n    return 0;\n}\n\n/* Inverse"),
    ("weight matrix read transposed", "acc = acc + S[m * K + k] * bf16_to_f32(W[n * ldw + k]);", "acc = acc + S[m * K + k] * bf16_to_f32(W[(k % N) * ldw + (n % K)]);"),
    ("bias subtracted", "if (bias) acc = acc + bf16_to_f32(bias[n]);", "if (bias) acc = acc - bf16_to_f32(bias[n]);"),
    ("bf16 rounding truncates", "u += 0x7FFFu + lsb;", "u += 0u;"),
    ("LoRA product uses L_B transposed", "acc = acc + bf16_to_f32(LA[n * R + r]) * bf16_to_f32(LB[r * K + k]);", "acc = acc + bf16_to_f32(LA[n * R + r]) * bf16_to_f32(LB[(k % R) * K + (r % K)]);"),
    ("E4M3 ties round away from zero", "if (frac > 0.5f || (frac == 0.5f && (r & 1))) r += 1;", "if (frac >= 0.5f) r += 1;"),
    ("E4M3 overflow is not saturated", "if (a >= 448.0f) return (uint8_t)(sign | 0x7E);", "if (a >= 448.0f) return (uint8_t)(sign | 0x7F);"),
    ("E4M3 subnormals flushed", "if (e < -6) e = -6;", "if (e < -6) return sign;"),
    ("activation multiplied by the scale instead of divided", "const float inv = 1.0f / x_scale;", "const float inv = x_scale;"),
    ("FP8 path forgets the group factor", "if (scope == ORC_GROUP) v = s[m * (K / 4) + k / 4] * v;\n                v = v * inv;", "v = v * inv;"),
]


def run_pins(lib):
    env = dict(os.environ, RTL_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                           "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


def build(src_text, out):
    c = out + ".c"
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", c, "-o", out, "-lm"],
                   check=True)
    return out


def test_unmodified_copy_passes(tmp_path):
    lib = build(open(SRC).read(), str(tmp_path / "orc_same.so"))
    r = run_pins(lib)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, what, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation target not found exactly once: %r" % old
    lib = build(src.replace(old, new), str(tmp_path / "orc_mut.so"))
    r = run_pins(lib)
    assert r.returncode != 0, "the pins did not notice: " + what
