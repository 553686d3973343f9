"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a temporary copy of
oracle/rsparse_oracle.c (a transposed operand, a dropped or negated term, a wrong list, a wrong compare,
an off-by-one, flushed subnormals, a lost tie rule ...), build it, and run tests/test_oracle_pins.py and
tests/test_oracle_variants.py against that library: every mutant must make at least one pin fail.  CPU only; the mistakes live in the
copy, never in the tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rsparse_oracle.c")

MUTANTS = [
    ("tie rule of the keep-predicate", "a >= (double)tau) : (a > (double)tau)", "a > (double)tau) : (a > (double)tau)"),
    ("U read transposed", "ld(U, (size_t)o * r + i, kind_w)", "ld(U, (size_t)i * d_out + o, kind_w)"),
    ("S V^T read transposed", "ld(SV, (size_t)i * d_in + c, kind_w)", "ld(SV, (size_t)c * r + i, kind_w)"),
    ("low-rank part dropped", ": ys + yr;", ": ys;"),
    ("low-rank part negated", ": ys + yr;", ": ys - yr;"),
    ("low-rank part over the kept channels", "int z = list_of(mb, d_in, 0, i_list);", "int z = list_of(mb, d_in, 1, i_list);"),
    ("W read transposed", "ld(W, (size_t)o * d_in + c, kind_w) * xs[c];\n            }\n            /* step 3b",
     "ld(W, (size_t)c * d_out + o, kind_w) * xs[c];\n            }\n            /* step 3b"),
    ("fp16 subnormals flushed", "v = ldexp((double)frac, -24);", "v = 0.0;"),
    ("quantile index off by one", "size_t idx = (size_t)floor(s * (double)n);", "size_t idx = (size_t)floor(s * (double)(n-1));"),
    ("last singular component skipped", "for (int i = 0; i < r; ++i)\n                yr", "for (int i = 0; i < r-1; ++i)\n                yr"),
    ("union mask as an intersection", "umask[c] |= mask", "umask[c] &= mask"),
    ("bf16 rounding truncates", "u += 0x7fffu + ((u >> 16) & 1u);", "u += 0u;"),
    ("bf16 ties round away from zero", "u += 0x7fffu + ((u >> 16) & 1u);", "u += 0x8000u;"),
    ("fp16 ties round up", "if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;", "if (rem >= 0x1000u) ++h;"),
    ("definition rounding: floor instead of nearest", "const double n = rint(q);                         /* nearest, ties to even */",
     "const double n = floor(q);"),
    ("plain SiLU with the wrong sign in the exponent", ": g / (1.0 + exp(-g));", ": g / (1.0 + exp(g));"),
    ("gated input without the up factor", "const float h = orc_silu32(g) * u;", "const float h = orc_silu32(g);"),
    ("4-bit zero point ignored", "((double)q[o * d_in + c] - (double)z[o * G + g])", "((double)q[o * d_in + c])"),
    ("4-bit group index by row", "const size_t g = c / group;", "const size_t g = (c / group + o) % G;"),
    ("top-k: ties to the higher channel", "return x->c < y->c ? -1 : (x->c > y->c ? 1 : 0);", "return x->c > y->c ? -1 : (x->c < y->c ? 1 : 0);"),
    ("top-k: smallest magnitudes kept", "if (x->a != y->a) return x->a > y->a ? -1 : 1;", "if (x->a != y->a) return x->a < y->a ? -1 : 1;"),
    ("top-k: signed values instead of magnitudes", "m[n].a = fabs(v); m[n].c = c;", "m[n].a = v; m[n].c = c;"),
    ("top-k: one channel too many", "int kept = k < n ? k : n;", "int kept = k + 1 < n ? k + 1 : n;"),
    ("signed threshold compares the magnitude", "if (cmp_mode == 2) return x >= (double)tau;", "if (cmp_mode == 2) return fabs(x) >= (double)tau;"),
    ("bias subtracted", "bias ? ys + yr + bias[o]", "bias ? ys + yr - bias[o]"),
    ("multi-phase: upper threshold instead of the midpoint", "return 0.5 * (T[i] + T[i + 1]);", "return T[i];"),
    ("multi-phase residual: midpoint of the wrong interval", "Yr[o] += 0.5 * (T[j] + T[j + 1]) * bsum;", "Yr[o] += 0.5 * (T[j] + T[j]) * bsum;"),
    ("multi-phase: interval boundary to the wrong side", "if (x >= T[i + 1]) return i;", "if (x > T[i + 1]) return i;"),
    ("static bias: sum instead of mean", "bias[o] /= (double)N;", "bias[o] /= 1.0;"),
]


def _run_mutant(args):
    i, (name, old, new), tmp = args
    src = open(SRC).read()
    if old not in src:
        return name, "pattern not found in the oracle source (update the mutant)"
    c_path, lib = os.path.join(tmp, f"mut{i}.c"), os.path.join(tmp, f"mut{i}.so")
    with open(c_path, "w") as f:
        f.write(src.replace(old, new, 1))
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
                    "-w", "-o", lib, c_path, "-lm"], check=True)
    env = dict(os.environ, RSPARSE_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_variants.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    return name, None if r.returncode == 1 else f"survived (pytest exit code {r.returncode})"


def test_every_planted_mistake_is_caught(tmp_path):
    if os.environ.get("RSPARSE_ORACLE_LIB"):
        pytest.skip("already running against an altered oracle")
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run_mutant, [(i, m, str(tmp_path)) for i, m in enumerate(MUTANTS)]))
    bad = [f"{name}: {why}" for name, why in results if why]
    assert not bad, "\n".join(bad)
