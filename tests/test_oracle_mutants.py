"""The pins of the oracle have to notice a plausible mistake anywhere in it.  Each case below plants
one in a COPY of oracle/reshard_oracle.cpp (on the CPU; the real oracle is never touched), builds
it, and runs the pin tests against the broken build in a child process: they must fail (or the
child must die on the broken oracle's wild accesses)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "reshard_oracle.cpp")

MUTANTS = [
    ("ravel walks the shape backwards",
     "f = f * shape[k] + x[k];", "f = f * shape[n - 1 - k] + x[k];"),
    ("unravel starts at the slowest dimension",
     "for (int k = n - 1; k >= 0; --k) {\n    out[k] = flat % shape[k];",
     "for (int k = 0; k < n; ++k) {\n    out[k] = flat % shape[k];"),
    ("box offsets dropped on the saved side",
     "for (int d = 0; d < n; ++d) x[d] = p.offsets[d] + y[d];\n        const int64_t gi",
     "for (int d = 0; d < n; ++d) x[d] = y[d];\n        const int64_t gi"),
    ("box offsets dropped on the target side",
     "for (int d = 0; d < n; ++d) x[d] = p.offsets[d] + y[d];\n      const int64_t gi",
     "for (int d = 0; d < n; ++d) x[d] = y[d];\n      const int64_t gi"),
    ("flat_begin not subtracted from the stored position",
     "(concat_index - sh.flat_begin)", "(concat_index)"),
    ("strides ignored",
     "e += y[d] * sh.strides[d];", "e += y[d];"),
    ("parts of a shard all start at position 0 of the concatenation",
     "pos += volume(p.lengths, p.ndim);", "pos += 0 * volume(p.lengths, p.ndim);"),
    ("slice of the concatenation one element too long",
     "const int64_t last = std::min<int64_t>(sh.flat_end - r.concat_pos, pvol);\n      for (int64_t local = first; local < last; ++local) {\n        const int64_t ci",
     "const int64_t last = std::min<int64_t>(sh.flat_end - r.concat_pos + 1, pvol);\n      for (int64_t local = first; local < last; ++local) {\n        const int64_t ci"),
    ("slice of the concatenation starts one element late",
     "const int64_t first = std::max<int64_t>(sh.flat_begin - r.concat_pos, 0);\n    const int64_t last",
     "const int64_t first = std::max<int64_t>(sh.flat_begin - r.concat_pos + 1, 0);\n    const int64_t last"),
    ("saved overlap not detected",
     "if (cnt[gi]) return job.err.set(ORC_SAVED_OVERLAP", "if (false) return job.err.set(ORC_SAVED_OVERLAP"),
    ("uncovered elements silently skipped",
     "if (job.allow_uncovered) continue;", "continue;"),
    ("itemsize taken as one byte in the global image",
     "std::memcpy(&G[(size_t)gi * e], job.src[sh.buf] + b, e);", "std::memcpy(&G[(size_t)gi * e], job.src[sh.buf] + b, 1);"),
    ("shape disagreement not checked",
     "if (p.global_shape[d] != t0.global_shape[d]) return false;", "if (false) return false;"),
]


# mistakes in the dtype-converting load; its pins are tests/test_oracle_convert.py
CONVERT_MUTANTS = [
    ("ties go away from zero instead of to even",
     "else pick = (below & 1u) == 0 ? below : above;", "else pick = above;"),
    ("truncation instead of rounding",
     "if (down < up) pick = below;\n  else if (up < down) pick = above;", "if (down <= up || up < down) pick = below;\n  else if (up < down) pick = above;"),
    ("bfloat16 subnormals one binade off",
     "if (exp == 0) return std::ldexp(frac, -133);", "if (exp == 0) return std::ldexp(frac, -134);"),
    ("binary32 subnormals one binade off",
     "if (exp == 0) return std::ldexp(frac, -149);", "if (exp == 0) return std::ldexp(frac, -150);"),
    ("seven fraction bits taken as eight",
     "return std::ldexp(128.0 + frac, exp - 134);", "return std::ldexp(256.0 + frac, exp - 135);"),
    ("sign dropped",
     "return (uint16_t)((sign << 15) | pick);", "return (uint16_t)(pick);"),
    ("NaN rounded like a number",
     "if (mag > 0x7f800000u) {", "if (false) {"),
    ("narrowing applied with the wrong element size in the global image",
     "std::memcpy(&wide, &G[(size_t)gi * e], 4);", "std::memcpy(&wide, &G[(size_t)gi * et], 4);"),
    ("conversion without the flag",
     "if (job.convert == 1 && es == 4 && et == 2) e = es;", "if (es == 4 && et == 2) e = es;"),
    ("any wider element size converts",
     "if (job.convert == 1 && es == 4 && et == 2) e = es;", "if (job.convert == 1 && es > et) e = es;"),
]


@pytest.mark.parametrize("name,old,new", CONVERT_MUTANTS, ids=[m[0] for m in CONVERT_MUTANTS])
def test_convert_pins_catch_the_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    mutant_src = tmp_path / "mutant.cpp"
    mutant_src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-pthread", str(mutant_src), "-o", str(lib)])
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_convert.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode != 0, f"the pins did not notice: {name}\n{r.stdout[-2000:]}"


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_the_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    mutant_src = tmp_path / "mutant.cpp"
    mutant_src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-pthread", str(mutant_src), "-o", str(lib)])
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    # 1: a pin failed; a negative code: the broken oracle ran out of its arrays and the child died,
    # which is being noticed as well
    assert r.returncode != 0, f"the pins did not notice: {name}\n{r.stdout[-2000:]}"


def test_unmodified_oracle_passes_the_same_run(tmp_path):
    lib = tmp_path / "liborig.so"
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-pthread", SRC, "-o", str(lib)])
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_convert.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:]
