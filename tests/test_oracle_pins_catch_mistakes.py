"""The pins must be able to fail: each plausible mistake below is planted in a copy of the
oracle's C source (never in the GPU code), the copy is compiled, and the pin tests are run
against it in a subprocess.  Every mutant has to be caught by at least one pin."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sdl_ref.c")
PIN_FILES = ["tests/test_oracle_codec.py", "tests/test_oracle_step.py"]

MUTANTS = [
    ("ties go to the odd code", "(c & 1u) == 0u", "(c & 1u) == 1u"),
    ("element scaled by the wrong power of two", "ldexp(fabs((double)x), 127 - (int)sb)", "ldexp(fabs((double)x), 126 - (int)sb)"),
    ("E3M0 exponent bias off by one", "ldexp(1.0, (int)E - 3)", "ldexp(1.0, (int)E - 2)"),
    ("nibbles packed high-first", "(c & 15u) << ((k & 1u) * 4u)", "(c & 15u) << (((k & 1u) ^ 1u) * 4u)"),
    ("scale byte off by one", "    return e_a - emax;", "    return e_a - emax + 1u;"),
    ("look-ahead uses the old momentum", "float look = dbar + mu_mom_new;", "float look = dbar + mu_mom;"),
    ("outer step goes uphill", "g[i] = g[i] - step;", "g[i] = g[i] + step;"),
    ("sum instead of mean", "float dbar = acc / (float)M;", "float dbar = acc;"),
    ("merge weights the global part with alpha", "float global_part = one_minus_alpha * g_new[i];", "float global_part = alpha * g_new[i];"),
    ("bf16 rounding ignores the tie rule", "u += 0x7fffu + lsb;", "u += 0x7fffu;"),
    ("local minus global", "d[i] = g[b0 + i] - bf16_to_f32(w[b0 + i]);", "d[i] = bf16_to_f32(w[b0 + i]) - g[b0 + i];"),
    ("E4M3 may emit the NaN code", "nearest_code(y, 0x7eu, e4m3_magnitude)", "nearest_code(y, 0x7fu, e4m3_magnitude)"),
    ("E4M3 subnormal quantum wrong", "ldexp((double)m, -9)", "ldexp((double)m, -8)"),
    ("sign bit dropped", "unsigned s = f32_bits(x) >> 31;", "unsigned s = 0; (void)x;"),
    ("momentum not decayed", "float mu_mom = mu * mom[i];", "float mu_mom = mom[i];"),
    ("round-to-nearest variant uses the default scale", "fmt == REF_FMT_E3M0_RN ? 3u : 4u", "fmt == REF_FMT_E3M0_RN ? 4u : 4u"),
    ("round-to-nearest variant two binades up", "fmt == REF_FMT_E3M0_RN ? 3u : 4u", "fmt == REF_FMT_E3M0_RN ? 2u : 4u"),
    ("block maximum skips the last element", "for (uint64_t i = 0; i < len; ++i) {\n        uint32_t m = f32_bits(d[i]) & 0x7fffffffu;", "for (uint64_t i = 0; i + 1 < len; ++i) {\n        uint32_t m = f32_bits(d[i]) & 0x7fffffffu;"),
]


def test_the_unmodified_source_contains_every_mutation_site():
    text = open(SRC).read()
    for name, old, _new in MUTANTS:
        assert text.count(old) == 1, (name, text.count(old))



@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch(name, old, new, tmp_path):
    text = open(SRC).read().replace(old, new)
    src = tmp_path / "sdl_ref_mutant.c"
    lib = tmp_path / "libsdl_ref_mutant.so"
    src.write_text(text)
    oracle.compile_source(str(src), str(lib))
    env = dict(os.environ, SDL_ORACLE_LIB=str(lib))
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 1, f"mutant '{name}' survived the pins:\n{run.stdout[-2000:]}"
