"""The pins must bite: plausible mistakes planted in a COPY of the oracle (on the CPU, never in
the GPU path) have to fail at least one of the pinned checks.  Each mutant is the oracle source
with one line changed, compiled separately."""
import ctypes as C
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "nsml_oracle.c")

MUTANTS = {
    "tie goes to the higher index": ("if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;",
                                     "if (a->idx != b->idx) return a->idx > b->idx ? -1 : 1;"),
    "sign not cleared in the key": ("return f32_bits(x) & 0x7FFFFFFFu;", "return f32_bits(x);"),
    "smallest instead of largest": ("if (a->key != b->key) return a->key > b->key ? -1 : 1;",
                                    "if (a->key != b->key) return a->key < b->key ? -1 : 1;"),
    "k rounded down": ("double kd = ceil(ratio * (double)n);", "double kd = floor(ratio * (double)n);"),
    "residual keeps the sent value": ("volatile float res = v - deq;", "volatile float res = v;"),
    "residual sign flipped": ("volatile float res = v - deq;", "volatile float res = deq - v;"),
    "scale uses qmax + 1": ("volatile float s = m / (float)qmax;", "volatile float s = m / (float)(qmax + 1);"),
    "truncation instead of rounding": ("float rt = rintf(t);", "float rt = truncf(t);"),
    "nibbles swapped": ("*p = (j & 1) ? (uint8_t)(*p | (nib << 4)) : (uint8_t)(*p | nib);",
                        "*p = (j & 1) ? (uint8_t)(*p | nib) : (uint8_t)(*p | (nib << 4));"),
    "error feedback dropped": ("volatile float a = g[i] + r[i];", "volatile float a = g[i];"),
    "chunks span the whole payload": ("scales[j / chunk]", "scales[0]"),
    "fp16 rounds half up": ("if (rem > half || (rem == half && (kept & 1u))) h += 1u;",
                            "if (rem >= half) h += 1u;"),
}


def _build(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, (name, text.count(old))
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", *oracle.GCC_FLAGS, "-o", str(lib), str(src), "-lm"])
    return str(lib)


def _run_pins(lib):
    # run the pinned oracle tests in a child process whose oracle library is the mutant
    code = (
        "import sys, ctypes, pytest; sys.path.insert(0, %r); import oracle; "
        "oracle._LIB = %r; oracle.build = lambda force=False: oracle._LIB; "
        "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', "
        "%r, %r, %r, %r]))"
    ) % (os.path.dirname(HERE), lib,
         os.path.join(HERE, "test_oracle_select.py"), os.path.join(HERE, "test_oracle_quant.py"),
         os.path.join(HERE, "test_oracle_invariants.py"), os.path.join(HERE, "test_oracle_next.py"))
    return subprocess.call([sys.executable, "-c", code], stdout=subprocess.DEVNULL,
                           stderr=subprocess.DEVNULL, cwd=os.path.dirname(HERE))


def test_control_unmodified_copy_passes(tmp_path):
    """The same harness with an unmodified copy must pass, or the mutant results mean nothing."""
    text = open(SRC).read()
    src = tmp_path / "copy.c"
    src.write_text(text)
    lib = tmp_path / "libcopy.so"
    subprocess.check_call(["gcc", *oracle.GCC_FLAGS, "-o", str(lib), str(src), "-lm"])
    assert _run_pins(str(lib)) == 0


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(name, tmp_path):
    lib = _build(tmp_path, name, *MUTANTS[name])
    assert _run_pins(lib) != 0, f"no pin notices the mistake: {name}"
