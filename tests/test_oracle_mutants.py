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
    # Algorithm 2 Step 2 (weight-magnitude pruning)
    "pruned count rounded up": ("double np = floor(0.5 * (1.0 - ratio) * (double)n);",
                                "double np = ceil(0.5 * (1.0 - ratio) * (double)n);"),
    "pruning rate without the 0.5": ("double np = floor(0.5 * (1.0 - ratio) * (double)n);",
                                     "double np = floor((1.0 - ratio) * (double)n);"),
    "pruning rate uses ratio, not 1 - ratio": ("double np = floor(0.5 * (1.0 - ratio) * (double)n);",
                                               "double np = floor(0.5 * ratio * (double)n);"),
    "kept set one too large": ("uint64_t m = n - orc_pruned_count(ratio, n);",
                               "uint64_t m = n - orc_pruned_count(ratio, n) + 1;"),
    "kept set one too small": ("uint64_t m = n - orc_pruned_count(ratio, n);",
                               "uint64_t m = n - orc_pruned_count(ratio, n) - 1;"),
    "largest weights pruned": ("for (uint64_t j = 0; j < m; ++j) eligible[order[j].idx] = 1;",
                               "for (uint64_t j = n - m; j < n; ++j) eligible[order[j].idx] = 1;"),
    "pruned parameters can still be selected": ("if (eligible[i]) { order[m].key = mag_key(r[i]);",
                                                "if (1) { order[m].key = mag_key(r[i]);"),
    # receiver side and the norm of Algorithm 2 Step 1
    "accumulate overwrites": ("volatile float sum = dense[i] + tmp[i];", "volatile float sum = tmp[i];"),
    "accumulate subtracts": ("volatile float sum = dense[i] + tmp[i];", "volatile float sum = dense[i] - tmp[i];"),
    "norm without the square root": ("    return sqrt(total);\n}", "    return total;\n}"),
    "per-bucket norm without the square root": ("if (per_bucket) per_bucket[b] = sqrt(s);",
                                                "if (per_bucket) per_bucket[b] = s;"),
    "norm summed in binary32": ("        double s = 0.0;\n        for (uint64_t i = off[b]; i < off[b + 1]; ++i) s += (double)g[i] * (double)g[i];",
                                "        float s = 0.0f;\n        for (uint64_t i = off[b]; i < off[b + 1]; ++i) s += g[i] * g[i];"),
    "norm of absolute values (L1)": ("s += (double)g[i] * (double)g[i];", "s += fabs((double)g[i]);"),
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
        "%r, %r, %r, %r, %r]))"
    ) % (os.path.dirname(HERE), lib,
         os.path.join(HERE, "test_oracle_select.py"), os.path.join(HERE, "test_oracle_quant.py"),
         os.path.join(HERE, "test_oracle_invariants.py"), os.path.join(HERE, "test_oracle_next.py"),
         os.path.join(HERE, "test_oracle_pruned.py"))
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


# ---------------------------------------------------------------- the controller (Python)

CTL_SRC = os.path.join(os.path.dirname(HERE), "oracle", "controller.py")

# Only what the paper fixes (Algorithm 1, Eq. (1)-(3), the constants printed in Sec. 4.1); the
# start-up exit, the windows and the gate thresholds are readings and have no pin to bite.
CTL_MUTANTS = {
    "trigger at 1.0 * BDP": ("bdp_frac: float = 0.9", "bdp_frac: float = 1.0"),
    "trigger on >= instead of >": ("if last_payload_bytes > p.bdp_frac * s.bdp:",
                                   "if last_payload_bytes >= p.bdp_frac * s.bdp:"),
    "alpha 0.75": ("alpha: float = 0.5 ", "alpha: float = 0.75"),
    "beta2 0.02": ("beta2: float = 0.01 ", "beta2: float = 0.02 "),
    "floor 0.001": ("floor: float = 0.005 ", "floor: float = 0.001 "),
    "cap 0.5": ("cap: float = 1.0 ", "cap: float = 0.5 "),
    "initial ratio 0.02": ("init: float = 0.01 ", "init: float = 0.02 "),
    "Eq. (1) inverted": ("s.ebb.append(last_payload_bytes / last_tx_seconds)",
                         "s.ebb.append(last_tx_seconds / last_payload_bytes)"),
    "Eq. (2) is a sum": ("s.bdp = s.btlbw * s.rtprop", "s.bdp = s.btlbw + s.rtprop"),
    "BtlBw is the minimum EBB": ("s.btlbw = max(ebb)", "s.btlbw = min(ebb)"),
    "RTprop is the maximum RTT": ("s.rtprop = min(rtt)", "s.rtprop = max(rtt)"),
    "decrease is additive": ("s.ratio = max(p.floor, s.ratio * p.alpha)", "s.ratio = max(p.floor, s.ratio - p.alpha)"),
    "increase is multiplicative": ("s.ratio = min(p.cap, s.ratio + p.beta2)", "s.ratio = min(p.cap, s.ratio * (1.0 + p.beta2))"),
    "branches of Eq. (3) swapped": ("if last_payload_bytes > p.bdp_frac * s.bdp:",
                                    "if not (last_payload_bytes > p.bdp_frac * s.bdp):"),
    "floor not applied": ("s.ratio = max(p.floor, s.ratio * p.alpha)", "s.ratio = s.ratio * p.alpha"),
    "cap not applied": ("s.ratio = min(p.cap, s.ratio + p.beta2)", "s.ratio = s.ratio + p.beta2"),
    "quantized ratio not doubled": ("ratio_out = min(p.cap, 2.0 * s.ratio)", "ratio_out = s.ratio"),
}


def _run_ctl_pins(tmp_path, text):
    """Run the controller pins in a child whose ``oracle.controller`` is the given source."""
    pkg = tmp_path / "oracle"
    pkg.mkdir()
    (pkg / "controller.py").write_text(text)
    # the package's marshalling module is reused as is; only controller.py differs
    (pkg / "__init__.py").write_text(open(os.path.join(os.path.dirname(HERE), "oracle", "__init__.py")).read())
    os.symlink(os.path.join(os.path.dirname(HERE), "oracle", "nsml_oracle.c"), pkg / "nsml_oracle.c")
    code = ("import sys, pytest; sys.path.insert(0, %r); sys.path.insert(1, %r); "
            "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', '--noconftest', %r]))"
            ) % (str(tmp_path), os.path.dirname(HERE), os.path.join(HERE, "test_oracle_controller.py"))
    return subprocess.call([sys.executable, "-c", code], stdout=subprocess.DEVNULL,
                           stderr=subprocess.DEVNULL, cwd=str(tmp_path))


def test_controller_control_unmodified_copy_passes(tmp_path):
    assert _run_ctl_pins(tmp_path, open(CTL_SRC).read()) == 0


@pytest.mark.parametrize("name", sorted(CTL_MUTANTS))
def test_controller_pins_catch_mutant(name, tmp_path):
    old, new = CTL_MUTANTS[name]
    text = open(CTL_SRC).read()
    assert text.count(old) == 1, (name, text.count(old))
    assert _run_ctl_pins(tmp_path, text.replace(old, new)) != 0, f"no pin notices the mistake: {name}"
