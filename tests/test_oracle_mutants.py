"""Are the oracle's pins sharp?  Each case below plants one plausible mistake in a COPY of the
oracle's C source (a dropped term, a wrong sign, a swapped operand, an off-by-one), builds it
with the oracle's own compiler flags, points the oracle's Python wrapper at the mutant and
re-runs the pins: at least one pin must fail for every mutant, and the untouched copy must
pass them all.  CPU only; the GPU library is not involved."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins
from oracle import GRAD_BF16, GRAD_FP16

SRC = os.path.join(os.path.dirname(oracle.__file__), "adam_oracle.c")

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("epsilon inside the square root", "sqrt(vhat) + eps", "sqrt(vhat + eps)"),
    ("decoupled decay dropped", "if (adamw) pn -= lr * wd * pi;", ""),
    ("decay with the wrong sign", "if (adamw) pn -= lr * wd * pi;", "if (adamw) pn += lr * wd * pi;"),
    ("update with the wrong sign", "pn -= lr * mhat / (sqrt(vhat) + eps);", "pn += lr * mhat / (sqrt(vhat) + eps);"),
    ("bias corrections swapped", "double mhat = mn / bc1;\n        double vhat = vn / bc2;",
     "double mhat = mn / bc2;\n        double vhat = vn / bc1;"),
    ("first moment without (1 - beta1)", "b1 * mi + (1.0 - b1) * gi;", "b1 * mi + gi;"),
    ("second moment from g instead of g^2", "(1.0 - b2) * gi * gi;", "(1.0 - b2) * gi;"),
    ("betas swapped in the moments", "double mn = b1 * mi + (1.0 - b1) * gi;", "double mn = b2 * mi + (1.0 - b2) * gi;"),
    ("bias correction one step late", "bc1 = 1.0 - pow_int(b1, t);", "bc1 = 1.0 - pow_int(b1, t + 1);"),
    ("second bias correction missing", "bc2 = 1.0 - pow_int(b2, t);", "bc2 = 1.0;"),
    ("gradient multiplier ignored", "orc_decode16(g[i], dtype) * s;", "orc_decode16(g[i], dtype);"),
    ("L2 decay folded in with the moment", "if (!adamw) gi += wd * pi;", "if (!adamw) gi += wd * mi;"),
    ("L2 decay applied in both modes", "if (!adamw) gi += wd * pi;", "gi += wd * pi;"),
    ("working copy truncated, not rounded", "if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))",
     "if (0)"),
    ("working copy rounds ties away from even", "(lower == 0x8000u && (upper & 1u))", "(lower == 0x8000u)"),
    ("working copy cast from the old parameter", "p[i] = (float)pn;\n        q[i]", "q[i]"),
    ("exponent bias off by one", "int bias = (1 << (ebits - 1)) - 1;", "int bias = (1 << (ebits - 1));"),
    ("subnormals flushed", "mag = ldexp((double)f, 1 - bias - fbits);", "mag = 0.0;"),
    ("NaN taken for infinity only", "mag = (f == 0) ? INFINITY : NAN;", "mag = (f == 0) ? INFINITY : 1.0;"),
    ("sum of values, not of squares", "acc += y * y;", "acc += y;"),
    ("loss scale not removed in the norm", "double y = x * s;", "double y = x;"),
    ("non-finite elements added to the sum", "if (!isfinite(x)) {\n            ++bad;\n        } else {",
     "if (!isfinite(x)) ++bad;\n        {"),
    ("clip coefficient not capped at one", "return c < 1.0 ? c : 1.0;", "return c;"),
    ("clip coefficient without the guard term", "double c = max_norm / (norm + 1e-6);", "double c = max_norm / norm;"),
    ("fp16 working copy truncated", "double qd = nearbyint(a / step);", "double qd = floor(a / step);"),
    ("array cast with the formats swapped", "q[i] = lp_fp16 ? orc_f32_to_fp16(p[i]) : orc_f32_to_bf16(p[i]);\n}",
     "q[i] = lp_fp16 ? orc_f32_to_bf16(p[i]) : orc_f32_to_fp16(p[i]);\n}"),
    ("array cast stops one element short", "for (uint64_t i = 0; i < n; ++i) q[i] = lp_fp16",
     "for (uint64_t i = 0; i + 1 < n; ++i) q[i] = lp_fp16"),
]


def run_all_pins():
    """Every pin of test_oracle_pins, with the parameters it is run with there; the cheap
    closed forms first, the exhaustive bit-pattern sweeps last."""
    pins.test_golden_dyadic_example()
    pins.test_step1_closed_form()
    pins.test_constant_gradient_trajectory()
    pins.test_zero_gradient_is_pure_decay()
    pins.test_lr_zero_moves_moments_only()
    pins.test_clip_coefficient()
    pins.test_norm_exactly_representable()
    pins.test_nonfinite_elements_are_counted_and_left_out_of_the_sum()
    pins.test_power_of_two_loss_scale_is_exact()
    pins.test_overflow_iteration_is_skipped_and_scale_halved()
    pins.test_clipped_iteration_matches_manual_scaling()
    pins.test_speculate_then_rollback_equals_synchronous()
    for adamw in (1, 0):
        pins.test_against_torch_fp64_optimizer(adamw)
    for dt in (GRAD_BF16, GRAD_FP16):
        for n in BRUTE_SIZES:
            pins.test_bruteforce_exact_rational(dt, n)
    pins.test_norm_statistical()
    pins.test_decode_fp16_exhaustive_vs_numpy()
    pins.test_decode_bf16_exhaustive_vs_numpy()
    for dt in (GRAD_BF16, GRAD_FP16):
        pins.test_nonfinite_scan_exhaustive(dt)
    pins.test_bf16_rounding_exhaustive_vs_torch_and_definition()
    pins.test_fp16_rounding_exhaustive_vs_numpy()
    pins.test_cast_lp_is_the_pinned_rounding_element_by_element()


def _param_values(fn, name):
    for mark in getattr(fn, "pytestmark", []):
        if mark.name == "parametrize" and mark.args[0] == name:
            return list(mark.args[1])
    raise AssertionError(f"{fn.__name__} is not parametrized over {name}")


BRUTE_SIZES = _param_values(pins.test_bruteforce_exact_rational, "n")


class _Mutant:
    """Swap the shared library behind the oracle's Python wrapper, and put it back."""

    def __init__(self, so_path):
        self.so_path = so_path

    def __enter__(self):
        self.saved = (oracle._LIB, oracle._lib)
        oracle._LIB, oracle._lib = self.so_path, None
        real_build = oracle.build
        self.real_build = real_build
        oracle.build = lambda force=False: self.so_path      # the mutant is already built
        oracle.lib()
        return self

    def __exit__(self, *exc):
        oracle.build = self.real_build
        oracle._LIB, oracle._lib = self.saved
        return False


def _compile(text, path):
    src = path + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
                    "-fno-fast-math", "-o", path, src, "-lm"], check=True)
    return path


def test_unmodified_copy_passes_every_pin(tmp_path):
    text = open(SRC).read()
    with _Mutant(_compile(text, str(tmp_path / "copy.so"))):
        run_all_pins()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not found exactly once: {old!r}"
    so = _compile(text.replace(old, new), str(tmp_path / "mutant.so"))
    with _Mutant(so):
        with pytest.raises(AssertionError):
            run_all_pins()
    # and the wrapper is back on the real oracle
    assert oracle._LIB.endswith("liboracle.so")
    assert isinstance(oracle.lib(), ctypes.CDLL)
