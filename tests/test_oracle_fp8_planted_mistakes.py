"""Do the pins of the 8-bit oracle catch mistakes?  One plausible mistake at a time is planted in a copy of
oracle/moe_fp8.py; every one must make at least one pin of tests/test_oracle_fp8.py fail.  CPU only."""
import inspect
import os
import types

import pytest

import tests.test_oracle_fp8 as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "moe_fp8.py")).read()

MISTAKES = [
    ("exponent bias 8 (the E5M2-style off-by-one)", "E4M3_BIAS = 7", "E4M3_BIAS = 8"),
    ("subnormals scaled as normals", "sub = m / 8.0 * 2.0 ** (1 - E4M3_BIAS)", "sub = m / 8.0 * 2.0 ** (0 - E4M3_BIAS)"),
    ("ties away from zero", "pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))", "pick_hi = d_hi <= d_lo"),
    ("ties to the odd code", "(hi % 2 == 0)", "(hi % 2 == 1)"),
    ("truncation instead of rounding", "pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))", "pick_hi = d_hi == 0"),
    ("sign of negative zero dropped", "np.where(np.signbit(x), 0x80, 0)", "np.where(x < 0, 0x80, 0)"),
    ("shared exponent from the largest binade of 2^7", "E4M3_EMAX = 8 ", "E4M3_EMAX = 7 "),
    ("shared exponent rounds up", "shared = np.clip(exp - 1 - E4M3_EMAX, -127, 127)", "shared = np.clip(exp - E4M3_EMAX, -127, 127)"),
    ("scale applied as a multiplication", "scaled = B / np.exp2(s.astype(np.float64) - 127.0)[..., None]",
     "scaled = B * np.exp2(s.astype(np.float64) - 127.0)[..., None]"),
    ("blocks of 16", "BLOCK = 32 ", "BLOCK = 16 "),
    ("dequantisation ignores the scale bias", "np.exp2(np.asarray(scales, dtype=np.float64) - 127.0)", "np.exp2(np.asarray(scales, dtype=np.float64) - 128.0)"),
    ("gate and up swapped", "A[a:b] = silu(G) * U", "A[a:b] = silu(U) * G"),
    ("down projection of the neighbouring expert", "Yp[a:b] = A[a:b] @ mx_dequantise(Wdq[e], Wds[e]).T",
     "Yp[a:b] = A[a:b] @ mx_dequantise(Wdq[(e + 1) % Wdq.shape[0]], Wds[(e + 1) % Wdq.shape[0]]).T"),
    ("activation quantised from float64", "return mx_quantise(np.asarray(A, dtype=np.float64).astype(np.float32).astype(np.float64))",
     "return mx_quantise(np.asarray(A, dtype=np.float64))"),
]


def _load(source):
    mod = types.ModuleType("moe_fp8_copy")
    mod.__file__ = os.path.join(ROOT, "oracle", "moe_fp8.py")
    exec(compile(source, mod.__file__, "exec"), mod.__dict__)
    return mod


def _failing_pins(module):
    saved = pins.F
    pins.F = module
    failed = []
    try:
        for name, fn in sorted(vars(pins).items()):
            if name.startswith("test_") and callable(fn) and not inspect.signature(fn).parameters:
                try:
                    fn()
                except pytest.skip.Exception:
                    pass
                except Exception:
                    failed.append(name)
    finally:
        pins.F = saved
    return failed


def test_unmodified_oracle_passes_every_pin():
    assert _failing_pins(_load(SOURCE)) == []


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(name, old, new):
    assert SOURCE.count(old) == 1, "the oracle no longer contains this text once: %r" % old
    failed = _failing_pins(_load(SOURCE.replace(old, new)))
    assert failed, "no pin noticed: " + name
