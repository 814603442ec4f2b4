"""Do the oracle's pins catch mistakes?  (CPU only; test infrastructure.)

Each case plants one plausible mistake in a copy of the oracle's source -- a wrong sign, a dropped factor or
term, a swapped operand, a wrong index, an unstable order -- loads the copy as a module and runs the pins of
`tests/test_oracle_pins.py` against it.  Every planted mistake must make at least one pin fail, and the
unmodified source must pass them all, so a pin that only re-states the oracle would show up here as a
survivor.
"""
import inspect
import os
import types

import pytest

import tests.test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "moe_oracle.py")).read()

# (name, text in the oracle, what it is replaced with)
MISTAKES = [
    ("silu derivative: sign of the second term",
     "return s * (1.0 + g * (1.0 - s))", "return s * (1.0 - g * (1.0 - s))"),
    ("forward: silu on the up projection instead of the gate",
     "A[a:b] = silu(G[a:b]) * U[a:b]", "A[a:b] = silu(U[a:b]) * G[a:b]"),
    ("forward: down projection of the neighbouring expert",
     "Yp[a:b] = A[a:b] @ Wd[e].T", "Yp[a:b] = A[a:b] @ Wd[(e + 1) % E].T"),
    ("backward: factor U dropped from dG",
     "dG = dA * U[a:b] * silu_grad(G[a:b])", "dG = dA * silu_grad(G[a:b])"),
    ("backward: dU uses the derivative of silu",
     "dU = dA * silu(G[a:b])", "dU = dA * silu_grad(G[a:b])"),
    ("backward: up-projection term dropped from dXp",
     "dXp[a:b] = dG @ Wg[e] + dU @ Wu[e]", "dXp[a:b] = dG @ Wg[e]"),
    ("backward: dW_up takes the gate's gradient",
     "dWu[e] = dU.T @ Xp[a:b]", "dWu[e] = dG.T @ Xp[a:b]"),
    ("backward: dW_down from the pre-activations instead of the activations",
     "dWd[e] = dYp[a:b].T @ A[a:b]", "dWd[e] = dYp[a:b].T @ G[a:b]"),
    ("routing: ascending instead of descending logits",
     'order = np.argsort(-z, axis=1, kind="stable")', 'order = np.argsort(z, axis=1, kind="stable")'),
    ("routing: ties to the higher index",
     'order = np.argsort(-z, axis=1, kind="stable")',
     'order = (E - 1 - np.argsort(-z[:, ::-1], axis=1, kind="stable"))'),
    ("routing: renormalisation skipped",
     "    if renorm:\n        w = w / w.sum(axis=1, keepdims=True)\n    counts", "    counts"),
    ("routing: offsets are the inclusive scan",
     "    offsets[1:] = np.cumsum(counts)\n    return idx.astype(np.int32), w, counts, offsets",
     "    offsets[:-1] = np.cumsum(counts)\n    return idx.astype(np.int32), w, counts, offsets"),
    ("permutation: order inside an expert reversed",
     'pair_of_row = np.argsort(flat, kind="stable").astype(np.int32)',
     'pair_of_row = (P - 1 - np.argsort(flat[::-1], kind="stable")[::-1]).astype(np.int32)'),
    ("combine: weights of the slots swapped",
     "Y += w[:, j:j + 1] * Yp[rows[:, j]]", "Y += w[:, k - 1 - j:k - j] * Yp[rows[:, j]]"),
    ("combine backward: dw from the weighted row",
     'dw[:, j] = np.einsum("td,td->t", dY, Yp[rows[:, j]])', 'dw[:, j] = np.einsum("td,td->t", dY, w[:, j:j + 1] * Yp[rows[:, j]])'),
    ("combine backward: weight dropped from dYp",
     "dYp[rows[:, j]] = w[:, j:j + 1] * dY", "dYp[rows[:, j]] = dY"),
    ("routing backward: sign of the common term",
     "    if renorm:\n        np.put_along_axis(dz, idx, w * (dw - s), axis=1)",
     "    if renorm:\n        np.put_along_axis(dz, idx, w * (dw + s), axis=1)"),
    ("routing backward (no renormalisation): unselected experts get no gradient",
     "        dz = -p * s\n", "        dz = np.zeros((T, E))\n"),
    ("router linear: logits against the wrong axis of the weight",
     'return np.asarray(X, dtype=np.float64) @ np.asarray(Wr, dtype=np.float64).T',
     'return np.asarray(X, dtype=np.float64) @ np.asarray(Wr, dtype=np.float64)[:, ::-1].T'),
    ("router backward: hidden-state term through the transposed weight of the wrong expert order",
     "dXr = dz @ np.asarray(Wr, dtype=np.float64)", "dXr = dz[:, ::-1] @ np.asarray(Wr, dtype=np.float64)"),
    ("router backward: weight gradient from the unweighted rows",
     "dWr = dz.T @ np.asarray(X, dtype=np.float64)", "dWr = np.sign(dz).T @ np.asarray(X, dtype=np.float64)"),
    ("whole block: router term dropped from dX",
     'out["dX"] = out["dX"] + dXr', 'out["dX"] = out["dX"]'),
    ("sampled token: combine weight dropped from the backward",
     "da = wd.T @ (w_t[j] * dy)", "da = wd.T @ dy"),
]


def _load(source):
    mod = types.ModuleType("moe_oracle_copy")
    mod.__file__ = os.path.join(ROOT, "oracle", "moe_oracle.py")
    exec(compile(source, mod.__file__, "exec"), mod.__dict__)
    return mod


def _pin_calls():
    """Every pin of tests/test_oracle_pins.py as a zero-argument call (parametrised ones once per parameter set)."""
    calls = []
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            if not inspect.signature(fn).parameters:
                calls.append((name, fn))
            continue
        assert len(marks) == 1, name
        argnames = [a.strip() for a in marks[0].args[0].split(",")]
        for values in marks[0].args[1]:
            values = values if isinstance(values, (tuple, list)) else (values,)
            calls.append(("%s%r" % (name, tuple(values)), lambda fn=fn, kw=dict(zip(argnames, values)): fn(**kw)))
    return calls


def _failing_pins(module):
    saved = pins.O
    pins.O = module
    failed = []
    try:
        for name, call in _pin_calls():
            try:
                call()
            except Exception:          # an assertion, or arithmetic that no longer fits together
                failed.append(name)
    finally:
        pins.O = saved
    return failed


def test_unmodified_oracle_passes_every_pin():
    assert len(_pin_calls()) >= 15
    assert _failing_pins(_load(SOURCE)) == []


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(name, old, new):
    assert SOURCE.count(old) == 1, "the oracle no longer contains this line once: %r" % old
    failed = _failing_pins(_load(SOURCE.replace(old, new)))
    assert failed, "no pin noticed: " + name
