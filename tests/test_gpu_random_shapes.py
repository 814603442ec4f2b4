"""GPU parity of the whole layer on seeded random shapes.

The shapes are drawn once from a fixed seed: token counts from 1 to a few thousand, widths that are
multiples of 8 but of none of the tile sizes, expert counts that are not powers of two, top-k up to 8, and
logits with a per-expert bias of random strength so that some experts collect thousands of rows (several
reduction chunks, several row tiles) while others stay empty.  Every case runs both call sequences (rows
gathered inside the products, and the separate permute / combine-backward launches) and is compared with
the fp64 oracle element by element: integers bit for bit, floating point to the tolerance of the dtype.
"""
import sys

import numpy as np
import pytest

from oracle import moe_oracle as O
from tests.util import assert_close, q, to_dev, to_np, torch_dtype

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True, file=sys.stderr)


def _draw_cases(n, seed):
    r = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        E = int(r.integers(1, 41))
        k = int(r.integers(1, min(E, 8) + 1))
        T = int(r.choice([1, 2, 7, 63, 300, 1100, 2900])) if i < 7 else int(r.integers(1, 3000))
        d = 8 * int(r.integers(1, 66))
        f = 8 * int(r.integers(1, 50))
        skew = float(r.choice([0.0, 1.0, 3.0]))
        dt = "f32" if i % 6 == 5 else "bf16"
        if dt == "f32":                     # one thread per output: keep the product small
            T, d, f = min(T, 400), min(d, 128), min(f, 96)
        cases.append((i, T, k, d, f, E, dt, skew))
    return cases


CASES = _draw_cases(18, seed=20250802)


def _problem(i, T, k, d, f, E, dt, skew):
    r = np.random.default_rng(1000 + i)
    z = r.standard_normal((T, E)) - skew * np.log(1.0 + r.permutation(E))[None, :]
    X = q(r.standard_normal((T, d)), dt)
    dY = q(r.standard_normal((T, d)), dt)
    Wg = q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wu = q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wd = q(r.standard_normal((E, d, f)) * 0.05, dt)
    return dict(X=X, dY=dY, Wg=Wg, Wu=Wu, Wd=Wd, logits=z.astype(np.float32))


@pytest.mark.parametrize("case", CASES, ids=lambda c: "T%d_k%d_d%d_f%d_E%d_%s_s%g" % c[1:])
def test_layer_random_shape(case):
    import torch
    from paper_2508_02317_amd.layer import MoELayer
    i, T, k, d, f, E, dt, skew = case
    say("random shape %d: T=%d k=%d d=%d f=%d E=%d %s skew=%g" % case)
    inp = _problem(*case)
    fwd = O.moe_layer_fwd(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], k)
    bwd = O.moe_layer_bwd(fwd, inp["dY"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"])
    say("  rows per expert: max %d, empty %d of %d" % (fwd["counts"].max(), int((fwd["counts"] == 0).sum()), E))
    for gather in (True, False):
        layer = MoELayer(T, d, E, k, f, torch_dtype(dt), to_dev(inp["Wg"], dt), to_dev(inp["Wu"], dt),
                         to_dev(inp["Wd"], dt), gather=gather)
        x, dy, logits = to_dev(inp["X"], dt), to_dev(inp["dY"], dt), to_dev(inp["logits"])
        layer.forward(x, logits=logits)
        layer.backward(dy, logits=logits)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(layer.topk_idx), fwd["topk_idx"])
        assert np.array_equal(to_np(layer.counts), fwd["counts"])
        assert np.array_equal(to_np(layer.offsets), fwd["offsets"])
        assert np.array_equal(to_np(layer.row_of_pair), fwd["row_of_pair"])
        assert np.array_equal(to_np(layer.pair_of_row), fwd["pair_of_row"])
        tag = " (gather)" if gather else ""
        assert_close(to_np(layer.topk_w), fwd["topk_w"], "f32", "topk_w" + tag)
        assert_close(to_np(layer.y), fwd["Y"], dt, "Y" + tag)
        assert_close(to_np(layer.dx), bwd["dX"], dt, "dX" + tag)
        assert_close(to_np(layer.dw), bwd["dw"], dt, "dw" + tag)
        assert_close(to_np(layer.dlogits), bwd["dlogits"], dt, "dlogits" + tag)
        for e in range(E):
            if fwd["counts"][e] == 0:
                assert not to_np(layer.dw_gate)[e].any() and not to_np(layer.dw_down)[e].any()
        assert_close(to_np(layer.dw_gate), bwd["dWg"], dt, "dWg" + tag)
        assert_close(to_np(layer.dw_up), bwd["dWu"], dt, "dWu" + tag)
        assert_close(to_np(layer.dw_down), bwd["dWd"], dt, "dWd" + tag)
