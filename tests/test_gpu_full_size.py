"""GPU parity at the full configured sizes, in the launch configuration bench.py times.

The whole-layer fp64 oracle runs once per configuration (a few seconds at a3b_8k and a3b_ep_skew,
a quarter of a minute at a3b_long on the GPU machine's host cores) and EVERY element of every output is
compared with it, for both call sequences: routing indices, counts, offsets and the permutation maps
bit for bit; Y, dX, d topk_w, d logits and the three weight gradients of all E experts within the
tolerance of the element type.
"""
import sys
import time

import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2508_02317_amd.inputs import CONFIGS, make_inputs, quantise, select_local_share
from tests.util import TOL, rel_err, to_dev, to_np, torch_dtype

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True, file=sys.stderr)


def _run(cfg, inp, X, routing=None, gather=True):
    """gather=True is the call sequence bench.py times by default (rows read by token inside the products);
    gather=False the one with the separate permute / combine-backward launches (bench.py --no-gather)."""
    import torch
    from paper_2508_02317_amd.layer import MoELayer
    dt = cfg.dtype
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, torch_dtype(dt), to_dev(inp["Wg"], dt), to_dev(inp["Wu"], dt),
                     to_dev(inp["Wd"], dt), renorm=cfg.renorm, prerouted=routing is not None, gather=gather)
    x, dy = to_dev(X, dt), to_dev(inp["dY"], dt)
    if routing is None:
        logits = to_dev(inp["logits"])
        layer.forward(x, logits=logits)
        layer.backward(dy, logits=logits)
    else:
        layer.forward(x, topk_idx=to_dev(routing[0]), topk_w=to_dev(routing[1]))
        layer.backward(dy)
    torch.cuda.synchronize()
    return layer


_ORACLE = {}


def _oracle(name):
    """Inputs and the whole-layer oracle result of a configuration, computed once per test session."""
    if name in _ORACLE:
        return _ORACLE[name]
    cfg = CONFIGS[name]
    inp = make_inputs(cfg)
    t0 = time.perf_counter()
    if cfg.kind == "ep_share":
        ridx, rw, rcounts, _ = O.route_topk(inp["logits"], cfg.k_global, cfg.renorm)
        assert rcounts.max() > 5 * rcounts.mean()                      # a few experts get > 5x the mean
        tok, lidx, lw = select_local_share(ridx, rw, cfg.E, cfg.T)
        assert len(tok) == cfg.T
        lw32 = lw.astype(np.float32)
        X = inp["X"][tok]
        fwd = O.moe_layer_fwd(X, None, inp["Wg"], inp["Wu"], inp["Wd"], 1, routing=(lidx, lw32))
        bwd = O.moe_layer_bwd(fwd, inp["dY"], None, inp["Wg"], inp["Wu"], inp["Wd"])
        extra = dict(X=X, routing=(lidx, lw32), global_idx=ridx, global_counts=rcounts)
    else:
        fwd = O.moe_layer_fwd(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.k, cfg.renorm)
        bwd = O.moe_layer_bwd(fwd, inp["dY"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.renorm)
        extra = dict(X=inp["X"], routing=None)
    say("  oracle %s: whole layer fwd+bwd in %.1f s" % (name, time.perf_counter() - t0))
    # keep only what is compared: the expert-ordered fp64 intermediates are several GB at a3b_long
    keep_f = {k: fwd[k] for k in ("topk_idx", "topk_w", "counts", "offsets", "row_of_pair", "pair_of_row", "Y")}
    keep_b = {k: bwd[k] for k in ("dw", "dWg", "dWu", "dWd", "dX", "dlogits")}
    _ORACLE.clear()                                    # one configuration's reference at a time
    _ORACLE[name] = (cfg, inp, keep_f, keep_b, extra)
    return _ORACLE[name]


def _compare_everything(cfg, layer, fwd, bwd, with_routing):
    tol = TOL[cfg.dtype]
    if with_routing:
        assert np.array_equal(to_np(layer.topk_idx), fwd["topk_idx"])
        assert rel_err(to_np(layer.topk_w), fwd["topk_w"]) <= 1e-5
    assert np.array_equal(to_np(layer.counts), fwd["counts"])
    assert np.array_equal(to_np(layer.offsets), fwd["offsets"])
    assert np.array_equal(to_np(layer.row_of_pair), fwd["row_of_pair"])
    assert np.array_equal(to_np(layer.pair_of_row), fwd["pair_of_row"])
    errs = {"Y": rel_err(to_np(layer.y), fwd["Y"]), "dX": rel_err(to_np(layer.dx), bwd["dX"]),
            "dw": rel_err(to_np(layer.dw), bwd["dw"])}
    if with_routing:
        errs["dlogits"] = rel_err(to_np(layer.dlogits), bwd["dlogits"])
    # every expert's weight gradients, normalised per tensor (the stated bar) and, stricter, per expert for the
    # experts that have rows; experts without rows must hold exact zeros
    for key, got, ref in (("dWg", layer.dw_gate, bwd["dWg"]), ("dWu", layer.dw_up, bwd["dWu"]), ("dWd", layer.dw_down, bwd["dWd"])):
        got = to_np(got)
        errs[key] = rel_err(got, ref)
        worst = 0.0
        for e in range(cfg.E):
            if fwd["counts"][e] == 0:
                assert not got[e].any(), "%s[%d]: expert without rows must have a zero gradient" % (key, e)
            else:
                worst = max(worst, rel_err(got[e], ref[e]))
        errs[key + " worst expert"] = worst
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()))
    for key, v in errs.items():
        assert v <= tol, "%s: %.3e > %.1e" % (key, v, tol)


@pytest.mark.parametrize("name,gather", [("a3b_8k", True), ("a3b_8k", False), ("a3b_long", True), ("a3b_long", False)])
def test_full_size_layer(name, gather):
    cfg, inp, fwd, bwd, extra = _oracle(name)
    say("full size %s: T=%d P=%d gather=%s" % (name, cfg.T, cfg.P, gather))
    layer = _run(cfg, inp, extra["X"], gather=gather)
    if gather:
        assert layer.xp is None and layer.dyp is None              # no copies in expert order
    else:
        xp = to_np(layer.xp)                                       # bit copies, every row
        assert np.array_equal(xp, inp["X"].astype(np.float32)[fwd["pair_of_row"] // cfg.k])
    _compare_everything(cfg, layer, fwd, bwd, with_routing=True)


@pytest.mark.parametrize("gather", [True, False])
def test_full_size_ep_share_skewed(gather):
    cfg, inp, fwd, bwd, extra = _oracle("a3b_ep_skew")
    say("full size a3b_ep_skew: rows=%d local experts=%d gather=%s" % (cfg.T, cfg.E, gather))
    from paper_2508_02317_amd import libmoe as L
    gidx, gw, gcounts, _ = L.moe_route_topk(to_dev(inp["logits"]), cfg.k_global, cfg.renorm)
    assert np.array_equal(to_np(gidx), extra["global_idx"]) and np.array_equal(to_np(gcounts), extra["global_counts"])
    layer = _run(cfg, inp, extra["X"], routing=extra["routing"], gather=gather)
    say("  local counts: %s" % fwd["counts"].tolist())
    _compare_everything(cfg, layer, fwd, bwd, with_routing=False)


def test_full_size_block_from_hidden_states():
    """a3b_8k with the router linear in front: logits against the fp64 product, routing on the GPU's own
    logits, and every element of Y, dX (expert + router path), d logits, dW_router and the expert weight gradients."""
    import torch
    from paper_2508_02317_amd.layer import MoELayer
    cfg = CONFIGS["a3b_8k"]
    say("full size a3b_8k from hidden states: T=%d" % cfg.T)
    inp = make_inputs(cfg)
    dt = cfg.dtype
    Wr = np.ascontiguousarray(inp["Wr"].T)                           # [E, d]
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, torch_dtype(dt), to_dev(inp["Wg"], dt), to_dev(inp["Wu"], dt),
                     to_dev(inp["Wd"], dt), renorm=cfg.renorm, w_router=to_dev(Wr, dt), gather=True)
    layer.forward(to_dev(inp["X"], dt))
    layer.backward(to_dev(inp["dY"], dt))
    torch.cuda.synchronize()
    z = to_np(layer.logits)
    assert rel_err(z, O.router_logits(inp["X"], Wr)) <= 1e-5
    fwd = O.moe_layer_fwd(inp["X"], z, inp["Wg"], inp["Wu"], inp["Wd"], cfg.k, cfg.renorm)   # the oracle routes on the same fp32 logits
    bwd = O.moe_layer_bwd(fwd, inp["dY"], z, inp["Wg"], inp["Wu"], inp["Wd"], cfg.renorm)
    assert np.array_equal(to_np(layer.topk_idx), fwd["topk_idx"]) and np.array_equal(to_np(layer.offsets), fwd["offsets"])
    dz = to_np(layer.dlogits).astype(np.float64)
    dz_seen = quantise(dz.astype(np.float32), dt).astype(np.float64)  # the backward products use dz rounded to bf16
    dXr, rdWr = O.router_bwd(dz_seen, inp["X"], Wr)
    tol = TOL[dt]
    errs = {"Y": rel_err(to_np(layer.y), fwd["Y"]), "dX": rel_err(to_np(layer.dx), bwd["dX"] + dXr),
            "dlogits": rel_err(dz, bwd["dlogits"]), "dW_router": rel_err(to_np(layer.dw_router), rdWr),
            "dWg": rel_err(to_np(layer.dw_gate), bwd["dWg"]), "dWu": rel_err(to_np(layer.dw_up), bwd["dWu"]),
            "dWd": rel_err(to_np(layer.dw_down), bwd["dWd"])}
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()))
    for key, v in errs.items():
        assert v <= tol, "%s: %.3e > %.1e" % (key, v, tol)
