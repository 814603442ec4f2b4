"""GPU parity at the full configured sizes, in the launch configuration bench.py times.

The whole-layer oracle would take minutes at these sizes, so the integer outputs (routing,
counts, offsets, permutation maps) are compared in full and bit for bit, and the floating
point outputs on samples the oracle computes one by one straight from the definition:
rows of Y, dX, dw and dlogits for sampled tokens, and dW_gate / dW_up / dW_down of sampled
experts (each needs every row routed to that expert).
"""
import sys

import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2508_02317_amd.inputs import CONFIGS, make_inputs, select_local_share
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


def _check_sampled(cfg, inp, X, layer, idx, w, logits, tokens, experts):
    tol = TOL[cfg.dtype]
    y, dx, dwt, dz = to_np(layer.y), to_np(layer.dx), to_np(layer.dw), None
    if logits is not None:
        dz = to_np(layer.dlogits)
    refs = {"Y": [], "dX": [], "dw": [], "dlogits": []}
    gots = {"Y": [], "dX": [], "dw": [], "dlogits": []}
    for t in tokens:
        ry, rdx, rdw = O.token_fwd_bwd(X[t], idx[t], w[t], inp["dY"][t], inp["Wg"], inp["Wu"], inp["Wd"])
        refs["Y"].append(ry); gots["Y"].append(y[t])
        refs["dX"].append(rdx); gots["dX"].append(dx[t])
        refs["dw"].append(rdw); gots["dw"].append(dwt[t])
        if logits is not None:
            rdz = O.route_topk_bwd(rdw[None], w[t][None], idx[t][None], logits[t][None], cfg.E, cfg.renorm)[0]
            refs["dlogits"].append(rdz); gots["dlogits"].append(dz[t])
    errs = {}
    for key in refs:
        if refs[key]:
            errs[key] = rel_err(np.array(gots[key]), np.array(refs[key]))
    dwg, dwu, dwd = to_np(layer.dw_gate), to_np(layer.dw_up), to_np(layer.dw_down)
    for e in experts:
        rg, ru, rd = O.expert_weight_grads(e, X, inp["dY"], idx, w, inp["Wg"], inp["Wu"], inp["Wd"])
        if not rg.any():
            assert not dwg[e].any() and not dwu[e].any() and not dwd[e].any()
            continue
        errs["dWg[%d]" % e] = rel_err(dwg[e], rg)
        errs["dWu[%d]" % e] = rel_err(dwu[e], ru)
        errs["dWd[%d]" % e] = rel_err(dwd[e], rd)
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()))
    for key, v in errs.items():
        assert v <= tol, "%s: %.3e > %.1e" % (key, v, tol)


@pytest.mark.parametrize("name,gather", [("a3b_8k", True), ("a3b_8k", False), ("a3b_long", True), ("a3b_long", False)])
def test_full_size_layer(name, gather):
    cfg = CONFIGS[name]
    say("full size %s: T=%d P=%d gather=%s" % (name, cfg.T, cfg.P, gather))
    inp = make_inputs(cfg)
    layer = _run(cfg, inp, inp["X"], gather=gather)
    idx, w, counts, offsets = O.route_topk(inp["logits"], cfg.k, cfg.renorm)
    assert np.array_equal(to_np(layer.topk_idx), idx)
    assert np.array_equal(to_np(layer.counts), counts)
    assert np.array_equal(to_np(layer.offsets), offsets)
    assert rel_err(to_np(layer.topk_w), w) <= 1e-5
    row_of_pair, pair_of_row = O.permute_maps(idx, offsets)
    assert np.array_equal(to_np(layer.row_of_pair), row_of_pair)
    assert np.array_equal(to_np(layer.pair_of_row), pair_of_row)
    r = np.random.default_rng(cfg.seed)
    rows = r.choice(cfg.P, size=256, replace=False)
    if gather:
        assert layer.xp is None and layer.dyp is None              # no copies in expert order
    else:
        assert np.array_equal(to_np(layer.xp)[rows], inp["X"][pair_of_row[rows] // cfg.k])   # bit copies (sampled rows)
    tokens = sorted(r.choice(cfg.T, size=12, replace=False).tolist()) + [0, cfg.T - 1]
    experts = [int(np.argmax(counts)), int(np.argmin(counts))]
    _check_sampled(cfg, inp, inp["X"], layer, idx, w, inp["logits"], tokens, experts)


@pytest.mark.parametrize("gather", [True, False])
def test_full_size_ep_share_skewed(gather):
    cfg = CONFIGS["a3b_ep_skew"]
    say("full size a3b_ep_skew: rows=%d local experts=%d" % (cfg.T, cfg.E))
    inp = make_inputs(cfg)
    from paper_2508_02317_amd import libmoe as L
    gidx, gw, gcounts, _ = L.moe_route_topk(to_dev(inp["logits"]), cfg.k_global, cfg.renorm)
    ridx, rw, rcounts, _ = O.route_topk(inp["logits"], cfg.k_global, cfg.renorm)
    assert np.array_equal(to_np(gidx), ridx) and np.array_equal(to_np(gcounts), rcounts)
    assert rcounts.max() > 5 * rcounts.mean()                      # a few experts get > 5x the mean
    tok, lidx, lw = select_local_share(ridx, rw, cfg.E, cfg.T)
    assert len(tok) == cfg.T
    lw32 = lw.astype(np.float32)
    X = inp["X"][tok]
    layer = _run(cfg, inp, X, routing=(lidx, lw32), gather=gather)
    counts, offsets = O.counts_offsets(lidx, cfg.E)
    say("  local counts: %s" % counts.tolist())
    assert np.array_equal(to_np(layer.counts), counts) and np.array_equal(to_np(layer.offsets), offsets)
    row_of_pair, pair_of_row = O.permute_maps(lidx, offsets)
    assert np.array_equal(to_np(layer.row_of_pair), row_of_pair)
    r = np.random.default_rng(cfg.seed)
    tokens = sorted(r.choice(cfg.T, size=12, replace=False).tolist())
    # the hottest expert, a mid-sized one, a nearly empty one and (if any) an empty one
    order = np.argsort(counts)
    experts = sorted({int(order[-1]), int(order[len(order) // 2]), int(order[0]), int(order[1])})
    _check_sampled(cfg, inp, X, layer, lidx, lw32.astype(np.float64), None, tokens, experts)


def test_full_size_block_from_hidden_states():
    """a3b_8k with the router linear in front: logits against the fp64 product, routing on the GPU's own
    logits, the whole dW_router, and Y / dX (expert + router path) on sampled tokens."""
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
    idx, w, counts, offsets = O.route_topk(z, cfg.k, cfg.renorm)     # the oracle routes on the same fp32 logits
    assert np.array_equal(to_np(layer.topk_idx), idx) and np.array_equal(to_np(layer.offsets), offsets)
    r = np.random.default_rng(cfg.seed + 100)
    tokens = sorted(r.choice(cfg.T, size=10, replace=False).tolist())
    dz = to_np(layer.dlogits).astype(np.float64)
    from paper_2508_02317_amd.inputs import quantise
    dz_seen = quantise(dz.astype(np.float32), dt).astype(np.float64)  # the backward products use dz rounded to bf16
    got_y, got_dx, ref_y, ref_dx, ref_dz = [], [], [], [], []
    for t in tokens:
        ry, rdx, rdw = O.token_fwd_bwd(inp["X"][t], idx[t], w[t], inp["dY"][t], inp["Wg"], inp["Wu"], inp["Wd"])
        rdz = O.route_topk_bwd(rdw[None], w[t][None], idx[t][None], z[t][None], cfg.E, cfg.renorm)[0]
        ref_y.append(ry); ref_dz.append(rdz)
        ref_dx.append(rdx + dz_seen[t] @ Wr.astype(np.float64))
        got_y.append(to_np(layer.y)[t]); got_dx.append(to_np(layer.dx)[t])
    tol = TOL[dt]
    errs = {"Y": rel_err(np.array(got_y), np.array(ref_y)), "dX": rel_err(np.array(got_dx), np.array(ref_dx)),
            "dlogits": rel_err(dz[tokens], np.array(ref_dz))}
    _, rdWr = O.router_bwd(dz_seen, inp["X"], Wr)
    errs["dW_router"] = rel_err(to_np(layer.dw_router), rdWr)
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()))
    for key, v in errs.items():
        assert v <= tol, "%s: %.3e > %.1e" % (key, v, tol)
