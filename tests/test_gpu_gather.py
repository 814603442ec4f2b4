"""GPU parity of the *_gather entry points: the grouped FFN reading the layer input and the output gradient
by token, so that neither xp nor dyp is written.

Forward: the arithmetic is that of moe_grouped_gemm_swiglu_fwd on the gathered rows, so the outputs must match
the fp64 oracle within the usual tolerance and the other entry point bit for bit.  Backward: the reference is the
oracle's combine backward followed by its FFN backward (no rounding in between), with act = silu(G) * U taken
from the rounded G and U the GPU receives -- what the entry point is documented to compute.
"""
import sys

import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2508_02317_amd.inputs import CONFIGS, make_inputs, scaled, select_local_share
from tests.util import assert_close, q, to_dev, to_np, torch_dtype

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True, file=sys.stderr)


@pytest.fixture(scope="module")
def L():
    from paper_2508_02317_amd import libmoe
    return libmoe


CASES = [
    # T, k, d, f, E, dtype, routing kind
    (256, 2, 128, 256, 8, "f32", "normal"),
    (777, 2, 256, 384, 16, "bf16", "normal"),
    (600, 8, 512, 256, 128, "bf16", "normal"),       # many experts with a handful of rows, some empty
    (900, 1, 264, 136, 5, "bf16", "skew"),           # d, f not multiples of the tile sizes
    (64, 1, 128, 128, 4, "bf16", "one_expert"),      # every row on one expert, three empty
    (3, 1, 64, 64, 2, "bf16", "normal"),             # segments of one or two rows
    (130, 3, 72, 40, 6, "f32", "skew"),
    (5300, 2, 136, 72, 3, "bf16", "skew"),           # experts longer than one weight-gradient chunk (split path)
]


def _problem(T, k, d, f, E, dt, kind, seed):
    r = np.random.default_rng(seed)
    z = r.standard_normal((T, E))
    if kind == "skew":
        z = z - 2.0 * np.log(1 + np.arange(E))[None, :]
    if kind == "one_expert":
        z[:, 1] = 100.0
    idx, w, counts, offsets = O.route_topk(z.astype(np.float32), k)
    X = q(r.standard_normal((T, d)), dt)
    dY = q(r.standard_normal((T, d)), dt)
    Wg = q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wu = q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wd = q(r.standard_normal((E, d, f)) * 0.05, dt)
    Xp, row_of_pair, pair_of_row = O.permute(X, idx, offsets)
    return dict(idx=idx, w=w.astype(np.float32), counts=counts, offsets=offsets, X=X, dY=dY, Xp=Xp.astype(np.float32),
                Wg=Wg, Wu=Wu, Wd=Wd, row_of_pair=row_of_pair, pair_of_row=pair_of_row)


@pytest.mark.parametrize("T,k,d,f,E,dt,kind", CASES)
def test_gather_ffn_fwd_bwd(L, T, k, d, f, E, dt, kind):
    say("gather ffn T=%d k=%d d=%d f=%d E=%d %s %s" % (T, k, d, f, E, dt, kind))
    pr = _problem(T, k, d, f, E, dt, kind, seed=T + d + f)
    offs = pr["offsets"]
    G, U, A, Yp = O.grouped_ffn_fwd(pr["Xp"], pr["Wg"], pr["Wu"], pr["Wd"], offs)
    tx, twg, twu, twd = (to_dev(pr[n], dt) for n in ("X", "Wg", "Wu", "Wd"))
    toffs, tpair = to_dev(offs), to_dev(pr["pair_of_row"])

    # the maps alone
    _, row_of_pair, pair_of_row = L.moe_permute(None, to_dev(pr["idx"]), toffs, E)
    assert np.array_equal(to_np(row_of_pair), pr["row_of_pair"]) and np.array_equal(to_np(pair_of_row), pr["pair_of_row"])

    act, yp, g, u = L.moe_grouped_gemm_swiglu_fwd_gather(tx, k, tpair, twg, twu, twd, toffs, save_gu=True)
    assert_close(to_np(g), G, dt, "G")
    assert_close(to_np(u), U, dt, "U")
    assert_close(to_np(act), A, dt, "act")
    assert_close(to_np(yp), Yp, dt, "yp")
    # same arithmetic as the entry point that is handed xp
    act0, yp0, g0, u0 = L.moe_grouped_gemm_swiglu_fwd(to_dev(pr["Xp"], dt), twg, twu, twd, toffs, save_gu=True)
    for a, b, name in ((act, act0, "act"), (yp, yp0, "yp"), (g, g0, "G"), (u, u0, "U")):
        assert np.array_equal(to_np(a), to_np(b)), name + " differs from the un-gathered entry point"

    # backward, teacher-forced with the rounded G and U
    Gq, Uq = q(G, dt), q(U, dt)
    Aq = O.silu(Gq.astype(np.float64)) * Uq
    Ypq = np.zeros((T * k, d))
    for e in range(E):
        Ypq[offs[e]:offs[e + 1]] = Aq[offs[e]:offs[e + 1]] @ pr["Wd"][e].astype(np.float64).T
    dYp, rdw = O.unpermute_combine_bwd(pr["dY"], Ypq, pr["w"], pr["row_of_pair"], T, k)
    rdXp, rdWg, rdWu, rdWd = O.grouped_ffn_bwd(dYp, pr["Xp"], Gq, Uq, Aq, pr["Wg"], pr["Wu"], pr["Wd"], offs)
    tdy, tw = to_dev(pr["dY"], dt), to_dev(pr["w"])
    dxp, dwg, dwu, dwd, dtw = L.moe_grouped_gemm_swiglu_bwd_gather(tdy, tx, tw, tpair, to_dev(Gq, dt), to_dev(Uq, dt),
                                                                   twg, twu, twd, toffs)
    assert_close(to_np(dxp), rdXp, dt, "dxp")
    assert_close(to_np(dwg), rdWg, dt, "dw_gate")
    assert_close(to_np(dwu), rdWu, dt, "dw_up")
    assert_close(to_np(dwd), rdWd, dt, "dw_down")
    assert_close(to_np(dtw), rdw, dt, "dtopk_w")
    for e in np.flatnonzero(pr["counts"] == 0):
        assert not to_np(dwg)[e].any() and not to_np(dwu)[e].any() and not to_np(dwd)[e].any()
    # deterministic
    again = L.moe_grouped_gemm_swiglu_bwd_gather(tdy, tx, tw, tpair, to_dev(Gq, dt), to_dev(Uq, dt), twg, twu, twd, toffs)
    for a, b in zip((dxp, dwg, dwu, dwd, dtw), again):
        assert np.array_equal(to_np(a), to_np(b))
    # recompute variant: G and U not passed
    Af = O.silu(G) * U
    Ypf = np.zeros((T * k, d))
    for e in range(E):
        Ypf[offs[e]:offs[e + 1]] = Af[offs[e]:offs[e + 1]] @ pr["Wd"][e].astype(np.float64).T
    dYp2, rdw2 = O.unpermute_combine_bwd(pr["dY"], Ypf, pr["w"], pr["row_of_pair"], T, k)
    r2 = O.grouped_ffn_bwd(dYp2, pr["Xp"], G, U, Af, pr["Wg"], pr["Wu"], pr["Wd"], offs)
    got2 = L.moe_grouped_gemm_swiglu_bwd_gather(tdy, tx, tw, tpair, None, None, twg, twu, twd, toffs)
    for a, b, name in zip(got2, r2 + (rdw2,), ("dxp", "dw_gate", "dw_up", "dw_down", "dtopk_w")):
        assert_close(to_np(a), b, dt, name + " (recompute)")

    # the combine weight applied inside the forward products: act and yp leave scaled by the row's weight, G and U do not;
    # the plain sum of those yp rows is Y, and the backward takes the weighted activation as it is
    w_row = pr["w"].reshape(-1)[pr["pair_of_row"]][:, None].astype(np.float64)
    act_w, yp_w, g_w, u_w = L.moe_grouped_gemm_swiglu_fwd_gather(tx, k, tpair, twg, twu, twd, toffs, save_gu=True, topk_w=tw)
    assert np.array_equal(to_np(g_w), to_np(g)) and np.array_equal(to_np(u_w), to_np(u))
    assert_close(to_np(act_w), w_row * A, dt, "w * act")
    assert_close(to_np(yp_w), w_row * Yp, dt, "w * yp")
    y = L.moe_unpermute_combine_fwd(yp_w, None, to_dev(pr["row_of_pair"]), T, k)
    assert_close(to_np(y), O.unpermute_combine_fwd(Yp, pr["w"], pr["row_of_pair"], T, k), dt, "Y from weighted rows")
    got3 = L.moe_grouped_gemm_swiglu_bwd_gather(tdy, tx, tw, tpair, to_dev(Gq, dt), to_dev(Uq, dt), twg, twu, twd, toffs,
                                                act_w=to_dev(q(w_row * Aq, dt), dt))
    for a, b, name in zip(got3, (rdXp, rdWg, rdWu, rdWd, rdw), ("dxp", "dw_gate", "dw_up", "dw_down", "dtopk_w")):
        assert_close(to_np(a), b, dt, name + " (weighted activation from the forward)")


def _run_layer(cfg, inp, X, gather, routing=None, save_gu=True, weight_in_forward=None):
    import torch
    from paper_2508_02317_amd.layer import MoELayer
    dt = cfg.dtype
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, torch_dtype(dt), to_dev(inp["Wg"], dt), to_dev(inp["Wu"], dt),
                     to_dev(inp["Wd"], dt), renorm=cfg.renorm, prerouted=routing is not None, gather=gather, save_gu=save_gu,
                     weight_in_forward=weight_in_forward)
    x, dy = to_dev(X, dt), to_dev(inp["dY"], dt)
    if routing is None:
        logits = to_dev(inp["logits"])
        layer.forward(x, logits=logits)
        layer.backward(dy, logits=logits)
    else:
        layer.forward(x, topk_idx=to_dev(routing[0]), topk_w=to_dev(routing[1].astype(np.float32)))
        layer.backward(dy)
    torch.cuda.synchronize()
    return layer


def _check_layer(layer, cfg, fwd, bwd):
    dt = cfg.dtype
    assert np.array_equal(to_np(layer.topk_idx), fwd["topk_idx"])
    assert np.array_equal(to_np(layer.offsets), fwd["offsets"])
    assert np.array_equal(to_np(layer.row_of_pair), fwd["row_of_pair"])
    errs = {}
    errs["Y"] = assert_close(to_np(layer.y), fwd["Y"], dt, "Y")
    errs["dX"] = assert_close(to_np(layer.dx), bwd["dX"], dt, "dX")
    errs["dWg"] = assert_close(to_np(layer.dw_gate), bwd["dWg"], dt, "dWg")
    errs["dWu"] = assert_close(to_np(layer.dw_up), bwd["dWu"], dt, "dWu")
    errs["dWd"] = assert_close(to_np(layer.dw_down), bwd["dWd"], dt, "dWd")
    if bwd["dlogits"] is not None:
        errs["dlogits"] = assert_close(to_np(layer.dlogits), bwd["dlogits"], dt, "dlogits")
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()))


REDUCED = {
    "tiny": CONFIGS["tiny"],
    "small_r": scaled(CONFIGS["small"], T=777, d=256, f=384, E=16),
    "a3b_r": scaled(CONFIGS["a3b_8k"], T=1000, d=512, f=256, E=128),
    "long_r": scaled(CONFIGS["a3b_long"], T=1500, d=256, f=128, E=128),
}


@pytest.mark.parametrize("name", list(REDUCED))
@pytest.mark.parametrize("save_gu", [True, False])
def test_gather_layer_end_to_end_reduced(name, save_gu):
    cfg = REDUCED[name]
    say("gather layer %s T=%d d=%d E=%d k=%d f=%d %s save_gu=%s" % (name, cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, cfg.dtype, save_gu))
    inp = make_inputs(cfg)
    fwd = O.moe_layer_fwd(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.k, cfg.renorm)
    bwd = O.moe_layer_bwd(fwd, inp["dY"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.renorm)
    layer = _run_layer(cfg, inp, inp["X"], gather=True, save_gu=save_gu)      # the default: combine weight inside the forward products
    assert layer.weight_in_forward
    _check_layer(layer, cfg, fwd, bwd)
    assert layer.xp is None and layer.dyp is None
    # with the weight left to the combine, the forward is the same arithmetic as the layer that materialises xp
    late = _run_layer(cfg, inp, inp["X"], gather=True, save_gu=save_gu, weight_in_forward=False)
    _check_layer(late, cfg, fwd, bwd)
    plain = _run_layer(cfg, inp, inp["X"], gather=False, save_gu=save_gu)
    assert np.array_equal(to_np(late.y), to_np(plain.y))


def test_gather_layer_ep_share_reduced():
    cfg = scaled(CONFIGS["a3b_ep_skew"], T=2048, T_global=2048, d=256, f=128)
    say("gather layer ep_share reduced")
    inp = make_inputs(cfg)
    ridx, rw, _, _ = O.route_topk(inp["logits"], cfg.k_global)
    tok, lidx, lw = select_local_share(ridx, rw, cfg.E, cfg.T)
    lw32 = lw.astype(np.float32)
    X = inp["X"][tok]
    fwd = O.moe_layer_fwd(X, None, inp["Wg"], inp["Wu"], inp["Wd"], 1, routing=(lidx, lw32))
    bwd = O.moe_layer_bwd(fwd, inp["dY"], None, inp["Wg"], inp["Wu"], inp["Wd"])
    layer = _run_layer(cfg, inp, X, gather=True, routing=(lidx, lw32))
    _check_layer(layer, cfg, fwd, bwd)
    assert_close(to_np(layer.dw), bwd["dw"], "bf16", "dtopk_w")


def test_gather_layer_full_size_against_the_plain_layer():
    """At the benchmark's size the gathered layer is compared with the layer that writes xp and dyp (itself
    checked against the oracle on samples at this size): same routing, same forward bits, gradients within
    the bf16 tolerance of each other."""
    cfg = CONFIGS["a3b_8k"]
    say("gather full size a3b_8k")
    inp = make_inputs(cfg)
    a = _run_layer(cfg, inp, inp["X"], gather=True, weight_in_forward=False)
    b = _run_layer(cfg, inp, inp["X"], gather=False)
    assert np.array_equal(to_np(a.row_of_pair), to_np(b.row_of_pair))
    assert np.array_equal(to_np(a.y), to_np(b.y))
    for name in ("dx", "dw_gate", "dw_up", "dw_down", "dlogits", "dw"):
        e = assert_close(to_np(getattr(a, name)), to_np(getattr(b, name)).astype(np.float64), "bf16", name)
        say("  %s: %.2e" % (name, e))


def test_gather_layer_step_replays_from_a_graph():
    import torch
    from paper_2508_02317_amd.layer import MoELayer
    cfg = scaled(CONFIGS["a3b_8k"], T=1024, E=32, d=512, f=256)
    inp = make_inputs(cfg)
    dt = cfg.dtype
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, torch_dtype(dt), to_dev(inp["Wg"], dt), to_dev(inp["Wu"], dt),
                     to_dev(inp["Wd"], dt), renorm=cfg.renorm, gather=True)
    x, dy, logits = to_dev(inp["X"], dt), to_dev(inp["dY"], dt), to_dev(inp["logits"])

    def step():
        layer.forward(x, logits=logits)
        layer.backward(dy, logits=logits)

    tensors = (layer.y, layer.dx, layer.dw_gate, layer.dw_up, layer.dw_down, layer.dlogits)
    outs = lambda: [to_np(t).copy() for t in tensors]
    step()
    torch.cuda.synchronize()
    eager = outs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(3):
        for t in tensors:
            t.fill_(7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs(), eager):
            assert np.array_equal(a, b), "replay %d differs from the eager step" % rep
