"""GPU parity: every C-ABI entry point against the fp64 oracle, element by element.

Each entry point is fed oracle-made inputs (rounded to the dtype the GPU receives) so one
kernel's error cannot hide another's; the whole chain is then checked end to end.
Integer outputs (indices, counts, offsets, maps, copied rows) must match bit for bit;
floating point within max|got-ref|/max|ref| <= 1e-5 (fp32) or 2e-2 (bf16 inputs, fp32
accumulation).
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


# reduced-size versions of the five configurations: several tiles, ragged tails
REDUCED = {
    "tiny": CONFIGS["tiny"],
    "small_r": scaled(CONFIGS["small"], T=777, d=256, f=384, E=16),
    "a3b_r": scaled(CONFIGS["a3b_8k"], T=1000, d=512, f=256, E=128),
    "long_r": scaled(CONFIGS["a3b_long"], T=1500, d=256, f=128, E=128),
}


# --------------------------------------------------------------------------------- routing

ROUTE_CASES = [
    # T, E, k, renorm, kind
    (256, 8, 2, 1, "normal"), (1000, 128, 8, 1, "normal"), (333, 16, 2, 0, "normal"),
    (64, 128, 8, 1, "ties"), (17, 6, 3, 1, "equal"), (50, 5, 1, 1, "normal"), (50, 7, 7, 1, "normal"),
    (9, 1, 1, 1, "normal"), (40, 1000, 64, 0, "normal"), (130, 300, 5, 1, "ties"), (1, 64, 4, 1, "normal"),
    (5000, 128, 8, 1, "skew"), (0, 8, 2, 1, "normal"),
]


def _route_logits(T, E, kind, seed):
    r = np.random.default_rng(seed)
    if kind == "normal":
        z = r.standard_normal((T, E))
    elif kind == "ties":
        z = r.integers(-3, 4, size=(T, E)).astype(np.float64) * 0.5
        z[::3] = np.where(z[::3] == 0, -0.0, z[::3])       # signed zeros among the ties
    elif kind == "equal":
        z = np.full((T, E), 1.25)
    else:
        z = r.standard_normal((T, E)) - 1.2 * np.log(1 + np.arange(E))[None, :]
    return z.astype(np.float32)


@pytest.mark.parametrize("T,E,k,renorm,kind", ROUTE_CASES)
def test_route_topk(L, T, E, k, renorm, kind):
    say("route T=%d E=%d k=%d renorm=%d %s" % (T, E, k, renorm, kind))
    z = _route_logits(T, E, kind, seed=T + E + k)
    idx, w, counts, offsets = L.moe_route_topk(to_dev(z), k, renorm)
    ridx, rw, rcounts, roffsets = O.route_topk(z, k, renorm)
    assert np.array_equal(to_np(idx), ridx)
    assert np.array_equal(to_np(counts), rcounts)
    assert np.array_equal(to_np(offsets), roffsets)
    if T:
        assert_close(to_np(w), rw, "f32", "topk_w")
        if renorm:
            assert np.max(np.abs(to_np(w).sum(axis=1) - 1.0)) <= 1e-6


@pytest.mark.parametrize("T,E,k,renorm", [(300, 128, 8, 1), (257, 16, 2, 0), (64, 300, 5, 0), (10, 4, 4, 1)])
def test_route_topk_bwd(L, T, E, k, renorm):
    say("route_bwd T=%d E=%d k=%d renorm=%d" % (T, E, k, renorm))
    r = np.random.default_rng(T)
    z = r.standard_normal((T, E)).astype(np.float32)
    idx, w, _, _ = O.route_topk(z, k, renorm)
    w32 = w.astype(np.float32)
    dw = r.standard_normal((T, k)).astype(np.float32)
    ref = O.route_topk_bwd(dw, w32, idx, z, E, renorm)
    got = L.moe_route_topk_bwd(to_dev(dw), to_dev(w32), to_dev(idx), to_dev(z), E, renorm)
    assert_close(to_np(got), ref, "f32", "dlogits")
    if renorm:
        mask = np.ones((T, E), dtype=bool)
        np.put_along_axis(mask, idx.astype(np.int64), False, axis=1)
        assert np.all(to_np(got)[mask] == 0.0)


def test_expert_offsets(L):
    r = np.random.default_rng(3)
    for n, E in ((0, 4), (1, 1), (5000, 16), (70000, 128)):
        idx = r.integers(0, E, size=n).astype(np.int32)
        if n > 10:
            idx[idx == 2] = 0            # an empty expert
        counts, offsets = L.moe_expert_offsets(to_dev(idx), E)
        rc, ro = O.counts_offsets(idx, E)
        assert np.array_equal(to_np(counts), rc) and np.array_equal(to_np(offsets), ro)


# --------------------------------------------------------------------------------- permute

@pytest.mark.parametrize("T,d,E,k,dt", [(256, 128, 8, 2, "f32"), (1000, 512, 128, 8, "bf16"), (777, 264, 16, 2, "bf16"),
                                        (3, 8, 4, 4, "f32"), (2049, 2048, 128, 8, "bf16"), (1300, 64, 16, 1, "bf16")])
def test_permute(L, T, d, E, k, dt):
    say("permute T=%d d=%d E=%d k=%d %s" % (T, d, E, k, dt))
    r = np.random.default_rng(T + d)
    z = r.standard_normal((T, E)).astype(np.float32)
    z[:, E // 2] = -50.0 if E > k else z[:, E // 2]          # an empty expert
    X = q(r.standard_normal((T, d)), dt)
    idx, _, _, offsets = O.route_topk(z, k)
    rXp, rrow, rpair = O.permute(X, idx, offsets)
    xp, row_of_pair, pair_of_row = L.moe_permute(to_dev(X, dt), to_dev(idx), to_dev(offsets), E)
    assert np.array_equal(to_np(row_of_pair), rrow)
    assert np.array_equal(to_np(pair_of_row), rpair)
    assert np.array_equal(to_np(xp).astype(np.float64), rXp)      # bit copies
    assert sorted(to_np(row_of_pair).tolist()) == list(range(T * k))


# --------------------------------------------------------------------------------- combine

@pytest.mark.parametrize("T,d,E,k,dt", [(256, 128, 8, 2, "f32"), (500, 512, 32, 8, "bf16"), (77, 2048, 128, 8, "bf16"),
                                        (130, 72, 8, 3, "bf16"), (64, 40, 8, 5, "f32")])
def test_combine_fwd_bwd(L, T, d, E, k, dt):
    say("combine T=%d d=%d E=%d k=%d %s" % (T, d, E, k, dt))
    r = np.random.default_rng(T + k)
    z = r.standard_normal((T, E)).astype(np.float32)
    idx, w, _, offsets = O.route_topk(z, k)
    w32 = w.astype(np.float32)
    row_of_pair, _ = O.permute_maps(idx, offsets)
    Yp = q(r.standard_normal((T * k, d)), dt)
    dY = q(r.standard_normal((T, d)), dt)
    tw, trow, typ = to_dev(w32), to_dev(row_of_pair), to_dev(Yp, dt)
    y = L.moe_unpermute_combine_fwd(typ, tw, trow, T, k)
    assert_close(to_np(y), O.unpermute_combine_fwd(Yp, w32, row_of_pair, T, k), dt, "y")
    y1 = L.moe_unpermute_combine_fwd(typ, None, trow, T, k)
    assert_close(to_np(y1), O.unpermute_combine_fwd(Yp, None, row_of_pair, T, k), dt, "y unit weights")
    dyp, dw = L.moe_unpermute_combine_bwd(to_dev(dY, dt), typ, tw, trow)
    rdyp, rdw = O.unpermute_combine_bwd(dY, Yp, w32, row_of_pair, T, k)
    assert_close(to_np(dyp), rdyp, dt, "dyp")
    assert_close(to_np(dw), rdw, "f32", "dw", tol=1e-5)


def test_permute_then_combine_is_identity(L):
    import torch
    r = np.random.default_rng(11)
    T, d, E, k = 300, 256, 16, 4
    z = r.standard_normal((T, E)).astype(np.float32)
    X = q(r.standard_normal((T, d)), "bf16")
    idx, w, counts, offsets = L.moe_route_topk(to_dev(z), k)
    xp, row_of_pair, _ = L.moe_permute(to_dev(X, "bf16"), idx, offsets, E)
    quarter = torch.full((T, k), 0.25, dtype=torch.float32, device="cuda")
    y = L.moe_unpermute_combine_fwd(xp, quarter, row_of_pair, T, k)
    assert np.array_equal(to_np(y), X)


# --------------------------------------------------------------------------------- grouped FFN

FFN_CASES = [
    # P-rows via (T, k), d, f, E, dtype, routing kind
    (256, 2, 128, 256, 8, "f32", "normal"),
    (777, 2, 256, 384, 16, "bf16", "normal"),
    (600, 8, 512, 256, 128, "bf16", "normal"),       # many experts with a handful of rows, some empty
    (900, 1, 264, 136, 5, "bf16", "skew"),           # d, f not multiples of the tile sizes
    (64, 1, 128, 128, 4, "bf16", "one_expert"),      # every row on one expert, three empty
    (3, 1, 64, 64, 2, "bf16", "normal"),             # segments of one or two rows
    (130, 3, 72, 40, 6, "f32", "skew"),
]


def _ffn_problem(T, k, d, f, E, dt, kind, seed):
    r = np.random.default_rng(seed)
    z = r.standard_normal((T, E))
    if kind == "skew":
        z = z - 2.0 * np.log(1 + np.arange(E))[None, :]
    if kind == "one_expert":
        z[:, 1] = 100.0
    idx, w, counts, offsets = O.route_topk(z.astype(np.float32), k)
    X = q(r.standard_normal((T, d)), dt)
    Wg = q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wu = q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wd = q(r.standard_normal((E, d, f)) * 0.05, dt)
    Xp, row_of_pair, _ = O.permute(X, idx, offsets)
    return dict(idx=idx, w=w, counts=counts, offsets=offsets, Xp=Xp.astype(np.float32), Wg=Wg, Wu=Wu, Wd=Wd,
                row_of_pair=row_of_pair, r=r)


@pytest.mark.parametrize("T,k,d,f,E,dt,kind", FFN_CASES)
def test_grouped_ffn_fwd_bwd(L, T, k, d, f, E, dt, kind):
    say("ffn T=%d k=%d d=%d f=%d E=%d %s %s" % (T, k, d, f, E, dt, kind))
    pr = _ffn_problem(T, k, d, f, E, dt, kind, seed=T + d + f)
    P = T * k
    offs = pr["offsets"]
    G, U, A, Yp = O.grouped_ffn_fwd(pr["Xp"], pr["Wg"], pr["Wu"], pr["Wd"], offs)
    txp, twg, twu, twd = (to_dev(pr[n], dt) for n in ("Xp", "Wg", "Wu", "Wd"))
    toffs = to_dev(offs)
    act, yp, g, u = L.moe_grouped_gemm_swiglu_fwd(txp, twg, twu, twd, toffs, save_gu=True)
    assert_close(to_np(g), G, dt, "G")
    assert_close(to_np(u), U, dt, "U")
    assert_close(to_np(act), A, dt, "act")
    assert_close(to_np(yp), Yp, dt, "yp")
    # without saving the pre-activations the other outputs must not change
    act2, yp2, g2, u2 = L.moe_grouped_gemm_swiglu_fwd(txp, twg, twu, twd, toffs, save_gu=False)
    assert g2 is None and u2 is None
    assert np.array_equal(to_np(act2), to_np(act)) and np.array_equal(to_np(yp2), to_np(yp))

    # backward, teacher-forced: the GPU gets the oracle's forward intermediates, rounded
    dYp = q(pr["r"].standard_normal((P, d)), dt)
    Gq, Uq, Aq = q(G, dt), q(U, dt), q(A, dt)
    rdXp, rdWg, rdWu, rdWd = O.grouped_ffn_bwd(dYp, pr["Xp"], Gq, Uq, Aq, pr["Wg"], pr["Wu"], pr["Wd"], offs)
    dxp, dwg, dwu, dwd = L.moe_grouped_gemm_swiglu_bwd(to_dev(dYp, dt), txp, to_dev(Gq, dt), to_dev(Uq, dt),
                                                       to_dev(Aq, dt), twg, twu, twd, toffs)
    assert_close(to_np(dxp), rdXp, dt, "dxp")
    assert_close(to_np(dwg), rdWg, dt, "dw_gate")
    assert_close(to_np(dwu), rdWu, dt, "dw_up")
    assert_close(to_np(dwd), rdWd, dt, "dw_down")
    empty = np.flatnonzero(pr["counts"] == 0)
    for e in empty:
        assert not to_np(dwg)[e].any() and not to_np(dwu)[e].any() and not to_np(dwd)[e].any()
    # recompute variant: G and U not passed
    dxp2, dwg2, dwu2, dwd2 = L.moe_grouped_gemm_swiglu_bwd(to_dev(dYp, dt), txp, None, None, to_dev(Aq, dt),
                                                           twg, twu, twd, toffs)
    rdXp2, rdWg2, rdWu2, rdWd2 = O.grouped_ffn_bwd(dYp, pr["Xp"], G, U, Aq, pr["Wg"], pr["Wu"], pr["Wd"], offs)
    assert_close(to_np(dxp2), rdXp2, dt, "dxp (recompute)")
    assert_close(to_np(dwg2), rdWg2, dt, "dw_gate (recompute)")
    assert_close(to_np(dwu2), rdWu2, dt, "dw_up (recompute)")
    assert_close(to_np(dwd2), rdWd2, dt, "dw_down (recompute)")


def test_ffn_bwd_weight_gradients_of_long_experts(L):
    """Experts with more rows than one reduction chunk (2048 rows here) go through the split path: fp32
    partial tiles per chunk, summed in chunk order.  Counts cover 3.x chunks, exactly one chunk, exactly two
    chunks, one row over a chunk, short and empty experts."""
    dt, d, f = "bf16", 136, 72
    counts = np.array([6700, 2048, 0, 4096, 2049, 37, 0, 600], dtype=np.int64)
    E, P = len(counts), int(counts.sum())
    offs = np.zeros(E + 1, dtype=np.int32)
    offs[1:] = np.cumsum(counts)
    r = np.random.default_rng(11)
    Xp = q(r.standard_normal((P, d)), dt).astype(np.float32)
    Wg, Wu = q(r.standard_normal((E, f, d)) * 0.05, dt), q(r.standard_normal((E, f, d)) * 0.05, dt)
    Wd = q(r.standard_normal((E, d, f)) * 0.05, dt)
    G, U, A, _ = O.grouped_ffn_fwd(Xp, Wg, Wu, Wd, offs)
    dYp = q(r.standard_normal((P, d)), dt)
    Gq, Uq, Aq = q(G, dt), q(U, dt), q(A, dt)
    rdXp, rdWg, rdWu, rdWd = O.grouped_ffn_bwd(dYp, Xp, Gq, Uq, Aq, Wg, Wu, Wd, offs)
    args = (to_dev(dYp, dt), to_dev(Xp, dt), to_dev(Gq, dt), to_dev(Uq, dt), to_dev(Aq, dt), to_dev(Wg, dt),
            to_dev(Wu, dt), to_dev(Wd, dt), to_dev(offs))
    dxp, dwg, dwu, dwd = L.moe_grouped_gemm_swiglu_bwd(*args)
    assert_close(to_np(dxp), rdXp, dt, "dxp")
    for e in range(E):
        say("  expert %d rows %d" % (e, counts[e]))
        if counts[e] == 0:
            assert not to_np(dwg)[e].any() and not to_np(dwu)[e].any() and not to_np(dwd)[e].any()
            continue
        assert_close(to_np(dwg)[e], rdWg[e], dt, "dw_gate[%d]" % e)
        assert_close(to_np(dwu)[e], rdWu[e], dt, "dw_up[%d]" % e)
        assert_close(to_np(dwd)[e], rdWd[e], dt, "dw_down[%d]" % e)
    # the split path is deterministic: a second run gives the same bits
    again = L.moe_grouped_gemm_swiglu_bwd(*args)
    for a, b in zip((dxp, dwg, dwu, dwd), again):
        assert np.array_equal(to_np(a), to_np(b))


def test_ffn_zero_rows_writes_zero_weight_gradients(L):
    import torch
    E, d, f = 3, 64, 64
    w = lambda *s: torch.randn(s, device="cuda").to(torch.bfloat16)
    wg, wu, wd = w(E, f, d), w(E, f, d), w(E, d, f)
    empty = torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    ef = torch.empty((0, f), dtype=torch.bfloat16, device="cuda")
    offs = torch.zeros(E + 1, dtype=torch.int32, device="cuda")
    out = (torch.empty_like(empty), torch.full_like(wg, 7.0), torch.full_like(wu, 7.0), torch.full_like(wd, 7.0))
    L.moe_grouped_gemm_swiglu_bwd(empty, empty, ef, ef, ef, wg, wu, wd, offs, out=out)
    torch.cuda.synchronize()
    assert not out[1].any() and not out[2].any() and not out[3].any()


# --------------------------------------------------------------------------------- whole layer

def _run_layer(L, cfg, inp, routing=None):
    import torch
    from paper_2508_02317_amd.layer import MoELayer
    dt = cfg.dtype
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, torch_dtype(dt), to_dev(inp["Wg"], dt), to_dev(inp["Wu"], dt),
                     to_dev(inp["Wd"], dt), renorm=cfg.renorm, prerouted=routing is not None)
    x = to_dev(inp["X"], dt)
    dy = to_dev(inp["dY"], dt)
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
    assert np.array_equal(to_np(layer.counts), fwd["counts"])
    assert np.array_equal(to_np(layer.offsets), fwd["offsets"])
    assert np.array_equal(to_np(layer.row_of_pair), fwd["row_of_pair"])
    errs = {}
    errs["topk_w"] = assert_close(to_np(layer.topk_w), fwd["topk_w"], "f32", "topk_w")
    errs["Y"] = assert_close(to_np(layer.y), fwd["Y"], dt, "Y")
    errs["dX"] = assert_close(to_np(layer.dx), bwd["dX"], dt, "dX")
    errs["dWg"] = assert_close(to_np(layer.dw_gate), bwd["dWg"], dt, "dWg")
    errs["dWu"] = assert_close(to_np(layer.dw_up), bwd["dWu"], dt, "dWu")
    errs["dWd"] = assert_close(to_np(layer.dw_down), bwd["dWd"], dt, "dWd")
    if bwd["dlogits"] is not None:
        errs["dlogits"] = assert_close(to_np(layer.dlogits), bwd["dlogits"], dt, "dlogits")
    say("  errors: " + " ".join("%s=%.2e" % kv for kv in errs.items()))


@pytest.mark.parametrize("name", list(REDUCED))
def test_layer_end_to_end_reduced(L, name):
    cfg = REDUCED[name]
    say("layer %s T=%d d=%d E=%d k=%d f=%d %s" % (name, cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, cfg.dtype))
    inp = make_inputs(cfg)
    fwd = O.moe_layer_fwd(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.k, cfg.renorm)
    bwd = O.moe_layer_bwd(fwd, inp["dY"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.renorm)
    layer = _run_layer(L, cfg, inp)
    _check_layer(layer, cfg, fwd, bwd)


def test_layer_end_to_end_ep_share_reduced(L):
    cfg = scaled(CONFIGS["a3b_ep_skew"], T=2048, T_global=2048, d=256, f=128)
    say("layer ep_share reduced")
    inp = make_inputs(cfg)
    # global routing on the GPU must agree bit for bit with the oracle's before the share is cut
    gidx, gw, _, _ = L.moe_route_topk(to_dev(inp["logits"]), cfg.k_global)
    ridx, rw, rcounts, _ = O.route_topk(inp["logits"], cfg.k_global)
    assert np.array_equal(to_np(gidx), ridx)
    tok, lidx, lw = select_local_share(ridx, rw, cfg.E, cfg.T)
    assert len(tok) == cfg.T
    lw32 = lw.astype(np.float32)
    local = dict(inp, X=inp["X"][tok])
    fwd = O.moe_layer_fwd(local["X"], None, inp["Wg"], inp["Wu"], inp["Wd"], 1, routing=(lidx, lw32))
    bwd = O.moe_layer_bwd(fwd, inp["dY"], None, inp["Wg"], inp["Wu"], inp["Wd"])
    assert fwd["counts"].max() > 5 * cfg.T / cfg.E                 # really skewed
    layer = _run_layer(L, cfg, local, routing=(lidx, lw32))
    _check_layer(layer, cfg, fwd, bwd)


def test_layer_is_deterministic(L):
    cfg = REDUCED["a3b_r"]
    inp = make_inputs(cfg)
    a = _run_layer(L, cfg, inp)
    b = _run_layer(L, cfg, inp)
    for name in ("y", "dx", "dw_gate", "dw_up", "dw_down", "dlogits", "row_of_pair", "topk_w"):
        assert np.array_equal(to_np(getattr(a, name)), to_np(getattr(b, name))), name


def test_layer_small_config_full_size(L):
    cfg = CONFIGS["small"]
    say("layer small (full size)")
    inp = make_inputs(cfg)
    fwd = O.moe_layer_fwd(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.k, cfg.renorm)
    bwd = O.moe_layer_bwd(fwd, inp["dY"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.renorm)
    layer = _run_layer(L, cfg, inp)
    _check_layer(layer, cfg, fwd, bwd)


def test_dense_swiglu_mlp_is_the_one_expert_case(L):
    """E = 1, k = 1: routing weight 1 for every token, one segment of all rows -- the layer is a plain dense
    SwiGLU MLP, checked here against that closed form written with matrix products (no routing code)."""
    from paper_2508_02317_amd.layer import MoELayer
    T, d, f, dt = 700, 256, 384, "bf16"
    r = np.random.default_rng(5)
    X, dY = q(r.standard_normal((T, d)), dt), q(r.standard_normal((T, d)), dt)
    Wg, Wu = q(r.standard_normal((1, f, d)) * 0.05, dt), q(r.standard_normal((1, f, d)) * 0.05, dt)
    Wd = q(r.standard_normal((1, d, f)) * 0.05, dt)
    logits = np.zeros((T, 1), dtype=np.float32)
    layer = MoELayer(T, d, 1, 1, f, torch_dtype(dt), to_dev(Wg, dt), to_dev(Wu, dt), to_dev(Wd, dt))
    tl = to_dev(logits)
    layer.forward(to_dev(X, dt), logits=tl)
    layer.backward(to_dev(dY, dt), logits=tl)
    X64 = X.astype(np.float64)
    G, U = X64 @ Wg[0].astype(np.float64).T, X64 @ Wu[0].astype(np.float64).T
    sg = 1.0 / (1.0 + np.exp(-G))
    A = G * sg * U
    Y = A @ Wd[0].astype(np.float64).T
    dA = dY.astype(np.float64) @ Wd[0].astype(np.float64)
    dG, dU = dA * U * sg * (1.0 + G * (1.0 - sg)), dA * G * sg
    dX = dG @ Wg[0].astype(np.float64) + dU @ Wu[0].astype(np.float64)
    assert np.array_equal(to_np(layer.topk_w), np.ones((T, 1), dtype=np.float32))
    assert np.array_equal(to_np(layer.xp), X)                      # the permutation is the identity
    assert_close(to_np(layer.y), Y, dt, "Y")
    assert_close(to_np(layer.dx), dX, dt, "dX")
    assert_close(to_np(layer.dw_down)[0], dY.astype(np.float64).T @ A, dt, "dW_down")
    assert_close(to_np(layer.dw_gate)[0], dG.T @ X64, dt, "dW_gate")
    assert not to_np(layer.dlogits).any()                          # k = 1, renormalised: no gradient to the logit
