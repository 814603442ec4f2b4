"""Pins for the fp64 oracle (CPU only).

The oracle is checked against things other than itself: a dense brute-force evaluation
that shares no code with it, a hand-derived fixture, closed forms and library routines
for the special cases, structural invariants, and central finite differences taken on the
brute-force loss.
"""
import os

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import moe_brute as B
from oracle import moe_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_layer(seed, T, d, E, f, wscale=0.5):
    r = np.random.default_rng(seed)
    X = r.standard_normal((T, d))
    Wg = r.standard_normal((E, f, d)) * wscale
    Wu = r.standard_normal((E, f, d)) * wscale
    Wd = r.standard_normal((E, d, f)) * wscale
    z = r.standard_normal((T, E))
    dY = r.standard_normal((T, d))
    return X, z, Wg, Wu, Wd, dY


# ------------------------------------------------------------------ hand-derived fixture

def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, v = line.split()
            vals[key] = float(v)
    return vals


def test_hand_example():
    g = _read_golden("hand_example.txt")
    X = np.array([[1.0]])
    z = np.array([[np.log(3.0), 0.0]])
    Wg = np.array([[[0.0]], [[np.log(2.0)]]])
    Wu = np.array([[[5.0]], [[3.0]]])
    Wd = np.array([[[7.0]], [[0.5]]])
    fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, k=2)
    assert fwd["topk_idx"].tolist() == [[0, 1]]
    assert fwd["topk_w"][0, 0] == pytest.approx(g["w0"], abs=1e-15)
    assert fwd["topk_w"][0, 1] == pytest.approx(g["w1"], abs=1e-15)
    assert fwd["Y"][0, 0] == pytest.approx(g["Y"], abs=1e-15)
    bwd = O.moe_layer_bwd(fwd, np.array([[1.0]]), z, Wg, Wu, Wd)
    assert bwd["dw"][0, 0] == pytest.approx(0.0, abs=1e-15)
    assert bwd["dw"][0, 1] == pytest.approx(g["dw1"], abs=1e-15)
    assert bwd["dlogits"][0, 0] == pytest.approx(g["dz0"], abs=1e-15)
    assert bwd["dlogits"][0, 1] == pytest.approx(g["dz1"], abs=1e-15)


# ------------------------------------------------------------------ forward vs brute force

@pytest.mark.parametrize("T,d,E,f,k,renorm", [
    (5, 4, 4, 3, 2, 1), (1, 3, 2, 2, 1, 1), (4, 2, 3, 5, 3, 1), (3, 4, 1, 2, 1, 1),
    (6, 3, 5, 4, 2, 0), (4, 3, 4, 2, 4, 0)])
def test_forward_vs_scalar_brute(T, d, E, f, k, renorm):
    X, z, Wg, Wu, Wd, _ = _rand_layer(10 + T + E, T, d, E, f)
    Y = O.moe_layer_fwd(X, z, Wg, Wu, Wd, k, renorm)["Y"]
    Yb = np.array(B.layer_dense(X.tolist(), z.tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist(), k, renorm))
    assert np.max(np.abs(Y - Yb)) <= 1e-12 * max(1.0, np.max(np.abs(Yb)))


def test_forward_vs_matvec_brute_tiny_config():
    from paper_2508_02317_amd.inputs import CONFIGS, make_inputs
    cfg = CONFIGS["tiny"]
    inp = make_inputs(cfg)
    Y = O.moe_layer_fwd(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.k)["Y"]
    Yb = B.layer_dense_matvec(inp["X"], inp["logits"], inp["Wg"], inp["Wu"], inp["Wd"], cfg.k)
    assert np.max(np.abs(Y - Yb)) <= 1e-12 * np.max(np.abs(Yb))


def test_matvec_brute_vs_scalar_brute():
    # pins the orientation of the library mat-vecs used at the larger size
    X, z, Wg, Wu, Wd, _ = _rand_layer(3, 4, 3, 3, 2)
    Ya = np.array(B.layer_dense(X.tolist(), z.tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist(), 2))
    Yb = B.layer_dense_matvec(X, z, Wg, Wu, Wd, 2)
    assert np.max(np.abs(Ya - Yb)) <= 1e-13


# ------------------------------------------------------------------ special cases

def test_identical_experts_is_plain_swiglu_mlp():
    r = np.random.default_rng(1)
    T, d, E, f, k = 9, 6, 5, 7, 3
    X = r.standard_normal((T, d)); z = r.standard_normal((T, E))
    wg = r.standard_normal((f, d)); wu = r.standard_normal((f, d)); wd = r.standard_normal((d, f))
    Wg = np.broadcast_to(wg, (E, f, d)); Wu = np.broadcast_to(wu, (E, f, d)); Wd = np.broadcast_to(wd, (E, d, f))
    Y = O.moe_layer_fwd(X, z, Wg, Wu, Wd, k)["Y"]
    gate = X @ wg.T
    ref = ((gate * (1.0 / (1.0 + np.exp(-gate)))) * (X @ wu.T)) @ wd.T
    assert np.max(np.abs(Y - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_k1_weights_are_one_and_dz_zero():
    X, z, Wg, Wu, Wd, dY = _rand_layer(2, 7, 4, 5, 3)
    fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, 1)
    assert np.array_equal(fwd["topk_idx"][:, 0], np.argmax(z, axis=1))
    assert np.all(fwd["topk_w"] == 1.0)
    for t in range(7):
        e = int(np.argmax(z[t]))
        g = Wg[e] @ X[t]
        ref = Wd[e] @ (g / (1 + np.exp(-g)) * (Wu[e] @ X[t]))
        assert np.max(np.abs(fwd["Y"][t] - ref)) <= 1e-13 * max(1.0, np.max(np.abs(ref)))
    bwd = O.moe_layer_bwd(fwd, dY, z, Wg, Wu, Wd)
    assert np.all(bwd["dlogits"] == 0.0)


def test_kE_is_full_softmax_mixture():
    X, z, Wg, Wu, Wd, _ = _rand_layer(4, 5, 3, 4, 2)
    for renorm in (0, 1):
        idx, w, _, _ = O.route_topk(z, 4, renorm)
        p = scipy_softmax(z, axis=1)
        assert np.max(np.abs(w - np.take_along_axis(p, idx.astype(np.int64), axis=1))) <= 1e-15


# ------------------------------------------------------------------ routing invariants

def test_routing_weights_and_indices():
    r = np.random.default_rng(5)
    z = r.standard_normal((64, 16)).astype(np.float32)
    idx, w, counts, offsets = O.route_topk(z, 4, 1)
    assert idx.dtype == np.int32 and counts.dtype == np.int32 and offsets.dtype == np.int32
    assert np.all(w >= 0) and np.max(np.abs(w.sum(axis=1) - 1.0)) <= 1e-15
    for t in range(64):
        assert len(set(idx[t].tolist())) == 4
        zs = z[t, idx[t]].astype(np.float64)
        assert np.all(np.diff(zs) <= 0)                       # slot order = descending
        assert zs.min() >= np.delete(z[t], idx[t]).max()      # really the k largest
        assert np.max(np.abs(w[t] - scipy_softmax(zs))) <= 1e-15   # softmax restricted to S
    # renorm=0: plain softmax probabilities of the selected experts
    idx0, w0, _, _ = O.route_topk(z, 4, 0)
    assert np.array_equal(idx0, idx)
    p = scipy_softmax(z.astype(np.float64), axis=1)
    assert np.max(np.abs(w0 - np.take_along_axis(p, idx.astype(np.int64), axis=1))) <= 1e-15
    # counts / offsets
    assert counts.sum() == 64 * 4 and offsets[0] == 0 and offsets[-1] == 64 * 4
    assert np.all(np.diff(offsets) == counts)
    assert np.array_equal(counts, np.bincount(idx.ravel(), minlength=16))


def test_ties_go_to_lower_index():
    z = np.zeros((3, 6), dtype=np.float32)
    idx, w, _, _ = O.route_topk(z, 3)
    assert idx.tolist() == [[0, 1, 2]] * 3
    assert np.allclose(w, 1 / 3)
    # duplicated columns: the lower copy wins the last slot
    z = np.array([[1.0, 5.0, 1.0, 5.0, 0.0]], dtype=np.float32)
    idx, _, _, _ = O.route_topk(z, 3)
    assert idx.tolist() == [[1, 3, 0]]
    # signed zeros compare equal
    z = np.array([[0.0, -0.0, -1.0], [-0.0, 0.0, -1.0]], dtype=np.float32)
    idx, _, _, _ = O.route_topk(z, 1)
    assert idx.tolist() == [[0], [0]]
    # agrees with the scanning selection of the brute force
    r = np.random.default_rng(6)
    z = r.integers(-2, 3, size=(40, 9)).astype(np.float32)       # many ties
    idx, _, _, _ = O.route_topk(z, 4)
    _, chosen = B.dense_coefficients(z.tolist(), 4)
    assert idx.tolist() == chosen


# ------------------------------------------------------------------ permutation

def test_permutation_is_stable_bijection():
    r = np.random.default_rng(7)
    T, E, k, d = 50, 6, 3, 4
    z = r.standard_normal((T, E)); X = r.standard_normal((T, d))
    z[:, 4] = -100.0                                              # an empty expert
    idx, _, counts, offsets = O.route_topk(z, k)
    assert counts[4] == 0 and offsets[4] == offsets[5]
    Xp, row_of_pair, pair_of_row = O.permute(X, idx, offsets)
    P = T * k
    assert sorted(row_of_pair.tolist()) == list(range(P))
    assert np.array_equal(pair_of_row[row_of_pair], np.arange(P))
    flat = idx.ravel()
    for row in range(P):
        p = pair_of_row[row]
        e = flat[p]
        assert offsets[e] <= row < offsets[e + 1]
        assert np.array_equal(Xp[row], X[p // k])
    # stable: inside a segment the pair ids ascend; rank = number of earlier tokens choosing e
    for e in range(E):
        seg = pair_of_row[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            earlier = int(np.sum(idx[:t] == e))
            assert row_of_pair[t * k + j] == offsets[e] + earlier


def test_permute_then_combine_returns_X():
    r = np.random.default_rng(8)
    T, E, k, d = 20, 8, 4, 5
    z = r.standard_normal((T, E)); X = r.standard_normal((T, d))
    idx, w, _, offsets = O.route_topk(z, k)
    Xp, row_of_pair, _ = O.permute(X, idx, offsets)
    Y = O.unpermute_combine_fwd(Xp, np.full((T, k), 0.25), row_of_pair, T, k)
    assert np.array_equal(Y, X)
    Y = O.unpermute_combine_fwd(Xp, w, row_of_pair, T, k)
    assert np.max(np.abs(Y - X)) <= 1e-14


# ------------------------------------------------------------------ gradients

def _fd(fun, arr, h=1e-6, picks=None):
    """central differences of scalar fun() w.r.t. entries of arr (modified in place)."""
    flat = arr.reshape(-1)
    picks = range(flat.size) if picks is None else picks
    out = {}
    for i in picks:
        old = flat[i]
        flat[i] = old + h; fp = fun()
        flat[i] = old - h; fm = fun()
        flat[i] = old
        out[i] = (fp - fm) / (2 * h)
    return out


@pytest.mark.parametrize("k,renorm", [(2, 1), (3, 0), (1, 1), (4, 1)])
def test_gradients_by_finite_differences_on_brute_loss(k, renorm):
    T, d, E, f = 6, 4, 4, 5
    X, z, Wg, Wu, Wd, dY = _rand_layer(20 + k, T, d, E, f, wscale=0.7)
    fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, k, renorm)
    bwd = O.moe_layer_bwd(fwd, dY, z, Wg, Wu, Wd, renorm)
    coeff, _ = B.dense_coefficients(z.tolist(), k, renorm)        # routing frozen for X / weights
    loss = lambda: B.loss_dense(X, z, Wg, Wu, Wd, dY, k, renorm, coeff=coeff)
    r = np.random.default_rng(0)
    for name, arr, grad in (("X", X, bwd["dX"]), ("Wg", Wg, bwd["dWg"]), ("Wu", Wu, bwd["dWu"]),
                            ("Wd", Wd, bwd["dWd"])):
        picks = r.choice(arr.size, size=min(arr.size, 24), replace=False)
        fd = _fd(loss, arr, picks=picks)
        for i, v in fd.items():
            assert grad.reshape(-1)[i] == pytest.approx(v, rel=2e-6, abs=2e-7), (name, i)
    # logits: re-route on every evaluation; only tokens whose k-th / (k+1)-th gap is wide
    h = 1e-6
    loss_z = lambda: B.loss_dense(X, z, Wg, Wu, Wd, dY, k, renorm)
    zs = np.sort(z, axis=1)[:, ::-1]
    for t in range(T):
        if k < E and zs[t, k - 1] - zs[t, k] <= 10 * h:
            continue
        fd = _fd(loss_z, z, h=h, picks=[t * E + e for e in range(E)])
        for i, v in fd.items():
            assert bwd["dlogits"].reshape(-1)[i] == pytest.approx(v, rel=2e-6, abs=2e-7), ("z", i)


# ------------------------------------------------------------------ router linear, whole block

def _logits_by_loops(X, Wr):
    """z[t][e] = sum_i X[t][i] * Wr[e][i] with plain Python loops (no library product)."""
    return [[sum(float(X[t][i]) * float(Wr[e][i]) for i in range(len(X[t]))) for e in range(len(Wr))]
            for t in range(len(X))]


def test_router_linear_vs_scalar_loops():
    r = np.random.default_rng(41)
    T, d, E = 5, 7, 3
    X, Wr, dz = r.standard_normal((T, d)), r.standard_normal((E, d)), r.standard_normal((T, E))
    assert np.allclose(O.router_logits(X, Wr), np.array(_logits_by_loops(X, Wr)), rtol=1e-13, atol=1e-13)
    dXr, dWr = O.router_bwd(dz, X, Wr)
    for t in range(T):
        for i in range(d):
            assert dXr[t, i] == pytest.approx(sum(dz[t, e] * Wr[e, i] for e in range(E)), rel=1e-12, abs=1e-13)
    for e in range(E):
        for i in range(d):
            assert dWr[e, i] == pytest.approx(sum(dz[t, e] * X[t, i] for t in range(T)), rel=1e-12, abs=1e-13)
    # a one-hot upstream gradient picks one row of Wr / one row of X
    one = np.zeros((T, E)); one[2, 1] = 1.0
    dXr, dWr = O.router_bwd(one, X, Wr)
    assert np.array_equal(dXr[2], Wr[1]) and not dXr[[0, 1, 3, 4]].any()
    assert np.array_equal(dWr[1], X[2]) and not dWr[[0, 2]].any()


@pytest.mark.parametrize("k,renorm", [(2, 1), (3, 0)])
def test_whole_block_gradient_by_finite_differences(k, renorm):
    """L(X, Wr) = sum(dY * Y) with the logits recomputed from X and Wr by scalar loops and the dense
    brute-force layer on top: its finite differences w.r.t. X and Wr must equal the block backward
    (expert path + router path).  Tokens whose top-k boundary is close are left out, as the selection
    is treated as constant."""
    T, d, E, f = 6, 4, 4, 5
    X, _, Wg, Wu, Wd, dY = _rand_layer(50 + k, T, d, E, f, wscale=0.7)
    Wr = np.random.default_rng(60 + k).standard_normal((E, d))
    z = O.router_logits(X, Wr)
    zs = np.sort(z, axis=1)[:, ::-1]
    safe = [t for t in range(T) if k == E or zs[t, k - 1] - zs[t, k] > 1e-3]
    assert len(safe) >= 3
    fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, k, renorm)
    blk = O.moe_block_bwd(fwd, dY, z, X, Wr, Wg, Wu, Wd, renorm)
    assert np.allclose(blk["dX"], blk["dX_expert"] + blk["dX_router"])
    loss = lambda: B.loss_dense(X, _logits_by_loops(X, Wr), Wg, Wu, Wd, dY, k, renorm)
    fd = _fd(loss, X, picks=[t * d + i for t in safe for i in range(d)])
    for i, v in fd.items():
        assert blk["dX"].reshape(-1)[i] == pytest.approx(v, rel=5e-6, abs=5e-7), ("X", i)
    if len(safe) == T:                                   # dWr sums over every token
        fd = _fd(loss, Wr)
        for i, v in fd.items():
            assert blk["dWr"].reshape(-1)[i] == pytest.approx(v, rel=5e-6, abs=5e-7), ("Wr", i)
    # with k = 1 and renormalised weights the logits carry no gradient: the router term vanishes
    fwd1 = O.moe_layer_fwd(X, z, Wg, Wu, Wd, 1, 1)
    blk1 = O.moe_block_bwd(fwd1, dY, z, X, Wr, Wg, Wu, Wd, 1)
    assert not blk1["dX_router"].any() and not blk1["dWr"].any()


def test_dlogits_invariants_and_linearity():
    X, z, Wg, Wu, Wd, dY = _rand_layer(30, 12, 5, 6, 4)
    for renorm in (0, 1):
        fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, 3, renorm)
        bwd = O.moe_layer_bwd(fwd, dY, z, Wg, Wu, Wd, renorm)
        dz = bwd["dlogits"]
        assert np.max(np.abs(dz.sum(axis=1))) <= 1e-13 * max(1.0, np.max(np.abs(dz)))
        if renorm:
            mask = np.ones_like(dz, dtype=bool)
            np.put_along_axis(mask, fwd["topk_idx"].astype(np.int64), False, axis=1)
            assert np.all(dz[mask] == 0.0)
        bwd2 = O.moe_layer_bwd(fwd, 2.5 * dY, z, Wg, Wu, Wd, renorm)
        for key in ("dX", "dWg", "dWu", "dWd", "dlogits", "dw"):
            assert np.max(np.abs(bwd2[key] - 2.5 * bwd[key])) <= 1e-12 * max(1.0, np.max(np.abs(bwd[key])))


def test_empty_expert_gets_zero_weight_gradients():
    X, z, Wg, Wu, Wd, dY = _rand_layer(31, 10, 4, 5, 3)
    z[:, 2] = -50.0
    fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, 2)
    assert fwd["counts"][2] == 0
    bwd = O.moe_layer_bwd(fwd, dY, z, Wg, Wu, Wd)
    assert np.all(bwd["dWg"][2] == 0) and np.all(bwd["dWu"][2] == 0) and np.all(bwd["dWd"][2] == 0)


# ------------------------------------------------------------------ staged functions vs whole layer

def test_supplied_routing_and_sampled_outputs_match_whole_layer():
    X, z, Wg, Wu, Wd, dY = _rand_layer(40, 16, 5, 6, 4)
    k = 2
    fwd = O.moe_layer_fwd(X, z, Wg, Wu, Wd, k)
    bwd = O.moe_layer_bwd(fwd, dY, z, Wg, Wu, Wd)
    # the same layer seen as P pre-routed rows with k=1 and the pair's weight attached
    P = 16 * k
    Xrows = np.repeat(X, k, axis=0); dYrows = np.repeat(dY, k, axis=0)
    fwd1 = O.moe_layer_fwd(Xrows, None, Wg, Wu, Wd, 1,
                           routing=(fwd["topk_idx"].reshape(P, 1), fwd["topk_w"].reshape(P, 1)))
    Ysum = fwd1["Y"].reshape(16, k, -1).sum(axis=1)
    assert np.max(np.abs(Ysum - fwd["Y"])) <= 1e-13
    bwd1 = O.moe_layer_bwd(fwd1, dYrows, None, Wg, Wu, Wd)
    assert bwd1["dlogits"] is None
    assert np.max(np.abs(bwd1["dWd"] - bwd["dWd"])) <= 1e-12
    assert np.max(np.abs(bwd1["dX"].reshape(16, k, -1).sum(axis=1) - bwd["dX"])) <= 1e-12
    # one-by-one outputs
    for t in (0, 7, 15):
        y, dx, dw = O.token_fwd_bwd(X[t], fwd["topk_idx"][t], fwd["topk_w"][t], dY[t], Wg, Wu, Wd)
        assert np.max(np.abs(y - fwd["Y"][t])) <= 1e-13
        assert np.max(np.abs(dx - bwd["dX"][t])) <= 1e-12
        assert np.max(np.abs(dw - bwd["dw"][t])) <= 1e-12
    for e in range(6):
        g, u, dn = O.expert_weight_grads(e, X, dY, fwd["topk_idx"], fwd["topk_w"], Wg, Wu, Wd)
        assert np.max(np.abs(g - bwd["dWg"][e])) <= 1e-12
        assert np.max(np.abs(u - bwd["dWu"][e])) <= 1e-12
        assert np.max(np.abs(dn - bwd["dWd"][e])) <= 1e-12
