"""fp64 CPU oracle for one GPU's share of a top-k routed SwiGLU mixture-of-experts layer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its Python
binding, the timed legs of the benchmark) may import this module; it exists so that
tests, the smoke check and the benchmark's CPU-baseline leg have an independent,
plain statement of what the layer computes.  It shares no code with the HIP path.

What the paper fixes (Sec. 3.2.3, Sec. 3.2.5 "Efficient Kernels", App. B.6 listing of the
expert-parallel plan): tokens are routed to a sparse subset of experts; each expert is a
SwiGLU feed-forward block; the experts' three projections are stored as stacked,
expert-major tensors gate_proj / up_proj / down_proj (dim 0 = expert).  The paper gives
no formula, so the definition written out here is the standard dropless top-k MoE:

    S(t)    = the k experts with the largest router logit z[t, :], ordered by
              (logit descending, expert index ascending); slot j is the j-th of them
    p       = softmax(z[t, :]) over all E experts
    w[t, j] = p[e_j] / sum_{m<k} p[e_m]      (renorm=1)      or  p[e_j]   (renorm=0)
    FFN_e(x)= W_down[e] @ ( silu(W_gate[e] @ x) * (W_up[e] @ x) ),  silu(g) = g / (1 + exp(-g))
    Y[t]    = sum_j w[t, j] * FFN_{e_j}(X[t])

Weight layout (a reading; the paper fixes only dim 0): W_gate, W_up : [E, f, d];
W_down : [E, d, f]  ("out-features x in-features").

The permutation into expert-contiguous rows is an exact re-ordering of that definition;
the functions below expose each stage (route, permute, grouped FFN, combine and their
backward) so that each library call can be checked on its own with oracle-made inputs.
All arithmetic is float64; inputs are taken as given (already rounded to the dtype the
GPU receives) and nothing is rounded afterwards.

Pins (tests/test_oracle_*.py): dense brute-force evaluation (oracle/moe_brute.py),
closed forms and special cases (identical experts -> plain SwiGLU MLP, k=1 -> w=1 and
dz=0, k=E -> full softmax mixture), permutation bijection, weight sums, central finite
differences for every gradient (the router linear and the whole-block gradient included:
finite differences of the loss through the logits with the selection held fixed, and scalar
loops).  No function here is "parity unpinned"; what stays
unpinned is only whether the paper's own model renormalises and its weight dims 1-2,
because the paper does not say.
"""
import numpy as np


# --------------------------------------------------------------------------- routing

def route_topk(logits, k, renorm=1):
    """Top-k routing of `logits` [T, E] (Sec. 3.2.3: tokens are routed to their experts).

    Selection is on the raw logits; ties go to the lower expert index.  Returns
    topk_idx [T,k] int32 (slot order = logit descending, index ascending),
    topk_w [T,k] float64, counts [E] int32, offsets [E+1] int32 (exclusive scan).
    """
    z = np.asarray(logits, dtype=np.float64)
    T, E = z.shape
    assert 1 <= k <= E
    # stable sort of -z: descending value, equal values keep ascending index
    order = np.argsort(-z, axis=1, kind="stable")
    idx = order[:, :k]
    zmax = z.max(axis=1, keepdims=True) if T else z[:, :1]
    ez = np.exp(z - zmax)
    p = ez / ez.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx, axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    counts = np.bincount(idx.reshape(-1), minlength=E).astype(np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return idx.astype(np.int32), w, counts, offsets


def counts_offsets(topk_idx, E):
    """Per-expert pair counts and their exclusive scan for a given assignment."""
    counts = np.bincount(np.asarray(topk_idx).reshape(-1), minlength=E).astype(np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return counts, offsets


def permute_maps(topk_idx, offsets):
    """Stable expert-major order of the P = T*k (token, slot) pairs.

    row_of_pair[t*k+j] = offsets[e] + #{pairs p' < t*k+j with the same expert e};
    pair_of_row is the inverse map.
    """
    flat = np.asarray(topk_idx).reshape(-1)
    P = flat.size
    pair_of_row = np.argsort(flat, kind="stable").astype(np.int32)
    row_of_pair = np.empty(P, dtype=np.int32)
    row_of_pair[pair_of_row] = np.arange(P, dtype=np.int32)
    # the segment of expert e must start at offsets[e]
    if P:
        e_sorted = flat[pair_of_row]
        assert np.all(np.arange(P) >= np.asarray(offsets)[e_sorted])
        assert np.all(np.arange(P) < np.asarray(offsets)[e_sorted + 1])
    return row_of_pair, pair_of_row


def permute(X, topk_idx, offsets):
    """Gather token rows into expert-contiguous order: Xp[row_of_pair[t*k+j]] = X[t]."""
    X = np.asarray(X, dtype=np.float64)
    T, k = np.asarray(topk_idx).shape
    row_of_pair, pair_of_row = permute_maps(topk_idx, offsets)
    Xp = X[pair_of_row // k] if T else np.zeros((0, X.shape[1]))
    return Xp, row_of_pair, pair_of_row


# --------------------------------------------------------------------------- experts

def silu(g):
    return g / (1.0 + np.exp(-g))


def silu_grad(g):
    s = 1.0 / (1.0 + np.exp(-g))
    return s * (1.0 + g * (1.0 - s))


def grouped_ffn_fwd(Xp, Wg, Wu, Wd, offsets):
    """Per expert e, on rows offsets[e]..offsets[e+1]: G = Xp Wg[e]^T, U = Xp Wu[e]^T,
    A = silu(G) * U, Yp = A Wd[e]^T  (SwiGLU expert, Sec. 3.2.5; stacked weights, App. B.6)."""
    Xp = np.asarray(Xp, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64)
    Wu = np.asarray(Wu, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    E, f, d = Wg.shape
    P = Xp.shape[0]
    G = np.zeros((P, f)); U = np.zeros((P, f)); A = np.zeros((P, f)); Yp = np.zeros((P, d))
    for e in range(E):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b == a:
            continue
        G[a:b] = Xp[a:b] @ Wg[e].T
        U[a:b] = Xp[a:b] @ Wu[e].T
        A[a:b] = silu(G[a:b]) * U[a:b]
        Yp[a:b] = A[a:b] @ Wd[e].T
    return G, U, A, Yp


def grouped_ffn_bwd(dYp, Xp, G, U, A, Wg, Wu, Wd, offsets):
    """Backward of grouped_ffn_fwd.  Returns dXp, dWg, dWu, dWd; experts with no rows
    get zero weight gradients."""
    dYp = np.asarray(dYp, dtype=np.float64); Xp = np.asarray(Xp, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64); U = np.asarray(U, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64); Wu = np.asarray(Wu, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    E, f, d = Wg.shape
    dXp = np.zeros_like(Xp)
    dWg = np.zeros_like(Wg); dWu = np.zeros_like(Wu); dWd = np.zeros_like(Wd)
    for e in range(E):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b == a:
            continue
        dA = dYp[a:b] @ Wd[e]                    # [M, f]
        dWd[e] = dYp[a:b].T @ A[a:b]             # [d, f]
        dG = dA * U[a:b] * silu_grad(G[a:b])
        dU = dA * silu(G[a:b])
        dWg[e] = dG.T @ Xp[a:b]                  # [f, d]
        dWu[e] = dU.T @ Xp[a:b]
        dXp[a:b] = dG @ Wg[e] + dU @ Wu[e]
    return dXp, dWg, dWu, dWd


# --------------------------------------------------------------------------- combine

def unpermute_combine_fwd(Yp, topk_w, row_of_pair, T, k):
    """Y[t] = sum_j w[t,j] * Yp[row_of_pair[t*k+j]];  topk_w=None means all weights 1."""
    Yp = np.asarray(Yp, dtype=np.float64)
    rows = np.asarray(row_of_pair).reshape(T, k)
    w = np.ones((T, k)) if topk_w is None else np.asarray(topk_w, dtype=np.float64)
    Y = np.zeros((T, Yp.shape[1]))
    for j in range(k):
        Y += w[:, j:j + 1] * Yp[rows[:, j]]
    return Y


def unpermute_combine_bwd(dY, Yp, topk_w, row_of_pair, T, k):
    """dYp[row] = w[t,j] * dY[t];  dw[t,j] = <dY[t], Yp[row]>."""
    dY = np.asarray(dY, dtype=np.float64); Yp = np.asarray(Yp, dtype=np.float64)
    rows = np.asarray(row_of_pair).reshape(T, k)
    w = np.asarray(topk_w, dtype=np.float64)
    dYp = np.zeros_like(Yp)
    dw = np.zeros((T, k))
    for j in range(k):
        dYp[rows[:, j]] = w[:, j:j + 1] * dY
        dw[:, j] = np.einsum("td,td->t", dY, Yp[rows[:, j]])
    return dYp, dw


def route_topk_bwd(dw, topk_w, topk_idx, logits, E, renorm=1):
    """Gradient of the combine weights w.r.t. the router logits (selection held fixed).

    renorm=1: w = softmax of z restricted to S, so dz[e_j] = w_j (dw_j - sum_m w_m dw_m)
    and dz = 0 outside S.  renorm=0: w_j = p[e_j] with p the full softmax, so
    dz[e] = p_e (1[e in S] dw_e - sum_{m in S} p_m dw_m) for every e.
    """
    dw = np.asarray(dw, dtype=np.float64); w = np.asarray(topk_w, dtype=np.float64)
    idx = np.asarray(topk_idx)
    T, k = idx.shape
    dz = np.zeros((T, E))
    s = (w * dw).sum(axis=1, keepdims=True)
    if renorm:
        np.put_along_axis(dz, idx, w * (dw - s), axis=1)
    else:
        z = np.asarray(logits, dtype=np.float64)
        ez = np.exp(z - z.max(axis=1, keepdims=True))
        p = ez / ez.sum(axis=1, keepdims=True)
        dz = -p * s
        np.put_along_axis(dz, idx, w * (dw - s), axis=1)
    return dz


# --------------------------------------------------------------------------- whole layer

def moe_layer_fwd(X, logits, Wg, Wu, Wd, k, renorm=1, routing=None):
    """Whole forward.  `routing`, if given, is (topk_idx, topk_w) supplied from outside
    (the pre-routed expert-parallel share: every row already carries its local expert
    and its globally renormalised weight); then `logits` is ignored."""
    E = np.asarray(Wg).shape[0]
    if routing is None:
        idx, w, counts, offsets = route_topk(logits, k, renorm)
    else:
        idx, w = routing
        idx = np.asarray(idx, dtype=np.int32); w = np.asarray(w, dtype=np.float64)
        counts, offsets = counts_offsets(idx, E)
    T, kk = idx.shape
    Xp, row_of_pair, pair_of_row = permute(X, idx, offsets)
    G, U, A, Yp = grouped_ffn_fwd(Xp, Wg, Wu, Wd, offsets)
    Y = unpermute_combine_fwd(Yp, w, row_of_pair, T, kk)
    return dict(topk_idx=idx, topk_w=w, counts=counts, offsets=offsets, Xp=Xp,
                row_of_pair=row_of_pair, pair_of_row=pair_of_row, G=G, U=U, A=A, Yp=Yp, Y=Y)


def moe_layer_bwd(fwd, dY, logits, Wg, Wu, Wd, renorm=1):
    """Whole backward for L = sum(dY * Y).  dX is the expert-path gradient only (the
    router-linear term dz @ W_r^T is outside this path); dlogits is None when the routing
    was supplied from outside."""
    idx = fwd["topk_idx"]; w = fwd["topk_w"]
    T, k = idx.shape
    E = np.asarray(Wg).shape[0]
    dYp, dw = unpermute_combine_bwd(dY, fwd["Yp"], w, fwd["row_of_pair"], T, k)
    dXp, dWg, dWu, dWd = grouped_ffn_bwd(dYp, fwd["Xp"], fwd["G"], fwd["U"], fwd["A"],
                                         Wg, Wu, Wd, fwd["offsets"])
    dX = unpermute_combine_fwd(dXp, None, fwd["row_of_pair"], T, k)
    dlogits = None if logits is None else route_topk_bwd(dw, w, idx, logits, E, renorm)
    return dict(dYp=dYp, dw=dw, dXp=dXp, dWg=dWg, dWu=dWu, dWd=dWd, dX=dX, dlogits=dlogits)


# --------------------------------------------------------------------------- router linear
# The router that produces the logits is a bias-free linear map of the hidden state (Sec. 3.2.3
# speaks only of "routing"; a linear gate is the standard reading).  Weight layout, again a
# reading: W_router [E, d] ("out-features x in-features"), row e = the gate vector of expert e.

def router_logits(X, Wr):
    """z[t, e] = <X[t, :], Wr[e, :]>."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(Wr, dtype=np.float64).T


def router_bwd(dlogits, X, Wr):
    """Backward of router_logits for an upstream dlogits [T, E]:
    dWr[e, :] = sum_t dlogits[t, e] X[t, :];   dX_router[t, :] = sum_e dlogits[t, e] Wr[e, :]."""
    dz = np.asarray(dlogits, dtype=np.float64)
    dWr = dz.T @ np.asarray(X, dtype=np.float64)
    dXr = dz @ np.asarray(Wr, dtype=np.float64)
    return dXr, dWr


def moe_block_bwd(fwd, dY, logits, X, Wr, Wg, Wu, Wd, renorm=1):
    """Backward of the whole block, hidden state in to hidden-state gradient out, for
    L = sum(dY * Y) with logits = router_logits(X, Wr): the layer backward plus the router
    term.  The top-k selection is treated as constant.  Returns the layer's dict with dX
    replaced by the full gradient, plus dX_expert, dX_router and dWr."""
    out = moe_layer_bwd(fwd, dY, logits, Wg, Wu, Wd, renorm)
    dXr, dWr = router_bwd(out["dlogits"], X, Wr)
    out["dX_expert"] = out["dX"]
    out["dX_router"] = dXr
    out["dX"] = out["dX"] + dXr
    out["dWr"] = dWr
    return out


# --------------------------------------------------------------------------- sampled outputs
# For sizes where the whole layer takes minutes on a CPU, single outputs computed one by
# one straight from the definition.

def token_fwd_bwd(x, idx_t, w_t, dy, Wg, Wu, Wd):
    """For one token: y = sum_j w_j FFN_{e_j}(x), dx (expert path), dw_j = <dy, FFN_{e_j}(x)>."""
    x = np.asarray(x, dtype=np.float64); dy = np.asarray(dy, dtype=np.float64)
    y = np.zeros_like(dy); dx = np.zeros_like(x); dw = np.zeros(len(idx_t))
    for j, e in enumerate(idx_t):
        wg = np.asarray(Wg[e], dtype=np.float64); wu = np.asarray(Wu[e], dtype=np.float64)
        wd = np.asarray(Wd[e], dtype=np.float64)
        g = wg @ x; u = wu @ x
        a = silu(g) * u
        h = wd @ a
        y += w_t[j] * h
        dw[j] = dy @ h
        da = wd.T @ (w_t[j] * dy)
        dg = da * u * silu_grad(g); du = da * silu(g)
        dx += wg.T @ dg + wu.T @ du
    return y, dx, dw


def expert_weight_grads(e, X, dY, topk_idx, topk_w, Wg, Wu, Wd):
    """dWg[e], dWu[e], dWd[e] from all tokens routed to expert e, straight from the definition."""
    idx = np.asarray(topk_idx)
    tok, slot = np.nonzero(idx == e)
    f, d = np.asarray(Wg[e]).shape
    if tok.size == 0:
        return np.zeros((f, d)), np.zeros((f, d)), np.zeros((d, f))
    x = np.asarray(X[tok], dtype=np.float64)
    dyp = np.asarray(topk_w, dtype=np.float64)[tok, slot][:, None] * np.asarray(dY[tok], dtype=np.float64)
    wg = np.asarray(Wg[e], dtype=np.float64); wu = np.asarray(Wu[e], dtype=np.float64)
    wd = np.asarray(Wd[e], dtype=np.float64)
    g = x @ wg.T; u = x @ wu.T
    a = silu(g) * u
    da = dyp @ wd
    dg = da * u * silu_grad(g); du = da * silu(g)
    return dg.T @ x, du.T @ x, dyp.T @ a
