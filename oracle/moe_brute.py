"""Brute-force dense evaluation of the top-k SwiGLU mixture-of-experts layer, for tiny inputs.

TEST INFRASTRUCTURE ONLY (never imported by the product path).  This is the pin for
oracle/moe_oracle.py: it shares no code with it, uses no permutation, no offsets and no
sorting routine.  Every expert is evaluated for every token and the result is masked by a
dense coefficient matrix c[t, e] (= the combine weight if e was selected, else 0), i.e.
the textbook statement  Y[t] = sum_e c[t,e] * FFN_e(X[t])  of a sparsely activated
mixture (Sec. 3.2.3), with FFN_e the SwiGLU block (Sec. 3.2.5) on the stacked expert
weights (App. B.6).

`dense_coefficients` and `layer_dense` use Python scalar loops throughout (math.exp on
Python floats); `layer_dense_matvec` does the same with a library mat-vec per (token,
expert) so that the largest parity configuration is still feasible.
"""
import math


def dense_coefficients(logits, k, renorm=1):
    """c[t][e] and the selected list per token, by repeated scanning for the maximum.

    Selection: scan e = 0..E-1 and keep the first strictly larger value, k times over the
    not-yet-taken experts, so equal logits go to the lower index."""
    T = len(logits)
    coeff, chosen = [], []
    for t in range(T):
        z = [float(v) for v in logits[t]]
        E = len(z)
        taken = [False] * E
        sel = []
        for _ in range(k):
            best = -1
            for e in range(E):
                if taken[e]:
                    continue
                if best < 0 or z[e] > z[best]:
                    best = e
            taken[best] = True
            sel.append(best)
        m = max(z)
        ex = [math.exp(v - m) for v in z]
        den_all = math.fsum(ex)
        den_sel = math.fsum(ex[e] for e in sel)
        row = [0.0] * E
        for e in sel:
            row[e] = ex[e] / (den_sel if renorm else den_all)
        coeff.append(row)
        chosen.append(sel)
    return coeff, chosen


def _ffn_scalar(x, wg, wu, wd):
    f = len(wg); d = len(x)
    a = []
    for i in range(f):
        g = 0.0; u = 0.0
        for c in range(d):
            g += float(wg[i][c]) * float(x[c])
            u += float(wu[i][c]) * float(x[c])
        a.append(g / (1.0 + math.exp(-g)) * u)
    out = []
    for r in range(len(wd)):
        s = 0.0
        for i in range(f):
            s += float(wd[r][i]) * a[i]
        out.append(s)
    return out


def layer_dense(X, logits, Wg, Wu, Wd, k, renorm=1):
    """Y as nested Python lists; every expert evaluated for every token."""
    coeff, _ = dense_coefficients(logits, k, renorm)
    T = len(X); E = len(Wg); d = len(X[0])
    Y = []
    for t in range(T):
        acc = [0.0] * d
        for e in range(E):
            h = _ffn_scalar(X[t], Wg[e], Wu[e], Wd[e])
            for c in range(d):
                acc[c] += coeff[t][e] * h[c]
        Y.append(acc)
    return Y


def layer_dense_matvec(X, logits, Wg, Wu, Wd, k, renorm=1):
    """Same dense evaluation with numpy mat-vecs per (token, expert)."""
    import numpy as np
    coeff, _ = dense_coefficients(logits, k, renorm)
    X = np.asarray(X, dtype=np.float64)
    T, d = X.shape
    E = len(Wg)
    Y = np.zeros((T, d))
    for t in range(T):
        for e in range(E):
            g = np.asarray(Wg[e], dtype=np.float64) @ X[t]
            u = np.asarray(Wu[e], dtype=np.float64) @ X[t]
            a = g / (1.0 + np.exp(-g)) * u
            Y[t] += coeff[t][e] * (np.asarray(Wd[e], dtype=np.float64) @ a)
    return Y


def loss_dense(X, logits, Wg, Wu, Wd, dY, k, renorm=1, coeff=None):
    """L = sum(dY * Y) with the dense evaluation; `coeff`, if given, freezes the dense
    coefficient matrix (used by finite differences that must not re-route)."""
    import numpy as np
    X = np.asarray(X, dtype=np.float64); dY = np.asarray(dY, dtype=np.float64)
    if coeff is None:
        coeff, _ = dense_coefficients(logits, k, renorm)
    coeff = np.asarray(coeff, dtype=np.float64)
    T, d = X.shape
    E = len(Wg)
    L = 0.0
    for e in range(E):
        rows = np.nonzero(coeff[:, e])[0]
        if rows.size == 0:
            continue
        g = X[rows] @ np.asarray(Wg[e], dtype=np.float64).T
        u = X[rows] @ np.asarray(Wu[e], dtype=np.float64).T
        a = g / (1.0 + np.exp(-g)) * u
        h = a @ np.asarray(Wd[e], dtype=np.float64).T
        L += float(np.sum(coeff[rows, e][:, None] * h * dY[rows]))
    return L
