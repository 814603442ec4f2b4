"""fp64 CPU oracle for the expert forward products with 8-bit floating-point operands.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it shares no code,
table or constant with the HIP path.

What is fixed, and by whom.  The paper trains in "mixed precision" (App. A, Table 4 caption) and
names no 8-bit format, so everything below is a reading, taken from two public standards:

  * the element format is OCP 8-bit floating point E4M3 (OFP8 specification, Table 1): 1 sign bit,
    4 exponent bits with bias 7, 3 mantissa bits; exponent field 0 holds subnormals m/8 * 2^-6;
    there are no infinities; S.1111.111 is NaN; the largest finite value is S.1111.110 = 448.
  * operands are block-scaled as in the OCP Microscaling (MX) specification, format MXFP8 (E4M3):
    every 32 consecutive elements ALONG THE REDUCTION DIMENSION share one scale 2^(s - 127) with s
    an 8-bit code (E8M0; 255 is NaN and is never produced).  A matrix entry is scale * element.

Quantising a block V of 32 real numbers (MX specification, Sec. 6.3, with its open choices fixed):

    amax  = max |V_i|
    s     = clamp(floor(log2(amax)) - 8, -127, 127) + 127      (8 = exponent of E4M3's largest binade;
                                                                 amax = 0 gives s = 0)
    q_i   = E4M3( V_i / 2^(s - 127) )    rounded to nearest, ties to the even mantissa, and SATURATED:
                                         magnitudes beyond 448 become 448 (the specification leaves the
                                         overflow behaviour to the implementation; scaled magnitudes
                                         lie below 512, so only (448, 512) is affected)

The division by a power of two is exact, so the only rounding is the one to E4M3; with inputs that are
exactly representable in float32 a float32 implementation takes identical decisions, and codes and
scales can be compared bit for bit.

The forward products with such operands (Sec. 3.2.5 SwiGLU expert; App. B.6 stacked weights):

    G = dq(Xq) dq(Wgq[e])^T,  U = dq(Xq) dq(Wuq[e])^T,  A = silu(G) * U
    Aq = quantise(A rounded to float32) along f       (the kernel holds A in float32 when it quantises)
    Yp = dq(Aq) dq(Wdq[e])^T

with X and W_gate/W_up quantised along d and W_down along f.  Products of dequantised values are formed
in float64 here: every partial product is exact in float64 and so is any sum the sizes used here produce
to well below the comparison tolerance.

Pins (tests/test_oracle_fp8.py): the code points the OFP8 table lists, exhaustive decode/encode round trip,
brute-force nearest-value search with ties-to-even over dense samples, saturation, an independent
float8 conversion of a library (torch.float8_e4m3fn) inside its range, exact powers of two, the MX worked
cases (block maximum exactly a power of two, all-zero block, one element dominating), error bounds
(relative error at most 2^-4 for normal results), and the dequantised product against a per-element scalar loop.
"""
import numpy as np

BLOCK = 32                 # elements per scale, MX specification
E4M3_MAX = 448.0           # S.1111.110
E4M3_EMAX = 8              # 448 = 1.75 * 2^8
E4M3_BIAS = 7


def e4m3_decode(codes):
    """Value of each E4M3 code (uint8) as float64; the two NaN codes give NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    sub = m / 8.0 * 2.0 ** (1 - E4M3_BIAS)
    nor = (1.0 + m / 8.0) * np.exp2((e - E4M3_BIAS).astype(np.float64))
    v = sign * np.where(e == 0, sub, nor)
    return np.where((c & 0x7F) == 0x7F, np.nan, v)


def _positive_table():
    """The 127 non-negative finite values in code order (code 0x00 .. 0x7E); value grows with the code."""
    t = e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    assert np.all(np.diff(t) > 0)
    return t


def e4m3_encode(x):
    """Nearest E4M3 code of each real x: ties go to the code with an even mantissa (= the even code, since
    value grows with the code), magnitudes above 448 saturate to 448, the sign bit is kept (also for zero)."""
    x = np.asarray(x, dtype=np.float64)
    assert not np.isnan(x).any()
    tab = _positive_table()
    mag = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.clip(np.searchsorted(tab, mag, side="left"), 1, len(tab) - 1)   # tab[hi-1] <= mag <= tab[hi] (or mag == 0)
    lo = hi - 1
    d_lo = mag - tab[lo]
    d_hi = tab[hi] - mag
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return (code | np.where(np.signbit(x), 0x80, 0).astype(np.uint8)).astype(np.uint8)


def mx_scale_code(amax):
    """E8M0 code of the shared scale of blocks whose largest magnitude is amax (array, float64)."""
    amax = np.asarray(amax, dtype=np.float64)
    frac, exp = np.frexp(amax)                        # amax = frac * 2^exp, frac in [0.5, 1): floor(log2) = exp - 1
    shared = np.clip(exp - 1 - E4M3_EMAX, -127, 127)
    return np.where(amax > 0, shared + 127, 0).astype(np.uint8)


def mx_quantise(V):
    """Blocks of 32 along the last axis.  Returns (codes uint8 [..., K], scale codes uint8 [..., K/32])."""
    V = np.asarray(V, dtype=np.float64)
    K = V.shape[-1]
    assert K % BLOCK == 0
    B = V.reshape(V.shape[:-1] + (K // BLOCK, BLOCK))
    s = mx_scale_code(np.abs(B).max(axis=-1))
    scaled = B / np.exp2(s.astype(np.float64) - 127.0)[..., None]
    return e4m3_encode(scaled).reshape(V.shape), s


def mx_dequantise(codes, scales):
    """scale * element as float64; inverse layout of mx_quantise."""
    codes = np.asarray(codes, dtype=np.uint8)
    K = codes.shape[-1]
    B = e4m3_decode(codes).reshape(codes.shape[:-1] + (K // BLOCK, BLOCK))
    return (B * np.exp2(np.asarray(scales, dtype=np.float64) - 127.0)[..., None]).reshape(codes.shape)


def silu(g):
    return g / (1.0 + np.exp(-g))


def gate_up_fp8(Xq, Xs, Wgq, Wgs, Wuq, Wus, offsets):
    """A = silu(G) * U in float64 from quantised operands (rows in expert order, weights [E, f, d])."""
    X = mx_dequantise(Xq, Xs)
    P, f = X.shape[0], Wgq.shape[1]
    A = np.zeros((P, f))
    for e in range(Wgq.shape[0]):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b > a:
            G = X[a:b] @ mx_dequantise(Wgq[e], Wgs[e]).T
            U = X[a:b] @ mx_dequantise(Wuq[e], Wus[e]).T
            A[a:b] = silu(G) * U
    return A


def down_fp8(Aq, As, Wdq, Wds, offsets):
    """Yp = dq(Aq) dq(Wdq[e])^T in float64 (weights [E, d, f])."""
    A = mx_dequantise(Aq, As)
    Yp = np.zeros((A.shape[0], Wdq.shape[1]))
    for e in range(Wdq.shape[0]):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b > a:
            Yp[a:b] = A[a:b] @ mx_dequantise(Wdq[e], Wds[e]).T
    return Yp


def quantise_activation(A):
    """The activation as the second product receives it: rounded to float32 (the precision in which the
    kernel holds it), then MX-quantised along f."""
    return mx_quantise(np.asarray(A, dtype=np.float64).astype(np.float32).astype(np.float64))


def ffn_fwd_fp8(Xp, Wg, Wu, Wd, offsets):
    """The whole expert forward with 8-bit operands from unquantised inputs.  Returns a dict with every
    quantised operand, the float64 activation A and the result Yp."""
    Xq, Xs = mx_quantise(Xp)
    Wgq, Wgs = mx_quantise(Wg)
    Wuq, Wus = mx_quantise(Wu)
    Wdq, Wds = mx_quantise(Wd)
    A = gate_up_fp8(Xq, Xs, Wgq, Wgs, Wuq, Wus, offsets)
    Aq, As = quantise_activation(A)
    Yp = down_fp8(Aq, As, Wdq, Wds, offsets)
    return dict(Xq=Xq, Xs=Xs, Wgq=Wgq, Wgs=Wgs, Wuq=Wuq, Wus=Wus, Wdq=Wdq, Wds=Wds, A=A, Aq=Aq, As=As, Yp=Yp)
