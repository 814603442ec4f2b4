"""Pins of the 8-bit floating-point oracle (oracle/moe_fp8.py) against what the public formats fix: listed
code points, exhaustive round trips, brute-force nearest-value search, an independent library conversion,
worked block cases, error bounds and scalar loops.  No GPU."""
import os

import numpy as np
import pytest

from oracle import moe_fp8 as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ofp8_e4m3_points.txt")


def _finite_codes():
    c = np.arange(256, dtype=np.uint8)
    return c[(c & 0x7F) != 0x7F]


def test_listed_code_points():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        code, value = line.split()
        code, value = int(code, 16), float(value)
        got = F.e4m3_decode(np.array([code], dtype=np.uint8))[0]
        assert got == value and np.signbit(got) == np.signbit(value), (hex(code), got, value)
        assert F.e4m3_encode(np.array([value]))[0] == code
        n += 1
    assert n == 13
    assert np.isnan(F.e4m3_decode(np.array([0x7F, 0xFF], dtype=np.uint8))).all()


def test_decode_structure():
    """254 finite values, symmetric, strictly increasing with the code on the positive side, 8 values per binade."""
    pos = F.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    assert np.all(np.diff(pos) > 0) and pos[0] == 0.0 and pos[-1] == 448.0
    neg = F.e4m3_decode(np.arange(0x80, 0xFF, dtype=np.uint8))
    assert np.array_equal(neg, -pos)
    for e in range(-6, 9):                             # normal binades [2^e, 2^(e+1))
        inside = pos[(pos >= 2.0 ** e) & (pos < 2.0 ** (e + 1))]
        assert len(inside) == (8 if e < 8 else 7)      # the top binade loses 480 to NaN
        assert np.allclose(np.diff(inside), 2.0 ** (e - 3), rtol=0, atol=0)
    assert np.array_equal(pos[:8], np.arange(8) * 2.0 ** -9)      # subnormals


def test_round_trip_exhaustive():
    c = _finite_codes()
    assert np.array_equal(F.e4m3_encode(F.e4m3_decode(c)), c)


def _brute_encode(x):
    """Nearest finite value by exhaustive search; among equidistant ones the even code."""
    codes = np.arange(0x7F, dtype=np.int64)
    vals = F.e4m3_decode(codes.astype(np.uint8))
    out = np.zeros(len(x), dtype=np.uint8)
    for i, v in enumerate(x):
        m = min(abs(v), 448.0)
        dist = np.abs(vals - m)
        best = np.flatnonzero(dist == dist.min())
        c = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]
        out[i] = c | (0x80 if np.signbit(v) else 0)
    return out


def test_encode_is_nearest_ties_to_even():
    rng = np.random.default_rng(5)
    pos = F.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mid = (pos[:-1] + pos[1:]) / 2                      # every tie point
    x = np.concatenate([mid, -mid, np.nextafter(mid, 0), np.nextafter(mid, 1e9), rng.uniform(-500, 500, 4000),
                        rng.uniform(-0.05, 0.05, 4000), rng.standard_normal(4000) * 8, [0.0, -0.0, 448.0, 464.0, 479.9, 1e30, -1e30]])
    assert np.array_equal(F.e4m3_encode(x), _brute_encode(x))
    # the tie points, spelled out: the result has an even mantissa
    assert np.all(F.e4m3_encode(mid) % 2 == 0)
    assert F.e4m3_encode(np.array([464.0]))[0] == 0x7E and F.e4m3_encode(np.array([1e9]))[0] == 0x7E   # saturation, no NaN
    assert F.e4m3_encode(np.array([2.0 ** -10]))[0] == 0x00 and F.e4m3_encode(np.array([1.5 * 2.0 ** -10]))[0] == 0x01


def test_encode_matches_library_conversion_in_range():
    """torch's float8_e4m3fn cast is an independent implementation of the same format (round to nearest even).
    Compared below the point where overflow handling could differ."""
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("no float8 dtype")
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.uniform(-448, 448, 20000), rng.standard_normal(20000), rng.uniform(-0.02, 0.02, 20000)]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F.e4m3_encode(x.astype(np.float64)), lib)


def test_relative_error_bound():
    rng = np.random.default_rng(2)
    x = rng.uniform(2.0 ** -6, 448, 20000) * rng.choice([-1, 1], 20000)
    q = F.e4m3_decode(F.e4m3_encode(x))
    assert np.max(np.abs(q - x) / np.abs(x)) <= 2.0 ** -4          # half a unit in the last of 3 mantissa bits


def test_mx_scale_worked_cases():
    # block maximum exactly 2^n: scale 2^(n-8), the maximum becomes 256 = code 0x78
    for n in (-20, -1, 0, 5, 30):
        v = np.zeros(32); v[3] = 2.0 ** n; v[7] = -0.75 * 2.0 ** n
        q, s = F.mx_quantise(v)
        assert s[0] == n - 8 + 127
        assert q[3] == 0x78 and F.e4m3_decode(q[7:8])[0] == -192.0
        assert np.array_equal(F.mx_dequantise(q, s), v)
    # just below a power of two: one binade lower scale, and the scaled maximum (511.99..) saturates to 448
    v = np.zeros(32); v[0] = np.nextafter(1.0, 0)
    q, s = F.mx_quantise(v)
    assert s[0] == -1 - 8 + 127 and q[0] == 0x7E
    # all-zero block: scale code 0, codes 0 (or 0x80 for negative zero)
    q, s = F.mx_quantise(np.zeros(64))
    assert not s.any() and not q.any()
    # one dominating element pushes small ones to subnormals or zero
    v = np.full(32, 2.0 ** -20); v[0] = 1.0; v[1] = 2.0 ** -12; v[2] = 2.0 ** -17; v[3] = 2.0 ** -18
    q, s = F.mx_quantise(v)                                        # scale 2^-8: 2^-12 -> 2^-4, 2^-17 -> the smallest subnormal,
    assert s[0] == 119 and q[0] == 0x78 and q[1] == 0x18 and q[2] == 0x01 and q[3] == 0x00 and np.all(q[4:] == 0)   # 2^-18 -> a tie, to even (zero)
    # clamps at both ends of the scale range
    assert F.mx_scale_code(np.array([2.0 ** -140]))[0] == 0 and F.mx_scale_code(np.array([2.0 ** 200]))[0] == 254


def test_mx_blocks_are_independent_and_along_last_axis():
    rng = np.random.default_rng(3)
    V = rng.standard_normal((5, 3, 96)) * np.exp2(rng.integers(-10, 10, (5, 3, 1)))
    q, s = F.mx_quantise(V)
    assert q.shape == V.shape and s.shape == (5, 3, 3)
    for i in range(5):
        for j in range(3):
            for b in range(3):
                qb, sb = F.mx_quantise(V[i, j, 32 * b:32 * b + 32])
                assert np.array_equal(qb, q[i, j, 32 * b:32 * b + 32]) and sb[0] == s[i, j, b]
    # scaling a block by a power of two moves only its scale
    q2, s2 = F.mx_quantise(V * 8.0)
    assert np.array_equal(q2, q) and np.array_equal(s2.astype(int), s.astype(int) + 3)
    # relative error of every block against its maximum: at most 2^-4 of the element or half a subnormal step, plus saturation (448 vs < 512)
    dq = F.mx_dequantise(q, s)
    amax = np.abs(V.reshape(5, 3, 3, 32)).max(-1, keepdims=True)
    err = np.abs(dq - V).reshape(5, 3, 3, 32)
    assert np.all(err <= np.maximum(np.abs(V.reshape(5, 3, 3, 32)) * 2.0 ** -4, amax * 2.0 ** -9 * 2) + amax * 0.125)


def test_float32_arithmetic_takes_the_same_decisions():
    """With float32 inputs the quantiser's arithmetic is exact in float32 as well (power-of-two scaling, then a single
    rounding): a float32 re-statement of the steps gives identical codes."""
    rng = np.random.default_rng(9)
    V = (rng.standard_normal((64, 128)) * np.exp2(rng.integers(-30, 30, (64, 1)))).astype(np.float32)
    q, s = F.mx_quantise(V)
    B = V.reshape(64, 4, 32)
    amax = np.abs(B).max(-1)
    eb = (amax.view(np.uint32) >> 23) & 0xFF                      # biased float32 exponent of the block maximum
    s32 = np.maximum(eb.astype(np.int64) - 8, 0)
    assert np.array_equal(s32, s)
    inv = np.exp2(127.0 - s32).astype(np.float32)
    scaled = B * inv[..., None]                                   # float32 product, exact
    assert scaled.dtype == np.float32
    assert np.array_equal(F.e4m3_encode(scaled.astype(np.float64)).reshape(64, 128), q)


def test_products_against_scalar_loops():
    rng = np.random.default_rng(4)
    E, f, d = 3, 64, 96
    offsets = np.array([0, 4, 4, 9])
    Xp = rng.standard_normal((9, d)).astype(np.float32)
    Wg = (rng.standard_normal((E, f, d)) * 0.1).astype(np.float32)
    Wu = (rng.standard_normal((E, f, d)) * 0.1).astype(np.float32)
    Wd = (rng.standard_normal((E, d, f)) * 0.1).astype(np.float32)
    r = F.ffn_fwd_fp8(Xp, Wg, Wu, Wd, offsets)
    tab = {c: float(F.e4m3_decode(np.array([c], dtype=np.uint8))[0]) for c in range(256) if (c & 0x7F) != 0x7F}

    def val(q, s, *idx):
        return tab[int(q[idx])] * 2.0 ** (int(s[idx[:-1] + (idx[-1] // 32,)]) - 127)
    for row, e in ((0, 0), (3, 0), (4, 2), (8, 2)):
        for n in (0, 17, 63):
            g = sum(val(r["Xq"], r["Xs"], row, k) * val(r["Wgq"], r["Wgs"], e, n, k) for k in range(d))
            u = sum(val(r["Xq"], r["Xs"], row, k) * val(r["Wuq"], r["Wus"], e, n, k) for k in range(d))
            a = g / (1.0 + np.exp(-g)) * u
            assert abs(a - r["A"][row, n]) <= 1e-12 * max(1.0, abs(a))
        for m in (0, 50, 95):
            y = sum(val(r["Aq"], r["As"], row, k) * val(r["Wdq"], r["Wds"], e, m, k) for k in range(f))
            assert abs(y - r["Yp"][row, m]) <= 1e-12 * max(1.0, abs(y))
    # the activation is quantised from its float32 rounding
    Aq, As = F.mx_quantise(r["A"].astype(np.float32).astype(np.float64))
    assert np.array_equal(Aq, r["Aq"]) and np.array_equal(As, r["As"])


def test_activation_is_quantised_from_its_float32_value():
    """17 + 1e-9 lies above the tie between 16 and 18 in float64 but on it in float32, where ties go to the even mantissa."""
    A = np.zeros((1, 32)); A[0, 0] = 256.0; A[0, 1] = 17.0 + 1e-9
    q64, s64 = F.mx_quantise(A)
    q32, s32 = F.quantise_activation(A)
    assert s64[0, 0] == 127 and s32[0, 0] == 127
    assert F.e4m3_decode(q64[0, 1:2])[0] == 18.0 and F.e4m3_decode(q32[0, 1:2])[0] == 16.0


def test_quantised_forward_is_close_to_the_exact_forward():
    """Sanity of the whole reading: 8-bit operands reproduce the float64 forward to a few percent."""
    from oracle import moe_oracle as O
    rng = np.random.default_rng(6)
    E, f, d, P = 4, 128, 256, 64
    offsets = np.array([0, 16, 32, 48, 64])
    Xp = rng.standard_normal((P, d)).astype(np.float32)
    Wg = (rng.standard_normal((E, f, d)) / np.sqrt(d)).astype(np.float32)
    Wu = (rng.standard_normal((E, f, d)) / np.sqrt(d)).astype(np.float32)
    Wd = (rng.standard_normal((E, d, f)) / np.sqrt(f)).astype(np.float32)
    exact = O.grouped_ffn_fwd(Xp, Wg, Wu, Wd, offsets)[3]
    q = F.ffn_fwd_fp8(Xp, Wg, Wu, Wd, offsets)["Yp"]
    rel = np.linalg.norm(q - exact) / np.linalg.norm(exact)
    assert 1e-3 < rel < 8e-2, rel
