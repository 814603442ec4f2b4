"""GPU parity of the 8-bit (MXFP8) forward products against oracle/moe_fp8.py, through the C ABI.

The quantiser is exact arithmetic followed by one rounding, so its codes and scales are compared bit for bit.
The products are compared on operands quantised by the ORACLE (both sides consume identical codes and scales):
the activation codes may differ from the oracle's where the kernel's fp32 activation and the oracle's fp64 one
fall on different sides of a rounding boundary, so they are compared as values -- never more than one E4M3 step
of their block apart, and identical for all but a small fraction.  The second product is checked sharply on its own
entry point with the oracle's activation codes (Yp within the bf16 tolerance, element by element); the Yp of the fused
call inherits the differing activation codes, each of which moves an output by up to one E4M3 step of one term, so it is
held to a norm-wise bound (relative Frobenius error 5e-3) and a loose element-wise one."""
import sys

import numpy as np
import pytest

from oracle import moe_fp8 as F
from oracle import moe_oracle as O
from paper_2508_02317_amd.inputs import CONFIGS, make_inputs, scaled
from tests.util import TOL, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True, file=sys.stderr)


def pack_scales(s):
    """oracle scale codes [rows, K/32] uint8 -> the library's words [K/128, rows] int32 (byte j = block 4 g + j)."""
    rows, nb = s.shape
    words = np.ascontiguousarray(s.reshape(rows, nb // 4, 4)).view("<u4")[..., 0]
    return np.ascontiguousarray(words.T).view(np.int32)


def unpack_scales(w):
    """inverse of pack_scales: int32 [K/128, rows] -> uint8 [rows, K/32]"""
    g, rows = w.shape
    return np.ascontiguousarray(np.ascontiguousarray(w).view(np.uint32).T).view(np.uint8).reshape(rows, g * 4)


def test_pack_helpers_round_trip():
    s = np.arange(6 * 8, dtype=np.uint8).reshape(6, 8)
    assert np.array_equal(unpack_scales(pack_scales(s)), s)
    assert pack_scales(s)[1, 2] == int.from_bytes(bytes(s[2, 4:8]), "little")


@pytest.mark.parametrize("rows,K,seed", [(1, 128, 0), (77, 256, 1), (300, 384, 2), (1000, 2048, 3)])
def test_quantiser_bit_exact(rows, K, seed):
    import torch
    from paper_2508_02317_amd import libmoe as L
    rng = np.random.default_rng(seed)
    V = rng.standard_normal((rows, K)) * np.exp2(rng.integers(-40, 40, (rows, K // 32)).repeat(32, axis=1).astype(np.float64))
    V[0, :32] = 0.0                                       # an all-zero block
    if rows > 2:
        V[1, :32] = 0.0; V[1, 5] = 2.0 ** -3              # block maximum a power of two
        V[2, :32] = 0.25; V[2, 7] = -np.nextafter(np.float32(1.0), np.float32(0))   # scaled maximum just below 512: saturates
        V[2, 40:44] = [17.0, 18.0, 19.0, 0.0]             # (second block) ties between neighbouring codes
    src = torch.from_numpy(V.astype(np.float32)).cuda().to(torch.bfloat16)
    Vb = src.float().cpu().numpy().astype(np.float64)     # what the kernel receives
    say("mx8 quantise rows=%d K=%d" % (rows, K))
    codes, scales = L.moe_mx8_quantise(src)
    torch.cuda.synchronize()
    q_ref, s_ref = F.mx_quantise(Vb)
    assert np.array_equal(unpack_scales(to_np(scales)), s_ref)
    assert np.array_equal(to_np(codes), q_ref)


def _case(T, d, E, k, f, seed):
    cfg = scaled(CONFIGS["a3b_8k"], T=T, d=d, E=E, k=k, f=f, seed=seed)
    inp = make_inputs(cfg)
    idx, w, counts, offsets = O.route_topk(inp["logits"], k, 1)
    row_of_pair, pair_of_row = O.permute_maps(idx, offsets)
    return cfg, inp, offsets.astype(np.int32), pair_of_row.astype(np.int32)


FUSED_YP_FRO, FUSED_YP_MAX = 5e-3, 6e-2


def fro_err(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return np.linalg.norm(got - ref) / np.linalg.norm(ref)


def _step_of_block(scales):
    """one E4M3 step at the top binade of each block's range, as a value: 32 * 2^(s-127) (spacing of codes in [256, 448])"""
    return 32.0 * np.exp2(scales.astype(np.float64) - 127.0)


def _compare_forward(cfg, inp, offsets, pair_of_row, gather):
    import torch
    from paper_2508_02317_amd import libmoe as L
    k = cfg.k
    X = inp["X"].astype(np.float64)
    Xq, Xs = F.mx_quantise(X)                              # by token
    Wgq, Wgs = F.mx_quantise(inp["Wg"]); Wuq, Wus = F.mx_quantise(inp["Wu"]); Wdq, Wds = F.mx_quantise(inp["Wd"])
    tok = pair_of_row // k
    A = F.gate_up_fp8(Xq[tok], Xs[tok], Wgq, Wgs, Wuq, Wus, offsets)
    Aq, As = F.quantise_activation(A)
    Yp = F.down_fp8(Aq, As, Wdq, Wds, offsets)
    E, f, d = inp["Wg"].shape
    dev = lambda a: to_dev(np.ascontiguousarray(a))
    wargs = (dev(Wgq), dev(pack_scales(Wgs.reshape(E * f, -1))), dev(Wuq), dev(pack_scales(Wus.reshape(E * f, -1))),
             dev(Wdq), dev(pack_scales(Wds.reshape(E * d, -1))))
    if gather:
        actq, acts, yp = L.moe_grouped_gemm_swiglu_fwd_mx8(dev(Xq), dev(pack_scales(Xs)), *wargs, dev(offsets), pair_of_row=dev(pair_of_row), k=k)
    else:
        actq, acts, yp = L.moe_grouped_gemm_swiglu_fwd_mx8(dev(Xq[tok]), dev(pack_scales(Xs[tok])), *wargs, dev(offsets))
    torch.cuda.synchronize()
    got_s = unpack_scales(to_np(acts))
    got_q = to_np(actq)
    same_scale = got_s == As
    frac_scale = 1.0 - same_scale.mean()
    got_A = F.mx_dequantise(got_q, got_s)
    ref_A = F.mx_dequantise(Aq, As)
    step = np.maximum(_step_of_block(got_s), _step_of_block(As)).repeat(32, axis=1)
    worst = np.max(np.abs(got_A - ref_A) / step)
    frac_code = np.mean((got_q != Aq) | ~same_scale.repeat(32, axis=1))
    err_a = rel_err(got_A, A)                              # against the unquantised activation: the quantisation error itself
    err_y, fro_y = rel_err(to_np(yp), Yp), fro_err(to_np(yp), Yp)
    yp2 = L.moe_grouped_gemm_down_mx8(dev(Aq), dev(pack_scales(As)), wargs[4], wargs[5], dev(offsets))     # the oracle's codes in
    torch.cuda.synchronize()
    err_y2 = rel_err(to_np(yp2), Yp)
    say("  gather=%s: act scales differing %.2e, codes differing %.2e, worst |dA| = %.2f steps, act vs fp64 act %.2e, "
        "Yp fused max %.2e fro %.2e, Yp of the second product alone %.2e" % (gather, frac_scale, frac_code, worst, err_a, err_y, fro_y, err_y2))
    assert frac_scale <= 1e-3 and frac_code <= 5e-3
    assert worst <= 1.0 + 1e-9
    assert err_a <= 0.125 + 1e-3                           # the format's bound: saturation of a scaled maximum just below 512 to 448
    assert err_y2 <= TOL["bf16"]
    assert fro_y <= FUSED_YP_FRO and err_y <= FUSED_YP_MAX
    return to_np(actq), to_np(acts), to_np(yp)


@pytest.mark.parametrize("T,d,E,k,f,seed", [(64, 128, 2, 1, 128, 0), (300, 256, 5, 2, 384, 1), (777, 384, 16, 2, 256, 2), (1500, 512, 4, 4, 768, 3)])
def test_forward_products(T, d, E, k, f, seed):
    cfg, inp, offsets, pair_of_row = _case(T, d, E, k, f, seed)
    say("mx8 forward T=%d d=%d E=%d k=%d f=%d counts=%s" % (T, d, E, k, f, np.diff(offsets).tolist()))
    a = _compare_forward(cfg, inp, offsets, pair_of_row, gather=False)
    b = _compare_forward(cfg, inp, offsets, pair_of_row, gather=True)
    for x, y in zip(a, b):                                 # reading rows by token changes nothing
        assert np.array_equal(x, y)


def test_forward_with_empty_experts_and_single_rows():
    cfg, inp, _, _ = _case(40, 256, 8, 1, 256, 7)
    idx = np.zeros((40, 1), dtype=np.int32); idx[0] = 3; idx[1:] = 6        # experts 0-2, 4, 5, 7 empty; expert 3 has one row
    counts, offsets = O.counts_offsets(idx, 8)
    _, pair_of_row = O.permute_maps(idx, offsets)
    say("mx8 forward with empty experts counts=%s" % counts.tolist())
    _compare_forward(cfg, inp, offsets.astype(np.int32), pair_of_row.astype(np.int32), gather=True)


def test_rejects_unsupported_shapes():
    import torch
    from paper_2508_02317_amd import libmoe as L
    with pytest.raises(L.MoEError) as e:
        L.moe_mx8_quantise(torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == 2 or "multiple of 128" in str(e.value)


def test_full_size_a3b_8k():
    """The 30B-A3B-class layer at its full size, in the launch configuration the benchmark's 8-bit leg times (rows read by
    token): the GPU quantiser against the oracle's on the whole input and on all three weights, bit for bit; then every
    activation code / scale and every element of Yp of the forward on the oracle-quantised operands."""
    import time
    import torch
    from paper_2508_02317_amd import libmoe as L
    cfg = CONFIGS["a3b_8k"]
    say("mx8 full size a3b_8k: T=%d P=%d" % (cfg.T, cfg.P))
    inp = make_inputs(cfg)
    idx, w, counts, offsets = O.route_topk(inp["logits"], cfg.k, cfg.renorm)
    _, pair_of_row = O.permute_maps(idx, offsets)
    offsets = offsets.astype(np.int32); pair_of_row = pair_of_row.astype(np.int32)
    E, f, d, k, P = cfg.E, cfg.f, cfg.d, cfg.k, cfg.P
    t0 = time.perf_counter()
    Xq, Xs = F.mx_quantise(inp["X"])
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(torch.bfloat16)
    gq, gs = L.moe_mx8_quantise(bf(inp["X"]))
    assert np.array_equal(to_np(gq), Xq) and np.array_equal(unpack_scales(to_np(gs)), Xs)
    wq = {}
    for name in ("Wg", "Wu", "Wd"):
        W = inp[name]
        q_ref = np.empty(W.shape, dtype=np.uint8); s_ref = np.empty(W.shape[:2] + (W.shape[2] // 32,), dtype=np.uint8)
        for e in range(E):                                 # blocks are independent: one expert at a time bounds the temporaries
            q_ref[e], s_ref[e] = F.mx_quantise(W[e])
        cq, cs = L.moe_mx8_quantise(bf(W))
        assert np.array_equal(to_np(cq), q_ref), name
        assert np.array_equal(unpack_scales(to_np(cs)), s_ref.reshape(E * W.shape[1], -1)), name
        wq[name] = (q_ref, s_ref, cq, cs)
        say("  %s: codes and scales identical (%.0f s)" % (name, time.perf_counter() - t0))
    tok = pair_of_row // k
    A = np.empty((P, f)); Yp = np.empty((P, d)); Aq = np.empty((P, f), dtype=np.uint8); As = np.empty((P, f // 32), dtype=np.uint8)
    Xd = F.mx_dequantise(Xq, Xs)
    for e in range(E):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b == a:
            continue
        xe = Xd[tok[a:b]]
        G = xe @ F.mx_dequantise(wq["Wg"][0][e], wq["Wg"][1][e]).T
        U = xe @ F.mx_dequantise(wq["Wu"][0][e], wq["Wu"][1][e]).T
        A[a:b] = F.silu(G) * U
        Aq[a:b], As[a:b] = F.quantise_activation(A[a:b])
        Yp[a:b] = F.mx_dequantise(Aq[a:b], As[a:b]) @ F.mx_dequantise(wq["Wd"][0][e], wq["Wd"][1][e]).T
    say("  oracle forward done (%.0f s)" % (time.perf_counter() - t0))
    actq, acts, yp = L.moe_grouped_gemm_swiglu_fwd_mx8(gq, gs, wq["Wg"][2], wq["Wg"][3], wq["Wu"][2], wq["Wu"][3], wq["Wd"][2], wq["Wd"][3],
                                                       to_dev(offsets), pair_of_row=to_dev(pair_of_row), k=k)
    torch.cuda.synchronize()
    got_q, got_s = to_np(actq), unpack_scales(to_np(acts))
    same_scale = got_s == As
    frac_scale = 1.0 - same_scale.mean()
    frac_code = np.mean((got_q != Aq) | ~same_scale.repeat(32, axis=1))
    step = np.maximum(_step_of_block(got_s), _step_of_block(As)).repeat(32, axis=1)
    worst = np.max(np.abs(F.mx_dequantise(got_q, got_s) - F.mx_dequantise(Aq, As)) / step)
    err_y, fro_y = rel_err(to_np(yp), Yp), fro_err(to_np(yp), Yp)
    yp2 = L.moe_grouped_gemm_down_mx8(to_dev(Aq), to_dev(pack_scales(As)), wq["Wd"][2], wq["Wd"][3], to_dev(offsets))
    torch.cuda.synchronize()
    err_y2 = rel_err(to_np(yp2), Yp)
    say("  act scales differing %.2e, codes differing %.2e, worst |dA| = %.2f steps, Yp fused max %.2e fro %.2e, second product alone %.2e"
        % (frac_scale, frac_code, worst, err_y, fro_y, err_y2))
    assert frac_scale <= 1e-3 and frac_code <= 5e-3 and worst <= 1.0 + 1e-9
    assert err_y2 <= TOL["bf16"]
    assert fro_y <= FUSED_YP_FRO and err_y <= FUSED_YP_MAX


def test_forward_is_deterministic_and_replays_from_a_graph():
    """Quantiser and 8-bit forward allocate nothing and use one stream: captured into a HIP graph they replay
    bit-identically to the eager calls (eager work and synchronisations between the replays), and two eager calls agree."""
    import torch
    from paper_2508_02317_amd import libmoe as L
    cfg, inp, offsets, pair_of_row = _case(1024, 512, 32, 2, 256, 5)
    k = cfg.k
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(torch.bfloat16)
    x = bf(inp["X"])
    wq = [L.moe_mx8_quantise(bf(inp[n])) for n in ("Wg", "Wu", "Wd")]
    toffs, tpair = to_dev(offsets), to_dev(pair_of_row)
    P, d, f, E = cfg.P, cfg.d, cfg.f, cfg.E
    xq = L.moe_mx8_quantise(x)
    out = L.moe_grouped_gemm_swiglu_fwd_mx8(xq[0], xq[1], wq[0][0], wq[0][1], wq[1][0], wq[1][1], wq[2][0], wq[2][1], toffs,
                                            pair_of_row=tpair, k=k)
    ws = torch.empty(L.lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E), dtype=torch.uint8, device="cuda")

    def fwd():
        L.moe_mx8_quantise(x, out=xq)
        L.moe_grouped_gemm_swiglu_fwd_mx8(xq[0], xq[1], wq[0][0], wq[0][1], wq[1][0], wq[1][1], wq[2][0], wq[2][1], toffs,
                                          pair_of_row=tpair, k=k, out=out, ws=ws)

    outs = lambda: [to_np(t).copy() for t in (xq[0], xq[1]) + tuple(out)]
    fwd()
    torch.cuda.synchronize()
    eager = outs()
    fwd()
    torch.cuda.synchronize()
    for a, b in zip(outs(), eager):
        assert np.array_equal(a, b)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fwd()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        fwd()
    for rep in range(3):
        for t in out:
            t.fill_(3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs(), eager):
            assert np.array_equal(a, b), "replay %d differs from the eager calls" % rep
        say("  replay %d identical to eager" % rep)


def test_full_size_a3b_long_sampled():
    """The largest configuration (40960 tokens, 327680 rows): the quantiser bit for bit on the whole input, then the forward
    on GPU-quantised operands checked on sampled rows that the oracle computes one by one -- the first and last row of
    twelve experts (first, last, largest, smallest and eight others), rows at row-tile boundaries and in the last,
    partial tile of their expert."""
    import torch
    from paper_2508_02317_amd import libmoe as L
    cfg = CONFIGS["a3b_long"]
    say("mx8 full size a3b_long (sampled): T=%d P=%d" % (cfg.T, cfg.P))
    inp = make_inputs(cfg)
    idx, w, counts, offsets = O.route_topk(inp["logits"], cfg.k, cfg.renorm)
    _, pair_of_row = O.permute_maps(idx, offsets)
    E, f, d, k, P = cfg.E, cfg.f, cfg.d, cfg.k, cfg.P
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(torch.bfloat16)
    xq, xs = L.moe_mx8_quantise(bf(inp["X"]))
    Xq, Xs = F.mx_quantise(inp["X"])
    assert np.array_equal(to_np(xq), Xq) and np.array_equal(unpack_scales(to_np(xs)), Xs)
    wq = [L.moe_mx8_quantise(bf(inp[n])) for n in ("Wg", "Wu", "Wd")]
    actq, acts, yp = L.moe_grouped_gemm_swiglu_fwd_mx8(xq, xs, wq[0][0], wq[0][1], wq[1][0], wq[1][1], wq[2][0], wq[2][1],
                                                       to_dev(offsets.astype(np.int32)), pair_of_row=to_dev(pair_of_row.astype(np.int32)), k=k)
    torch.cuda.synchronize()
    got_q, got_s, got_y = to_np(actq), unpack_scales(to_np(acts)), to_np(yp)
    rng = np.random.default_rng(17)
    experts = sorted(set([0, E - 1, int(np.argmax(counts)), int(np.argmin(counts))] + rng.choice(E, 8, replace=False).tolist()))
    n_rows, flips, worst_y = 0, 0, 0.0
    for e in experts:
        a, b = int(offsets[e]), int(offsets[e + 1])
        if b == a:
            continue
        last_tile = a + ((b - a - 1) // 256) * 256
        rows = sorted(set([a, b - 1, min(a + 255, b - 1), min(a + 256, b - 1), last_tile, (a + b) // 2]))
        Wg, Gs = F.mx_quantise(inp["Wg"][e]); Wu, Us = F.mx_quantise(inp["Wu"][e]); Wd, Ds = F.mx_quantise(inp["Wd"][e])
        assert np.array_equal(to_np(wq[0][0][e]), Wg) and np.array_equal(to_np(wq[2][0][e]), Wd)       # the GPU's weight codes for this expert
        wg, wu, wd = F.mx_dequantise(Wg, Gs), F.mx_dequantise(Wu, Us), F.mx_dequantise(Wd, Ds)
        tok = pair_of_row[rows] // k
        x = F.mx_dequantise(Xq[tok], Xs[tok])
        A = F.silu(x @ wg.T) * (x @ wu.T)
        Aq, As = F.quantise_activation(A)
        Y = F.mx_dequantise(Aq, As) @ wd.T
        same = got_s[rows] == As
        assert same.mean() >= 0.99
        step = np.maximum(_step_of_block(got_s[rows]), _step_of_block(As)).repeat(32, axis=1)
        dA = np.abs(F.mx_dequantise(got_q[rows], got_s[rows]) - F.mx_dequantise(Aq, As)) / step
        assert dA.max() <= 1.0 + 1e-9
        flips += int(((got_q[rows] != Aq) | ~same.repeat(32, axis=1)).sum())
        n_rows += len(rows)
        worst_y = max(worst_y, float(np.max(np.abs(got_y[rows] - Y)) / np.max(np.abs(Y))))
    say("  %d rows of %d experts: %d of %d activation codes differ, Yp max error %.2e" % (n_rows, len(experts), flips, n_rows * f, worst_y))
    assert flips <= 5e-3 * n_rows * f
    assert worst_y <= FUSED_YP_MAX
