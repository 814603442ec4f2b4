"""ctypes binding of libmoe_gfx950.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/moe.h) and does
nothing but check tensor dtypes / contiguity, allocate outputs and workspaces with torch
when the caller did not pass them, and hand raw device pointers and the current HIP
stream to the library.  All arithmetic of the MoE layer runs inside the library's
kernels.  There is no fallback: if the shared library has not been built, importing this
module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_gfx950.so")

MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE, MOE_ERR_HIP = range(5)
MOE_F32, MOE_BF16 = 0, 1

EXPORTS = [
    "moe_version", "moe_last_error",
    "moe_route_topk_workspace_bytes", "moe_route_topk", "moe_route_topk_bwd",
    "moe_route_topk_noalloc_max_bytes", "moe_route_topk_noalloc",
    "moe_expert_offsets_workspace_bytes", "moe_expert_offsets",
    "moe_permute_workspace_bytes", "moe_permute",
    "moe_grouped_gemm_swiglu_fwd_workspace_bytes", "moe_grouped_gemm_swiglu_fwd",
    "moe_grouped_gemm_swiglu_bwd_workspace_bytes", "moe_grouped_gemm_swiglu_bwd",
    "moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes", "moe_grouped_gemm_swiglu_fwd_gather",
    "moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes", "moe_grouped_gemm_swiglu_bwd_gather",
    "moe_unpermute_combine_fwd", "moe_unpermute_combine_bwd",
    "moe_router_logits_workspace_bytes", "moe_router_logits", "moe_router_bwd_workspace_bytes", "moe_router_bwd",
    "moe_mx8_quantise", "moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes", "moe_grouped_gemm_swiglu_fwd_mx8",
    "moe_grouped_gemm_down_mx8",
    "moe_set_launch_hook",
]


# void hook(const char* kernel_name, int phase, void* stream, void* user)
LAUNCH_HOOK = ctypes.CFUNCTYPE(None, ctypes.c_char_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p)


class MoEError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("libmoe status %d: %s" % (code, message))
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libmoe_gfx950.so is not built (%s missing). Build it with "
            "`python -m paper_2508_02317_amd.build`; there is no fallback path." % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.moe_version.restype = ctypes.c_char_p
    lib.moe_version.argtypes = []
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_last_error.argtypes = []
    lib.moe_route_topk_workspace_bytes.restype = sz
    lib.moe_route_topk_workspace_bytes.argtypes = [i32, i32, i32]
    lib.moe_route_topk.restype = ctypes.c_int32
    lib.moe_route_topk.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_route_topk_noalloc_max_bytes.restype = sz
    lib.moe_route_topk_noalloc_max_bytes.argtypes = []
    lib.moe_route_topk_noalloc.restype = ctypes.c_int32
    lib.moe_route_topk_noalloc.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.moe_route_topk_bwd.restype = ctypes.c_int32
    lib.moe_route_topk_bwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]
    lib.moe_expert_offsets_workspace_bytes.restype = sz
    lib.moe_expert_offsets_workspace_bytes.argtypes = [i32, i32]
    lib.moe_expert_offsets.restype = ctypes.c_int32
    lib.moe_expert_offsets.argtypes = [vp, i32, i32, vp, vp, vp, sz, vp]
    lib.moe_permute_workspace_bytes.restype = sz
    lib.moe_permute_workspace_bytes.argtypes = [i32, i32, i32]
    lib.moe_permute.restype = ctypes.c_int32
    lib.moe_permute.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes.restype = sz
    lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.moe_grouped_gemm_swiglu_fwd.restype = ctypes.c_int32
    lib.moe_grouped_gemm_swiglu_fwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes.restype = sz
    lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.moe_grouped_gemm_swiglu_bwd.restype = ctypes.c_int32
    lib.moe_grouped_gemm_swiglu_bwd.argtypes = [vp] * 8 + [i32] * 5 + [vp] * 6 + [sz, vp]
    lib.moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes.restype = sz
    lib.moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.moe_grouped_gemm_swiglu_fwd_gather.restype = ctypes.c_int32
    lib.moe_grouped_gemm_swiglu_fwd_gather.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes.restype = sz
    lib.moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.moe_grouped_gemm_swiglu_bwd_gather.restype = ctypes.c_int32
    lib.moe_grouped_gemm_swiglu_bwd_gather.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_unpermute_combine_fwd.restype = ctypes.c_int32
    lib.moe_unpermute_combine_fwd.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.moe_unpermute_combine_bwd.restype = ctypes.c_int32
    lib.moe_unpermute_combine_bwd.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.moe_router_logits_workspace_bytes.restype = sz
    lib.moe_router_logits_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.moe_router_logits.restype = ctypes.c_int32
    lib.moe_router_logits.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.moe_router_bwd_workspace_bytes.restype = sz
    lib.moe_router_bwd_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.moe_router_bwd.restype = ctypes.c_int32
    lib.moe_router_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.moe_mx8_quantise.restype = ctypes.c_int32
    lib.moe_mx8_quantise.argtypes = [vp, ctypes.c_int64, i32, vp, vp, vp]
    lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes.restype = sz
    lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.moe_grouped_gemm_swiglu_fwd_mx8.restype = ctypes.c_int32
    lib.moe_grouped_gemm_swiglu_fwd_mx8.argtypes = [vp, vp, i32, i32, vp] + [vp] * 6 + [i32] * 4 + [vp] * 5 + [sz, vp]
    lib.moe_grouped_gemm_down_mx8.restype = ctypes.c_int32
    lib.moe_grouped_gemm_down_mx8.argtypes = [vp] * 4 + [i32] * 4 + [vp] * 3 + [sz, vp]
    lib.moe_set_launch_hook.restype = ctypes.c_int32
    lib.moe_set_launch_hook.argtypes = [LAUNCH_HOOK, vp]
    return lib


lib = _load()


def moe_version():
    return lib.moe_version().decode()


def moe_last_error():
    return lib.moe_last_error().decode()


def moe_set_launch_hook(hook):
    """hook: a LAUNCH_HOOK instance (kept alive by the caller) or None to remove it."""
    _check(lib.moe_set_launch_hook(hook if hook is not None else LAUNCH_HOOK(), None))


def _check(status):
    if status != MOE_OK:
        raise MoEError(status, moe_last_error())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise TypeError("libmoe supports float32 and bfloat16 tensors, got %s" % t.dtype)


def _need(t, dtype=None, name="tensor"):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(nbytes, ws, device):
    if ws is None:
        ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    return ws, ws.numel()


# --------------------------------------------------------------------------------------------

def moe_route_topk(logits, k, renorm=1, out=None, ws=None):
    """-> topk_idx [T,k] i32, topk_w [T,k] f32, counts [E] i32, offsets [E+1] i32."""
    _need(logits, torch.float32, "logits")
    T, E = logits.shape
    dev = logits.device
    if out is None:
        out = (torch.empty((T, k), dtype=torch.int32, device=dev), torch.empty((T, k), dtype=torch.float32, device=dev),
               torch.empty(E, dtype=torch.int32, device=dev), torch.empty(E + 1, dtype=torch.int32, device=dev))
    idx, w, counts, offsets = out
    ws, nbytes = _ws(lib.moe_route_topk_workspace_bytes(T, E, k), ws, dev)
    _check(lib.moe_route_topk(_ptr(logits), T, E, k, int(renorm), _ptr(idx), _ptr(w), _ptr(counts), _ptr(offsets),
                              _ptr(ws), nbytes, _stream()))
    return idx, w, counts, offsets


def moe_route_topk_noalloc(logits, k, renorm, out):
    """moe_route_topk without a workspace (histogram rows in the library's static device array); `out` =
    (topk_idx, topk_w, counts, offsets) must be given: nothing is allocated here either."""
    _need(logits, torch.float32, "logits")
    T, E = logits.shape
    idx, w, counts, offsets = out
    _check(lib.moe_route_topk_noalloc(_ptr(logits), T, E, k, int(renorm), _ptr(idx), _ptr(w), _ptr(counts), _ptr(offsets),
                                      _stream()))
    return idx, w, counts, offsets


def moe_expert_offsets(topk_idx, E, out=None, ws=None):
    """-> counts [E] i32, offsets [E+1] i32 of a known assignment."""
    _need(topk_idx, torch.int32, "topk_idx")
    n = topk_idx.numel()
    dev = topk_idx.device
    if out is None:
        out = (torch.empty(E, dtype=torch.int32, device=dev), torch.empty(E + 1, dtype=torch.int32, device=dev))
    counts, offsets = out
    ws, nbytes = _ws(lib.moe_expert_offsets_workspace_bytes(n, E), ws, dev)
    _check(lib.moe_expert_offsets(_ptr(topk_idx), n, E, _ptr(counts), _ptr(offsets), _ptr(ws), nbytes, _stream()))
    return counts, offsets


def moe_route_topk_bwd(dw, topk_w, topk_idx, logits, E, renorm=1, out=None):
    """-> dlogits [T,E] f32."""
    _need(dw, torch.float32, "dw"); _need(topk_w, torch.float32, "topk_w"); _need(topk_idx, torch.int32, "topk_idx")
    T, k = topk_idx.shape
    if out is None:
        out = torch.empty((T, E), dtype=torch.float32, device=dw.device)
    _check(lib.moe_route_topk_bwd(_ptr(dw), _ptr(topk_w), _ptr(topk_idx), _ptr(logits), T, E, k, int(renorm),
                                  _ptr(out), _stream()))
    return out


def moe_permute(x, topk_idx, offsets, E, out=None, ws=None):
    """-> xp [P,d], row_of_pair [P] i32, pair_of_row [P] i32.  x None: only the two maps (xp is None)."""
    _need(topk_idx, torch.int32, "topk_idx"); _need(offsets, torch.int32, "offsets")
    T, k = topk_idx.shape
    P = T * k
    dev = topk_idx.device
    if x is not None:
        _need(x, None, "x")
        d = x.shape[1]
    else:
        d = 8
    if out is None:
        out = (torch.empty((P, d), dtype=x.dtype, device=dev) if x is not None else None,
               torch.empty(P, dtype=torch.int32, device=dev), torch.empty(P, dtype=torch.int32, device=dev))
    xp, row_of_pair, pair_of_row = out
    if x is None:
        xp = None
    ws, nbytes = _ws(lib.moe_permute_workspace_bytes(T, E, k), ws, dev)
    _check(lib.moe_permute(_ptr(x), _dtype_code(x) if x is not None else MOE_BF16, T, d, E, k, _ptr(topk_idx), _ptr(offsets),
                           _ptr(xp), _ptr(row_of_pair), _ptr(pair_of_row), _ptr(ws), nbytes, _stream()))
    return xp, row_of_pair, pair_of_row


def moe_grouped_gemm_swiglu_fwd(xp, w_gate, w_up, w_down, offsets, save_gu=True, out=None, ws=None):
    """-> act [P,f], yp [P,d], g_save, u_save ([P,f] or None)."""
    _need(xp, None, "xp"); _need(offsets, torch.int32, "offsets")
    for name, w in (("w_gate", w_gate), ("w_up", w_up), ("w_down", w_down)):
        _need(w, xp.dtype, name)
    P, d = xp.shape
    E, f, _ = w_gate.shape
    dev = xp.device
    if out is None:
        mk = lambda *s: torch.empty(s, dtype=xp.dtype, device=dev)
        out = (mk(P, f), mk(P, d), mk(P, f) if save_gu else None, mk(P, f) if save_gu else None)
    act, yp, g, u = out
    code = _dtype_code(xp)
    ws, nbytes = _ws(lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes(code, P, d, f, E), ws, dev)
    _check(lib.moe_grouped_gemm_swiglu_fwd(_ptr(xp), _ptr(w_gate), _ptr(w_up), _ptr(w_down), code, P, d, f, E,
                                           _ptr(offsets), _ptr(g), _ptr(u), _ptr(act), _ptr(yp), _ptr(ws), nbytes,
                                           _stream()))
    return act, yp, g, u


def moe_grouped_gemm_swiglu_bwd(dyp, xp, g_save, u_save, act, w_gate, w_up, w_down, offsets, out=None, ws=None):
    """-> dxp [P,d], dw_gate [E,f,d], dw_up [E,f,d], dw_down [E,d,f]."""
    _need(dyp, xp.dtype, "dyp"); _need(xp, None, "xp"); _need(act, xp.dtype, "act")
    P, d = xp.shape
    E, f, _ = w_gate.shape
    if out is None:
        out = (torch.empty_like(xp), torch.empty_like(w_gate), torch.empty_like(w_up), torch.empty_like(w_down))
    dxp, dwg, dwu, dwd = out
    code = _dtype_code(xp)
    have_saved = int(g_save is not None)
    ws, nbytes = _ws(lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes(code, P, d, f, E, have_saved), ws, xp.device)
    _check(lib.moe_grouped_gemm_swiglu_bwd(_ptr(dyp), _ptr(xp), _ptr(g_save), _ptr(u_save), _ptr(act), _ptr(w_gate),
                                           _ptr(w_up), _ptr(w_down), code, P, d, f, E, _ptr(offsets), _ptr(dxp),
                                           _ptr(dwg), _ptr(dwu), _ptr(dwd), _ptr(ws), nbytes, _stream()))
    return dxp, dwg, dwu, dwd


def moe_grouped_gemm_swiglu_fwd_gather(x, k, pair_of_row, w_gate, w_up, w_down, offsets, save_gu=True, out=None, ws=None, topk_w=None):
    """Forward without xp: rows are read as x[pair_of_row[r] // k].  -> act [P,f], yp [P,d], g_save, u_save.
    With topk_w [T,k], act and yp leave scaled by each row's combine weight."""
    if topk_w is not None:
        _need(topk_w, torch.float32, "topk_w")
    _need(x, None, "x"); _need(pair_of_row, torch.int32, "pair_of_row"); _need(offsets, torch.int32, "offsets")
    for name, w in (("w_gate", w_gate), ("w_up", w_up), ("w_down", w_down)):
        _need(w, x.dtype, name)
    T, d = x.shape
    P = T * k
    E, f, _ = w_gate.shape
    dev = x.device
    if out is None:
        mk = lambda *s: torch.empty(s, dtype=x.dtype, device=dev)
        out = (mk(P, f), mk(P, d), mk(P, f) if save_gu else None, mk(P, f) if save_gu else None)
    act, yp, g, u = out
    code = _dtype_code(x)
    ws, nbytes = _ws(lib.moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes(code, P, d, f, E), ws, dev)
    _check(lib.moe_grouped_gemm_swiglu_fwd_gather(_ptr(x), T, k, _ptr(pair_of_row), _ptr(topk_w), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                                  code, P, d, f, E, _ptr(offsets), _ptr(g), _ptr(u), _ptr(act), _ptr(yp),
                                                  _ptr(ws), nbytes, _stream()))
    return act, yp, g, u


def moe_mx8_quantise(src, out=None):
    """bf16 [..., K] -> (E4M3 codes uint8 [..., K], packed scale words int32 [K/128, rows]) with rows = the product of the
    leading dimensions; byte j of word (g, row) is the power-of-two scale code of elements 128 g + 32 j .. + 31 of the row."""
    _need(src, torch.bfloat16, "src")
    K = src.shape[-1]
    rows = src.numel() // K if K else 0
    if out is None:
        out = (torch.empty(src.shape, dtype=torch.uint8, device=src.device),
               torch.empty((max(K // 128, 0), rows), dtype=torch.int32, device=src.device))
    codes, scales = out
    _check(lib.moe_mx8_quantise(_ptr(src), rows, K, _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def moe_grouped_gemm_swiglu_fwd_mx8(xq, xs, wgq, wgs, wuq, wus, wdq, wds, offsets, pair_of_row=None, k=1, out=None, ws=None):
    """Expert forward with 8-bit block-scaled operands (from moe_mx8_quantise).  xq [T, d] codes read by token through
    pair_of_row [P] (P = T * k), or [P, d] in expert order when pair_of_row is None.
    -> act codes uint8 [P, f], act scale words int32 [f/128, P], yp bf16 [P, d]."""
    _need(xq, torch.uint8, "xq"); _need(xs, torch.int32, "xs"); _need(offsets, torch.int32, "offsets")
    for name, w in (("wgq", wgq), ("wuq", wuq), ("wdq", wdq)):
        _need(w, torch.uint8, name)
    for name, w in (("wgs", wgs), ("wus", wus), ("wds", wds)):
        _need(w, torch.int32, name)
    T, d = xq.shape
    E, f, _ = wgq.shape
    if pair_of_row is not None:
        _need(pair_of_row, torch.int32, "pair_of_row")
        P = T * k
    else:
        P, k = T, 1
    dev = xq.device
    if out is None:
        out = (torch.empty((P, f), dtype=torch.uint8, device=dev), torch.empty((max(f // 128, 0), P), dtype=torch.int32, device=dev),
               torch.empty((P, d), dtype=torch.bfloat16, device=dev))
    actq, acts, yp = out
    ws, nbytes = _ws(lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E), ws, dev)
    _check(lib.moe_grouped_gemm_swiglu_fwd_mx8(_ptr(xq), _ptr(xs), T, k, _ptr(pair_of_row), _ptr(wgq), _ptr(wgs), _ptr(wuq), _ptr(wus),
                                               _ptr(wdq), _ptr(wds), P, d, f, E, _ptr(offsets), _ptr(actq), _ptr(acts), _ptr(yp),
                                               _ptr(ws), nbytes, _stream()))
    return actq, acts, yp


def moe_grouped_gemm_down_mx8(actq, acts, wdq, wds, offsets, out=None, ws=None):
    """The second product alone on given activation codes [P, f] and scale words [f/128, P].  -> yp bf16 [P, d]."""
    _need(actq, torch.uint8, "actq"); _need(acts, torch.int32, "acts"); _need(wdq, torch.uint8, "wdq"); _need(wds, torch.int32, "wds")
    _need(offsets, torch.int32, "offsets")
    P, f = actq.shape
    E, d, _ = wdq.shape
    yp = out if out is not None else torch.empty((P, d), dtype=torch.bfloat16, device=actq.device)
    ws, nbytes = _ws(lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E), ws, actq.device)
    _check(lib.moe_grouped_gemm_down_mx8(_ptr(actq), _ptr(acts), _ptr(wdq), _ptr(wds), P, d, f, E, _ptr(offsets), _ptr(yp),
                                         _ptr(ws), nbytes, _stream()))
    return yp


def moe_grouped_gemm_swiglu_bwd_gather(dy, x, topk_w, pair_of_row, g_save, u_save, w_gate, w_up, w_down, offsets,
                                       out=None, ws=None, act_w=None):
    """Combine backward and FFN backward without dyp / xp.
    -> dxp [P,d], dw_gate [E,f,d], dw_up [E,f,d], dw_down [E,d,f], dtopk_w [T,k] f32.
    act_w [P,f]: the weighted activation the forward wrote when it was given topk_w (None: formed here)."""
    if act_w is not None:
        _need(act_w, x.dtype, "act_w")
    _need(dy, x.dtype, "dy"); _need(x, None, "x"); _need(topk_w, torch.float32, "topk_w")
    _need(pair_of_row, torch.int32, "pair_of_row"); _need(offsets, torch.int32, "offsets")
    T, d = x.shape
    k = topk_w.shape[1]
    P = T * k
    E, f, _ = w_gate.shape
    if out is None:
        out = (torch.empty((P, d), dtype=x.dtype, device=x.device), torch.empty_like(w_gate), torch.empty_like(w_up),
               torch.empty_like(w_down), torch.empty((T, k), dtype=torch.float32, device=x.device))
    dxp, dwg, dwu, dwd, dtw = out
    code = _dtype_code(x)
    have_saved = int(g_save is not None)
    ws, nbytes = _ws(lib.moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes(code, P, d, f, E, have_saved), ws, x.device)
    _check(lib.moe_grouped_gemm_swiglu_bwd_gather(_ptr(dy), _ptr(x), T, k, _ptr(topk_w), _ptr(pair_of_row), _ptr(g_save),
                                                  _ptr(u_save), _ptr(act_w), _ptr(w_gate), _ptr(w_up), _ptr(w_down), code, P, d, f, E,
                                                  _ptr(offsets), _ptr(dxp), _ptr(dwg), _ptr(dwu), _ptr(dwd), _ptr(dtw),
                                                  _ptr(ws), nbytes, _stream()))
    return dxp, dwg, dwu, dwd, dtw


def moe_unpermute_combine_fwd(yp, topk_w, row_of_pair, T, k, out=None):
    """-> y [T,d]; topk_w None = unit weights (backward of moe_permute)."""
    _need(yp, None, "yp"); _need(row_of_pair, torch.int32, "row_of_pair")
    if topk_w is not None:
        _need(topk_w, torch.float32, "topk_w")
    d = yp.shape[1]
    if out is None:
        out = torch.empty((T, d), dtype=yp.dtype, device=yp.device)
    _check(lib.moe_unpermute_combine_fwd(_ptr(yp), _dtype_code(yp), T, d, k, _ptr(topk_w), _ptr(row_of_pair),
                                         _ptr(out), _stream()))
    return out


def moe_unpermute_combine_bwd(dy, yp, topk_w, row_of_pair, out=None):
    """-> dyp [P,d], dw [T,k] f32."""
    _need(dy, yp.dtype, "dy"); _need(yp, None, "yp"); _need(topk_w, torch.float32, "topk_w")
    T, d = dy.shape
    k = topk_w.shape[1]
    if out is None:
        out = (torch.empty_like(yp), torch.empty((T, k), dtype=torch.float32, device=dy.device))
    dyp, dw = out
    _check(lib.moe_unpermute_combine_bwd(_ptr(dy), _ptr(yp), _dtype_code(yp), T, d, k, _ptr(topk_w), _ptr(row_of_pair),
                                         _ptr(dyp), _ptr(dw), _stream()))
    return dyp, dw


def moe_router_logits(x, w_router, out=None, ws=None):
    """-> logits [T,E] f32 = x [T,d] @ w_router [E,d]^T."""
    _need(x, None, "x"); _need(w_router, x.dtype, "w_router")
    T, d = x.shape
    E = w_router.shape[0]
    dt = _dtype_code(x)
    if out is None:
        out = torch.empty((T, E), dtype=torch.float32, device=x.device)
    ws, n = _ws(lib.moe_router_logits_workspace_bytes(dt, T, d, E), ws, x.device)
    _check(lib.moe_router_logits(_ptr(x), _ptr(w_router), dt, T, d, E, _ptr(out), _ptr(ws), n, _stream()))
    return out


def moe_router_bwd(dlogits, x, w_router, dx=None, out_dw=None, ws=None):
    """-> dx [T,d] (dx given: the router term is added to it in place), dw_router [E,d]."""
    _need(dlogits, torch.float32, "dlogits"); _need(x, None, "x"); _need(w_router, x.dtype, "w_router")
    T, d = x.shape
    E = w_router.shape[0]
    dt = _dtype_code(x)
    accumulate = dx is not None
    if dx is None:
        dx = torch.empty_like(x)
    else:
        _need(dx, x.dtype, "dx")
    if out_dw is None:
        out_dw = torch.empty_like(w_router)
    ws, n = _ws(lib.moe_router_bwd_workspace_bytes(dt, T, d, E), ws, x.device)
    _check(lib.moe_router_bwd(_ptr(dlogits), _ptr(x), _ptr(w_router), dt, T, d, E, int(accumulate), _ptr(dx), _ptr(out_dw),
                              _ptr(ws), n, _stream()))
    return dx, out_dw

