"""The C-ABI library loads without a GPU, exports every symbol the header declares, and
rejects bad arguments on the host before launching anything (CPU only)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2508_02317_amd import libmoe
    return libmoe


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = _declared_functions()
    assert len(names) >= 13
    raw = ctypes.CDLL(L.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(L.EXPORTS) == names
    assert re.fullmatch(r"\d+\.\d+\.\d+", L.moe_version())


def test_workspace_queries_are_host_functions(L):
    assert L.lib.moe_route_topk_workspace_bytes(8192, 128, 8) >= 128 * 4
    assert L.lib.moe_permute_workspace_bytes(8192, 128, 8) >= 8192 * 8 * 4
    fwd = L.lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128)
    bwd = L.lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128, 1)
    bwd_re = L.lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128, 0)
    assert bwd >= fwd + 2 * 65536 * 768 * 2           # room for [dG | dU]
    assert bwd_re >= bwd + 2 * 65536 * 768 * 2        # plus recomputed G, U
    assert L.lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes(L.MOE_F32, -1, 8, 8, 1) == 0


def test_bad_arguments_are_rejected_before_any_launch(L):
    lib = L.lib
    one = ctypes.c_void_p(16)     # non-null, aligned, never dereferenced: validation fails first
    # k > E
    assert lib.moe_route_topk(one, 4, 8, 9, 1, one, one, one, one, one, 1 << 20, None) == L.MOE_ERR_INVALID_ARG
    assert "k=9" in L.moe_last_error()
    # E above the built maximum
    assert lib.moe_route_topk(one, 4, 2048, 2, 1, one, one, one, one, one, 1 << 30, None) == L.MOE_ERR_UNSUPPORTED
    # null output
    assert lib.moe_route_topk(one, 4, 8, 2, 1, None, one, one, one, one, 1 << 20, None) == L.MOE_ERR_INVALID_ARG
    # workspace too small / null
    assert lib.moe_route_topk(one, 4, 8, 2, 1, one, one, one, one, one, 1, None) == L.MOE_ERR_WORKSPACE
    assert lib.moe_route_topk(one, 4, 8, 2, 1, one, one, one, one, None, 1 << 20, None) == L.MOE_ERR_WORKSPACE
    # permute: unknown dtype, d not a multiple of 8, misaligned pointer
    assert lib.moe_permute(one, 7, 4, 8, 8, 2, one, one, one, one, one, one, 1 << 20, None) == L.MOE_ERR_UNSUPPORTED
    assert lib.moe_permute(one, 0, 4, 12, 8, 2, one, one, one, one, one, one, 1 << 20, None) == L.MOE_ERR_UNSUPPORTED
    odd = ctypes.c_void_p(20)
    assert lib.moe_permute(odd, 0, 4, 8, 8, 2, one, one, one, one, one, one, 1 << 20, None) == L.MOE_ERR_INVALID_ARG
    # ffn: g_save without u_save, non-positive sizes, workspace
    args = [one, one, one, one, 1, 16, 64, 64, 2, one, one, None, one, one, one, 1 << 30, None]
    assert lib.moe_grouped_gemm_swiglu_fwd(*args) == L.MOE_ERR_INVALID_ARG
    args = [one, one, one, one, 1, 16, 0, 64, 2, one, None, None, one, one, one, 1 << 30, None]
    assert lib.moe_grouped_gemm_swiglu_fwd(*args) == L.MOE_ERR_INVALID_ARG
    args = [one, one, one, one, 1, 16, 64, 64, 2, one, None, None, one, one, one, 8, None]
    assert lib.moe_grouped_gemm_swiglu_fwd(*args) == L.MOE_ERR_WORKSPACE
    bargs = [one] * 8 + [1, 16, 64, 60, 2] + [one] * 6 + [1 << 30, None]
    assert lib.moe_grouped_gemm_swiglu_bwd(*bargs) == L.MOE_ERR_UNSUPPORTED
    # combine: k above the built maximum, null pointer
    assert lib.moe_unpermute_combine_fwd(one, 1, 4, 64, 65, one, one, one, None) == L.MOE_ERR_UNSUPPORTED
    assert lib.moe_unpermute_combine_fwd(None, 1, 4, 64, 2, one, one, one, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_unpermute_combine_bwd(one, one, 1, 4, 64, 2, None, one, one, one, None) == L.MOE_ERR_INVALID_ARG
    # route backward needs logits when renorm == 0
    assert lib.moe_route_topk_bwd(one, one, one, None, 4, 8, 2, 0, one, None) == L.MOE_ERR_INVALID_ARG
    # router linear: E not a multiple of 8 for bf16, null pointers, workspace, misalignment; fp32 has no such limit
    assert lib.moe_router_logits(one, one, 1, 16, 64, 12, one, one, 1 << 20, None) == L.MOE_ERR_UNSUPPORTED
    assert "E=12" in L.moe_last_error()
    assert lib.moe_router_logits(one, None, 1, 16, 64, 16, one, one, 1 << 20, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_router_logits(one, one, 1, 16, 64, 16, one, one, 8, None) == L.MOE_ERR_WORKSPACE
    assert lib.moe_router_logits(odd, one, 0, 16, 64, 12, one, one, 1 << 20, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_router_logits(one, one, 1, 0, 64, 16, one, one, 1 << 20, None) == L.MOE_OK      # no tokens
    assert lib.moe_router_bwd(one, one, one, 1, 16, 64, 2048, 0, one, one, one, 1 << 30, None) == L.MOE_ERR_UNSUPPORTED
    assert lib.moe_router_bwd(one, one, one, 1, 16, 64, 16, 0, None, one, one, 1 << 30, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_router_bwd(one, one, one, 1, 16, 64, 16, 0, one, one, one, 8, None) == L.MOE_ERR_WORKSPACE
    assert lib.moe_router_bwd_workspace_bytes(L.MOE_BF16, 8192, 2048, 128) >= 8192 * 128 * 2
    # 8-bit operands: reduction length a multiple of 128, null pointers, misalignment, workspace; nothing to do is fine
    assert lib.moe_mx8_quantise(one, 4, 96, one, one, None) == L.MOE_ERR_UNSUPPORTED
    assert "multiple of 128" in L.moe_last_error()
    assert lib.moe_mx8_quantise(one, 4, 128, None, one, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_mx8_quantise(odd, 4, 128, one, one, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_mx8_quantise(one, -1, 128, one, one, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_mx8_quantise(None, 0, 128, None, None, None) == L.MOE_OK
    mx = lambda T, k, pair, P, d, f, ws: lib.moe_grouped_gemm_swiglu_fwd_mx8(one, one, T, k, pair, one, one, one, one, one, one, P, d, f, 2,
                                                                             one, one, one, one, one, ws, None)
    assert mx(16, 1, None, 16, 128, 192, 1 << 30) == L.MOE_ERR_UNSUPPORTED           # f not a multiple of 128
    assert mx(8, 2, one, 17, 128, 128, 1 << 30) == L.MOE_ERR_INVALID_ARG             # P != T * k
    assert mx(1 << 22, 1, one, 1 << 22, 2048, 128, 1 << 40) == L.MOE_ERR_UNSUPPORTED   # token rows beyond 32-bit byte offsets
    assert mx(16, 1, None, 16, 128, 128, 8) == L.MOE_ERR_WORKSPACE
    assert mx(0, 1, None, 0, 128, 128, 0) == L.MOE_OK
    assert lib.moe_grouped_gemm_swiglu_fwd_mx8(one, None, 16, 1, None, one, one, one, one, one, one, 16, 128, 128, 2, one, one, one, one,
                                               one, 1 << 30, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_grouped_gemm_down_mx8(one, one, one, None, 16, 128, 128, 2, one, one, one, 1 << 30, None) == L.MOE_ERR_INVALID_ARG
    assert lib.moe_grouped_gemm_down_mx8(one, one, one, one, 16, 128, 128, 2, one, one, one, 8, None) == L.MOE_ERR_WORKSPACE
    assert lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(65536, 2048, 768, 128) >= 65536 * 4
    # gathered FFN: P must be T * k, a token's row offset must fit 32 bits, null list, workspace
    gf = lambda T, k, P, d, ws: lib.moe_grouped_gemm_swiglu_fwd_gather(one, T, k, one, None, one, one, one, 1, P, d, 64, 2, one, None, None, one,
                                                                     one, one, ws, None)
    assert gf(8, 2, 17, 64, 1 << 30) == L.MOE_ERR_INVALID_ARG
    assert "T * k" in L.moe_last_error()
    assert gf(1 << 20, 1, 1 << 20, 4096, 1 << 40) == L.MOE_ERR_UNSUPPORTED
    assert gf(8, 2, 16, 64, 8) == L.MOE_ERR_WORKSPACE
    assert lib.moe_grouped_gemm_swiglu_fwd_gather(one, 8, 2, None, None, one, one, one, 1, 16, 64, 64, 2, one, None, None, one, one, one,
                                                  1 << 30, None) == L.MOE_ERR_INVALID_ARG
    gb = [one, one, 8, 2, one, one, one, one, None, one, one, one, 1, 16, 64, 64, 2, one, one, one, one, one, None, one, 1 << 30, None]
    assert lib.moe_grouped_gemm_swiglu_bwd_gather(*gb) == L.MOE_ERR_INVALID_ARG       # null dtopk_w
    gb[22] = one; gb[3] = 3
    assert lib.moe_grouped_gemm_swiglu_bwd_gather(*gb) == L.MOE_ERR_INVALID_ARG       # P != T * k
    fw = lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128)
    assert lib.moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128) >= fw + 65536 * 4
    bw = lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128, 1)
    assert lib.moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes(L.MOE_BF16, 65536, 2048, 768, 128, 1) >= bw + 65536 * 768 * 2
    # the maps alone: x and xp both null is fine, only one of them is not
    assert lib.moe_permute(None, 1, 4, 8, 8, 2, one, one, one, one, one, one, 1 << 20, None) == L.MOE_ERR_INVALID_ARG
    # zero tokens is a no-op, not an error (nothing is launched for the movers)
    assert lib.moe_unpermute_combine_fwd(None, 1, 0, 64, 2, None, None, None, None) == L.MOE_OK


def test_binding_refuses_to_load_without_library(L, monkeypatch, tmp_path):
    import importlib.util
    src = os.path.join(ROOT, "paper_2508_02317_amd", "libmoe.py")
    target = tmp_path / "libmoe_copy.py"
    target.write_text(open(src).read())
    spec = importlib.util.spec_from_file_location("libmoe_copy", str(target))
    mod = importlib.util.module_from_spec(spec)
    with pytest.raises(ImportError):
        spec.loader.exec_module(mod)      # no .so next to the copy -> loud failure, no fallback
