"""The allocation-free routing entry point against moe_route_topk, through the C ABI (GPU)."""
import ctypes
import sys

import numpy as np
import pytest

from tests.util import to_dev, to_np

pytestmark = pytest.mark.gpu


def _route_both(L, z, k, renorm):
    import torch
    T, E = z.shape
    dev = z.device
    mk = lambda: (torch.full((T, k), -7, dtype=torch.int32, device=dev), torch.full((T, k), -7.0, dtype=torch.float32, device=dev),
                  torch.full((E,), -7, dtype=torch.int32, device=dev), torch.full((E + 1,), -7, dtype=torch.int32, device=dev))
    ref = L.moe_route_topk(z, k, renorm, out=mk())
    got = mk()
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = L.lib.moe_route_topk_noalloc(ptr(z), T, E, k, renorm, ptr(got[0]), ptr(got[1]), ptr(got[2]), ptr(got[3]),
                                      ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == L.MOE_OK, L.moe_last_error()
    torch.cuda.synchronize()
    return ref, got


def test_noalloc_route_matches_route_twice_second_call_smaller():
    from paper_2508_02317_amd import libmoe as L
    r = np.random.default_rng(11)
    # two calls in a row on the same GPU; the second, smaller one sees the histogram rows the first one left
    for T, E, k, renorm in ((8192, 128, 8, 1), (1000, 48, 3, 0)):
        print("noalloc route T=%d E=%d k=%d renorm=%d" % (T, E, k, renorm), flush=True, file=sys.stderr)
        z = to_dev(r.standard_normal((T, E)).astype(np.float32))
        ref, got = _route_both(L, z, k, renorm)
        for name, a, b in zip(("topk_idx", "topk_w", "counts", "offsets"), ref, got):
            assert np.array_equal(to_np(a), to_np(b)), name          # same kernels: bit-identical, weights included
        assert int(to_np(got[3])[-1]) == T * k


def test_noalloc_route_rejects_what_does_not_fit():
    from paper_2508_02317_amd import libmoe as L
    one = ctypes.c_void_p(256)
    cap = L.lib.moe_route_topk_noalloc_max_bytes()
    assert cap == 2 << 20
    assert L.lib.moe_route_topk_workspace_bytes(1 << 20, 1024, 2) > cap
    assert L.lib.moe_route_topk_noalloc(one, 1 << 20, 1024, 2, 1, one, one, one, one, None) == L.MOE_ERR_UNSUPPORTED
    assert "static scratch" in L.moe_last_error()
