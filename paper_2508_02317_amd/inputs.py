"""Seeded synthetic inputs for the MoE-layer hot path.

This module holds no arithmetic of the method itself (no top-k, no softmax, no expert
FFN, no permutation): it draws tensors, rounds them to the dtype the GPU receives, forms
the router logits with a plain fp64 matrix product, and offers pure index selection for
the pre-routed expert-parallel share.  Both the CPU oracle's tests and the HIP path's
harness take their inputs from here so that they see bit-identical values.

The shapes stand in for the paper's workloads (a Qwen3-30B-A3B-based omni-modal MoE
trained on packed multimodal sequences, Sec. 4 and App. A Table 4): one flat [T, d] token
matrix per micro-batch, 128 experts with top-8 routing, expert ffn width 768.  None of
the paper's datasets or weights is used.

Every tensor has its own counter-based Philox stream keyed by (seed, tensor id), so the
value of one tensor does not depend on the shape of another.
"""
from dataclasses import dataclass, replace
import os

import numpy as np


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int          # tokens seen by the layer (for "ep_share": rows already routed to this GPU)
    d: int          # hidden size
    E: int          # experts held by this GPU
    k: int          # experts per token (1 for the pre-routed share)
    f: int          # expert ffn width
    dtype: str      # "f32" | "bf16"
    seed: int
    renorm: int = 1
    kind: str = "layer"      # "layer" | "ep_share" | "mixed_modal"
    E_global: int = 0        # ep_share: experts of the global problem
    k_global: int = 0        # ep_share: top-k of the global problem
    T_global: int = 0        # ep_share: tokens routed globally before selection
    zipf_s: float = 0.0      # ep_share: exponent of the rank bias added to the logits

    @property
    def P(self):
        return self.T * self.k


CONFIGS = {
    # tiny fp32 parity case
    "tiny": MoEConfig("tiny", T=256, d=128, E=8, k=2, f=256, dtype="f32", seed=0),
    # small bf16 case, near-uniform routing
    "small": MoEConfig("small", T=4096, d=1024, E=16, k=2, f=2048, dtype="bf16", seed=1),
    # 30B-A3B-class layer: one 8K-token micro-batch
    "a3b_8k": MoEConfig("a3b_8k", T=8192, d=2048, E=128, k=8, f=768, dtype="bf16", seed=2),
    # one expert-parallel rank's share under Zipf-skewed routing: 16 local experts of 128
    "a3b_ep_skew": MoEConfig("a3b_ep_skew", T=16384, d=2048, E=16, k=1, f=768, dtype="bf16", seed=3,
                             kind="ep_share", E_global=128, k_global=8, T_global=16384, zipf_s=1.2),
    # sequence-parallel shard (160K / 4) mixing text rows and image/audio-patch rows
    "a3b_long": MoEConfig("a3b_long", T=40960, d=2048, E=128, k=8, f=768, dtype="bf16", seed=4,
                          kind="mixed_modal"),
}


def scaled(cfg, **kw):
    """A copy of `cfg` with some sizes replaced (reduced-size parity cases)."""
    return replace(cfg, **kw)


# ----------------------------------------------------------------------------- dtype helpers

def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.array(a, dtype=np.float32, order="C", copy=True)
    _round_to_bf16_inplace(a)
    return a


def _round_to_bf16_inplace(a):
    bits = a.reshape(-1).view(np.uint32)
    step = 1 << 22                                   # bounded temporaries
    for s in range(0, bits.size, step):
        b = bits[s:s + step]
        lsb = (b >> np.uint32(16)) & np.uint32(1)
        lsb += np.uint32(0x7FFF)
        b += lsb
        b &= np.uint32(0xFFFF0000)


def bf16_bits(a):
    """uint16 bit patterns of float32 values that are already bfloat16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b):
    """float32 values of uint16 bfloat16 bit patterns."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantise(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


# ----------------------------------------------------------------------------- generators

_TENSOR_IDS = {"X": 1, "Wr": 2, "Wg": 3, "Wu": 4, "Wd": 5, "dY": 6, "runs": 7}


def _rng(seed, tensor, chunk=0):
    return np.random.Generator(np.random.Philox(key=[int(seed) * 16 + _TENSOR_IDS[tensor], int(chunk)]))


_CHUNK_ROWS = 1024      # leading-dimension rows per Philox stream of a 2-D tensor


def _normal(seed, tensor, shape, std, dtype, row_scale=None):
    """N(0, std) values rounded to `dtype`.  The tensor is drawn in slabs along its leading
    dimension (one expert of a stacked weight, 1024 rows of a matrix), each slab from its
    own Philox stream, so the values do not depend on how many threads draw them."""
    out = np.empty(shape, dtype=np.float32)
    slab = 1 if len(shape) == 3 else _CHUNK_ROWS
    n_slabs = (shape[0] + slab - 1) // slab

    def draw(c):
        view = out[c * slab:(c + 1) * slab]
        _rng(seed, tensor, c).standard_normal(size=view.shape, dtype=np.float32, out=view)
        if std != 1.0:
            view *= np.float32(std)
        if row_scale is not None:
            view *= row_scale[c * slab:(c + 1) * slab, None]
        if dtype == "bf16":
            _round_to_bf16_inplace(view)

    if out.size < (1 << 22) or n_slabs == 1:
        for c in range(n_slabs):
            draw(c)
    else:
        from concurrent.futures import ThreadPoolExecutor
        workers = max(1, min(16, len(os.sched_getaffinity(0)), n_slabs))
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(draw, range(n_slabs)))
    return out


def modality_row_scale(cfg):
    """Per-row activation scale for the mixed-modality shard: contiguous alternating runs
    of text rows (std 1) and image/audio-patch rows (std 4), run lengths 64..2048 rows."""
    rng = _rng(cfg.seed, "runs")
    scale = np.ones(cfg.T, dtype=np.float32)
    pos, patch = 0, False
    while pos < cfg.T:
        n = int(rng.integers(64, 2049))
        if patch:
            scale[pos:pos + n] = 4.0
        pos += n
        patch = not patch
    return scale


def zipf_rank(e, n_ranks_per_gpu=16, n_gpus=8):
    """Popularity rank (1 = hottest) of global expert e, chosen so that each GPU's 16
    consecutive experts span hot to cold: rank(e) = (e mod 16) * 8 + e // 16 + 1."""
    e = np.asarray(e)
    return (e % n_ranks_per_gpu) * n_gpus + e // n_ranks_per_gpu + 1


def make_inputs(cfg):
    """Draw all inputs of one configuration.

    Returns a dict of float32 numpy arrays whose values are exactly representable in
    cfg.dtype: X [T', d], Wr [d, E'], Wg, Wu [E, f, d], Wd [E, d, f], dY [T, d], and
    logits [T', E'] float32 (= fp64 X @ Wr, plus the rank bias for the skewed case,
    rounded once to fp32).  For kind == "ep_share", T' = T_global and E' = E_global: the
    caller routes the global problem and then applies `select_local_share`.
    """
    ep = cfg.kind == "ep_share"
    Tg = cfg.T_global if ep else cfg.T
    Eg = cfg.E_global if ep else cfg.E
    row_scale = modality_row_scale(cfg) if cfg.kind == "mixed_modal" else None
    X = _normal(cfg.seed, "X", (Tg, cfg.d), 1.0, cfg.dtype, row_scale)
    Wr = _normal(cfg.seed, "Wr", (cfg.d, Eg), 0.02, cfg.dtype)
    Wg = _normal(cfg.seed, "Wg", (cfg.E, cfg.f, cfg.d), 0.02, cfg.dtype)
    Wu = _normal(cfg.seed, "Wu", (cfg.E, cfg.f, cfg.d), 0.02, cfg.dtype)
    Wd = _normal(cfg.seed, "Wd", (cfg.E, cfg.d, cfg.f), 0.02, cfg.dtype)
    dY = _normal(cfg.seed, "dY", (cfg.T, cfg.d), 1.0, cfg.dtype)
    z = X.astype(np.float64) @ Wr.astype(np.float64)
    if ep:
        z = z - cfg.zipf_s * np.log(zipf_rank(np.arange(Eg)).astype(np.float64))[None, :]
    logits = z.astype(np.float32)
    return dict(X=X, Wr=Wr, Wg=Wg, Wu=Wu, Wd=Wd, dY=dY, logits=logits)


def select_local_share(topk_idx, topk_w, n_local, max_rows):
    """Pure index selection for the expert-parallel share: keep, in (token, slot) order,
    the routed pairs whose expert id is < n_local, truncated to max_rows rows.

    Returns token_of_row [R] (which global token each local row is a copy of),
    local_idx [R, 1] int32 (expert id on this GPU) and local_w [R, 1] (the pair's weight
    from the global top-k renormalisation)."""
    idx = np.asarray(topk_idx)
    tok, slot = np.nonzero(idx < n_local)        # row-major order = token, then slot
    tok, slot = tok[:max_rows], slot[:max_rows]
    local_idx = idx[tok, slot].astype(np.int32)[:, None]
    local_w = np.asarray(topk_w)[tok, slot][:, None]
    return tok.astype(np.int64), local_idx, local_w
