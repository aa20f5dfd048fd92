"""Seeded synthetic inputs for the PSD denoising-step hot path.

This module only *draws* inputs: model shapes, random-init weights, RoPE tables, prompts,
and synthetic (top-1, confidence) tables for the decision kernels.  It holds none of the
method's arithmetic (no forward pass, no softmax, no policy, no drafting, no acceptance),
so both the CPU oracle's tests and the HIP path's tests may import it.

Stand-ins: the paper measures with trained Dream-7B / LLaDA-1.5 / openPangu-7B checkpoints
on few-shot GSM8K / HumanEval / MBPP prompts (Sec. 4.1, App. A, App. B.1).  Neither the
weights nor the prompts exist here; what follows takes only their shapes (7-8B layouts,
block length 32, a few hundred prompt tokens, 256-1024 generated tokens).

Recipe
------
* every weight tensor has its own counter-based stream
  ``numpy.random.default_rng([seed, layer + 1, tensor_id])`` so that any single tensor (or
  any single layer) can be regenerated without drawing the rest;
* matrices ~ N(0, 0.02^2); ``wo`` and ``w_down`` additionally scaled by 1/sqrt(2 n_layers);
  norm gains = 1; QKV biases (only where ``qkv_bias``) ~ N(0, 0.02^2);
* bf16 configs: every tensor is rounded once (nearest-even) to a bf16-representable fp32
  value, so the CPU and the GPU side consume identical numbers;
* prompts: token id = r - 1 with rank r from the truncated Zipf law p(r) ~ r^-1.1 over
  r = 1..V-1 (inverse CDF on ``default_rng(seed).random()``); config 1 uses uniform ids in
  [0, V-2]; the mask id V-1 never appears in a prompt.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

# ----------------------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------------------


@dataclass(frozen=True)
class ModelShape:
    name: str
    dtype: str            # "fp32" | "bf16"
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_head: int
    d_ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float
    qkv_bias: bool
    seed: int
    logit_scale: float = 1.0
    attention: str = "bidirectional"     # or "block_causal": full attention inside a decoding block, causal across blocks

    @property
    def mask_id(self) -> int:
        return self.vocab - 1


@dataclass(frozen=True)
class Workload:
    """One BASELINE configuration: a model shape plus the decode job run on it."""
    index: int
    shape: ModelShape
    batch: int            # B independent sequences
    prompt_len: int       # P
    gen_len: int          # G
    block_len: int        # L
    n_drafts: int         # K, root included
    prompt_kind: str      # "uniform" | "zipf"
    prompt_seeds: tuple
    tau: float = 0.9
    k_min: int = 1
    k_max: int = 0

    @property
    def seq_len(self) -> int:
        return self.prompt_len + self.gen_len


_TINY = ModelShape("tiny-fp32", "fp32", 2, 64, 4, 4, 16, 256, 256, 1e-5, 1e4, False, 0)
_SMALL = ModelShape("small-bf16", "bf16", 8, 512, 8, 8, 64, 1408, 32000, 1e-5, 1e4, False, 2)
_LLADA = ModelShape("llada8b-shaped", "bf16", 32, 4096, 32, 32, 128, 12288, 126464, 1e-5, 5e5, False, 3)
_DREAM = ModelShape("dream7b-shaped", "bf16", 28, 3584, 28, 4, 128, 18944, 152064, 1e-6, 1e6, True, 4)

WORKLOADS: Dict[int, Workload] = {
    1: Workload(1, _TINY, 1, 16, 32, 32, 2, "uniform", (0,)),
    2: Workload(2, _SMALL, 1, 128, 256, 32, 4, "zipf", (2,)),
    3: Workload(3, _LLADA, 1, 256, 256, 32, 4, "zipf", (3,)),
    4: Workload(4, _DREAM, 1, 512, 512, 32, 6, "zipf", (4,)),
    5: Workload(5, replace(_LLADA, seed=5), 16, 256, 1024, 64, 8, "zipf", tuple(range(100, 116))),
}


def cut_down(shape: ModelShape, **changes) -> ModelShape:
    """A smaller variant of a shape (fewer layers, narrower vocab ...) for bounded CPU work."""
    return replace(shape, **changes)


# ----------------------------------------------------------------------------------------
# bf16 rounding (input preparation only)
# ----------------------------------------------------------------------------------------


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array whose values are exactly representable in bf16 (nearest-even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """bf16-representable fp32 array -> uint16 bit patterns (exact)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------

_TENSOR_IDS = {
    "tok_emb": 1, "lm_head": 2, "final_norm": 3,
    "attn_norm": 10, "wq": 11, "wk": 12, "wv": 13, "bq": 14, "bk": 15, "bv": 16, "wo": 17,
    "ffn_norm": 18, "w_gate": 19, "w_up": 20, "w_down": 21,
}
LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
_INIT_STD = 0.02


def tensor_shape(shape: ModelShape, name: str):
    d, hq, hkv, f, v = (shape.d_model, shape.n_heads * shape.d_head, shape.n_kv_heads * shape.d_head,
                        shape.d_ffn, shape.vocab)
    return {
        "tok_emb": (v, d), "lm_head": (v, d), "final_norm": (d,),
        "attn_norm": (d,), "ffn_norm": (d,),
        "wq": (hq, d), "wk": (hkv, d), "wv": (hkv, d), "bq": (hq,), "bk": (hkv,), "bv": (hkv,),
        "wo": (d, hq), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }[name]


def draw_tensor(shape: ModelShape, name: str, layer: int = -1) -> Optional[np.ndarray]:
    """One weight tensor as fp32 (bf16-representable for bf16 shapes); None for absent biases.

    ``layer`` = -1 for the three model-level tensors.  Row-major [out, in].
    """
    if name in ("bq", "bk", "bv") and not shape.qkv_bias:
        return None
    dims = tensor_shape(shape, name)
    if name.endswith("norm"):
        return np.ones(dims, dtype=np.float32)
    rng = np.random.default_rng([shape.seed, layer + 1, _TENSOR_IDS[name]])
    std = _INIT_STD
    if name in ("wo", "w_down"):
        std = _INIT_STD / math.sqrt(2.0 * shape.n_layers)
    w = rng.standard_normal(dims, dtype=np.float32)
    w *= np.float32(std)
    if shape.dtype == "bf16":
        w = round_to_bf16(w)
    return w


def draw_layer(shape: ModelShape, layer: int) -> Dict[str, Optional[np.ndarray]]:
    return {name: draw_tensor(shape, name, layer) for name in LAYER_TENSORS}


@dataclass
class HostModel:
    """All weights of one model as host fp32 arrays plus the RoPE tables."""
    shape: ModelShape
    max_seq: int
    tok_emb: np.ndarray
    final_norm: np.ndarray
    lm_head: np.ndarray
    layers: List[Dict[str, Optional[np.ndarray]]]
    rope_cos: np.ndarray = field(repr=False, default=None)
    rope_sin: np.ndarray = field(repr=False, default=None)


def rope_tables(shape: ModelShape, max_seq: int):
    """cos/sin of pos * theta^(-2j/d_head), j < d_head/2; computed in fp64, stored as fp32.

    The tables are an *input* of the forward on both sides (the paper does not specify a
    positional scheme; the architecture is taken from the benchmark configurations).
    """
    half = shape.d_head // 2
    inv_freq = shape.rope_theta ** (-np.arange(half, dtype=np.float64) * 2.0 / shape.d_head)
    ang = np.arange(max_seq, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def draw_model(shape: ModelShape, max_seq: int, threads: int = 8) -> HostModel:
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        layer_futs = [ex.submit(draw_layer, shape, l) for l in range(shape.n_layers)]
        emb = ex.submit(draw_tensor, shape, "tok_emb")
        head = ex.submit(draw_tensor, shape, "lm_head")
        layers = [f.result() for f in layer_futs]
        tok_emb, lm_head = emb.result(), head.result()
    cos, sin = rope_tables(shape, max_seq)
    return HostModel(shape, max_seq, tok_emb, draw_tensor(shape, "final_norm"), lm_head, layers, cos, sin)


# ----------------------------------------------------------------------------------------
# prompts and sequence state
# ----------------------------------------------------------------------------------------


def draw_prompt(vocab: int, length: int, seed: int, kind: str = "zipf", exponent: float = 1.1) -> np.ndarray:
    rng = np.random.default_rng(seed)
    if kind == "uniform":
        return rng.integers(0, vocab - 1, size=length, dtype=np.int64).astype(np.int32)
    ranks = np.arange(1, vocab, dtype=np.float64)          # r = 1 .. V-1
    cdf = np.cumsum(ranks ** (-exponent))
    cdf /= cdf[-1]
    u = rng.random(length)
    r = np.searchsorted(cdf, u, side="left")                 # 0-based rank index = token id
    return np.minimum(r, vocab - 2).astype(np.int32)


def initial_state(w: Workload) -> np.ndarray:
    """tokens int32 [B, N]: prompt followed by G mask ids."""
    out = np.full((w.batch, w.seq_len), w.shape.mask_id, dtype=np.int32)
    for b in range(w.batch):
        out[b, : w.prompt_len] = draw_prompt(w.shape.vocab, w.prompt_len, w.prompt_seeds[b], w.prompt_kind)
    return out


# ----------------------------------------------------------------------------------------
# synthetic (top1, conf) tables for exercising the decision kernels without a model
# ----------------------------------------------------------------------------------------


def draw_block_state(seed: int, N: int, block_start: int, L: int, vocab: int, frac_masked: float = 0.7,
                     conf_kind: str = "uniform", tie_levels: int = 0):
    """A random sequence state plus a (top1, conf) table for its active block.

    conf_kind "uniform": U(0,1) confidences, so both the threshold clause and the k_min
    fallback fire; "low": U(0, 0.2) (only the fallback fires); "high": U(0.85, 1).
    tie_levels > 0 quantises confidences to that many levels to force exact ties.
    Non-masked block positions carry the sentinel (token, -1).
    """
    rng = np.random.default_rng(seed)
    mask_id = vocab - 1
    tokens = rng.integers(0, vocab - 1, size=N, dtype=np.int64).astype(np.int32)
    masked = rng.random(L) < frac_masked
    blk = tokens[block_start: block_start + L]
    blk[masked] = mask_id
    tokens[block_start + L:] = mask_id               # later blocks are still fully masked
    lo, hi = {"uniform": (0.0, 1.0), "low": (0.0, 0.2), "high": (0.85, 1.0)}[conf_kind]
    conf = (lo + (hi - lo) * rng.random(L)).astype(np.float32)
    if tie_levels > 0:
        conf = (np.floor(conf * tie_levels) / tie_levels).astype(np.float32)
        conf = np.maximum(conf, np.float32(1.0 / (4 * tie_levels)))
    top1 = rng.integers(0, vocab - 1, size=L, dtype=np.int64).astype(np.int32)
    top1 = np.where(masked, top1, blk).astype(np.int32)
    conf = np.where(masked, conf, np.float32(-1.0)).astype(np.float32)
    return tokens, top1, conf


def draw_verifier_tables(seed: int, drafts: np.ndarray, block_start: int, L: int, vocab: int,
                         top1_t: np.ndarray, agree: float = 0.7, conf_kind: str = "uniform"):
    """Synthetic verifier outputs (v_top1, v_conf) [K, L] for given drafts.

    With probability ``agree`` the verifier's top-1 at a masked position repeats the step-t
    prediction ``top1_t`` (so that drafts are accepted at assorted depths), else it is a
    fresh random token.  Sentinels on positions that are not masked in the draft.
    """
    rng = np.random.default_rng(seed)
    K = drafts.shape[0]
    mask_id = vocab - 1
    lo, hi = {"uniform": (0.0, 1.0), "low": (0.0, 0.2), "high": (0.85, 1.0)}[conf_kind]
    v_top1 = np.empty((K, L), dtype=np.int32)
    v_conf = np.empty((K, L), dtype=np.float32)
    for k in range(K):
        blk = drafts[k, block_start: block_start + L]
        masked = blk == mask_id
        fresh = rng.integers(0, vocab - 1, size=L, dtype=np.int64).astype(np.int32)
        keep = rng.random(L) < agree
        pred = np.where(keep, top1_t, fresh).astype(np.int32)
        c = (lo + (hi - lo) * rng.random(L)).astype(np.float32)
        v_top1[k] = np.where(masked, pred, blk)
        v_conf[k] = np.where(masked, c, np.float32(-1.0))
    return v_top1, v_conf
