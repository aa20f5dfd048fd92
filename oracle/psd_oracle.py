"""CPU oracle for the Parallel Speculative Decoding (PSD) denoising step.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 NumPy implementation of what the
hot path computes, written from the paper (Sec. 3.1, Sec. 3.2, Eq. 1, Eq. 2, Alg. 1).  It
shares no code with the HIP library, and only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it.  The product path never does.

PSD is a heuristic procedure (its output depends on every decision), so the oracle is the
procedure itself, step by step, in the paper's order and notation:

    stage 1   forward -> (x_hat, c) on the masked positions of the active block   (Sec. 3.1)
              T = pi(x, c), commit x_hat on T                                      (Eq. 1)
    stage 2   sigma = residual masks sorted by step-t confidence, K drafts         (Eq. 2)
    stage 3   one batched forward over the K drafts, hierarchical acceptance over
              the draft DAG, advance to the deepest accepted draft                 (Alg. 1)

The transformer itself (RMSNorm, rotary embedding, bidirectional softmax attention with
optional grouped KV heads, SwiGLU feed-forward) is not described by the paper beyond
"bidirectional attention"; its layout comes from the benchmark configurations.  One model
family of the paper (App. A) uses context-causal block attention instead -- full attention
inside a block, causal across blocks -- which `block_causal` selects; PSD itself is unchanged.
The evaluation protocol's EOS early stopping with truncated token statistics (App. B.1) is an
option of the decode loop (`eos_id`).  `ApproximateCache` is a second model call for
bidirectional models: block rows recomputed against per-layer keys / values frozen at block entry.

Precision: everything is fp64.  The benchmark configurations other than the first are "bf16" models (bf16
operands, wider accumulation): for those, `operands="bf16"` additionally rounds the INPUTS of every
contraction (normed activations, rotated queries and keys, values, attention probabilities, attention output,
SwiGLU output, final hidden rows) to bf16, nearest-even via fp32, while sums, the residual stream, softmax
and the LM-head reduction stay fp64.  That is the computation a bf16 model defines; without the option the
oracle is the same network in exact arithmetic, from which any bf16 evaluation of an 8B-parameter shape
differs by a few 1e-2 in the logits whatever the kernels do.

Pins: every function here is pinned by tests/test_oracle_*.py (closed forms, special cases
that reduce to library routines, brute force on tiny inputs, the greedy and K=1
reductions).  Two things the paper does not publish stay "parity unpinned" against the
paper itself: the calibrated topology of the draft DAG, and the LocalLeap policy.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------
# policy and graph descriptions
# ----------------------------------------------------------------------------------------


@dataclass(frozen=True)
class Policy:
    """Transfer policy pi(tau, k_min, k_max) (Sec. 3.2 "Spatial parallel unmasking"; App. B.2).

    Greedy decoding is tau = +inf, k_min = 1.  Confidence Parallel Decoding is tau = 0.9;
    k_min = 1 is the fallback that keeps the loop moving when nothing exceeds tau.
    """
    tau: float = 0.9
    k_min: int = 1
    k_max: int = 0        # 0 = unbounded

    def __post_init__(self):
        # confidences are fp32 values; the threshold is compared in that same precision
        object.__setattr__(self, "tau", float(np.float32(self.tau)))


@dataclass(frozen=True)
class Graph:
    """Draft DAG (Sec. 3.2 "Temporal speculative drafting").

    Node k speculates on the ranks in ``rank_sets[k]`` of the speculative ordering sigma:
    rank r (0-based) stands for position sigma_{r+1}.  Node 0 is the root (empty set).
    Edges are not stored: (p, k) is an edge iff S_p is a strict subset of S_k.
    """
    rank_sets: Tuple[frozenset, ...]

    @property
    def K(self) -> int:
        return len(self.rank_sets)


def chain_graph(K: int, width: int = 1) -> Graph:
    """Prefix chain: node k fills the k*width most confident residual positions."""
    return Graph(tuple(frozenset(range(k * width)) for k in range(K)))


# ----------------------------------------------------------------------------------------
# O1: transformer forward (fp64)
# ----------------------------------------------------------------------------------------


def to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to bf16 (8 significant bits) of the fp32 image of x; returned as fp64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32).astype(F64)


def _operand(x: np.ndarray, operands: Optional[str]) -> np.ndarray:
    """x as it enters a contraction: unchanged, or rounded to bf16."""
    if operands is None:
        return x
    if operands == "bf16":
        return to_bf16(x)
    raise ValueError(f"operands={operands!r}")


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate-half rotary embedding. x: [N, heads, d_head]; cos/sin: [N, d_head/2]."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def block_causal_visibility(N: int, L: int) -> np.ndarray:
    """visible[i, j] for context-causal block attention (App. A, the block-diffusion model family): position i
    sees every position of its own block of L (full attention inside the block) and of all earlier blocks
    (causal across blocks), and nothing later.  Blocks are [0, L), [L, 2L), ... from the start of the sequence."""
    blk = np.arange(N) // L
    return blk[None, :] <= blk[:, None]


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, operands: Optional[str] = None,
              visible: Optional[np.ndarray] = None) -> np.ndarray:
    """Softmax attention. q: [Nq, H, dh]; k, v: [Nk, Hkv, dh] -> [Nq, H, dh].  Bidirectional (every query sees
    every key) unless `visible` [Nq, Nk] says which keys j query i may see.

    Query head j reads KV head j // (H / Hkv).  With operands="bf16" the probabilities enter the second
    contraction rounded (as exp(s - max), before the division by their exact sum).
    """
    N, H, dh = q.shape
    group = H // k.shape[1]
    out = np.empty_like(q)
    for j in range(H):
        kj, vj = k[:, j // group, :], v[:, j // group, :]
        s = q[:, j, :] @ kj.T / np.sqrt(F64(dh))
        if visible is not None:
            s = np.where(visible, s, -np.inf)
        if operands is None:
            out[:, j, :] = softmax_rows(s) @ vj
        else:
            e = np.exp(s - s.max(axis=-1, keepdims=True))
            out[:, j, :] = (_operand(e, operands) @ vj) / e.sum(axis=-1, keepdims=True)
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _w(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


def layer_forward(h: np.ndarray, lw: dict, shape, cos: np.ndarray, sin: np.ndarray,
                  operands: Optional[str] = None, visible: Optional[np.ndarray] = None,
                  kv_out: Optional[list] = None, kv_frozen: Optional[tuple] = None) -> np.ndarray:
    """One pre-norm transformer layer on the residual stream h [N, d] (cos / sin: the rotary rows of these N
    positions).  kv_out: a list that receives this layer's (rotated keys, values), each [N, Hkv, dh], as the
    attention uses them.  kv_frozen = (k, v): further keys and values, from positions that are not among the
    rows of h, which every query also sees (the approximate cache)."""
    N = h.shape[0]
    H, Hkv, dh = shape.n_heads, shape.n_kv_heads, shape.d_head
    a = _operand(rmsnorm(h, _w(lw["attn_norm"]), shape.rms_eps), operands)
    q = a @ _w(lw["wq"]).T
    k = a @ _w(lw["wk"]).T
    v = a @ _w(lw["wv"]).T
    if lw.get("bq") is not None:
        q, k, v = q + _w(lw["bq"]), k + _w(lw["bk"]), v + _w(lw["bv"])
    q = _operand(rope(q.reshape(N, H, dh), cos, sin), operands)
    k = _operand(rope(k.reshape(N, Hkv, dh), cos, sin), operands)
    v = _operand(v.reshape(N, Hkv, dh), operands)
    if kv_out is not None:
        kv_out.append((k, v))
    if kv_frozen is not None:
        k, v = np.concatenate([kv_frozen[0], k]), np.concatenate([kv_frozen[1], v])
    o = _operand(attention(q, k, v, operands, visible).reshape(N, H * dh), operands)
    h = h + o @ _w(lw["wo"]).T
    f = _operand(rmsnorm(h, _w(lw["ffn_norm"]), shape.rms_eps), operands)
    g = _operand(silu(f @ _w(lw["w_gate"]).T) * (f @ _w(lw["w_up"]).T), operands)
    h = h + g @ _w(lw["w_down"]).T
    return h


def forward_hidden(model, tokens: np.ndarray, operands: Optional[str] = None,
                   block_causal: Optional[int] = None, kv_out: Optional[list] = None) -> np.ndarray:
    """Final-normed hidden states y [N, d] for one sequence (mask positions hold mask_id,
    which has an ordinary embedding row).  Positions are 0..N-1.  block_causal = L switches the
    attention of every layer from bidirectional to context-causal blocks of L."""
    tokens = np.asarray(tokens)
    N = tokens.shape[0]
    cos, sin = _w(model.rope_cos[:N]), _w(model.rope_sin[:N])
    h = _w(model.tok_emb[tokens])
    visible = None if block_causal is None else block_causal_visibility(N, block_causal)
    for lw in model.layers:
        h = layer_forward(h, lw, model.shape, cos, sin, operands, visible, kv_out)
    return _operand(rmsnorm(h, _w(model.final_norm), model.shape.rms_eps), operands)


def forward_hidden_frozen(model, tokens: np.ndarray, block_start: int, L: int, frozen: list,
                          operands: Optional[str] = None) -> np.ndarray:
    """Final-normed hidden states of the block rows only, [L, d], with every layer's keys and values of the
    positions OUTSIDE the block taken from `frozen` (one (k, v) pair per layer, [N - L, Hkv, dh]) instead of
    being recomputed: the forward of a bidirectional model under an approximate KV cache.  The block rows keep
    their positions block_start .. block_start + L - 1."""
    blk = slice(block_start, block_start + L)
    cos, sin = _w(model.rope_cos[blk]), _w(model.rope_sin[blk])
    h = _w(model.tok_emb[np.asarray(tokens)[blk]])
    for lw, kv in zip(model.layers, frozen):
        h = layer_forward(h, lw, model.shape, cos, sin, operands, None, None, kv)
    return _operand(rmsnorm(h, _w(model.final_norm), model.shape.rms_eps), operands)


class ApproximateCache:
    """Model call of a fully bidirectional model under an approximate KV cache over prefix and suffix.

    The paper notes that KV-cache sharing can cut redundant computation (Sec. 3.2 stage 3) without fixing a
    scheme; for bidirectional models any cache is an approximation.  The scheme here is the published
    "dual cache" idea for block-wise diffusion decoding, restated: the first model call on a block (Alg. 1's
    stage-1 call on the state the block is entered with) is an exact forward over the whole sequence, and it
    freezes, per layer, the rotated keys and the values of every position outside the block.  Every later
    call on that block (verification batches, later iterations) recomputes the block rows only and attends
    to the frozen keys / values for the rest, which by then are stale: they were computed from the block's
    earlier content.  Entering another block refreshes.  Calls are (tokens, block_start, L) ->
    (top1, conf) like any model call of the loop; `logits` keeps the last call's block logits."""

    def __init__(self, model, operands: Optional[str] = None):
        self.model, self.operands = model, operands
        self.block, self.outside, self.frozen, self.logits = None, None, None, None
        self.refreshes = 0

    def _outside(self, tokens, block_start, L):
        return np.concatenate([tokens[:block_start], tokens[block_start + L:]])

    def __call__(self, tokens: np.ndarray, block_start: int, L: int):
        tokens = np.asarray(tokens)
        m = self.model
        if self.block != (block_start, L):
            kv = []
            y = forward_hidden(m, tokens, self.operands, None, kv)[block_start: block_start + L]
            keep = np.r_[0:block_start, block_start + L:tokens.shape[0]]
            self.frozen = [(k[keep], v[keep]) for k, v in kv]
            self.block, self.outside = (block_start, L), self._outside(tokens, block_start, L).copy()
            self.refreshes += 1
        else:
            if not np.array_equal(self._outside(tokens, block_start, L), self.outside):
                raise ValueError("the cache holds keys and values of other tokens outside the block")
            y = forward_hidden_frozen(m, tokens, block_start, L, self.frozen, self.operands)
        z = m.shape.logit_scale * (y @ _w(m.lm_head).T)
        self.logits = z
        x_hat, c = top1_confidence(z, m.shape.mask_id)
        blk = tokens[block_start: block_start + L]
        masked = blk == m.shape.mask_id
        return np.where(masked, x_hat, blk).astype(np.int32), np.where(masked, c, -1.0).astype(np.float32)


def block_logits(model, tokens: np.ndarray, block_start: int, L: int, operands: Optional[str] = None,
                 block_causal: bool = False) -> np.ndarray:
    """z = logit_scale * y W_lm^T on the block rows, [L, V] (mask column not yet excluded).  block_causal:
    context-causal block attention with the decoding block length L (block_start a multiple of L)."""
    if block_causal and block_start % L:
        raise ValueError("context-causal blocks are aligned to multiples of the block length")
    y = forward_hidden(model, tokens, operands, L if block_causal else None)[block_start: block_start + L]
    return model.shape.logit_scale * (y @ _w(model.lm_head).T)


# ----------------------------------------------------------------------------------------
# O2: top-1 token and confidence (Sec. 3.1)
# ----------------------------------------------------------------------------------------


def top1_confidence(z: np.ndarray, mask_id: int) -> Tuple[np.ndarray, np.ndarray]:
    """x_hat = argmax_v p(v), c = max_v p(v) with p = softmax(z) over the vocabulary V,
    which does not contain the mask token (Sec. 3.1): its logit is excluded.
    Ties in the argmax go to the lowest token id."""
    z = np.array(z, dtype=F64, copy=True)
    z[..., mask_id] = -np.inf
    x_hat = np.argmax(z, axis=-1)
    z_top = np.take_along_axis(z, x_hat[..., None], axis=-1)
    c = 1.0 / np.exp(z - z_top).sum(axis=-1)
    return x_hat.astype(np.int32), c


def forward_confidence(model, tokens: np.ndarray, block_start: int, L: int,
                       return_logits: bool = False, operands: Optional[str] = None, block_causal: bool = False):
    """(top1 int32 [L], conf fp32 [L]) for the active block of one sequence.

    Masked block positions carry the prediction; the others carry the sentinel
    (tokens[i], -1).  The confidence is rounded to fp32 here, the precision in which both
    sides take every later decision.
    """
    tokens = np.asarray(tokens)
    z = block_logits(model, tokens, block_start, L, operands, block_causal)
    x_hat, c = top1_confidence(z, model.shape.mask_id)
    blk = tokens[block_start: block_start + L]
    masked = blk == model.shape.mask_id
    top1 = np.where(masked, x_hat, blk).astype(np.int32)
    conf = np.where(masked, c, -1.0).astype(np.float32)
    if return_logits:
        return top1, conf, z
    return top1, conf


# ----------------------------------------------------------------------------------------
# O3: transfer policy and Eq. 1
# ----------------------------------------------------------------------------------------


def confidence_order(positions: Sequence[int], conf: np.ndarray) -> List[int]:
    """Positions ordered by confidence descending, ties by lower position first."""
    return sorted(positions, key=lambda i: (-float(conf[i]), i))


def policy_select(masked_positions: Sequence[int], conf: np.ndarray, policy: Policy) -> List[int]:
    """T = pi(x, c) over block-local positions (Sec. 3.2; App. B.2).

    T = {i : c_i > tau}  union  {the k_min most confident};  capped to the k_max most
    confident of those when k_max > 0.  Returned in confidence order.
    """
    order = confidence_order(masked_positions, conf)
    chosen = [i for r, i in enumerate(order) if float(conf[i]) > policy.tau or r < policy.k_min]
    if policy.k_max > 0:
        chosen = chosen[: policy.k_max]
    return chosen


def masked_in_block(tokens: np.ndarray, block_start: int, L: int, mask_id: int) -> List[int]:
    """Block-local indices of the positions still holding the mask token."""
    return [j for j in range(L) if int(tokens[block_start + j]) == mask_id]


def select_unmask(tokens: np.ndarray, block_start: int, L: int, top1: np.ndarray, conf: np.ndarray,
                  policy: Policy, mask_id: int):
    """Apply pi and the state update of Eq. 1. Returns (new tokens, transfer_mask uint8 [L])."""
    T = policy_select(masked_in_block(tokens, block_start, L, mask_id), conf, policy)
    new = np.array(tokens, dtype=np.int32, copy=True)
    transfer = np.zeros(L, dtype=np.uint8)
    for j in T:
        new[block_start + j] = top1[j]
        transfer[j] = 1
    return new, transfer


# ----------------------------------------------------------------------------------------
# O4: speculative ordering and draft assembly (Eq. 2)
# ----------------------------------------------------------------------------------------


def node_positions(graph: Graph, sigma: Sequence[int]) -> List[frozenset]:
    """S_k as block-local position sets; ranks beyond the m residual masks are dropped."""
    m = len(sigma)
    return [frozenset(sigma[r] for r in ranks if r < m) for ranks in graph.rank_sets]


def build_drafts(tokens_next: np.ndarray, block_start: int, L: int, top1_t: np.ndarray, conf_t: np.ndarray,
                 graph: Graph, mask_id: int):
    """sigma, m and the K drafts from the post-commit state x^(t+1) and the step-t (x_hat, c).

    Returns (sigma int32 [L] padded with -1, m, drafts int32 [K, N]).
    """
    residual = masked_in_block(tokens_next, block_start, L, mask_id)
    order = confidence_order(residual, conf_t)
    m = len(order)
    S = node_positions(graph, order)
    drafts = np.tile(np.asarray(tokens_next, dtype=np.int32), (graph.K, 1))
    for k in range(graph.K):
        for j in S[k]:
            drafts[k, block_start + j] = top1_t[j]
    sigma = np.full(L, -1, dtype=np.int32)
    sigma[:m] = order
    return sigma, m, drafts


# ----------------------------------------------------------------------------------------
# O6 / O7: hierarchical acceptance and state advance (Alg. 1, stage 3)
# ----------------------------------------------------------------------------------------


def edge_accepts(p: int, k: int, S: List[frozenset], drafts: np.ndarray, block_start: int, L: int,
                 v_top1: np.ndarray, v_conf: np.ndarray, policy: Policy, mask_id: int) -> bool:
    """A_pi on every newly speculated position of edge (p, k).

    Position i passes when parent p's verifier prediction equals the drafted token AND the
    policy, applied to p's verifier output over p's own masked positions, would itself
    commit i ("the same acceptance criterion that pi uses to commit tokens").
    """
    T_p = set(policy_select(masked_in_block(drafts[p], block_start, L, mask_id), v_conf[p], policy))
    for j in S[k] - S[p]:
        if int(v_top1[p, j]) != int(drafts[k, block_start + j]) or j not in T_p:
            return False
    return True


def hierarchical_accept(drafts: np.ndarray, block_start: int, L: int, sigma: np.ndarray, m: int,
                        graph: Graph, policy: Policy, v_top1: np.ndarray, v_conf: np.ndarray, mask_id: int):
    """Accepted set A (uint8 [K]) and k* = the accepted node revealing the most positions.

    Nodes are visited by |S_k| ascending (a topological order of the strict-subset DAG),
    ties by node index; k* ties go to the lowest node index.
    """
    S = node_positions(graph, [int(s) for s in sigma[:m]])
    K = graph.K
    accepted = np.zeros(K, dtype=np.uint8)
    accepted[0] = 1
    for k in sorted(range(1, K), key=lambda n: (len(S[n]), n)):
        for p in range(K):
            if accepted[p] and S[p] < S[k] and edge_accepts(p, k, S, drafts, block_start, L,
                                                            v_top1, v_conf, policy, mask_id):
                accepted[k] = 1
                break
    k_star = min((k for k in range(K) if accepted[k]), key=lambda n: (-len(S[n]), n))
    return accepted, int(k_star)


def advance(drafts: np.ndarray, k_star: int, block_start: int, L: int, v_top1: np.ndarray,
            v_conf: np.ndarray, policy: Policy, mask_id: int):
    """x <- draft k*, then one more application of pi on k*'s verifier output (Alg. 1,
    last line of stage 3).  Returns (tokens, number of post-verify commits)."""
    x = np.array(drafts[k_star], dtype=np.int32, copy=True)
    if not masked_in_block(x, block_start, L, mask_id):
        return x, 0
    x, transfer = select_unmask(x, block_start, L, v_top1[k_star], v_conf[k_star], policy, mask_id)
    return x, int(transfer.sum())


# ----------------------------------------------------------------------------------------
# O8: the block loop (Alg. 1) and the outer semi-autoregressive loop
# ----------------------------------------------------------------------------------------


@dataclass
class Stats:
    invocations: int = 0
    tokens_policy: int = 0
    tokens_draft: int = 0
    tokens_postverify: int = 0
    depth_hist: List[int] = field(default_factory=lambda: [0] * 32)
    tokens_counted: int = 0     # resolved positions at or before the EOS position (all of them without an EOS)
    stopped: bool = False       # an EOS token was produced and early stopping was on
    eos_pos: int = -1           # position of the first EOS token in the sequence when stopped

    @property
    def tokens(self) -> int:
        return self.tokens_policy + self.tokens_draft + self.tokens_postverify

    @property
    def tpf(self) -> float:
        return self.tokens / max(1, self.invocations)

    @property
    def tpf_counted(self) -> float:
        """Tokens per forward over the tokens up to and including the EOS position (App. B.1)."""
        return self.tokens_counted / max(1, self.invocations)


ConfidenceFn = Callable[[np.ndarray, int, int], Tuple[np.ndarray, np.ndarray]]


def first_eos(tokens: np.ndarray, block_start: int, L: int, eos_id: Optional[int]) -> Optional[int]:
    """Position of the first EOS token inside the block, None without one (or without early stopping)."""
    if eos_id is None:
        return None
    hits = [i for i in range(block_start, block_start + L) if tokens[i] == eos_id]
    return hits[0] if hits else None


def decode_block(confidence_fn: ConfidenceFn, tokens: np.ndarray, block_start: int, L: int, policy: Policy,
                 graph: Graph, mask_id: int, stats: Optional[Stats] = None, trace: Optional[list] = None,
                 eos_id: Optional[int] = None, single_forward: bool = False):
    """Alg. 1 on one block of one sequence.  ``confidence_fn(tokens, block_start, L)`` is the
    model call (forward + top-1 confidence); a batched verification is K such calls counted
    as one invocation.

    EOS early stopping (App. B.1), when ``eos_id`` is given: decoding ends as soon as an EOS token
    has been produced -- read as: after every update of the state (the stage-1 commit, and the
    advance with its post-verification commit) the block is searched for ``eos_id`` and the loop
    ends if it is there, whatever is still masked.  ``tokens_counted`` is the number of positions this call
    resolved at or before the first EOS position (tokens unmasked beyond it are discarded from
    the statistic, in whichever iteration they were unmasked); without an EOS every resolved
    position counts.

    ``single_forward`` (a variant, NOT the literal Alg. 1): the last line of stage 3 commits the verifier's
    predictions of the accepted draft k* that pass the policy; the literal loop then calls the model again on
    the committed state (stage 1 of the next iteration).  The variant lets that post-verification commit BE
    the next iteration's stage-1 commit and builds the next drafts from k*'s verifier output (x_hat_k*, c_k*)
    -- the model's exact prediction on draft k*, i.e. on the state just before that commit -- so that an
    iteration costs one model call (the batched verification) instead of two.  Only the call that enters a
    block is a stage-1 call.  Every commit still comes from an exact forward of an exact state; what goes
    stale is only the table the SPECULATION is drawn from.  Results differ from the literal loop in
    general."""
    stats = stats if stats is not None else Stats()
    x = np.array(tokens, dtype=np.int32, copy=True)
    if eos_id is not None and eos_id == mask_id:
        raise ValueError("the EOS token cannot be the mask token")
    masked_on_entry = [block_start + j for j in masked_in_block(x, block_start, L, mask_id)]

    def finish(x):
        eos = first_eos(x, block_start, L, eos_id)
        if eos is not None:
            stats.stopped, stats.eos_pos = True, eos
        limit = eos if eos is not None else block_start + L - 1
        stats.tokens_counted += sum(1 for i in masked_on_entry if i <= limit and x[i] != mask_id)
        return x, stats

    have_tables = False      # single_forward: (top1, conf) already hold the output the last commit was taken from
    while masked_in_block(x, block_start, L, mask_id):
        if not have_tables:
            top1, conf = confidence_fn(x, block_start, L)                   # stage 1
            stats.invocations += 1
            x, transfer = select_unmask(x, block_start, L, top1, conf, policy, mask_id)
            stats.tokens_policy += int(transfer.sum())
            if trace is not None:
                trace.append(("commit", [block_start + j for j in range(L) if transfer[j]]))
            if first_eos(x, block_start, L, eos_id) is not None:
                break
            if not masked_in_block(x, block_start, L, mask_id):
                break
        sigma, m, drafts = build_drafts(x, block_start, L, top1, conf, graph, mask_id)   # stage 2
        v = [confidence_fn(drafts[k], block_start, L) for k in range(graph.K)]            # stage 3
        stats.invocations += 1
        v_top1 = np.stack([t for t, _ in v])
        v_conf = np.stack([c for _, c in v])
        accepted, k_star = hierarchical_accept(drafts, block_start, L, sigma, m, graph, policy,
                                               v_top1, v_conf, mask_id)
        depth = len(node_positions(graph, [int(s) for s in sigma[:m]])[k_star])
        x, n_post = advance(drafts, k_star, block_start, L, v_top1, v_conf, policy, mask_id)
        stats.tokens_draft += depth
        stats.tokens_postverify += n_post
        stats.depth_hist[depth] += 1
        if trace is not None:
            trace.append(("verify", k_star, depth, n_post, accepted.copy()))
        if first_eos(x, block_start, L, eos_id) is not None:
            break
        if single_forward:
            # the post-verification commit above was the next iteration's stage-1 commit; its drafts come
            # from the same output, the verifier's tables of draft k*
            top1, conf, have_tables = v_top1[k_star], v_conf[k_star], True
    return finish(x)


def decode(confidence_fn: ConfidenceFn, tokens: np.ndarray, prompt_len: int, L: int, policy: Policy,
           graph: Graph, mask_id: int, stats: Optional[Stats] = None, trace: Optional[list] = None,
           eos_id: Optional[int] = None, single_forward: bool = False):
    """Semi-autoregressive generation: blocks left to right, the next block starts only once
    the current one is fully resolved (App. B.1).  Later blocks stay masked meanwhile.  With
    ``eos_id`` the generation ends with the block that produced an EOS token."""
    stats = stats if stats is not None else Stats()
    x = np.array(tokens, dtype=np.int32, copy=True)
    N = x.shape[0]
    for block_start in range(prompt_len, N, L):
        x, stats = decode_block(confidence_fn, x, block_start, min(L, N - block_start), policy, graph,
                                mask_id, stats, trace, eos_id, single_forward)
        if stats.stopped:
            break
    return x, stats


def model_confidence_fn(model, operands: Optional[str] = None, block_causal: bool = False) -> ConfidenceFn:
    return lambda tokens, block_start, L: forward_confidence(model, tokens, block_start, L, operands=operands,
                                                             block_causal=block_causal)
