"""CPU oracle for the ESP (Embedding-Space Probing) speculate-and-verify decode step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the HIP
library must compute.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import it; it imports nothing from the package and shares no
code, tables or helpers with the GPU path.  All floating point is numpy float64
unless a passage below says otherwise (the paper fixes no precision; it treats the
decoder f_theta of Sec. 2, Eq. 1 as a black box).  Inputs that are bf16 on the GPU
arrive here as the same values held in float32/float64 arrays.

What follows the paper, and where:
  block layout, positions, tree mask ... Sec. 3.3 (Fig. 3), App. C, App. E (Fig. 7)
  proposal (Top-K of mask-row softmax) . Sec. 2 Eq. 2, Sec. 3.3
  pruning .............................. Sec. 3.5, App. F.6
  dynamic tree ......................... Sec. 3.4, Alg. 1, App. C (Fig. 6)
  verification ......................... Sec. 2 Eq. 3, Sec. 3.3, Sec. 4 (tau)
  mask embedding init / update ......... Sec. 3.1 Eq. 4, Eq. 5
The decoder itself (pre-norm, RMSNorm, rotary embedding, grouped-query attention,
SwiGLU MLP, untied LM head) is the textbook architecture named by the workload
shapes, not something the paper defines.

Pins (tests/test_oracle_*.py): library decoder (transformers Llama / Qwen3) on a
chain and on a tree with an explicit 4-D mask; path-by-path sequential decoding
(Sec. 2, App. C); brute-force path enumeration for verification; losslessness
against plain greedy decoding; full-sort Top-K; brute-force Alg. 1; block-complexity
closed form and the worked BC=30 example; the Lemma of Sec. 3.2 as a property.
Parity unpinned: none of the functions below; absolute activation values of the
random-weight workloads are pinned only through the library decoder.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64

LAYOUT_PER_NODE = 0    # every node row owns k mask rows (Sec. 3.3, Fig. 3): R = (k+1) N
LAYOUT_ROOT_CHAIN = 1  # only the root owns a chain of k mask rows: R = N + k


# --------------------------------------------------------------------------------------
# model description (plain containers, no arithmetic)
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class Model:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rope_theta: float
    rms_eps: float
    qk_norm: bool
    weights: dict  # embed, lm_head, final_norm, layers[...] as arrays ([out, in] matrices)


def as_f64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------------------
# decoder building blocks (textbook definitions)
# --------------------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    x = as_f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * as_f64(gain)


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, half-split pairing: element i pairs with i + hd/2,
    pair i turns by angle pos * theta^(-2 i / hd).  x is [rows, heads, hd]."""
    x = as_f64(x)
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = F64(theta) ** (-(np.arange(half, dtype=F64) * 2.0) / hd)
    ang = as_f64(pos)[:, None] * inv_freq[None, :]          # [rows, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(v: np.ndarray) -> np.ndarray:
    v = as_f64(v)
    e = np.exp(v - np.max(v))
    return e / np.sum(e)


def silu(v: np.ndarray) -> np.ndarray:
    return v / (1.0 + np.exp(-v))


# --------------------------------------------------------------------------------------
# block layout: rows, positions, visibility (Sec. 3.3 Fig. 3; App. C; App. E Fig. 7)
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class Block:
    """One forward block.  Rows 0..N-1 are tree nodes in (depth, creation) order, row 0
    the last accepted token; mask rows follow at the end (Fig. 3)."""
    tok: np.ndarray          # [N] token ids of the node rows
    parent: np.ndarray       # [N] tree parent of each node row, -1 for the root
    k: int                   # mask tokens per chain
    layout: int
    # derived, all of length R:
    kind: np.ndarray = None      # 0 node, 1 mask
    attach: np.ndarray = None    # node row a mask row hangs on (node rows: themselves)
    mask_j: np.ndarray = None    # 1..k for mask rows, 0 for node rows
    depth: np.ndarray = None     # node depth; for a mask row depth(attach) + j
    visible: np.ndarray = None   # [R, R] bool: row r may attend to block row c

    @property
    def n_nodes(self) -> int:
        return len(self.tok)

    @property
    def n_rows(self) -> int:
        return len(self.kind)

    def mask_row(self, node: int, j: int) -> int:
        """Row index of mask j (1-based) of `node`."""
        if self.layout == LAYOUT_PER_NODE:
            return self.n_nodes + node * self.k + (j - 1)
        if node != 0:
            raise ValueError("root-chain layout has mask rows on the root only")
        return self.n_nodes + (j - 1)


def make_block(tok: Sequence[int], parent: Sequence[int], k: int, layout: int) -> Block:
    tok = np.asarray(tok, dtype=np.int64)
    parent = np.asarray(parent, dtype=np.int64)
    n = len(tok)
    if n < 1 or parent[0] != -1:
        raise ValueError("row 0 must be the root")
    node_depth = np.zeros(n, dtype=np.int64)
    for i in range(1, n):
        if not (0 <= parent[i] < i):
            raise ValueError("parents must precede children")
        node_depth[i] = node_depth[parent[i]] + 1
    owners = list(range(n)) if layout == LAYOUT_PER_NODE else [0]
    if k == 0:
        owners = []
    r_total = n + k * len(owners)
    kind = np.zeros(r_total, dtype=np.int64)
    attach = np.arange(r_total, dtype=np.int64)
    mask_j = np.zeros(r_total, dtype=np.int64)
    depth = np.zeros(r_total, dtype=np.int64)
    depth[:n] = node_depth
    row = n
    for a in owners:
        for j in range(1, k + 1):
            kind[row], attach[row], mask_j[row] = 1, a, j
            depth[row] = node_depth[a] + j      # positions continue past the node (Fig. 7)
            row += 1
    # visibility from the parent pointers: a node sees itself and its ancestors; mask j
    # of node a sees a, a's ancestors and masks 1..j of the same chain (App. C).
    vis = np.zeros((r_total, r_total), dtype=bool)
    for r in range(r_total):
        a = int(attach[r])
        c = a
        while c >= 0:
            vis[r, c] = True
            c = int(parent[c])
        if kind[r] == 1:
            first = r - (int(mask_j[r]) - 1)
            vis[r, first:r + 1] = True
    blk = Block(tok, parent, k, layout, kind, attach, mask_j, depth, vis)
    return blk


def block_complexity(widths: Sequence[int]) -> int:
    """Rows of one forward pass for a static tree [K_1..K_k] (Sec. 3.3)."""
    k = len(widths)
    return (k + 1) * (1 + int(sum(widths)))


# --------------------------------------------------------------------------------------
# decoder forward of a block against a KV cache
# --------------------------------------------------------------------------------------
def block_inputs(model: Model, blk: Block, mask_embed: np.ndarray) -> np.ndarray:
    """h0: node rows take E[token], mask row j takes the mask vector m_j (Sec. 3.1)."""
    emb = model.weights["embed"]
    h = np.zeros((blk.n_rows, model.d_model), dtype=F64)
    for r in range(blk.n_rows):
        if blk.kind[r] == 0:
            h[r] = as_f64(emb[int(blk.tok[r])])
        else:
            h[r] = as_f64(mask_embed[int(blk.mask_j[r]) - 1])
    return h


def tree_attention(q: np.ndarray, k_cache, v_cache, k_blk, v_blk, visible: np.ndarray) -> np.ndarray:
    """Tree-masked grouped-query attention of one layer (Sec. 3.3, App. C).  q [R, hq, hd]
    (already rotated); k_cache/v_cache [L, hkv, hd] all visible to every row; k_blk/v_blk
    [R, hkv, hd] of the block rows, row r seeing block row c iff visible[r, c].  Query head h
    reads kv head h // (hq / hkv); scores scaled by 1/sqrt(hd); softmax with max subtraction."""
    q = as_f64(q)
    kc, vc, kb, vb = as_f64(k_cache), as_f64(v_cache), as_f64(k_blk), as_f64(v_blk)
    R, hq, hd = q.shape
    group = hq // kb.shape[1]
    scale = 1.0 / np.sqrt(F64(hd))
    att = np.zeros((R, hq, hd), dtype=F64)
    for r in range(R):
        cols = np.nonzero(visible[r])[0]
        for hh in range(hq):
            g = hh // group
            keys = np.concatenate([kc[:, g, :], kb[cols, g, :]], axis=0)
            vals = np.concatenate([vc[:, g, :], vb[cols, g, :]], axis=0)
            p = softmax((keys @ q[r, hh]) * scale)
            att[r, hh] = p @ vals
    return att


def tree_forward(model: Model, blk: Block, mask_embed, k_cache, v_cache, cache_len: int,
                 h0: Optional[np.ndarray] = None, want_logits_rows=None):
    """Forward all rows of `blk` in one call.  k_cache/v_cache: [n_layers][>=cache_len,
    n_kv_heads, head_dim].  Row r sits at position cache_len + depth[r] and attends to
    cache slots 0..cache_len-1 and to the block rows its visibility row allows.

    Returns (logits [R, V] (or only the requested rows), hidden [R, d] after the final
    norm, k_new, v_new [n_layers, R, n_kv_heads, head_dim])."""
    w = model.weights
    R, d, hd = blk.n_rows, model.d_model, model.head_dim
    hq, hkv = model.n_q_heads, model.n_kv_heads
    h = block_inputs(model, blk, mask_embed) if h0 is None else as_f64(h0).copy()
    pos = cache_len + blk.depth
    k_new = np.zeros((model.n_layers, R, hkv, hd), dtype=F64)
    v_new = np.zeros((model.n_layers, R, hkv, hd), dtype=F64)
    for l in range(model.n_layers):
        lw = w["layers"][l]
        x = rmsnorm(h, lw["norm_attn"], model.rms_eps)
        q = (x @ as_f64(lw["wq"]).T).reshape(R, hq, hd)
        kk = (x @ as_f64(lw["wk"]).T).reshape(R, hkv, hd)
        vv = (x @ as_f64(lw["wv"]).T).reshape(R, hkv, hd)
        if model.qk_norm:   # per-head RMSNorm over head_dim, before the rotation
            q = rmsnorm(q, lw["q_norm"], model.rms_eps)
            kk = rmsnorm(kk, lw["k_norm"], model.rms_eps)
        q = rope(q, pos, model.rope_theta)
        kk = rope(kk, pos, model.rope_theta)
        k_new[l], v_new[l] = kk, vv
        att = tree_attention(q, k_cache[l][:cache_len], v_cache[l][:cache_len], kk, vv, blk.visible)
        h = h + att.reshape(R, hq * hd) @ as_f64(lw["wo"]).T
        x = rmsnorm(h, lw["norm_mlp"], model.rms_eps)
        gate = x @ as_f64(lw["w_gate"]).T
        up = x @ as_f64(lw["w_up"]).T
        h = h + (silu(gate) * up) @ as_f64(lw["w_down"]).T
    hidden = rmsnorm(h, w["final_norm"], model.rms_eps)
    rows = np.arange(R) if want_logits_rows is None else np.asarray(want_logits_rows, dtype=np.int64)
    logits = lm_head_logits(model, hidden[rows])
    return logits, hidden, k_new, v_new


def lm_head_logits(model: Model, hidden_rows: np.ndarray) -> np.ndarray:
    """LM head on final-norm hidden states: logits = hidden @ lm_head^T (untied head)."""
    return as_f64(hidden_rows) @ as_f64(model.weights["lm_head"]).T


def sequence_forward(model: Model, embeds: np.ndarray, positions: Sequence[int],
                     k_cache, v_cache, cache_len: int):
    """Ordinary causal decoding, one row at a time with a growing cache: row t attends to
    cache slots 0..cache_len-1 and rows 0..t of `embeds`.  A separate code path from
    tree_forward (no visibility matrix), used as the definition the tree forward must
    reproduce path by path.  Returns (logits [T, V], k_rows, v_rows [n_layers, T, hkv, hd])."""
    w = model.weights
    T, hd = len(embeds), model.head_dim
    hq, hkv = model.n_q_heads, model.n_kv_heads
    group = hq // hkv
    ks = [[as_f64(k_cache[l][i]) for i in range(cache_len)] for l in range(model.n_layers)]
    vs = [[as_f64(v_cache[l][i]) for i in range(cache_len)] for l in range(model.n_layers)]
    logits = np.zeros((T, model.vocab), dtype=F64)
    for t in range(T):
        h = as_f64(embeds[t]).copy()
        p1 = np.asarray([positions[t]])
        for l in range(model.n_layers):
            lw = w["layers"][l]
            x = rmsnorm(h, lw["norm_attn"], model.rms_eps)
            q = (as_f64(lw["wq"]) @ x).reshape(1, hq, hd)
            kk = (as_f64(lw["wk"]) @ x).reshape(1, hkv, hd)
            vv = (as_f64(lw["wv"]) @ x).reshape(1, hkv, hd)
            if model.qk_norm:
                q = rmsnorm(q, lw["q_norm"], model.rms_eps)
                kk = rmsnorm(kk, lw["k_norm"], model.rms_eps)
            q = rope(q, p1, model.rope_theta)[0]
            kk = rope(kk, p1, model.rope_theta)[0]
            ks[l].append(kk)
            vs[l].append(vv[0])
            kmat = np.stack(ks[l])      # [len, hkv, hd]
            vmat = np.stack(vs[l])
            out = np.zeros((hq, hd), dtype=F64)
            for hh in range(hq):
                g = hh // group
                p = softmax((kmat[:, g, :] @ q[hh]) / np.sqrt(F64(hd)))
                out[hh] = p @ vmat[:, g, :]
            h = h + as_f64(lw["wo"]) @ out.reshape(-1)
            x = rmsnorm(h, lw["norm_mlp"], model.rms_eps)
            h = h + as_f64(lw["w_down"]) @ (silu(as_f64(lw["w_gate"]) @ x) * (as_f64(lw["w_up"]) @ x))
        logits[t] = as_f64(w["lm_head"]) @ rmsnorm(h, w["final_norm"], model.rms_eps)
    k_rows = np.stack([np.stack(ks[l][cache_len:]) for l in range(model.n_layers)])
    v_rows = np.stack([np.stack(vs[l][cache_len:]) for l in range(model.n_layers)])
    return logits, k_rows, v_rows


# --------------------------------------------------------------------------------------
# verification (Sec. 2 Eq. 3; Sec. 3.3; tau of Sec. 4)
# --------------------------------------------------------------------------------------
def argmax_lowest(v: np.ndarray) -> int:
    """Index of the maximum, lowest index on ties."""
    return int(np.argmax(v))   # numpy returns the first maximum


def verify_accept(tok: Sequence[int], parent: Sequence[int], g: Sequence[int]):
    """Greedy longest accepted path.  g[r] is the base model's own next token after node
    r.  A child is accepted iff its token equals g at its parent; the walk stops at the
    first miss and g at the last accepted node is emitted as the bonus token.
    Returns (n_star, accepted_rows, emitted_tokens); len(emitted) = len(accepted) + 1."""
    cur = 0
    accepted: List[int] = []
    while True:
        nxt = -1
        for c in range(len(tok)):
            if parent[c] == cur and int(tok[c]) == int(g[cur]):
                nxt = c
                break
        if nxt < 0:
            break
        accepted.append(nxt)
        cur = nxt
    emitted = [int(tok[c]) for c in accepted] + [int(g[cur])]
    return cur, accepted, emitted


def calls_reduction_percent(tau: float) -> float:
    """Model calls scale as 1/tau (Sec. 4): reduction over one call per token, percent."""
    return 100.0 * (1.0 - 1.0 / tau)


# --------------------------------------------------------------------------------------
# sample matching at temperature 1 (Sec. 4 "Experiments", App. "Impact of Sampling")
# --------------------------------------------------------------------------------------
def counter_uniform(seed: int, position: int, ids: np.ndarray) -> np.ndarray:
    """Counter-based uniform numbers in (0, 1), one per (seed, position, token id): a 32-bit
    integer mix (multiply-xorshift finaliser of the MurmurHash3 family) of the three
    counters, of which the top 23 bits are used, centred in their cell (so that the value is
    exact in float32 as well).  The GPU path
    implements the same generator; random numbers are inputs of the method, not part of it."""
    x = (np.asarray(ids, dtype=np.uint64) * 0x9E3779B1 + np.uint64(position & 0xFFFFFFFF) * 0x85EBCA77
         + np.uint64(seed & 0xFFFFFFFF) * 0xC2B2AE3D) & 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x85EBCA6B) & 0xFFFFFFFF
    x ^= x >> 13
    x = (x * 0xC2B2AE35) & 0xFFFFFFFF
    x ^= x >> 16
    return ((x >> 9).astype(np.float64) + 0.5) / float(1 << 23)


def sample_token(logits_row: np.ndarray, seed: int, position: int) -> int:
    """One draw from softmax(logits) at temperature 1 by the Gumbel-max rule: the arg-max of
    logit + g with g = -ln(-ln u) i.i.d. standard Gumbel is distributed as the softmax.
    `position` is the absolute position of the token being drawn, so the draw at a position
    is the same whether the position is reached by plain decoding or inside a tree."""
    u = counter_uniform(seed, position, np.arange(len(logits_row)))
    return argmax_lowest(as_f64(logits_row) - np.log(-np.log(u)))


# --------------------------------------------------------------------------------------
# proposal: softmax + Top-K' (Sec. 2 Eq. 2, Sec. 3.3)
# --------------------------------------------------------------------------------------
def softmax_topk(logits_row: np.ndarray, kp: int):
    """Full-vocabulary softmax (temperature 1), then the kp most probable tokens ordered
    by (probability descending, token id ascending).  Probabilities are returned rounded
    to float32, the precision the tree arithmetic uses."""
    p = softmax(logits_row)
    order = np.lexsort((np.arange(len(p)), -p))[:kp]
    return order.astype(np.int64), p[order].astype(np.float32)


# --------------------------------------------------------------------------------------
# pruning + dynamic tree (Sec. 3.4 Alg. 1, Sec. 3.5, App. C)
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class TreeParams:
    B: int                     # node budget including the root (Alg. 1 "Budget B")
    k: int                     # mask tokens = maximum depth
    K: int                     # cap on children per expanded node
    expand_width: int = 1      # nodes expanded per depth: 1 = Top-1 expansion (App. C); <=0 = all
    prune_parent: bool = True  # drop a candidate equal to its parent's token (Sec. 3.5)
    prune_last: bool = False   # also drop the last generated (root) token at depths >= 2
    static_widths: Optional[Sequence[int]] = None   # fixed [K_1..K_k]: no selection step


def build_prune_tree(params: TreeParams, lists_id: Sequence[Sequence[int]],
                     lists_p: Sequence[Sequence[float]], root_tok: int,
                     n_depths: Optional[int] = None):
    """Next draft tree from the candidate lists of the mask rows.

    lists_id[i-1] / lists_p[i-1]: tokens and float32 probabilities of mask i, best first.
    Every expansion at depth i draws from the same list i; only the parent's cumulative
    probability and the pruning filter differ between parents.  Cumulative probability
    of a child is one float32 product P(parent) * p.  Returns (tok, parent, prob) in
    block row order: root first, then kept nodes by (depth, creation)."""
    B, k = params.B, params.k
    depth_limit = k if n_depths is None else min(k, n_depths)
    # node records: [token, parent creation index, depth, P, creation index]
    tok = [int(root_tok)]
    par = [-1]
    dep = [0]
    prob = [np.float32(1.0)]
    frontier = [0]                 # the set N of Alg. 1 (creation indices)
    pool: List[int] = []           # the set C of Alg. 1
    for i in range(1, depth_limit + 1):
        cand_ids = lists_id[i - 1]
        cand_ps = lists_p[i - 1]
        at_depth = [n for n in frontier if dep[n] == i - 1]
        at_depth.sort(key=lambda n: (-float(prob[n]), n))
        if params.expand_width > 0:
            at_depth = at_depth[:params.expand_width]
        if params.static_widths is not None:
            want = int(params.static_widths[i - 1])
        else:
            want = min(params.K, B - i)
        fresh = []
        for n in at_depth:
            taken = 0
            for t, p in zip(cand_ids, cand_ps):
                if taken >= want:
                    break
                t = int(t)
                if params.prune_parent and t == tok[n]:
                    continue
                if params.prune_last and i >= 2 and t == tok[0]:
                    continue
                tok.append(t)
                par.append(n)
                dep.append(i)
                prob.append(np.float32(prob[n]) * np.float32(p))
                fresh.append(len(tok) - 1)
                taken += 1
        pool = pool + fresh
        if i < depth_limit:
            if params.static_widths is not None:
                frontier = fresh
            else:
                pool.sort(key=lambda n: (-float(prob[n]), n))
                frontier = pool[:max(B - i, 0)]
                pool = pool[max(B - i, 0):]
    everyone = list(range(1, len(tok)))
    if params.static_widths is None:
        everyone.sort(key=lambda n: (-float(prob[n]), n))
        everyone = everyone[:max(B - 1, 0)]
    keep = sorted(everyone, key=lambda n: (dep[n], n))
    new_row = {0: 0}
    for row, n in enumerate(keep, start=1):
        new_row[n] = row
    out_tok = [tok[0]] + [tok[n] for n in keep]
    out_par = [-1] + [new_row[par[n]] for n in keep]    # KeyError = not ancestor-closed
    out_p = [prob[0]] + [prob[n] for n in keep]
    return (np.asarray(out_tok, dtype=np.int64), np.asarray(out_par, dtype=np.int64),
            np.asarray(out_p, dtype=np.float32))


# --------------------------------------------------------------------------------------
# mask embeddings (Sec. 3.1 Eq. 4, Eq. 5)
# --------------------------------------------------------------------------------------
def mask_mean_init(model: Model, prompt: Sequence[int], k: int) -> np.ndarray:
    """m_i = mean of the prompt's token embeddings, the same vector for every i."""
    emb = model.weights["embed"]
    m = np.zeros(model.d_model, dtype=F64)
    for t in prompt:
        m += as_f64(emb[int(t)])
    m /= len(prompt)
    return np.tile(m[None, :], (k, 1))


def mask_last_k_init(model: Model, prompt: Sequence[int], k: int) -> np.ndarray:
    """Hard initialisation (Sec. 4, mask-design ablation, variant a): the embeddings of the last
    k prompt tokens.  The printed index would skip those very tokens, so the words are followed:
    mask i is the prompt token k - i places before the end, m_i = e_{t-k+i}, in prompt order."""
    if len(prompt) < k:
        raise ValueError("prompt shorter than k")
    emb = model.weights["embed"]
    return np.stack([as_f64(emb[int(t)]) for t in prompt[len(prompt) - k:]], axis=0)


def embed_table_stats(model: Model) -> Tuple[np.ndarray, float]:
    """Gaussian fit to the embedding table (Sec. 4, variant b; App. on masks outside the embedding
    distribution): mu = mean over the V rows (one value per dimension), sigma = one scalar, the
    root mean square deviation of all V * d entries from their dimension's mean (the paper's
    covariance is sigma^2 I)."""
    emb = as_f64(model.weights["embed"])
    mu = emb.mean(axis=0)
    sigma = float(np.sqrt(np.mean((emb - mu[None, :]) ** 2)))
    return mu, sigma


def mask_gaussian_init(model: Model, k: int, z: np.ndarray | None, shift: float = 0.0) -> np.ndarray:
    """m_i = mu + (shift + z_i) sigma.  z: [k, d] standard normal draws handed in by the caller
    (variant b, shift 0), or None with shift 5 or 10 for the out-of-distribution rows of the
    appendix table."""
    mu, sigma = embed_table_stats(model)
    zz = np.zeros((k, model.d_model), dtype=F64) if z is None else as_f64(z)
    return mu[None, :] + (shift + zz) * sigma


def mask_ema_update(mask_embed: np.ndarray, token_embed: np.ndarray, lam: float) -> np.ndarray:
    """m <- m + lambda (e - m) with e the embedding of the last generated token."""
    return as_f64(mask_embed) + lam * (as_f64(token_embed)[None, :] - as_f64(mask_embed))


# --------------------------------------------------------------------------------------
# one step and the generation loop (Sec. 3.3; Fig. 1 right)
# --------------------------------------------------------------------------------------
@dataclasses.dataclass
class DecodeState:
    k_cache: list            # [n_layers] arrays [len, hkv, hd] (float64)
    v_cache: list
    cache_len: int
    tok: np.ndarray          # current tree, node rows
    parent: np.ndarray
    mask_embed: np.ndarray   # [k, d]


@dataclasses.dataclass
class StepResult:
    logits: np.ndarray
    g: np.ndarray
    n_star: int
    accepted: List[int]
    emitted: List[int]
    lists_id: list
    lists_p: list
    n_depths: int
    next_tok: np.ndarray
    next_parent: np.ndarray
    next_prob: np.ndarray


def round_like(x: np.ndarray, store_dtype: str) -> np.ndarray:
    """Round values to the storage type of the workload's KV cache / mask vectors."""
    if store_dtype == "f64":
        return as_f64(x)
    if store_dtype == "f32":
        return as_f64(np.asarray(x, dtype=np.float32))
    if store_dtype == "bf16":
        u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000       # round to nearest even
        return as_f64(u.astype(np.uint32).view(np.float32))
    raise ValueError(store_dtype)


def esp_step(model: Model, st: DecodeState, params: TreeParams, layout: int, kp: int,
             store_dtype: str = "f64", ema_lambda: float = 0.0,
             sample_seed: Optional[int] = None) -> StepResult:
    """One speculate-and-verify step: forward tree + masks, verify, commit the accepted
    rows' K/V, take Top-K' at the mask rows that follow the accepted node, build the next
    tree.  Mutates `st` to the state before the next step.  With sample_seed the base
    model's token after node r is a temperature-1 sample (sample matching) instead of the
    arg-max; the token drawn for a position does not depend on how it is reached."""
    blk = make_block(st.tok, st.parent, params.k, layout)
    logits, _, k_new, v_new = tree_forward(model, blk, st.mask_embed, st.k_cache, st.v_cache,
                                           st.cache_len)
    n = blk.n_nodes
    if sample_seed is None:
        g = np.asarray([argmax_lowest(logits[r]) for r in range(n)], dtype=np.int64)
    else:   # node r sits at position cache_len + depth(r); its successor one further
        g = np.asarray([sample_token(logits[r], sample_seed, st.cache_len + int(blk.depth[r]) + 1)
                        for r in range(n)], dtype=np.int64)
    n_star, accepted, emitted = verify_accept(blk.tok, blk.parent, g)
    # commit: root then the accepted rows, in path order, become cache slots L, L+1, ...
    for l in range(model.n_layers):
        keep = [0] + accepted
        st.k_cache[l] = np.concatenate([st.k_cache[l][:st.cache_len],
                                        round_like(k_new[l][keep], store_dtype)], axis=0)
        st.v_cache[l] = np.concatenate([st.v_cache[l][:st.cache_len],
                                        round_like(v_new[l][keep], store_dtype)], axis=0)
    st.cache_len += 1 + len(accepted)
    # proposals: the mask rows aligned to the accepted position (Sec. 3.3)
    a = len(accepted)
    if layout == LAYOUT_PER_NODE:
        rows = [blk.mask_row(n_star, j) for j in range(1, params.k + 1)]
    else:
        # root chain: mask j predicts the token j+1 places after the old root; the new
        # root sits a+1 places after it, so depth i of the next tree is seeded by mask a+i
        rows = [blk.mask_row(0, a + i) for i in range(1, params.k - a + 1)]
    lists_id, lists_p = [], []
    for r in rows:
        ids, ps = softmax_topk(logits[r], kp)
        lists_id.append(ids)
        lists_p.append(ps)
    nt, npar, nprob = build_prune_tree(params, lists_id, lists_p, emitted[-1], n_depths=len(rows))
    if ema_lambda != 0.0:
        e = as_f64(model.weights["embed"][int(emitted[-1])])
        st.mask_embed = round_like(mask_ema_update(st.mask_embed, e, ema_lambda), store_dtype)
    st.tok, st.parent = nt, npar
    return StepResult(logits, g, n_star, accepted, emitted, lists_id, lists_p, len(rows),
                      nt, npar, nprob)


def prefill(model: Model, prompt: Sequence[int], store_dtype: str = "f64"):
    """Cache for prompt[:-1] by ordinary causal decoding (chain block, no mask rows);
    the last prompt token becomes the root of the first step (prefill = generation only,
    Sec. 3.3).  Returns (k_cache, v_cache, cache_len)."""
    t = len(prompt) - 1
    empty = [np.zeros((0, model.n_kv_heads, model.head_dim)) for _ in range(model.n_layers)]
    if t == 0:
        return empty, [e.copy() for e in empty], 0
    blk = make_block(prompt[:t], [-1] + list(range(t - 1)), 0, LAYOUT_PER_NODE)
    _, _, k_new, v_new = tree_forward(model, blk, np.zeros((0, model.d_model)), empty, empty, 0,
                                      want_logits_rows=[])
    return ([round_like(k_new[l], store_dtype) for l in range(model.n_layers)],
            [round_like(v_new[l], store_dtype) for l in range(model.n_layers)], t)


def esp_generate(model: Model, prompt: Sequence[int], n_new: int, params: TreeParams,
                 layout: int, kp: int, store_dtype: str = "f64", ema_lambda: float = 0.0,
                 sample_seed: Optional[int] = None):
    """Prompt -> at least n_new tokens by repeated esp_step.  The first step has the root
    alone (plus its masks), so it emits one token and seeds the first tree.
    Returns (tokens[:n_new], per-step results)."""
    kc, vc, L = prefill(model, prompt, store_dtype)
    m0 = round_like(mask_mean_init(model, prompt, params.k), store_dtype)
    st = DecodeState(kc, vc, L, np.asarray([prompt[-1]]), np.asarray([-1]), m0)
    out: List[int] = []
    steps = []
    while len(out) < n_new:
        res = esp_step(model, st, params, layout, kp, store_dtype, ema_lambda, sample_seed)
        out.extend(res.emitted)
        steps.append(res)
    return out[:n_new], steps


def greedy_generate(model: Model, prompt: Sequence[int], n_new: int, store_dtype: str = "f64",
                    sample_seed: Optional[int] = None):
    """Plain autoregressive decoding (Sec. 2 Eq. 1): one token per model call, through the
    sequential code path; arg-max, or with sample_seed a temperature-1 sample per position."""
    kc, vc, L = prefill(model, prompt, store_dtype)
    emb = model.weights["embed"]
    cur = int(prompt[-1])
    out: List[int] = []
    for _ in range(n_new):
        logits, k_rows, v_rows = sequence_forward(model, as_f64(emb[cur])[None, :], [L], kc, vc, L)
        for l in range(model.n_layers):
            kc[l] = np.concatenate([kc[l][:L], round_like(k_rows[l], store_dtype)], axis=0)
            vc[l] = np.concatenate([vc[l][:L], round_like(v_rows[l], store_dtype)], axis=0)
        L += 1
        cur = argmax_lowest(logits[0]) if sample_seed is None else sample_token(logits[0], sample_seed, L)
        out.append(cur)
    return out
