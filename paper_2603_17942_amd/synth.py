"""Seeded synthetic inputs for the ESP decode step (weights, prompts, KV fill, trees).

This module holds NO arithmetic of the method: it only draws numbers.  Both the
CPU oracle's tests and the HIP path's tests/bench take their inputs from here, so
that the two sides see the same bytes.  The generator is counter based (a
splitmix64-style finaliser of seed/stream/index, written with torch integer ops),
so the same element has the same bits on the CPU and on the GPU and any slice of
a tensor can be regenerated without materialising the rest.

Normal-like values are a centred, scaled sum of eight uniform 16-bit lanes
(Irwin-Hall, |x| < 4.9 sigma): an approximation of N(0, sigma^2) that needs no
transcendental function and is therefore bit-identical on every device.
"""
from __future__ import annotations

import dataclasses
import math

import torch

_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> two's-complement int64 value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLD = _s64(0x9E3779B97F4A7C15)
_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, n: int) -> torch.Tensor:
    """Logical shift right of int64 lanes (torch's >> is arithmetic)."""
    return (x >> n) & ((1 << (64 - n)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def hash64(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits per index (int64 tensor, wraps mod 2^64)."""
    base = _s64(seed * 0xD1342543DE82EF95 + stream * 0xA0761D6478BD642F + 0x2545F4914F6CDD1D)
    return _mix(_mix(idx * _GOLD + base) + _GOLD)


_LANE_MEAN = 8 * 32767.5
_LANE_STD = math.sqrt(8 * (65536.0 ** 2 - 1.0) / 12.0)


def normal_like(shape, std: float, seed: int, stream: int, device="cpu",
                dtype=torch.float32, chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of `shape` with approx. N(0, std^2) entries (see module docstring)."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        acc = torch.zeros(hi - lo, dtype=torch.int64, device=device)
        for half in range(2):
            h = hash64(seed, 2 * stream + half, idx)
            for lane in range(4):
                acc += _lsr(h, 16 * lane) & 0xFFFF
        v = (acc.to(torch.float64) - _LANE_MEAN) * (std / _LANE_STD)
        out[lo:hi] = v.to(torch.float32).to(dtype)
    return out.reshape(*shape)


def uniform_ints(n: int, high: int, seed: int, stream: int, device="cpu") -> torch.Tensor:
    """n integers uniform in [0, high) as int32."""
    idx = torch.arange(n, dtype=torch.int64, device=device)
    h = _lsr(hash64(seed, stream, idx), 33)
    return (h % high).to(torch.int32)


@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
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
    dtype: str  # "f32" | "bf16"

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


# Shapes of the workloads (decoder sizes as published for these model families;
# rope/eps values are this build's stated choices for random-weight models).
SHAPES = {
    "tiny": ModelShape("tiny", 2, 256, 4, 4, 64, 688, 4096, 1.0e4, 1.0e-5, False, "f32"),
    "llama3_8b": ModelShape("llama3_8b", 32, 4096, 32, 8, 128, 14336, 128256, 5.0e5, 1.0e-5, False, "bf16"),
    "qwen3_8b": ModelShape("qwen3_8b", 36, 4096, 32, 8, 128, 12288, 151936, 1.0e6, 1.0e-6, True, "bf16"),
}

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}

# stream ids of the weight tensors (layer l uses 16*l + id)
_ST = dict(embed=1, lm_head=2, wq=3, wk=4, wv=5, wo=6, w_gate=7, w_up=8, w_down=9,
           norm_attn=10, norm_mlp=11, q_norm=12, k_norm=13, final_norm=14)


def make_weights(shape: ModelShape, seed: int = 1, device="cpu", std: float = 0.02,
                 unit_gains: bool = True) -> dict:
    """Random weights of `shape`.  Matrices are [out, in] row-major, N(0, std^2)-like,
    already rounded to the model dtype.  Norm gains are 1 (or 1 + small noise when
    unit_gains is False, so that tests can tell a dropped gain)."""
    dt = _TORCH_DT[shape.dtype]
    d, hd = shape.d_model, shape.head_dim
    nq, nkv, ff = shape.n_q_heads * hd, shape.n_kv_heads * hd, shape.d_ff

    def mat(rows, cols, stream):
        return normal_like((rows, cols), std, seed, stream, device, dt)

    def gain(n, stream):
        if unit_gains:
            return torch.ones(n, dtype=dt, device=device)
        return (1.0 + normal_like((n,), 0.1, seed, stream, device, torch.float32)).to(dt)

    w = {"embed": mat(shape.vocab, d, _ST["embed"]),
         "lm_head": mat(shape.vocab, d, _ST["lm_head"]),
         "final_norm": gain(d, _ST["final_norm"]),
         "layers": []}
    for l in range(shape.n_layers):
        s = lambda name: 16 * (l + 1) + _ST[name]
        w["layers"].append({
            "wq": mat(nq, d, s("wq")), "wk": mat(nkv, d, s("wk")), "wv": mat(nkv, d, s("wv")),
            "wo": mat(d, nq, s("wo")),
            "w_gate": mat(ff, d, s("w_gate")), "w_up": mat(ff, d, s("w_up")),
            "w_down": mat(d, ff, s("w_down")),
            "norm_attn": gain(d, s("norm_attn")), "norm_mlp": gain(d, s("norm_mlp")),
            "q_norm": gain(hd, s("q_norm")), "k_norm": gain(hd, s("k_norm")),
        })
    return w


def make_prompt(n_tokens: int, vocab: int, seed: int = 2, device="cpu") -> torch.Tensor:
    return uniform_ints(n_tokens, vocab, seed, 0, device)


def make_kv_fill(shape: ModelShape, length: int, seed: int = 5, device="cpu", std: float = 1.0):
    """Synthetic KV-cache contents: K and V as [n_layers, length, n_kv_heads, head_dim]
    in the model dtype, N(0, std^2)-like.  Stands in for a prefilled cache where running
    the prompt through a CPU decoder is not feasible."""
    dt = _TORCH_DT[shape.dtype]
    dims = (shape.n_layers, length, shape.n_kv_heads, shape.head_dim)
    return (normal_like(dims, std, seed, 0, device, dt), normal_like(dims, std, seed, 1, device, dt))


def make_random_tree(n_nodes: int, max_depth: int, vocab: int, seed: int = 7,
                     max_children: int = 8):
    """Random rooted tree in (depth, creation) row order: returns (tok[int32 n], parent[int32 n]).
    parent[0] = -1; parents precede children; depth <= max_depth; at most max_children children
    per node; sibling tokens distinct."""
    n_draw = 8 * n_nodes + 16
    r = _lsr(hash64(seed, 3, torch.arange(n_draw, dtype=torch.int64)), 33).tolist()
    toks = uniform_ints(n_draw, vocab, seed, 4).tolist()
    cur = [0]

    def draw():
        cur[0] += 1
        return r[cur[0] % n_draw]

    tok, parent = [toks[0]], [-1]
    prev_level = [0]
    remaining = n_nodes - 1
    ti = 1
    for d in range(1, max_depth + 1):
        if remaining == 0:
            break
        cap = len(prev_level) * min(max_children, vocab)
        share = -(-remaining // (max_depth - d + 1))            # even split of what is left
        size = min(cap, remaining if d == max_depth else max(1, share + draw() % (share + 1) - share // 2))
        size = min(size, remaining)
        kids = {p: set() for p in prev_level}
        level = []
        guard = 0
        while len(level) < size:
            guard += 1
            if guard > 64 * n_draw:
                raise ValueError("could not place the nodes")
            p = prev_level[draw() % len(prev_level)]
            if len(kids[p]) >= max_children:
                continue
            t = toks[ti % n_draw]
            ti += 1
            if t in kids[p]:
                continue
            kids[p].add(t)
            tok.append(t)
            parent.append(p)
            level.append(len(tok) - 1)
        remaining -= size
        prev_level = level
    if remaining:
        raise ValueError("tree cannot hold that many nodes")
    return (torch.tensor(tok, dtype=torch.int32), torch.tensor(parent, dtype=torch.int32))
