"""Thin ctypes binding over libesp_hip.so (include/esp.h).  Argument marshalling only: every
step of the decode path runs inside the library's HIP kernels.  PyTorch supplies device memory
and the stream.  There is no CPU fallback: importing this module without the built library, or
calling it without a GPU, raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

from . import synth

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libesp_hip.so")

ESP_OK = 0
ESP_F32, ESP_BF16 = 0, 1
LAYOUT_PER_NODE, LAYOUT_ROOT_CHAIN = 0, 1
MAX_MASKS, MAX_ROWS_PER_SEQ, MAX_TOPK, MAX_TREE_NODES = 8, 1024, 32, 256
DEV_LEN_OVER_BOUND, DEV_BAD_TREE, DEV_BAD_TOKEN = 1, 2, 4
STATUS_NAMES = {0: "ESP_OK", 1: "ESP_EINVAL", 2: "ESP_ESHAPE", 3: "ESP_ECAPACITY", 4: "ESP_EDTYPE",
                5: "ESP_EDEVICE", 6: "ESP_ESTATE"}

_vp, _i32, _i64, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", _i32), ("d_model", _i32), ("n_q_heads", _i32), ("n_kv_heads", _i32),
                ("head_dim", _i32), ("d_ff", _i32), ("vocab", _i32), ("rope_theta", _f32),
                ("rms_eps", _f32), ("qk_norm", _i32), ("dtype", _i32)]


class Weights(C.Structure):
    _fields_ = [("embed", _vp), ("lm_head", _vp), ("final_norm", _vp),
                ("wqkv", C.POINTER(_vp)), ("wo", C.POINTER(_vp)), ("w_gate_up", C.POINTER(_vp)),
                ("w_down", C.POINTER(_vp)), ("norm_attn", C.POINTER(_vp)), ("norm_mlp", C.POINTER(_vp)),
                ("q_norm", C.POINTER(_vp)), ("k_norm", C.POINTER(_vp))]


class Kv(C.Structure):
    _fields_ = [("k", _vp), ("v", _vp), ("len", _vp), ("base", _vp), ("seq_cap", _vp),
                ("capacity", _i64), ("len_bound", _i32)]


class Block(C.Structure):
    _fields_ = [("batch", _i32), ("rows_per_seq", _i32), ("k_masks", _i32), ("layout", _i32),
                ("anc_words", _i32), ("n_rows", _vp), ("n_nodes", _vp), ("tok", _vp), ("parent", _vp),
                ("depth", _vp), ("mask_j", _vp), ("attach", _vp), ("anc", _vp)]


class TreeParams(C.Structure):
    _fields_ = [("B", _i32), ("k", _i32), ("K", _i32), ("expand_width", _i32), ("prune_parent", _i32),
                ("prune_last", _i32), ("layout", _i32), ("static_widths", _i32 * MAX_MASKS)]


EXPORTS = ["esp_status_str", "esp_workspace_bytes", "esp_create", "esp_destroy", "esp_last_device_status",
           "esp_tree_forward", "esp_verify_accept", "esp_mask_topk", "esp_build_prune_tree",
           "esp_block_from_tree", "esp_mask_mean", "esp_mask_ema", "esp_set_mask_batch", "esp_mask_ema_batch", "esp_mask_last_k", "esp_mask_gaussian", "esp_kv_store", "esp_kv_load",
           "esp_gemm_scratch_bytes", "esp_gemm", "esp_gemm_argmax_scratch_bytes", "esp_gemm_argmax", "esp_attn_tree", "esp_softmax_topk_scratch_bytes",
           "esp_softmax_topk", "esp_softmax_topk_static", "esp_profile_enable", "esp_profile_read", "esp_pack_weight", "esp_set_sampling"]
SITES = {"gemm_layer": 0, "attn": 1, "attn_merge": 2, "lm_head": 3, "topk": 4, "tree": 5, "glue": 6}

_lib = None


class EspError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {STATUS_NAMES.get(code, code)}")
        self.code = code


def load_library() -> C.CDLL:
    """Loads the in-tree HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_17942_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    lib.esp_status_str.restype = C.c_char_p
    lib.esp_status_str.argtypes = [C.c_int]
    lib.esp_workspace_bytes.restype = C.c_size_t
    lib.esp_workspace_bytes.argtypes = [P(ModelDesc), _i32, _i32, _i64]
    lib.esp_create.argtypes = [P(ModelDesc), P(Weights), _i32, _i32, _i64, _vp, C.c_size_t, _vp, P(_vp)]
    lib.esp_destroy.argtypes = [_vp]
    lib.esp_last_device_status.argtypes = [_vp, P(_i32)]
    lib.esp_tree_forward.argtypes = [_vp, P(Block), _vp, P(Kv), _vp, _vp, _vp]
    lib.esp_verify_accept.argtypes = [_vp, P(Block), _vp, P(Kv), _vp, _vp, _vp, _vp]
    lib.esp_mask_topk.argtypes = [_vp, P(Block), _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp]
    lib.esp_build_prune_tree.argtypes = [_vp, P(TreeParams), _vp, _vp, _i32, _vp, _vp, _vp, P(Block)]
    lib.esp_block_from_tree.argtypes = [_vp, P(Block)]
    lib.esp_mask_mean.argtypes = [_vp, _vp, _i32, _i32, _vp]
    lib.esp_mask_ema.argtypes = [_vp, _vp, _vp, _f32, _i32, _vp]
    lib.esp_set_mask_batch.argtypes = [_vp, _i32]
    lib.esp_mask_ema_batch.argtypes = [_vp, _i32, _vp, _vp, _f32, _i32, _vp]
    lib.esp_mask_last_k.argtypes = [_vp, _vp, _i32, _i32, _vp]
    lib.esp_mask_gaussian.argtypes = [_vp, _vp, _f32, _i32, _vp]
    lib.esp_kv_store.argtypes = [_vp, P(Kv), _i32, _i32, _i32, _i32, _vp, _vp]
    lib.esp_kv_load.argtypes = [_vp, P(Kv), _i32, _i32, _i32, _i32, _vp, _vp]
    lib.esp_gemm_scratch_bytes.restype = C.c_size_t
    lib.esp_gemm_scratch_bytes.argtypes = [_i32, _i32, _i32]
    lib.esp_gemm.argtypes = [_vp, _i32, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _vp, C.c_size_t]
    lib.esp_gemm_argmax_scratch_bytes.restype = C.c_size_t
    lib.esp_gemm_argmax_scratch_bytes.argtypes = [_i32, _i32]
    lib.esp_gemm_argmax.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _vp, C.c_size_t, _vp]
    lib.esp_pack_weight.argtypes = [_vp, _vp, _vp, _i32, _i32]
    lib.esp_attn_tree.argtypes = [_vp, P(Block), P(Kv), _i32, _vp, _vp]
    lib.esp_softmax_topk_scratch_bytes.restype = C.c_size_t
    lib.esp_softmax_topk_scratch_bytes.argtypes = [_i32, _i32, _i32]
    lib.esp_softmax_topk.argtypes = [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, C.c_size_t]
    lib.esp_softmax_topk_static.argtypes = [_vp, _vp, _i32, _i32, _i32, _vp, _vp]
    lib.esp_profile_enable.argtypes = [_vp, C.c_uint32]
    lib.esp_set_sampling.argtypes = [_vp, C.c_int32, C.c_uint32]
    lib.esp_profile_read.argtypes = [_vp, _i32, P(_i64), P(C.c_double)]
    for name in EXPORTS:
        getattr(lib, name)          # AttributeError here = a declared entry point is not exported
    _lib = lib
    return lib


def _check(code: int, where: str):
    if code != ESP_OK:
        raise EspError(code, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous()
    return t.data_ptr()


def _stream_ptr() -> Optional[int]:
    s = torch.cuda.current_stream().cuda_stream
    return s if s else None


def _dtype_code(shape: synth.ModelShape) -> int:
    return ESP_BF16 if shape.dtype == "bf16" else ESP_F32


def model_desc(shape: synth.ModelShape) -> ModelDesc:
    return ModelDesc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                     shape.d_ff, shape.vocab, shape.rope_theta, shape.rms_eps, int(shape.qk_norm),
                     _dtype_code(shape))


class KvCache:
    """Device KV pool in the library's layout plus the per-sequence bookkeeping arrays."""

    def __init__(self, shape: synth.ModelShape, seq_caps: Sequence[int], device="cuda"):
        dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        caps = [(int(c) + 63) // 64 * 64 for c in seq_caps]
        bases, off = [], 0
        for c in caps:
            bases.append(off)
            off += c
        self.capacity = off
        self.batch = len(caps)
        L, H, D = shape.n_layers, shape.n_kv_heads, shape.head_dim
        self.k = torch.zeros((L, H, self.capacity, D), dtype=dt, device=device)
        self.v = torch.zeros((L, H, self.capacity, D), dtype=dt, device=device)   # same plane size; block order
        self.len = torch.zeros(self.batch, dtype=torch.int32, device=device)
        self.base = torch.tensor(bases, dtype=torch.int32, device=device)
        self.seq_cap = torch.tensor(caps, dtype=torch.int32, device=device)
        self.bases, self.caps = bases, caps
        self.len_bound = 0      # host's upper bound of len[b]; the caller advances it

    def struct(self) -> Kv:
        return Kv(_ptr(self.k), _ptr(self.v), _ptr(self.len), _ptr(self.base), _ptr(self.seq_cap),
                  self.capacity, int(self.len_bound))

    def set_len(self, lens: Sequence[int]):
        self.len.copy_(torch.tensor(list(lens), dtype=torch.int32))
        self.len_bound = int(max(lens))


class BlockBuffers:
    """Device arrays of one forward block (esp_block)."""

    def __init__(self, batch: int, rows_per_seq: int, k_masks: int, layout: int, device="cuda"):
        self.batch, self.rows_per_seq, self.k_masks, self.layout = batch, rows_per_seq, k_masks, layout
        self.anc_words = (rows_per_seq + 63) // 64
        n = batch * rows_per_seq
        i32 = dict(dtype=torch.int32, device=device)
        self.n_rows = torch.zeros(batch, **i32)
        self.n_nodes = torch.zeros(batch, **i32)
        self.tok = torch.zeros(n, **i32)
        self.parent = torch.zeros(n, **i32)
        self.depth = torch.zeros(n, **i32)
        self.mask_j = torch.zeros(n, **i32)
        self.attach = torch.zeros(n, **i32)
        self.anc = torch.zeros((n, self.anc_words), dtype=torch.int64, device=device)

    def struct(self) -> Block:
        return Block(self.batch, self.rows_per_seq, self.k_masks, self.layout, self.anc_words,
                     _ptr(self.n_rows), _ptr(self.n_nodes), _ptr(self.tok), _ptr(self.parent),
                     _ptr(self.depth), _ptr(self.mask_j), _ptr(self.attach), _ptr(self.anc))

    def upload_trees(self, toks: Sequence[Sequence[int]], parents: Sequence[Sequence[int]]):
        """Copies node tokens / parents of each sequence to the device (marshalling only; the
        derived arrays are produced by esp_block_from_tree)."""
        tok = torch.zeros(self.batch * self.rows_per_seq, dtype=torch.int32)
        par = torch.zeros(self.batch * self.rows_per_seq, dtype=torch.int32)
        nn = []
        for b, (t, p) in enumerate(zip(toks, parents)):
            n = len(t)
            nn.append(n)
            tok[b * self.rows_per_seq: b * self.rows_per_seq + n] = torch.as_tensor(t, dtype=torch.int32)
            par[b * self.rows_per_seq: b * self.rows_per_seq + n] = torch.as_tensor(p, dtype=torch.int32)
        self.tok.copy_(tok)
        self.parent.copy_(par)
        self.n_nodes.copy_(torch.tensor(nn, dtype=torch.int32))


class Engine:
    """One esp_ctx plus the device tensors it works on.  Method names follow the C entry points."""

    GUARD_BYTE = 0xA5

    def __init__(self, shape: synth.ModelShape, weights: dict, max_batch: int, max_rows_per_seq: int,
                 max_kv_len: int, device="cuda", guard_bytes: int = 0):
        """guard_bytes > 0 places the workspace between two guard regions of that many bytes filled
        with GUARD_BYTE (guards_intact() checks them): a test hook, no effect on the library."""
        if not torch.cuda.is_available():
            raise RuntimeError("the ESP HIP path needs a GPU; there is no CPU fallback")
        self.lib = load_library()
        self.shape, self.device = shape, device
        self.dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.desc = model_desc(shape)
        L = shape.n_layers
        # the library takes q/k/v and gate/up as one matrix each: concatenate rows once at load
        self._keep = []
        lw = weights["layers"]

        def dev(t):
            t = t.to(device=device, dtype=self.dt).contiguous()
            self._keep.append(t)
            return t

        def mat(t):
            """Matrix for the GEMMs: bf16 models hand over the streaming layout."""
            t = t.to(device=device, dtype=self.dt).contiguous()
            if self.dt == torch.bfloat16:
                t = pack_weight(t)
            self._keep.append(t)
            return t

        arrs = {n: (_vp * L)() for n in ("wqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_mlp",
                                          "q_norm", "k_norm")}
        for l in range(L):
            w = lw[l]
            arrs["wqkv"][l] = mat(torch.cat([w["wq"], w["wk"], w["wv"]], 0)).data_ptr()
            arrs["wo"][l] = mat(w["wo"]).data_ptr()
            arrs["w_gate_up"][l] = mat(self._fuse_gate_up(w["w_gate"], w["w_up"])).data_ptr()
            arrs["w_down"][l] = mat(w["w_down"]).data_ptr()
            arrs["norm_attn"][l] = dev(w["norm_attn"]).data_ptr()
            arrs["norm_mlp"][l] = dev(w["norm_mlp"]).data_ptr()
            arrs["q_norm"][l] = dev(w["q_norm"]).data_ptr()
            arrs["k_norm"][l] = dev(w["k_norm"]).data_ptr()
        self.embed = dev(weights["embed"])
        self.lm_head = mat(weights["lm_head"])
        self.final_norm = dev(weights["final_norm"])
        self._arrs = arrs
        pp = lambda n: C.cast(arrs[n], C.POINTER(_vp))
        wst = Weights(self.embed.data_ptr(), self.lm_head.data_ptr(), self.final_norm.data_ptr(),
                      pp("wqkv"), pp("wo"), pp("w_gate_up"), pp("w_down"), pp("norm_attn"),
                      pp("norm_mlp"), pp("q_norm"), pp("k_norm"))
        nbytes = self.lib.esp_workspace_bytes(C.byref(self.desc), max_batch, max_rows_per_seq, max_kv_len)
        if nbytes == 0:
            raise EspError(1, "esp_workspace_bytes")
        guard = (int(guard_bytes) + 255) // 256 * 256
        self.workspace = torch.full((nbytes + 256 + 2 * guard,), self.GUARD_BYTE, dtype=torch.uint8, device=device)
        ws_ptr = (self.workspace.data_ptr() + guard + 255) // 256 * 256
        self._ws_off, self._ws_bytes = ws_ptr - self.workspace.data_ptr(), nbytes
        ctx = _vp()
        _check(self.lib.esp_create(C.byref(self.desc), C.byref(wst), max_batch, max_rows_per_seq, max_kv_len,
                                   ws_ptr, nbytes, _stream_ptr(), C.byref(ctx)), "esp_create")
        self.ctx = ctx
        self.max_batch, self.max_rows = max_batch, max_rows_per_seq

    def _fuse_gate_up(self, gate: torch.Tensor, up: torch.Tensor) -> torch.Tensor:
        """The fused gate/up matrix of esp_weights: fp32 models stack all gate rows on all up rows;
        bf16 models alternate blocks of 32 rows (gate block j, up block j, ...), the order in which
        the projection kernel pairs them for its SwiGLU epilogue."""
        if self.dt != torch.bfloat16:
            return torch.cat([gate, up], 0)
        ff, d = gate.shape
        assert ff % 32 == 0
        return torch.stack([gate.reshape(ff // 32, 32, d), up.reshape(ff // 32, 32, d)], 1).reshape(2 * ff, d)

    def guards_intact(self) -> bool:
        """True when every byte of the allocation outside the workspace still holds GUARD_BYTE."""
        lo = self.workspace[:self._ws_off]
        hi = self.workspace[self._ws_off + self._ws_bytes:]
        return bool((lo == self.GUARD_BYTE).all().item()) and bool((hi == self.GUARD_BYTE).all().item())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.esp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the four calls of a step ------------------------------------------------------------
    def tree_forward(self, blk: BlockBuffers, mask_embed: Optional[torch.Tensor], kv: KvCache,
                     hidden_out: torch.Tensor, node_argmax: Optional[torch.Tensor],
                     logits_dbg: Optional[torch.Tensor] = None):
        b, k = blk.struct(), kv.struct()
        if mask_embed is not None:       # [batch, k, d]: one set of mask vectors per sequence; [k, d]: shared
            self.set_mask_batch(mask_embed.dim() == 3)
        _check(self.lib.esp_tree_forward(self.ctx, C.byref(b), _ptr(mask_embed), C.byref(k), _ptr(hidden_out),
                                         _ptr(node_argmax), _ptr(logits_dbg)), "esp_tree_forward")

    def verify_accept(self, blk: BlockBuffers, node_argmax, kv: KvCache, n_emit, emit_tok, accepted_row,
                      star_row):
        b, k = blk.struct(), kv.struct()
        _check(self.lib.esp_verify_accept(self.ctx, C.byref(b), _ptr(node_argmax), C.byref(k), _ptr(n_emit),
                                          _ptr(emit_tok), _ptr(accepted_row), _ptr(star_row)),
               "esp_verify_accept")

    def mask_topk(self, blk: BlockBuffers, star_row, n_emit, hidden, kp: int, topk_id, topk_p, n_lists,
                  logits_out=None):
        b = blk.struct()
        _check(self.lib.esp_mask_topk(self.ctx, C.byref(b), _ptr(star_row), _ptr(n_emit), _ptr(hidden), kp,
                                      _ptr(topk_id), _ptr(topk_p), _ptr(n_lists), _ptr(logits_out)),
               "esp_mask_topk")

    def build_prune_tree(self, params: TreeParams, topk_id, topk_p, kp: int, n_lists, n_emit, emit_tok,
                         nxt: BlockBuffers):
        b = nxt.struct()
        _check(self.lib.esp_build_prune_tree(self.ctx, C.byref(params), _ptr(topk_id), _ptr(topk_p), kp,
                                             _ptr(n_lists), _ptr(n_emit), _ptr(emit_tok), C.byref(b)),
               "esp_build_prune_tree")

    # ---- stage-level / auxiliary ------------------------------------------------------------------
    def block_from_tree(self, blk: BlockBuffers):
        b = blk.struct()
        _check(self.lib.esp_block_from_tree(self.ctx, C.byref(b)), "esp_block_from_tree")

    def mask_mean(self, tokens: torch.Tensor, k: int, mask_embed: torch.Tensor):
        _check(self.lib.esp_mask_mean(self.ctx, _ptr(tokens), tokens.numel(), k, _ptr(mask_embed)), "esp_mask_mean")

    def mask_last_k(self, tokens: torch.Tensor, k: int, mask_embed: torch.Tensor):
        _check(self.lib.esp_mask_last_k(self.ctx, _ptr(tokens), tokens.numel(), k, _ptr(mask_embed)),
               "esp_mask_last_k")

    def mask_gaussian(self, z: Optional[torch.Tensor], shift: float, k: int, mask_embed: torch.Tensor):
        _check(self.lib.esp_mask_gaussian(self.ctx, _ptr(z) if z is not None else None, shift, k, _ptr(mask_embed)),
               "esp_mask_gaussian")

    def mask_ema(self, n_emit, emit_tok, lam: float, k: int, mask_embed: torch.Tensor):
        _check(self.lib.esp_mask_ema(self.ctx, _ptr(n_emit), _ptr(emit_tok), lam, k, _ptr(mask_embed)),
               "esp_mask_ema")

    def set_mask_batch(self, per_sequence: bool):
        _check(self.lib.esp_set_mask_batch(self.ctx, int(bool(per_sequence))), "esp_set_mask_batch")

    def mask_ema_batch(self, batch: int, n_emit, emit_tok, lam: float, k: int, mask_embed: torch.Tensor):
        _check(self.lib.esp_mask_ema_batch(self.ctx, batch, _ptr(n_emit), _ptr(emit_tok), lam, k, _ptr(mask_embed)),
               "esp_mask_ema_batch")

    def kv_store(self, kv: KvCache, layer: int, seq: int, first_slot: int, k_rows, v_rows):
        k = kv.struct()
        _check(self.lib.esp_kv_store(self.ctx, C.byref(k), layer, kv.bases[seq], first_slot, k_rows.shape[0],
                                     _ptr(k_rows), _ptr(v_rows)), "esp_kv_store")

    def kv_load(self, kv: KvCache, layer: int, seq: int, first_slot: int, n_slots: int):
        s = self.shape
        k_rows = torch.empty((n_slots, s.n_kv_heads, s.head_dim), dtype=self.dt, device=self.device)
        v_rows = torch.empty_like(k_rows)
        k = kv.struct()
        _check(self.lib.esp_kv_load(self.ctx, C.byref(k), layer, kv.bases[seq], first_slot, n_slots,
                                    _ptr(k_rows), _ptr(v_rows)), "esp_kv_load")
        return k_rows, v_rows

    def attn_tree(self, blk: BlockBuffers, kv: KvCache, layer: int, q: torch.Tensor, out: torch.Tensor):
        b, k = blk.struct(), kv.struct()
        _check(self.lib.esp_attn_tree(self.ctx, C.byref(b), C.byref(k), layer, _ptr(q), _ptr(out)),
               "esp_attn_tree")

    def set_sampling(self, enabled: bool, seed: int = 0):
        """Sample matching (temperature 1) instead of greedy verification for later forwards."""
        _check(self.lib.esp_set_sampling(self.ctx, int(bool(enabled)), int(seed) & 0xFFFFFFFF), "esp_set_sampling")

    def profile_enable(self, sites: Sequence[str]):
        mask = 0
        for name in sites:
            mask |= 1 << SITES[name]
        _check(self.lib.esp_profile_enable(self.ctx, mask), "esp_profile_enable")

    def profile_read(self, site: str):
        """(launch spans, total ms) of a site since the last read; synchronises."""
        n, ms = _i64(0), C.c_double(0.0)
        _check(self.lib.esp_profile_read(self.ctx, SITES[site], C.byref(n), C.byref(ms)), "esp_profile_read")
        return n.value, ms.value

    def device_status(self) -> int:
        v = _i32(0)
        _check(self.lib.esp_last_device_status(self.ctx, C.byref(v)), "esp_last_device_status")
        return v.value


def tree_params(B: int, k: int, K: int, expand_width: int = 1, prune_parent: bool = True,
                prune_last: bool = False, layout: int = LAYOUT_PER_NODE,
                static_widths: Optional[Sequence[int]] = None) -> TreeParams:
    sw = (_i32 * MAX_MASKS)()
    if static_widths is not None:
        for i, wdt in enumerate(static_widths):
            sw[i] = int(wdt)
    return TreeParams(B, k, K, expand_width, int(prune_parent), int(prune_last), layout, sw)


def pack_weight(w: torch.Tensor) -> torch.Tensor:
    """Row-major bf16 [N,K] -> the library's streaming layout (esp_pack_weight), same shape tag."""
    lib = load_library()
    assert w.dtype == torch.bfloat16 and w.dim() == 2 and w.is_contiguous()
    out = torch.empty_like(w)
    _check(lib.esp_pack_weight(_stream_ptr(), _ptr(w), _ptr(out), w.shape[0], w.shape[1]), "esp_pack_weight")
    return out


def gemm(A: torch.Tensor, W: torch.Tensor, packed: bool = False, out: Optional[torch.Tensor] = None,
         scratch: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[M,N] fp32 = A[M,K] @ W[N,K]^T through esp_gemm (W row-major, or packed by pack_weight).
    out / scratch (uint8, esp_gemm_scratch_bytes) may be passed in to keep allocation out of a loop."""
    lib = load_library()
    M, K = A.shape
    N = W.shape[0]
    code = ESP_BF16 if A.dtype == torch.bfloat16 else ESP_F32
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    nb = lib.esp_gemm_scratch_bytes(M, N, K)
    if scratch is None:
        scratch = torch.empty(max(nb, 256), dtype=torch.uint8, device=A.device)
    assert scratch.numel() >= nb and out.shape == (M, N) and out.dtype == torch.float32
    _check(lib.esp_gemm(_stream_ptr(), code, _ptr(A), _ptr(W), int(packed), _ptr(out), M, N, K, _ptr(scratch),
                        nb), "esp_gemm")
    return out


def gemm_argmax(A: torch.Tensor, W_packed: torch.Tensor, out: Optional[torch.Tensor] = None,
                scratch: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[M] int32 = arg-max over n of A[M,K] @ W[N,K]^T (bf16, W packed), lowest n on ties, through
    esp_gemm_argmax: the logits are never written."""
    lib = load_library()
    M, K = A.shape
    N = W_packed.shape[0]
    assert A.dtype == torch.bfloat16 and W_packed.dtype == torch.bfloat16
    if out is None:
        out = torch.empty(M, dtype=torch.int32, device=A.device)
    nb = lib.esp_gemm_argmax_scratch_bytes(M, N)
    if scratch is None:
        scratch = torch.empty(max(nb, 256), dtype=torch.uint8, device=A.device)
    assert scratch.numel() >= nb and out.numel() >= M and out.dtype == torch.int32
    _check(lib.esp_gemm_argmax(_stream_ptr(), _ptr(A), _ptr(W_packed), M, N, K, _ptr(scratch), nb, _ptr(out)),
           "esp_gemm_argmax")
    return out


def softmax_topk(logits: torch.Tensor, kp: int, bufs=None):
    """(ids, probs) of the kp largest softmax probabilities per row; bufs = (ids, probs, scratch)
    may be passed in to keep allocation out of a loop."""
    lib = load_library()
    rows, vocab = logits.shape
    nb = lib.esp_softmax_topk_scratch_bytes(rows, vocab, kp)
    if bufs is None:
        ids = torch.empty((rows, kp), dtype=torch.int32, device=logits.device)
        ps = torch.empty((rows, kp), dtype=torch.float32, device=logits.device)
        scratch = torch.empty(max(nb, 256), dtype=torch.uint8, device=logits.device)
    else:
        ids, ps, scratch = bufs
        assert scratch.numel() >= nb
    _check(lib.esp_softmax_topk(_stream_ptr(), _ptr(logits), rows, vocab, kp, _ptr(ids), _ptr(ps), _ptr(scratch),
                                nb), "esp_softmax_topk")
    return ids, ps


def softmax_topk_static(logits: torch.Tensor, kp: int, ids: torch.Tensor, ps: torch.Tensor):
    """esp_softmax_topk_static: as softmax_topk, but with the library's own device array as scratch
    (no workspace argument, no allocation).  ids / ps are written in place."""
    lib = load_library()
    rows, vocab = logits.shape
    assert ids.shape == (rows, kp) and ids.dtype == torch.int32 and ps.shape == (rows, kp) and ps.dtype == torch.float32
    _check(lib.esp_softmax_topk_static(_stream_ptr(), _ptr(logits), rows, vocab, kp, _ptr(ids), _ptr(ps)),
           "esp_softmax_topk_static")
    return ids, ps
