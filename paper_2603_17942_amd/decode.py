"""Sequencing of the C-ABI calls into prefill, one ESP step and a generation loop.
No arithmetic of the method happens here: buffers are allocated once and the four entry
points of a step are enqueued in order on the current stream (paper Sec. 3.3, Fig. 1 right).
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B
from . import synth


def rows_for(n_nodes: int, k: int, layout: int) -> int:
    """Rows of a block with n_nodes tree nodes: block complexity (Sec. 3.3) or nodes + k."""
    return n_nodes * (k + 1) if layout == B.LAYOUT_PER_NODE else n_nodes + k


class EspDecoder:
    default_max_rows = 0     # lower bound of the row capacity new engines are created with

    def __init__(self, shape: synth.ModelShape, weights: dict, params: B.TreeParams, kp: int,
                 seq_caps: Sequence[int], prefill_chunk: int = 256, max_nodes: Optional[int] = None,
                 ema_lambda: float = 0.0, device="cuda", engine: Optional[B.Engine] = None):
        self.shape, self.params, self.kp, self.device = shape, params, kp, device
        self.k, self.layout = params.k, params.layout
        self.batch = len(seq_caps)
        self.ema_lambda = ema_lambda
        nodes = max_nodes if max_nodes is not None else params.B
        if params.static_widths[0] > 0:
            nodes = 1 + sum(params.static_widths[i] for i in range(params.k))
        self.rows_per_seq = rows_for(nodes, self.k, self.layout)
        self.prefill_chunk = prefill_chunk
        max_rows = max(self.rows_per_seq, prefill_chunk, EspDecoder.default_max_rows)
        self.kv = B.KvCache(shape, seq_caps, device)
        # an engine (weights + workspace) can be shared by decoders that fit its limits
        self.eng = engine if engine is not None else \
            B.Engine(shape, weights, self.batch, max_rows, max(self.kv.caps), device)
        dt = self.eng.dt
        M = self.batch * self.rows_per_seq
        i32 = dict(dtype=torch.int32, device=device)
        self.cur = B.BlockBuffers(self.batch, self.rows_per_seq, self.k, self.layout, device)
        self.nxt = B.BlockBuffers(self.batch, self.rows_per_seq, self.k, self.layout, device)
        self.hidden = torch.zeros((M, shape.d_model), dtype=dt, device=device)
        self.node_argmax = torch.zeros(M, **i32)
        self.n_emit = torch.zeros(self.batch, **i32)
        self.emit_tok = torch.zeros((self.batch, B.MAX_MASKS + 1), **i32)
        self.accepted_row = torch.zeros((self.batch, B.MAX_MASKS + 1), **i32)
        self.star_row = torch.zeros(self.batch, **i32)
        self.topk_id = torch.zeros((self.batch, self.k, kp), **i32)
        self.topk_p = torch.zeros((self.batch, self.k, kp), dtype=torch.float32, device=device)
        self.n_lists = torch.zeros(self.batch, **i32)
        # mask vectors: one [k, d] set per sequence (Eq. 4 / Eq. 5 are per generation); a batch of one
        # keeps the plain [k, d] form
        self.per_seq_masks = self.batch > 1
        self.mask_embed = torch.zeros((self.batch, self.k, shape.d_model) if self.per_seq_masks
                                      else (self.k, shape.d_model), dtype=dt, device=device)
        self.mask_init = "mean"         # "mean" | "last_k" | "gaussian" (with mask_z [k, d] fp32 or None, mask_shift)
        self.mask_z, self.mask_shift = None, 0.0
        self.logits_dbg = None          # set to a [M, vocab] fp32 tensor to capture logits
        self.mask_logits = None         # set to a [batch, k, vocab] fp32 tensor to capture them

    # ---- prefill = generation only (Sec. 3.3): cache for prompt[:-1], root = prompt[-1] ----------
    def prefill(self, prompts: Sequence[Sequence[int]]):
        assert len(prompts) == self.batch
        lens = [len(p) - 1 for p in prompts]
        self.kv.set_len([0] * self.batch)
        done = [0] * self.batch
        chunk = self.prefill_chunk
        blk = B.BlockBuffers(self.batch, chunk, 0, B.LAYOUT_PER_NODE, self.device)
        hidden = torch.zeros((self.batch * chunk, self.shape.d_model), dtype=self.eng.dt, device=self.device)
        while any(done[b] < lens[b] for b in range(self.batch)):
            toks, pars, adv = [], [], []
            for b in range(self.batch):
                n = min(chunk, lens[b] - done[b])
                if n <= 0:
                    # keep the sequence alive with a 1-row block that is not committed
                    toks.append([int(prompts[b][-1])]); pars.append([-1]); adv.append(0)
                else:
                    toks.append([int(t) for t in prompts[b][done[b]:done[b] + n]])
                    pars.append([-1] + list(range(n - 1))); adv.append(n)
            blk.upload_trees(toks, pars)
            self.eng.block_from_tree(blk)
            self.eng.tree_forward(blk, None, self.kv, hidden, None, None)
            for b in range(self.batch):
                done[b] += adv[b]
            self.kv.len.add_(torch.tensor(adv, dtype=torch.int32, device=self.device))
            self.kv.len_bound = max(done)
        for b in range(self.batch if self.per_seq_masks else 1):
            ptok = torch.tensor([int(t) for t in prompts[b]], dtype=torch.int32, device=self.device)
            dst = self.mask_embed[b] if self.per_seq_masks else self.mask_embed
            if self.mask_init == "mean":            # Eq. 4, the paper's default
                self.eng.mask_mean(ptok, self.k, dst)
            elif self.mask_init == "last_k":        # Sec. 4 variant a
                self.eng.mask_last_k(ptok, self.k, dst)
            elif self.mask_init == "gaussian":      # Sec. 4 variant b; mask_z: the caller's normal draws
                self.eng.mask_gaussian(self.mask_z, self.mask_shift, self.k, dst)
            else:
                raise ValueError(f"unknown mask_init {self.mask_init!r}")
        self.cur.upload_trees([[int(p[-1])] for p in prompts], [[-1]] * self.batch)
        self.eng.block_from_tree(self.cur)

    def set_tree(self, toks, parents):
        self.cur.upload_trees(toks, parents)
        self.eng.block_from_tree(self.cur)

    # ---- one speculate-and-verify step ---------------------------------------------------------------
    def step(self):
        e = self.eng
        e.tree_forward(self.cur, self.mask_embed, self.kv, self.hidden, self.node_argmax, self.logits_dbg)
        e.verify_accept(self.cur, self.node_argmax, self.kv, self.n_emit, self.emit_tok, self.accepted_row,
                        self.star_row)
        e.mask_topk(self.cur, self.star_row, self.n_emit, self.hidden, self.kp, self.topk_id, self.topk_p,
                    self.n_lists, self.mask_logits)
        e.build_prune_tree(self.params, self.topk_id, self.topk_p, self.kp, self.n_lists, self.n_emit,
                           self.emit_tok, self.nxt)
        if self.ema_lambda != 0.0:
            if self.per_seq_masks:
                e.mask_ema_batch(self.batch, self.n_emit, self.emit_tok, self.ema_lambda, self.k, self.mask_embed)
            else:
                e.mask_ema(self.n_emit, self.emit_tok, self.ema_lambda, self.k, self.mask_embed)
        self.cur, self.nxt = self.nxt, self.cur
        self.kv.len_bound += self.k + 1      # a step commits at most k+1 tokens

    # ---- HIP-graph replay of the step ------------------------------------------------------------------
    def capture_step_pair(self, n_replays: int, stream: "torch.cuda.Stream") -> "torch.cuda.CUDAGraph":
        """Captures two consecutive steps (the block buffers swap every step, so a pair returns to
        the same buffers) into a HIP graph on `stream`, the stream the engine was created on (not
        the default stream).  Everything a step needs lives on the device; the one host value,
        the cache-length bound that sizes the attention launch, is fixed here for n_replays
        replays.  Every launch site must have run once before (kernel attributes are set on first
        use), i.e. call step() at least twice before capturing."""
        self.kv.len_bound += (2 * n_replays + 2) * (self.k + 1)
        bound0 = self.kv.len_bound
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            self.step()
            self.step()
        self.kv.len_bound = bound0 + 2 * (self.k + 1)
        return g

    def emitted(self) -> List[List[int]]:
        """Tokens emitted by the last step, per sequence (synchronises)."""
        ne = self.n_emit.cpu().tolist()
        et = self.emit_tok.cpu().tolist()
        # the host is in step with the device here: replace the running upper bound of the cache
        # length (k+1 per step) by the true value
        self.kv.len_bound = int(self.kv.len.max())
        return [et[b][:ne[b]] for b in range(self.batch)]

    def generate(self, prompts, n_new: int) -> List[List[int]]:
        self.prefill(prompts)
        out = [[] for _ in range(self.batch)]
        while min(len(o) for o in out) < n_new:
            self.step()
            for b, toks in enumerate(self.emitted()):
                out[b].extend(toks)
        return [o[:n_new] for o in out]
