"""Shared test plumbing: turn synthetic torch inputs into the oracle's containers."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import esp_oracle as O  # noqa: E402
from paper_2603_17942_amd import synth  # noqa: E402


def to_np(t):
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64) if t.is_floating_point() \
        else t.detach().cpu().numpy()


def oracle_model(shape: synth.ModelShape, weights: dict, layers=None) -> O.Model:
    """Oracle Model over the same weight values (held as float64 arrays)."""
    n_layers = shape.n_layers if layers is None else layers
    w = {"embed": to_np(weights["embed"]), "lm_head": to_np(weights["lm_head"]),
         "final_norm": to_np(weights["final_norm"]),
         "layers": [{k: to_np(v) for k, v in weights["layers"][l].items()} for l in range(n_layers)]}
    return O.Model(n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.d_ff, shape.vocab, shape.rope_theta, shape.rms_eps, shape.qk_norm, w)


def small_shape(**kw) -> synth.ModelShape:
    base = dict(name="unit", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                d_ff=96, vocab=211, rope_theta=1.0e4, rms_eps=1.0e-5, qk_norm=False, dtype="f32")
    base.update(kw)
    return synth.ModelShape(**base)


def read_golden(path):
    """Golden text fixture: '#' lines are comments/citations; other lines are
    whitespace-separated fields."""
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append(line.split())
    return rows


def identical_logits_leg(dec, seq, tok, parent, k, layout, kp, tree_params, L_before, logits_rows_gpu,
                         mask_logits_gpu, check_p_rtol=2e-4):
    """The integer chain of a step, checked exactly and unconditionally on the GPU's OWN logits:
    the oracle's arg-max -> longest accepted path -> softmax/Top-K' -> pruned tree run on the
    logits the GPU wrote (the fp32 values, held in float64), and every integer the step produced
    must equal them bit for bit (tree / prune / accept are exact given identical logits).

    dec: decoder after step(); seq: sequence index; tok/parent: the tree the step ran on;
    logits_rows_gpu: [rows of the sequence, vocab] fp32 logits of all block rows (debug output of
    esp_tree_forward); mask_logits_gpu: [k, vocab] logits esp_mask_topk computed for its rows.
    Returns a dict of what was compared (for printing)."""
    tok = np.asarray(tok, dtype=np.int64)
    parent = np.asarray(parent, dtype=np.int64)
    n = len(tok)
    blk = O.make_block(tok, parent, k, layout)
    R = blk.n_rows
    rb = seq * dec.rows_per_seq
    lg = np.asarray(logits_rows_gpu)          # fp32 as written by the GPU; rows go to float64 one at a time
    # (1) the base model's own next token at every tree row: arg-max, lowest id on ties
    g = np.asarray([O.argmax_lowest(lg[r].astype(np.float64)) for r in range(n)], dtype=np.int64)
    g_gpu = dec.node_argmax[rb:rb + n].cpu().numpy()
    assert np.array_equal(g_gpu, g), ("arg-max", seq, np.nonzero(g_gpu != g)[0][:8])
    # (2) longest accepted path, bonus token, cache length
    n_star, accepted, emitted = O.verify_accept(tok, parent, g)
    ne = int(dec.n_emit[seq])
    assert ne == len(emitted), (seq, ne, emitted)
    assert dec.emit_tok[seq, :ne].tolist() == emitted, seq
    assert dec.accepted_row[seq, :ne].tolist() == [0] + accepted, seq
    assert int(dec.star_row[seq]) == n_star, seq
    assert int(dec.kv.len[seq]) == L_before + ne, seq
    # (3) the proposal rows aligned to the accepted position and their Top-K'
    a = len(accepted)
    if layout == O.LAYOUT_PER_NODE:
        rows = [blk.mask_row(n_star, j) for j in range(1, k + 1)]
    else:
        rows = [blk.mask_row(0, a + i) for i in range(1, k - a + 1)]
    assert int(dec.n_lists[seq]) == len(rows), seq
    ids_gpu = dec.topk_id[seq].cpu().numpy()
    ps_gpu = dec.topk_p[seq].cpu().numpy()
    ml = np.asarray(mask_logits_gpu)
    same_as_dbg = 0
    lists_id, lists_p = [], []
    for i, r in enumerate(rows):
        same_as_dbg += int(np.array_equal(ml[i], lg[r]))
        ids, ps = O.softmax_topk(ml[i].astype(np.float64), kp)
        assert ids_gpu[i].tolist() == ids.tolist(), ("Top-K' ids", seq, i)
        np.testing.assert_allclose(ps_gpu[i], ps, rtol=check_p_rtol, atol=1e-30)
        lists_id.append(ids_gpu[i].astype(np.int64))
        lists_p.append(ps_gpu[i].astype(np.float32))
    # (4) pruning + Alg. 1 on the lists the GPU holds (ids equal the oracle's; probabilities are
    # the GPU's own fp32 values, so that the cumulative products are the identical numbers)
    nt, npar, _ = O.build_prune_tree(tree_params, lists_id, lists_p, emitted[-1], n_depths=len(rows))
    nn = int(dec.cur.n_nodes[seq])            # dec.cur is already the next block
    assert nn == len(nt), (seq, nn, len(nt))
    assert dec.cur.tok[rb:rb + nn].tolist() == nt.tolist(), seq
    assert dec.cur.parent[rb:rb + nn].tolist() == npar.tolist(), seq
    nb = O.make_block(nt, npar, k, layout)
    assert int(dec.cur.n_rows[seq]) == nb.n_rows
    assert dec.cur.depth[rb:rb + nb.n_rows].tolist() == nb.depth.tolist()
    return {"accepted": a, "lists": len(rows), "mask_rows_bit_equal_to_debug_rows": same_as_dbg, "next_nodes": nn}
