#!/usr/bin/env python3
"""Benchmark of the ESP speculate-and-verify decode step on one MI355X.

One "step" = the whole hot path through the C ABI: esp_tree_forward (tree + mask rows against
the KV cache, LM head + argmax at the tree rows), esp_verify_accept (+ KV commit), esp_mask_topk
(LM head + softmax + Top-K' at the accepted node's mask rows) and esp_build_prune_tree.
Workload: Llama-3-8B-shaped random bf16 decoder, KV cache of a 2048-token random prompt (prefilled
on the GPU), 4 mask tokens, Top-K 8, tree of 64 nodes, batch 1.  All inputs are synthetic and
resident in HBM before the timed region.

Besides that workload the line carries: the other layout, HIP-graph replay, the one-row
autoregressive baseline, a block-complexity sweep, steps with planted acceptance (mean 1.7 tokens per
step), stage figures (attention at a 32768-token cache, LM head at 1344 rows, softmax + Top-K'), the
other workloads as whole steps (32768-token cache; batch 16 with ragged lengths; Qwen3-8B shape) and
the CPU oracle's rate.

Prints ONE JSON line.  --gpus above 1 is refused: this build is single-GPU by construction.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0


def layer_gemm_shapes(s):
    nqkv = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim
    return [(nqkv, s.d_model), (s.d_model, s.n_q_heads * s.head_dim), (2 * s.d_ff, s.d_model), (s.d_model, s.d_ff)]


def gemm_algorithmic_bytes(M, N, K):
    """Weights once + activations in (bf16) + one fp32 result out."""
    return 2 * N * K + 2 * M * K + 4 * M * N


def layer_algorithmic_bytes(s, M):
    """Bytes the four projections of a layer must move for M rows: every weight once, the bf16
    activations in, and what each result is handed on as (fp32 for QKV, O and down, whose consumers
    add the residual or rotate in fp32; bf16 [M, d_ff] for the gate/up projection, whose SwiGLU runs
    in the epilogue)."""
    (nq, d), (_, ko), (n_gu, _), (_, ff) = layer_gemm_shapes(s)
    return (2 * nq * d + 2 * M * d + 4 * M * nq) + (2 * d * ko + 2 * M * ko + 4 * M * d) + \
        (2 * n_gu * d + 2 * M * d + 2 * M * ff) + (2 * d * ff + 2 * M * ff + 4 * M * d)


HBM_SUSTAINED_GBS = 6200.0      # plain streaming kernel on this GPU (measured), for context
MFMA_SUSTAINED_TFLOPS = 1880.0  # back-to-back MFMA loop on this GPU (measured; the clock drops under matrix load)


PMC_SUMMARY = os.path.join(ROOT, "profiles", "esp_step_llama3_8b_kv2048_hbm_traffic_pmc.txt")


def measured_traffic(layout, rows):
    """HBM bytes per launch of the layer-projection GEMM, averaged over its four launches per
    layer, from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, both scaled by
    a copy kernel of known size; the summary states the commands and the scale).  None when the
    summary has no line for this layout and row count."""
    try:
        for line in open(PMC_SUMMARY):
            if not line.startswith("bench-traffic "):
                continue
            kv = dict(f.split("=", 1) for f in line.split()[1:])
            if kv.get("layout") == layout and int(kv.get("rows", -1)) == rows:
                return float(kv["hbm_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass
    return None


TRACE_SUMMARY = os.path.join(ROOT, "profiles", "esp_step_llama3_8b_kv2048_kernel_trace.txt")


def traced_kernel_us(layout, rows):
    """Mean duration of a layer-projection kernel from the committed rocprofv3 kernel-trace summary of this
    benchmark (begin-to-end time stamps of the kernels themselves).  None when the summary has no line for
    this layout and row count."""
    try:
        for line in open(TRACE_SUMMARY):
            if not line.startswith("bench-kernel "):
                continue
            kv = dict(f.split("=", 1) for f in line.split()[1:])
            if kv.get("layout") == layout and int(kv.get("rows", -1)) == rows:
                return float(kv["gemm_layer_avg_us"])
    except (OSError, ValueError, KeyError):
        pass
    return None


PREFILL_CHUNK = int(os.environ.get("ESP_BENCH_PREFILL_CHUNK", "512"))   # rows per prefill block


def run_config(B, decode, synth, torch, shape, weights, eng_holder, layout, n_nodes, k, K, kp, L, steps, warmup,
               prompt, profile_every=4):
    params = B.tree_params(n_nodes, k, K, 0, True, False, layout)
    cap = L + (steps + warmup + 16) * (k + 1) + 1024
    dec = decode.EspDecoder(shape, weights, params, kp, [cap], prefill_chunk=PREFILL_CHUNK, engine=eng_holder.get("eng"))
    eng_holder["eng"] = dec.eng
    eng = dec.eng
    torch.cuda.synchronize()
    tp0 = time.perf_counter()
    dec.prefill([prompt])                        # chain blocks of PREFILL_CHUNK rows through esp_tree_forward (Sec. 3.3)
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - tp0) * 1e3
    dec.step()                                   # root-only step: seeds the first 64-node tree
    for _ in range(warmup):
        dec.step()
    torch.cuda.synchronize()
    n_nodes_now = int(dec.cur.n_nodes[0])
    rows_now = int(dec.cur.n_rows[0])
    len0 = int(dec.kv.len[0])
    eng.profile_read("gemm_layer")               # drop anything recorded so far
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        on = (i % profile_every) == profile_every - 1
        eng.profile_enable(["gemm_layer"] if on else [])
        dec.step()
        marks[i + 1].record()                    # per-step durations (percentiles) from consecutive events
    eng.profile_enable([])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    emitted = int(dec.kv.len[0]) - len0
    n_spans, span_ms = eng.profile_read("gemm_layer")
    # untimed breakdown pass over every launch site
    sites = list(B.SITES)
    for s in sites:
        eng.profile_read(s)
    eng.profile_enable(sites)
    nb = 3
    for _ in range(nb):
        dec.step()
    eng.profile_enable([])
    breakdown = {}
    for s in sites:
        n, ms = eng.profile_read(s)
        breakdown[s] = {"launches_per_step": n / nb, "ms_per_step": ms / nb}
    status = eng.device_status()
    assert status == 0, f"device status {status}"
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    return dict(dec=dec, ms_per_step=(t1 - t0) * 1e3 / steps, emitted=emitted, prefill_ms=prefill_ms,
                step_ms_p10_p50_p90=[round(pct(0.1), 4), round(pct(0.5), 4), round(pct(0.9), 4)], n_spans=n_spans, span_ms=span_ms,
                breakdown=breakdown, n_nodes=n_nodes_now, rows=rows_now, len_end=int(dec.kv.len[0]))


def run_case(B, decode, synth, torch, shape, weights, eng_holder, layout, n_nodes, k, K, kp, lens, steps, warmup,
             node_counts=None, ema=0.0):
    """A step workload with the KV cache filled directly (seeded N(0,1) bf16, the same values in every
    layer: a prompt of tens of thousands of tokens is not prefilled here).  lens: cache length per
    sequence.  node_counts: None = rolling steps (every step verifies the tree the step before built,
    which fills the node budget); a list = every timed step starts from the same seeded random trees
    with that many nodes per sequence (block arrays and cache lengths are put back by device-side
    copies inside the timed region: a few microseconds)."""
    batch = len(lens)
    params = B.tree_params(n_nodes, k, K, 0, True, False, layout)
    caps = [l + (steps + warmup + 24) * (k + 1) + 1024 for l in lens]
    dec = decode.EspDecoder(shape, weights, params, kp, caps, prefill_chunk=64, ema_lambda=ema,
                            engine=eng_holder.get("eng"))
    eng_holder["eng"] = dec.eng
    eng = dec.eng
    one = shape.replace(n_layers=1)
    kf, vf = synth.make_kv_fill(one, max(lens), seed=5, device="cuda")
    for b in range(batch):
        kb, vb = kf[0][:lens[b]].contiguous(), vf[0][:lens[b]].contiguous()
        for l in range(shape.n_layers):
            eng.kv_store(dec.kv, l, b, 0, kb, vb)
    del kf, vf
    dec.kv.set_len(lens)
    eng.mask_mean(synth.make_prompt(256, shape.vocab, seed=2).to("cuda", torch.int32), k,
                  dec.mask_embed[0] if dec.per_seq_masks else dec.mask_embed)
    if dec.per_seq_masks:
        dec.mask_embed.copy_(dec.mask_embed[0].clone())
    counts = node_counts if node_counts is not None else [n_nodes] * batch
    trees = [synth.make_random_tree(counts[b], k, shape.vocab, seed=7 + b) for b in range(batch)]
    dec.set_tree([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    fixed = node_counts is not None
    if fixed:
        names = [n for n, t in vars(dec.cur).items() if torch.is_tensor(t)]
        saved = {n: getattr(dec.cur, n).clone() for n in names}
        len0 = dec.kv.len.clone()
        bound0 = dec.kv.len_bound

        def restore():
            for n in names:
                getattr(dec.cur, n).copy_(saved[n])
            dec.kv.len.copy_(len0)
            dec.kv.len_bound = bound0
    else:
        def restore():
            pass
    for _ in range(warmup):
        restore()
        dec.step()
    torch.cuda.synchronize()
    rows_now = int(dec.cur.n_rows.sum()) if not fixed else int(saved["n_rows"].sum())
    nodes_now = int(dec.cur.n_nodes.sum()) if not fixed else int(saved["n_nodes"].sum())
    eng.profile_read("gemm_layer")
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    lsum0 = int(dec.kv.len.sum())
    emitted = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        restore()
        dec.step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    emitted = (int(dec.kv.len.sum()) - lsum0) if not fixed else steps * (int(dec.kv.len.sum()) - int(len0.sum()))
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    sites = list(B.SITES)
    for st in sites:
        eng.profile_read(st)
    eng.profile_enable(sites)
    nb = 2
    for _ in range(nb):
        restore()
        dec.step()
    eng.profile_enable([])
    breakdown = {}
    for st in sites:
        n, ms = eng.profile_read(st)
        breakdown[st] = {"launches_per_step": n / nb, "ms_per_step": ms / nb}
    status = eng.device_status()
    assert status == 0, f"device status {status}"
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    ms_per_step = (t1 - t0) * 1e3 / steps
    M = batch * dec.rows_per_seq                       # rows every launch is sized for
    g = breakdown["gemm_layer"]
    g_ms = g["ms_per_step"] / max(g["launches_per_step"], 1)
    lay_bytes = layer_algorithmic_bytes(shape, rows_now) / 4
    lay_flops = sum(2.0 * rows_now * N * Kd for N, Kd in layer_gemm_shapes(shape)) / 4
    a = breakdown["attn"]
    a_ms = (a["ms_per_step"] + breakdown["attn_merge"]["ms_per_step"]) / max(a["launches_per_step"], 1)
    kv_rows = int(sum(lens)) + rows_now
    attn_bytes = kv_rows * shape.n_kv_heads * shape.head_dim * 2 * 2 + 2 * rows_now * shape.n_q_heads * shape.head_dim * 2
    attn_flops = sum(4.0 * (dec.rows_per_seq if not fixed else int(saved["n_rows"][b])) * shape.n_q_heads * shape.head_dim *
                     (lens[b] + dec.rows_per_seq) for b in range(batch))
    res = {"layout": "per_node" if layout == B.LAYOUT_PER_NODE else "root_chain", "batch": batch,
           "rows_per_step": rows_now, "rows_launched": M, "tree_nodes": nodes_now, "kv_len": lens if batch <= 2 else
           {"min": min(lens), "max": max(lens), "sum": int(sum(lens))},
           "ms_per_step": ms_per_step, "step_ms_p10_p50_p90": [round(pct(0.1), 4), round(pct(0.5), 4), round(pct(0.9), 4)],
           "tokens_per_s": emitted / (ms_per_step * steps / 1e3), "tau_measured": emitted / (steps * batch),
           "steps": steps, "trees": "fixed seeded random trees" if fixed else "rolling (built by the step before)",
           "breakdown_ms_per_step": {st: round(v["ms_per_step"], 4) for st, v in breakdown.items()},
           "roofline": {"kernel": "layer projections (QKV, O, gate/up, down), mean of the four launches",
                        "bound": "hbm" if rows_now < 300 else "mfma",
                        "bytes_per_launch": lay_bytes, "flops_per_launch": lay_flops, "avg_launch_ms": g_ms,
                        "hbm_gbs": lay_bytes / (g_ms * 1e-3) / 1e9, "hbm_frac": lay_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "mfma_tflops": lay_flops / (g_ms * 1e-3) / 1e12,
                        "mfma_frac": lay_flops / (g_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
           "roofline_attn": {"kernel": "k_attn_ring + k_attn_merge_ring, per layer", "bound": "hbm",
                             "bytes_per_launch": attn_bytes, "avg_launch_ms": a_ms,
                             "achieved": attn_bytes / (a_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": attn_bytes / (a_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "mfma_tflops": attn_flops / (a_ms * 1e-3) / 1e12}}
    del dec
    return res


PLANTED_DEPTHS = [0] * 20 + [1] * 12 + [2] * 8   # accepted nodes per step: mean 0.70


def planted_acceptance(B, torch, dec, seed=11):
    """Steps with planted acceptance: random weights accept nothing, so before each timed step the
    tree the method built is edited on the device -- along one path from the root, down to a planted
    depth, a child's token is replaced by the token the base model itself produces at its parent
    (found by running the forward on the same block, untimed).  The timed step then verifies and
    commits that path like any other.  The planted depths are a shuffled multiset (20 steps accept
    nothing, 12 one node, 8 two nodes) whose mean, 1.70 tokens per step with the bonus token, lies in
    the range the paper reports for trained 8B models (Table 1: 1.63 to 1.74).  Depth stops at two:
    with random weights the Top-K' probabilities are nearly flat, so the pruned 64-node tree the method
    builds is the root, its 8 children and 55 grandchildren."""
    import random
    depths = list(PLANTED_DEPTHS)
    random.Random(seed).shuffle(depths)
    steps = len(depths)
    eng, k = dec.eng, dec.k
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    lens = []
    for i in range(steps):
        n = int(dec.cur.n_nodes[0])
        tok = dec.cur.tok[:n].tolist()
        par = dec.cur.parent[:n].tolist()
        children = [[] for _ in range(n)]
        for c in range(1, n):
            children[par[c]].append(c)
        height = [0] * n                          # parents precede children: one backward sweep
        for c in range(n - 1, 0, -1):
            height[par[c]] = max(height[par[c]], height[c] + 1)
        node = 0
        for d in range(min(depths[i], k)):
            if not children[node]:
                break
            eng.tree_forward(dec.cur, dec.mask_embed, dec.kv, dec.hidden, dec.node_argmax, None)
            g = int(dec.node_argmax[node])
            hit = [c for c in children[node] if tok[c] == g]
            # no child carries the token already: overwrite the child with the deepest subtree below it
            c = hit[0] if hit else max(children[node], key=lambda x: height[x])
            dec.cur.tok[c] = g
            tok[c] = g
            node = c
        torch.cuda.synchronize()
        l0 = int(dec.kv.len[0])
        e0[i].record()
        dec.step()
        e1[i].record()
        torch.cuda.synchronize()
        lens.append(int(dec.kv.len[0]) - l0)
        dec.kv.len_bound = int(dec.kv.len[0])
    ms = sum(a.elapsed_time(b) for a, b in zip(e0, e1))
    assert eng.device_status() == 0
    hist = {str(n): lens.count(n) for n in sorted(set(lens))}
    return {"tokens_per_s": sum(lens) / (ms * 1e-3), "tau_measured": sum(lens) / steps, "ms_per_step": ms / steps,
            "steps": steps, "planted_tokens_per_step": 1.0 + sum(min(d, k) for d in depths) / steps,
            "tokens_per_step_histogram": hist,
            "note": "acceptance planted on the device before each timed step (see the docstring of "
                    "planted_acceptance); tau is what the verifier then measured, not the paper's"}


def ar_baseline(B, torch, dec, steps):
    """Plain autoregressive decoding with the same kernels: one row per forward (the last token),
    arg-max at the LM head, token and cache length advanced on the device.  Gives the cost of an
    ESP step relative to an ordinary decode step."""
    eng, kv = dec.eng, dec.kv
    blk = B.BlockBuffers(1, 1, 0, B.LAYOUT_PER_NODE)
    blk.upload_trees([[1]], [[-1]])
    eng.block_from_tree(blk)
    hidden = torch.zeros((1, dec.shape.d_model), dtype=eng.dt, device="cuda")
    nxt = torch.zeros(1, dtype=torch.int32, device="cuda")
    one = torch.ones(1, dtype=torch.int32, device="cuda")

    def step():
        eng.tree_forward(blk, None, kv, hidden, nxt, None)
        blk.tok[:1].copy_(nxt)
        kv.len.add_(one)
        kv.len_bound += 1
    return time_gpu(torch, step, steps, warm=3)


def cpu_baseline(torch, synth, shape, weights, n_nodes, k, K, kp, L, layout):
    """The oracle as it stands, timed on the host: one decoder layer of the workload (of 32) plus
    the whole remainder of the step (LM head on all rows, softmax/Top-K, tree, verification),
    extrapolated to the full depth."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import esp_oracle as O

    def f64(t):
        return t.detach().to("cpu", torch.float32).numpy().astype(np.float64)

    lw = {n: f64(v) for n, v in weights["layers"][0].items()}
    ow = {"embed": f64(weights["embed"]), "lm_head": f64(weights["lm_head"]),
          "final_norm": f64(weights["final_norm"]), "layers": [lw]}
    m = O.Model(1, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff, shape.vocab,
                shape.rope_theta, shape.rms_eps, shape.qk_norm, ow)
    one = shape.replace(n_layers=1)
    kf, vf = synth.make_kv_fill(one, L, seed=5)
    tok, par = synth.make_random_tree(n_nodes, k, shape.vocab, seed=7)
    masks = f64(synth.normal_like((k, shape.d_model), 0.02, 6, 0))
    kc, vc = [f64(kf[0])], [f64(vf[0])]
    blk = O.make_block(tok.numpy(), par.numpy(), k, layout)
    n_timed = 6                                  # layers' worth of oracle work actually run
    t0 = time.perf_counter()
    for _ in range(n_timed):
        O.tree_forward(m, blk, masks, kc, vc, L, want_logits_rows=[])
    t_layer = (time.perf_counter() - t0) / n_timed
    st = O.DecodeState(kc, vc, L, tok.numpy().astype(np.int64), par.numpy().astype(np.int64), masks)
    t0 = time.perf_counter()
    res = O.esp_step(m, st, O.TreeParams(B=n_nodes, k=k, K=K, expand_width=0), layout, kp, "bf16")
    t_full = time.perf_counter() - t0
    t_step = shape.n_layers * t_layer + max(t_full - t_layer, 0.0)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": len(res.emitted) / t_step, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"oracle (numpy fp64) on one decoder layer of the same block ({blk.n_rows} rows, L={L}) run "
                      f"{n_timed} times, {t_layer:.1f} s each, plus the rest of the step (LM head on all "
                      f"rows, softmax/Top-K, verification, tree) {max(t_full - t_layer, 0.0):.1f} s; step time "
                      f"extrapolated as {shape.n_layers} x layer + rest = {t_step:.1f} s"}


def time_gpu(torch, fn, iters, warm=2):
    """Mean ms per call of fn, timed with events on the stream the library launches on."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def stage_rooflines(B, synth, torch, shape, lm_head_packed):
    """Stage-level figures for the pieces whose roofline the step workload cannot show: tree
    attention at a 32768-token cache (one layer, rotating over 4 layers of KV so the reads come
    from HBM), the LM-head GEMM at a batched-verification row count (MFMA-bound), and the fused
    softmax + Top-K' over many logit rows."""
    out = {}
    L, nl = 32768, 4
    sh = shape.replace(n_layers=nl, vocab=1024, d_ff=256)
    w = synth.make_weights(sh, seed=1, device="cuda")
    eng = B.Engine(sh, w, 1, 320, L + 1024)
    kv = B.KvCache(sh, [L + 512])
    kf, vf = synth.make_kv_fill(sh.replace(n_layers=1), L + 320, seed=5, device="cuda")
    for l in range(nl):
        eng.kv_store(kv, l, 0, 0, kf[0].contiguous(), vf[0].contiguous())
    kv.set_len([L])
    for layout, rows in [(B.LAYOUT_ROOT_CHAIN, 68), (B.LAYOUT_PER_NODE, 320)]:
        tok, par = synth.make_random_tree(64, 4, sh.vocab, seed=9)
        blk = B.BlockBuffers(1, rows, 4, layout)
        blk.upload_trees([tok.tolist()], [par.tolist()])
        eng.block_from_tree(blk)
        q = synth.normal_like((rows, sh.n_q_heads, sh.head_dim), 1.0, 3, layout, "cuda", torch.bfloat16)
        o = torch.zeros_like(q)
        cnt = [0]

        def call():
            eng.attn_tree(blk, kv, cnt[0] % nl, q, o)
            cnt[0] += 1
        ms = time_gpu(torch, call, 20, warm=3)
        byts = (L + rows) * sh.n_kv_heads * sh.head_dim * 2 * 2 + 2 * rows * sh.n_q_heads * sh.head_dim * 2
        flops = 4.0 * rows * sh.n_q_heads * sh.head_dim * (L + rows)
        out[f"attn_L32768_rows{rows}"] = {
            "kernel": "k_attn_ring + k_attn_merge_ring", "bound": "hbm", "achieved": byts / ms / 1e6, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": byts / ms / 1e6 / HBM_PEAK_GBS,
            "frac_of_sustained_6200": byts / ms / 1e6 / HBM_SUSTAINED_GBS, "bytes_per_launch": byts, "avg_launch_ms": ms,
            "mfma_tflops": flops / ms / 1e9, "mfma_frac": flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS}
    # tree building (Alg. 1) at block complexity 30 and 60 (6 and 12 nodes, k = 4): the dynamic tree,
    # a fixed tree built in full on every call (two width lists alternate on one block, which
    # defeats the reuse) and the same fixed tree with its rows reused (only the tokens are written)
    k, kp = 4, 10
    ids = torch.stack([torch.randperm(sh.vocab, device="cuda")[:kp] for _ in range(k)]).to(torch.int32)[None].contiguous()
    ps = torch.sort(torch.rand((1, k, kp), device="cuda"), dim=-1, descending=True).values.contiguous()
    i32 = dict(dtype=torch.int32, device="cuda")
    n_lists, n_emit = torch.full((1,), k, **i32), torch.ones(1, **i32)
    emit = torch.zeros((1, B.MAX_MASKS + 1), **i32)
    out["tree_build_us"] = {}
    for nodes, wa, wb in ((6, [2, 1, 1, 1], [1, 2, 1, 1]), (12, [5, 3, 2, 1], [5, 3, 1, 2])):
        blk = B.BlockBuffers(1, nodes * (k + 1), k, B.LAYOUT_PER_NODE)
        dyn = B.tree_params(nodes, k, 8, 0, True, False, B.LAYOUT_PER_NODE)
        sa = B.tree_params(nodes, k, 8, 1, True, False, B.LAYOUT_PER_NODE, wa)
        sb = B.tree_params(nodes, k, 8, 1, True, False, B.LAYOUT_PER_NODE, wb)
        flip = [0]

        def alternate():
            flip[0] ^= 1
            eng.build_prune_tree(sa if flip[0] else sb, ids, ps, kp, n_lists, n_emit, emit, blk)
        t_dyn = time_gpu(torch, lambda: eng.build_prune_tree(dyn, ids, ps, kp, n_lists, n_emit, emit, blk), 50, warm=3)
        t_full = time_gpu(torch, alternate, 50, warm=3)
        t_reuse = time_gpu(torch, lambda: eng.build_prune_tree(sa, ids, ps, kp, n_lists, n_emit, emit, blk), 50, warm=3)
        out["tree_build_us"][f"block_complexity_{nodes * (k + 1)}"] = {
            "dynamic": round(t_dyn * 1e3, 2), "static_built_in_full": round(t_full * 1e3, 2),
            "static_rows_reused": round(t_reuse * 1e3, 2)}
    assert eng.device_status() == 0
    eng.close()
    del eng, kv, kf, vf, w
    torch.cuda.empty_cache()

    M, N, K = 1344, shape.vocab, shape.d_model           # 16 sequences x (80 + 4) rows
    A = synth.normal_like((M, K), 1.0, 21, 0, "cuda", torch.bfloat16)
    C_out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    scratch = torch.empty(max(B.load_library().esp_gemm_scratch_bytes(M, N, K), 256), dtype=torch.uint8, device="cuda")
    ms_logits = time_gpu(torch, lambda: B.gemm(A, lm_head_packed, True, C_out, scratch), 5, warm=2)
    # the step's path above 128 tree rows: arg-max in the epilogue, no [rows, vocab] logits written
    am = torch.empty(M, dtype=torch.int32, device="cuda")
    am_scratch = torch.empty(B.load_library().esp_gemm_argmax_scratch_bytes(M, N), dtype=torch.uint8, device="cuda")
    ms = time_gpu(torch, lambda: B.gemm_argmax(A, lm_head_packed, am, am_scratch), 5, warm=2)
    fl = 2.0 * M * N * K
    out["lm_head_rows1344"] = {"kernel": "k_gemm_bf16_ring<5,2,argmax> + k_argmax_tiles (LM head, 1344 rows)",
                               "bound": "mfma", "achieved": fl / ms / 1e9,
                               "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                               "frac": fl / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                               "frac_of_sustained_1880": fl / ms / 1e9 / 1880.0, "avg_launch_ms": ms,
                               "with_logits_written_ms": ms_logits}
    del am, am_scratch
    del A, scratch
    for rows in (4, 64, 256, 1024, 1344, 4096):
        if rows <= M:
            lg = C_out[:rows]                      # logits of the GEMM above
        else:
            del C_out
            C_out = torch.empty((rows, N), dtype=torch.float32, device="cuda").normal_(0.0, 2.0)
            lg = C_out
        bufs = (torch.empty((rows, 10), dtype=torch.int32, device="cuda"),
                torch.empty((rows, 10), dtype=torch.float32, device="cuda"),
                torch.empty(max(B.load_library().esp_softmax_topk_scratch_bytes(rows, N, 10), 256), dtype=torch.uint8,
                            device="cuda"))
        ms = time_gpu(torch, lambda: B.softmax_topk(lg, 10, bufs), 10, warm=2)
        byts = rows * N * 4
        out[f"softmax_topk_rows{rows}"] = {"kernel": "k_topk_stream + k_topk_merge", "bound": "hbm",
                                           "achieved": byts / ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                           "frac": byts / ms / 1e6 / HBM_PEAK_GBS, "bytes_per_launch": byts,
                                           "avg_launch_ms": ms}
    del C_out
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layout", choices=["per_node", "root_chain"], default="per_node")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-alt", action="store_true", help="skip the second layout")
    ap.add_argument("--kv-len", type=int, default=2048)
    ap.add_argument("--no-stages", action="store_true", help="skip the stage-level roofline figures")
    ap.add_argument("--no-sweep", action="store_true", help="skip the block-complexity sweep")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--no-planted", action="store_true", help="skip the planted-acceptance run")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other workloads (long context, batch 16, Qwen3 shape)")
    ap.add_argument("--fast-weights", action="store_true",
                    help="draw the weights with torch.Tensor.normal_ (one kernel per tensor) instead of the "
                         "counter-based generator; for counter-collection runs, where tens of thousands of "
                         "generator dispatches only slow the profiler down")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_17942_amd import binding as B
    from paper_2603_17942_amd import decode, synth

    B.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU fallback of the hot path)"
    # everything runs on one non-default stream (the engine binds to the stream it is created on),
    # so that a step can also be captured into a HIP graph
    side = torch.cuda.Stream()
    torch.cuda.set_stream(side)
    shape = synth.SHAPES["llama3_8b"]
    n_nodes, k, K, kp, L = 64, 4, 8, 10, args.kv_len
    t_setup = time.perf_counter()
    if args.fast_weights:
        torch.manual_seed(1)
        weights = synth.make_weights(shape.replace(n_layers=0), seed=1, device="cuda")
        bf = dict(dtype=torch.bfloat16, device="cuda")
        d, hd, ff = shape.d_model, shape.head_dim, shape.d_ff
        nq, nkv = shape.n_q_heads * hd, shape.n_kv_heads * hd
        for _ in range(shape.n_layers):
            weights["layers"].append({
                "wq": torch.empty((nq, d), **bf).normal_(0, 0.02), "wk": torch.empty((nkv, d), **bf).normal_(0, 0.02),
                "wv": torch.empty((nkv, d), **bf).normal_(0, 0.02), "wo": torch.empty((d, nq), **bf).normal_(0, 0.02),
                "w_gate": torch.empty((ff, d), **bf).normal_(0, 0.02),
                "w_up": torch.empty((ff, d), **bf).normal_(0, 0.02),
                "w_down": torch.empty((d, ff), **bf).normal_(0, 0.02),
                "norm_attn": torch.ones(d, **bf), "norm_mlp": torch.ones(d, **bf),
                "q_norm": torch.ones(hd, **bf), "k_norm": torch.ones(hd, **bf)})
    else:
        weights = synth.make_weights(shape, seed=1, device="cuda")
    prompt = synth.make_prompt(L + 1, shape.vocab, seed=2).tolist()
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    layouts = {"per_node": B.LAYOUT_PER_NODE, "root_chain": B.LAYOUT_ROOT_CHAIN}
    holder = {}
    # the engine is sized for the larger layout so that both runs share the weights
    decode.EspDecoder.default_max_rows = n_nodes * (k + 1)
    main_r = run_config(B, decode, synth, torch, shape, weights, holder, layouts[args.layout], n_nodes, k, K, kp, L,
                        args.steps, args.warmup, prompt)
    alt_name = "root_chain" if args.layout == "per_node" else "per_node"
    alt_r = None
    if not args.no_alt:
        alt_r = run_config(B, decode, synth, torch, shape, weights, holder, layouts[alt_name], n_nodes, k, K, kp, L,
                           args.steps, args.warmup, prompt)

    def summarise(r, layout_name):
        rows = r["rows"]
        tokens_per_s = r["emitted"] / (r["ms_per_step"] * args.steps / 1e3)
        shapes = layer_gemm_shapes(shape)
        per_launch_fp32 = sum(gemm_algorithmic_bytes(rows, N, Kd) for N, Kd in shapes) / len(shapes)
        per_launch = layer_algorithmic_bytes(shape, rows) / len(shapes)
        avg_ms = r["span_ms"] / max(r["n_spans"], 1)
        achieved = per_launch / (avg_ms * 1e-3) / 1e9 if r["n_spans"] else None
        flops = sum(2.0 * rows * N * Kd for N, Kd in shapes) / len(shapes)
        attn = r["breakdown"]["attn"]
        Lnow = r["len_end"]
        attn_bytes = (Lnow + rows) * shape.n_kv_heads * shape.head_dim * 2 * 2 + \
            2 * rows * shape.n_q_heads * shape.head_dim * 2
        attn_ms = attn["ms_per_step"] / max(attn["launches_per_step"], 1)
        return dict(rows=rows, n_nodes=r["n_nodes"], tokens_per_s=tokens_per_s, ms_per_step=r["ms_per_step"],
                    pct=r["step_ms_p10_p50_p90"],
                    tau=r["emitted"] / args.steps,
                    roofline={"kernel": "k_gemm_bf16 (layer projections: QKV, O, gate/up, down)", "bound": "hbm",
                              "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                              "traffic": measured_traffic(layout_name, rows),
                              "bytes_per_launch": per_launch, "bytes_per_launch_all_fp32_out": per_launch_fp32,
                              "avg_launch_ms": avg_ms, "launches_timed": r["n_spans"],
                              "avg_kernel_us_rocprof": traced_kernel_us(layout_name, rows),
                              "frac_of_sustained_6200": (achieved / HBM_SUSTAINED_GBS) if achieved else None,
                              "mfma_tflops": flops / (avg_ms * 1e-3) / 1e12 if r["n_spans"] else None,
                              "mfma_frac": flops / (avg_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS if r["n_spans"] else None,
                              "mfma_frac_of_sustained_1880": flops / (avg_ms * 1e-3) / 1e12 / MFMA_SUSTAINED_TFLOPS
                              if r["n_spans"] else None},
                    roofline_attn={"kernel": "k_attn_ring", "bound": "hbm",
                                   "achieved": attn_bytes / (attn_ms * 1e-3) / 1e9 if attn_ms else None,
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "bytes_per_launch": attn_bytes,
                                   "avg_launch_ms": attn_ms, "kv_len": Lnow},
                    breakdown_ms_per_step={s: round(v["ms_per_step"], 4) for s, v in r["breakdown"].items()})

    sm = summarise(main_r, args.layout)
    weight_bytes = shape.n_layers * sum(2 * N * Kd for N, Kd in layer_gemm_shapes(shape)) + \
        2 * 2 * shape.vocab * shape.d_model
    out = {
        "metric": "verified tree-step latency (ms) & tokens/s at 8B shape",
        "value": sm["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sm["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-3-8B-shaped random bf16 decoder, KV cache from a "
                               f"{L}-token random prompt, ESP step with k=4 mask tokens, Top-K=8, tree of 64 nodes, "
                               "batch 1", "layout": args.layout, "rows_per_step": sm["rows"],
                   "tree_nodes": sm["n_nodes"], "kv_len": L, "tau_measured": sm["tau"],
                   "hbm_floor_ms": weight_bytes / (HBM_PEAK_GBS * 1e9) * 1e3},
        "step_ms_p10_p50_p90": sm["pct"],
        "roofline": sm["roofline"], "roofline_attn": sm["roofline_attn"],
        "breakdown_ms_per_step": sm["breakdown_ms_per_step"],
        "setup_s": round(t_setup, 1),
        "prefill": {"prompt_tokens": L, "chunk_rows": PREFILL_CHUNK, "ms": round(main_r["prefill_ms"], 2),
                    "tokens_per_s": round((L - 1) / (main_r["prefill_ms"] * 1e-3), 0),
                    "note": "untimed setup of the step workload, host-synchronised once at the end"},
    }
    if alt_r is not None:
        sa = summarise(alt_r, alt_name)
        out["alt_layout"] = {"layout": alt_name, "rows_per_step": sa["rows"], "tokens_per_s": sa["tokens_per_s"],
                             "ms_per_step": sa["ms_per_step"], "step_ms_p10_p50_p90": sa["pct"],
                             "roofline": sa["roofline"],
                             "roofline_attn": sa["roofline_attn"],
                             "breakdown_ms_per_step": sa["breakdown_ms_per_step"]}
    def graph_replay(r, eager_ms):
        """Two consecutive steps captured into a HIP graph, replayed; same work as the eager step."""
        n = max(args.steps // 2, 5)
        g = r["dec"].capture_step_pair(n + 3, side)
        ms = time_gpu(torch, g.replay, n, warm=2) / 2
        assert r["dec"].eng.device_status() == 0
        return {"ms_per_step": ms, "vs_eager": eager_ms / ms}

    if not args.no_graph:
        out["hip_graph_replay"] = graph_replay(main_r, sm["ms_per_step"])
        if alt_r is not None:
            out["alt_layout"]["hip_graph_replay"] = graph_replay(alt_r, out["alt_layout"]["ms_per_step"])
    # ordinary decode step with the same kernels, and what the paper's acceptance lengths would make of
    # the measured step-cost ratio (random weights accept nothing, so tau_measured is 1)
    ar_ms = ar_baseline(B, torch, main_r["dec"], 20)
    ratio = sm["ms_per_step"] / ar_ms
    out["ar_baseline"] = {"ms_per_step": ar_ms, "tokens_per_s": 1e3 / ar_ms, "esp_step_cost_ratio": ratio}
    if alt_r is not None:
        out["alt_layout"]["esp_step_cost_ratio"] = out["alt_layout"]["ms_per_step"] / ar_ms
    if not args.no_sweep:
        # the paper's operating points: block complexity (k+1) x nodes of 10..120 rows, PER_NODE layout
        sweep = []
        for nodes in (2, 6, 12, 24):
            r = run_config(B, decode, synth, torch, shape, weights, holder, B.LAYOUT_PER_NODE, nodes, k, K, kp, L,
                           10, 2, prompt)
            sweep.append({"block_complexity": r["rows"], "tree_nodes": r["n_nodes"],
                          "ms_per_step": round(r["ms_per_step"], 4),
                          "esp_step_cost_ratio": round(r["ms_per_step"] / ar_ms, 4)})
            del r
        for e in sweep:
            if e["block_complexity"] == 60:
                # random weights accept nothing (tau_measured = 1); with the acceptance lengths the paper
                # reports at BC = 60 on trained 8B models (1.63-1.74), this step-cost ratio would give:
                e["derived_speedup_at_paper_tau"] = {"tau_1.63": round(1.63 / e["esp_step_cost_ratio"], 3),
                                                     "tau_1.74": round(1.74 / e["esp_step_cost_ratio"], 3),
                                                     "note": "derived from the paper's tau, not measured here"}
        out["bc_sweep_per_node"] = sweep
    if not args.no_planted:
        out["planted_acceptance"] = planted_acceptance(B, torch, main_r["dec"])
        out["planted_acceptance"]["layout"] = args.layout
        out["planted_acceptance"]["speedup_over_ar"] = out["planted_acceptance"]["tokens_per_s"] * ar_ms / 1e3
        if alt_r is not None:
            pa = planted_acceptance(B, torch, alt_r["dec"])
            pa["layout"] = alt_name
            pa["speedup_over_ar"] = pa["tokens_per_s"] * ar_ms / 1e3
            out["alt_layout"]["planted_acceptance"] = pa
    if not args.no_stages:
        out["stage_rooflines"] = stage_rooflines(B, synth, torch, shape, holder["eng"].lm_head)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, synth, shape, weights, n_nodes, k, K, kp, L,
                                           layouts[args.layout])
    if not args.no_configs:
        del main_r, alt_r
        cfgs = {}
        # configs[3]: long context, full-depth Llama step; the root-chain layout (68 rows) is the headline
        holder["eng"].close()
        holder.clear()
        torch.cuda.empty_cache()
        h4 = {"eng": B.Engine(shape, weights, 1, 320, 32768 + 2048)}
        cfgs["config4_llama3_8b_kv32768"] = [
            run_case(B, decode, synth, torch, shape, weights, h4, lay, 64, 4, 8, 10, [32768], 10, 2)
            for lay in (B.LAYOUT_ROOT_CHAIN, B.LAYOUT_PER_NODE)]
        h4["eng"].close()
        del h4
        torch.cuda.empty_cache()
        # configs[4]: batch 16, ragged cache lengths and node counts (seeds as in the parity test)
        lens5 = (512 + synth.uniform_ints(16, 7681, 3, 0)).tolist()
        nodes5 = (32 + synth.uniform_ints(16, 97, 4, 0)).tolist()
        cfgs["config5_llama3_8b_batch16_ragged"] = []
        for lay in (B.LAYOUT_ROOT_CHAIN, B.LAYOUT_PER_NODE):
            h5 = {}
            cfgs["config5_llama3_8b_batch16_ragged"].append(
                run_case(B, decode, synth, torch, shape, weights, h5, lay, 128, 4, 8, 10, lens5, 6, 2, node_counts=nodes5))
            h5["eng"].close()
            del h5
            torch.cuda.empty_cache()
        del weights
        torch.cuda.empty_cache()
        # configs[2]: Qwen3-8B shape (QK-norm, 36 layers, 151936-token vocabulary), EMA mask update
        qshape = synth.SHAPES["qwen3_8b"]
        qw = synth.make_weights(qshape, seed=1, device="cuda")
        h3 = {}
        decode.EspDecoder.default_max_rows = 96 * 6
        cfgs["config3_qwen3_8b_kv4096"] = [
            run_case(B, decode, synth, torch, qshape, qw, h3, lay, 96, 5, 10, 12, [4096], 10, 2, ema=0.1)
            for lay in (B.LAYOUT_PER_NODE, B.LAYOUT_ROOT_CHAIN)]
        h3["eng"].close()
        del h3, qw
        torch.cuda.empty_cache()
        out["configs"] = cfgs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
