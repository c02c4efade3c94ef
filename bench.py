#!/usr/bin/env python3
"""Benchmark of the ESP speculate-and-verify decode step on one MI355X.

One "step" = the whole hot path through the C ABI: esp_tree_forward (tree + mask rows against
the KV cache, LM head + argmax at the tree rows), esp_verify_accept (+ KV commit), esp_mask_topk
(LM head + softmax + Top-K' at the accepted node's mask rows) and esp_build_prune_tree.
Workload: Llama-3-8B-shaped random bf16 decoder, KV cache of a 2048-token random prompt (prefilled
on the GPU), 4 mask tokens, Top-K 8, tree of 64 nodes, batch 1.  All inputs are synthetic and
resident in HBM before the timed region.

Prints ONE JSON line (see the design doc for the fields).  --gpus above 1 is refused: this build is
single-GPU by construction.
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
    dec.prefill([prompt])                        # chunks of 256 rows through esp_tree_forward (Sec. 3.3)
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
            "kernel": "k_attn_mfma + k_attn_merge", "bound": "hbm", "achieved": byts / ms / 1e6, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": byts / ms / 1e6 / HBM_PEAK_GBS, "bytes_per_launch": byts, "avg_launch_ms": ms,
            "mfma_tflops": flops / ms / 1e9}
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layout", choices=["per_node", "root_chain"], default="per_node")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-alt", action="store_true", help="skip the second layout")
    ap.add_argument("--kv-len", type=int, default=2048)
    ap.add_argument("--no-stages", action="store_true", help="skip the stage-level roofline figures")
    ap.add_argument("--no-sweep", action="store_true", help="skip the block-complexity sweep")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
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
        per_launch = sum(gemm_algorithmic_bytes(rows, N, Kd) for N, Kd in shapes) / len(shapes)
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
                              "bytes_per_launch": per_launch, "avg_launch_ms": avg_ms, "launches_timed": r["n_spans"],
                              "mfma_tflops": flops / (avg_ms * 1e-3) / 1e12 if r["n_spans"] else None},
                    roofline_attn={"kernel": "k_attn_mfma", "bound": "hbm",
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
    if not args.no_stages:
        out["stage_rooflines"] = stage_rooflines(B, synth, torch, shape, holder["eng"].lm_head)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, synth, shape, weights, n_nodes, k, K, kp, L,
                                           layouts[args.layout])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
