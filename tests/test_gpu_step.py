"""Whole-step and loop parity on the GPU: esp_tree_forward -> esp_verify_accept -> esp_mask_topk
-> esp_build_prune_tree through the C ABI against the oracle, on the seeded workloads.

Tolerances: logits row-wise max |diff| / max |oracle| <= 1e-4 (fp32 model) or 2e-2 (bf16 model);
integer results (argmax, accepted path, emitted tokens, trees) are compared exactly wherever the
oracle's deciding gap exceeds that band, and checked for validity otherwise."""
import numpy as np
import pytest
import torch

from util import O, identical_logits_leg, oracle_model, small_shape, synth, to_np

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 1e-4}


@pytest.fixture(scope="module")
def B():
    from paper_2603_17942_amd import binding
    binding.load_library()
    assert torch.cuda.is_available(), "GPU tests need a GPU; there is no fallback path"
    return binding


def rel_err_rows(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    den = np.max(np.abs(want), axis=-1, keepdims=True)
    den[den == 0] = 1.0
    return float(np.max(np.abs(got - want) / den))


def decisive(logits_row, tol):
    """True when the oracle's arg-max is separated from the runner-up by more than the band."""
    top2 = np.sort(logits_row)[-2:]
    return (top2[1] - top2[0]) > 2 * tol * np.max(np.abs(logits_row))


def topk_decisive(logits_row, kp, tol):
    """Positions j < kp of the oracle's ranking whose neighbours are both further than the band."""
    order = np.argsort(-logits_row, kind="stable")[:kp + 1]
    v = logits_row[order]
    band = 2 * tol * np.max(np.abs(logits_row))
    ok = []
    for j in range(kp):
        up = j == 0 or (v[j - 1] - v[j]) > band
        down = (v[j] - v[j + 1]) > band
        ok.append(up and down)
    return order[:kp], ok


def oracle_state_after_prefill(m, prompt, k, store):
    kc, vc, L = O.prefill(m, prompt, store)
    masks = O.round_like(O.mask_mean_init(m, prompt, k), store)
    return O.DecodeState(kc, vc, L, np.asarray([prompt[-1]]), np.asarray([-1]), masks)


def compare_step(dec, res, blk_nodes, rows_per_seq, shape, kp, tol, logits_gpu, mask_logits_gpu, check_tree=True):
    """GPU buffers of the step just run vs the oracle's StepResult.  Returns False when a near-tie
    of the oracle made an integer decision non-comparable (everything up to it was checked)."""
    R = res.logits.shape[0]
    err = rel_err_rows(logits_gpu[:R], res.logits)
    print(f"  logits: worst row-wise relative error {err:.2e} (tolerance {tol:.0e})", flush=True)
    assert err <= tol, f"logits rel err {err}"
    g_gpu = dec.node_argmax[:blk_nodes].cpu().numpy()
    for r in range(blk_nodes):
        if decisive(res.logits[r], tol):
            assert g_gpu[r] == res.g[r], r
        else:   # valid choice: within the band of the oracle's maximum
            band = 2 * tol * np.max(np.abs(res.logits[r]))
            assert res.logits[r][g_gpu[r]] >= np.max(res.logits[r]) - band
            if g_gpu[r] != res.g[r]:
                return False
    ne = int(dec.n_emit[0])
    assert dec.emit_tok[0, :ne].tolist() == res.emitted
    assert dec.accepted_row[0, :ne].tolist() == [0] + res.accepted
    assert int(dec.star_row[0]) == res.n_star
    assert int(dec.n_lists[0]) == res.n_depths
    ids_gpu = dec.topk_id[0].cpu().numpy()
    ps_gpu = dec.topk_p[0].cpu().numpy()
    same_lists = True
    scale = max(1.0, float(np.max(np.abs(res.logits))))
    for i in range(res.n_depths):
        want_p = np.asarray(res.lists_p[i], np.float64)
        np.testing.assert_allclose(ps_gpu[i], want_p, rtol=max(20 * tol * scale, 1e-3))
        # relative probability gap ~ logit gap: decisive when it exceeds twice the logit band
        gap_ok = [(want_p[j] - want_p[j + 1]) > 4 * tol * scale * want_p[j] for j in range(kp - 1)] + [False]
        for j in range(kp):
            if (j == 0 or gap_ok[j - 1]) and gap_ok[j]:
                assert ids_gpu[i, j] == res.lists_id[i][j], (i, j)
            elif ids_gpu[i, j] != res.lists_id[i][j]:
                same_lists = False
    if not same_lists:
        return False
    if check_tree:
        nn = int(dec.cur.n_nodes[0])       # dec.cur is already the next block
        assert nn == len(res.next_tok)
        assert dec.cur.tok[:nn].tolist() == res.next_tok.tolist()
        assert dec.cur.parent[:nn].tolist() == res.next_parent.tolist()
    return True


# ---------------------------------------------------------------------------------------------
# configuration 1: tiny fp32 decoder, prompt 128, k = 3, K = 4, tree <= 15 nodes
# ---------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny_setup(B):
    from paper_2603_17942_amd import decode
    shape = synth.SHAPES["tiny"]
    w = synth.make_weights(shape, seed=1)
    prompt = synth.make_prompt(128, shape.vocab, seed=2).tolist()
    m = oracle_model(shape, w)
    return decode, shape, w, prompt, m


def make_decoder(B, decode, shape, w, params, kp, cap=512, **kw):
    return decode.EspDecoder(shape, w, params, kp, [cap], prefill_chunk=64, **kw)


def test_config1_prefill_kv_and_one_step(B, tiny_setup):
    decode, shape, w, prompt, m = tiny_setup
    k, K, kp, Bn = 3, 4, 6, 15
    params = B.tree_params(Bn, k, K, 1, True, False, B.LAYOUT_PER_NODE)
    dec = make_decoder(B, decode, shape, w, params, kp)
    dec.prefill([prompt])
    assert dec.eng.device_status() == 0
    st = oracle_state_after_prefill(m, prompt, k, "f32")
    # prefilled cache and mask vector
    for l in range(shape.n_layers):
        kk, vv = dec.eng.kv_load(dec.kv, l, 0, 0, 127)
        assert rel_err_rows(to_np(kk).reshape(127, -1), st.k_cache[l].reshape(127, -1)) < 1e-4
        assert rel_err_rows(to_np(vv).reshape(127, -1), st.v_cache[l].reshape(127, -1)) < 1e-4
    assert rel_err_rows(to_np(dec.mask_embed), st.mask_embed) < 1e-5
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=1)
    M = dec.rows_per_seq
    dec.logits_dbg = torch.zeros((M, shape.vocab), dtype=torch.float32, device="cuda")
    # step 1: root alone (+ its masks); step 2: the first real tree
    for step in range(2):
        n_nodes = int(dec.cur.n_nodes[0])
        res = O.esp_step(m, st, op, O.LAYOUT_PER_NODE, kp, "f32")
        dec.step()
        assert dec.eng.device_status() == 0
        ok = compare_step(dec, res, n_nodes, M, shape, kp, TOL["f32"], dec.logits_dbg.cpu().numpy(), None)
        assert ok, "near-tie in the seeded workload: pick another seed"
        assert int(dec.kv.len[0]) == st.cache_len
    assert int(dec.cur.n_nodes[0]) <= 13     # Top-1 expansion with K = 4, k = 3


def gpu_greedy(B, decode, shape, w, prompt, n_new, cap=512):
    """Plain autoregressive greedy decoding on the GPU path: a tree of the root alone."""
    params = B.tree_params(1, 1, 1, 1, True, False, B.LAYOUT_ROOT_CHAIN)
    dec = decode.EspDecoder(shape, w, params, 1, [cap], prefill_chunk=64)
    out = dec.generate([prompt], n_new)[0]
    assert dec.eng.device_status() == 0
    dec.eng.close()
    return out


def planted(vocab, continuation, depth, rng_seed):
    tok, parent, prev = [None], [-1], 0
    noise = synth.uniform_ints(4 * depth + 4, vocab, rng_seed, 1).tolist()
    for d in range(depth):
        first = len(tok)
        tok.append(int(continuation[d])); parent.append(prev)
        t = noise[d]
        if t != continuation[d]:
            tok.append(int(t)); parent.append(prev)
        prev = first
    return tok, parent


@pytest.mark.parametrize("layout", [0, 1])
def test_config1_loop_is_lossless_and_matches_oracle(B, tiny_setup, layout):
    """32-token loop: (a) GPU ESP == GPU plain greedy token for token (losslessness, Sec. 2);
    (b) GPU ESP == oracle ESP step by step (emitted tokens and accept lengths).  Every second step
    the tree is replaced by one carrying the true continuation so that acceptance > 0 occurs."""
    decode, shape, w, prompt, m = tiny_setup
    n_new, k, K, kp, Bn = 32, 3, 4, 6, 15
    ref_gpu = gpu_greedy(B, decode, shape, w, prompt, n_new + 8)
    ref_cpu = O.greedy_generate(m, prompt, n_new + 8, "f32")
    assert ref_gpu == ref_cpu
    params = B.tree_params(Bn, k, K, 1, True, False, layout)
    dec = make_decoder(B, decode, shape, w, params, kp, ema_lambda=0.1)
    dec.prefill([prompt])
    st = oracle_state_after_prefill(m, prompt, k, "f32")
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=1)
    out, step, accepted = [], 0, 0
    while len(out) < n_new:
        res = O.esp_step(m, st, op, layout, kp, "f32", ema_lambda=0.1)
        dec.step()
        got = dec.emitted()[0]
        assert got == res.emitted, (step, got, res.emitted)
        out.extend(got)
        accepted += len(got) - 1
        step += 1
        if step % 2 == 1:
            tok, parent = planted(shape.vocab, ref_gpu[len(out):], 3, 100 + step)
            tok[0] = out[-1]
            dec.set_tree([tok], [parent])
            st.tok, st.parent = np.asarray(tok), np.asarray(parent)
    assert dec.eng.device_status() == 0
    assert out[:n_new] == ref_gpu[:n_new]
    assert accepted >= 8
    assert rel_err_rows(to_np(dec.mask_embed), st.mask_embed) < 1e-4      # Eq. 5 updates agree


# ---------------------------------------------------------------------------------------------
# bf16 models (MFMA GEMM + MFMA attention), reduced sizes the oracle finishes in seconds
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("qk_norm,layout,n_nodes,k,L", [(False, 0, 13, 4, 300), (True, 0, 20, 3, 1000),
                                                        (True, 1, 64, 4, 130)])
def test_bf16_step_against_oracle(B, qk_norm, layout, n_nodes, k, L):
    from paper_2603_17942_amd import decode
    print(f"bf16 step qk_norm={qk_norm} layout={layout} n={n_nodes} k={k} L={L}", flush=True)
    shape = small_shape(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=1280, vocab=4096, n_layers=3,
                        dtype="bf16", qk_norm=qk_norm, rope_theta=5.0e5)
    w = synth.make_weights(shape, seed=8, unit_gains=False)
    m = oracle_model(shape, w)
    kp, K = 8, 6
    params = B.tree_params(n_nodes, k, K, 0, True, False, layout)
    dec = decode.EspDecoder(shape, w, params, kp, [L + 1024], prefill_chunk=64)
    # synthetic cache contents and a random incoming tree
    kf, vf = synth.make_kv_fill(shape, L, seed=9, device="cuda")
    for l in range(shape.n_layers):
        dec.eng.kv_store(dec.kv, l, 0, 0, kf[l].contiguous(), vf[l].contiguous())
    dec.kv.set_len([L])
    tok, par = synth.make_random_tree(n_nodes, k, shape.vocab, seed=10)
    dec.set_tree([tok.tolist()], [par.tolist()])
    masks = synth.normal_like((k, shape.d_model), 0.02, 12, 0, "cuda", torch.bfloat16)
    dec.mask_embed.copy_(masks)
    M = dec.rows_per_seq
    dec.logits_dbg = torch.zeros((M, shape.vocab), dtype=torch.float32, device="cuda")
    dec.mask_logits = torch.zeros((1, k, shape.vocab), dtype=torch.float32, device="cuda")
    st = O.DecodeState([to_np(kf[l]) for l in range(shape.n_layers)], [to_np(vf[l]) for l in range(shape.n_layers)],
                       L, tok.numpy().astype(np.int64), par.numpy().astype(np.int64), to_np(masks))
    op = O.TreeParams(B=n_nodes, k=k, K=K, expand_width=0)
    res = O.esp_step(m, st, op, layout, kp, "bf16")
    dec.step()
    assert dec.eng.device_status() == 0
    lg_gpu = dec.logits_dbg.cpu().numpy()
    # oracle leg: logits within the band; integers where the oracle's margin is decisive
    full = compare_step(dec, res, n_nodes, M, shape, kp, TOL["bf16"], lg_gpu, None)
    banded = sum(not decisive(res.logits[r], TOL["bf16"]) for r in range(n_nodes))
    # identical-logits leg: every integer of the step, exactly, on the logits the GPU produced
    info = identical_logits_leg(dec, 0, tok.numpy(), par.numpy(), k, layout, kp, op, L, lg_gpu[:res.logits.shape[0]],
                                dec.mask_logits[0].cpu().numpy())
    print(f"  oracle-logits chain compared to the end: {full}; tree rows inside the band: {banded} of {n_nodes}; "
          f"identical-logits leg: {info}", flush=True)
    # the path without debug outputs (arg-max in the LM-head epilogue, logits kept or never written)
    # takes the same integer decisions from the same state
    fused = decode.EspDecoder(shape, w, params, kp, [L + 1024], prefill_chunk=64, engine=dec.eng)
    for l in range(shape.n_layers):
        fused.eng.kv_store(fused.kv, l, 0, 0, kf[l].contiguous(), vf[l].contiguous())
    fused.kv.set_len([L])
    fused.set_tree([tok.tolist()], [par.tolist()])
    fused.mask_embed.copy_(masks)
    fused.step()
    assert fused.eng.device_status() == 0
    assert torch.equal(fused.node_argmax[:n_nodes], dec.node_argmax[:n_nodes])
    assert fused.emitted() == dec.emitted()
    assert torch.equal(fused.topk_id, dec.topk_id) and torch.equal(fused.topk_p, dec.topk_p)
    assert torch.equal(fused.cur.tok, dec.cur.tok) and torch.equal(fused.cur.parent, dec.cur.parent)
    assert torch.equal(fused.cur.anc, dec.cur.anc) and int(fused.kv.len[0]) == int(dec.kv.len[0])
    # hidden states of the block rows against the oracle's K/V written into the cache
    R = res.logits.shape[0]
    blk = O.make_block(tok.numpy(), par.numpy(), k, layout)
    _, _, k_new, v_new = O.tree_forward(m, blk, to_np(masks),
                                        [to_np(kf[l]) for l in range(shape.n_layers)],
                                        [to_np(vf[l]) for l in range(shape.n_layers)], L, want_logits_rows=[])
    ne = int(dec.n_emit[0])
    rows = dec.accepted_row[0, :ne].tolist()
    for l in range(shape.n_layers):
        kk, vv = dec.eng.kv_load(dec.kv, l, 0, L, ne)
        assert rel_err_rows(to_np(kk).reshape(ne, -1), k_new[l][rows].reshape(ne, -1)) < 2e-2
        assert rel_err_rows(to_np(vv).reshape(ne, -1), v_new[l][rows].reshape(ne, -1)) < 2e-2


def test_bf16_loop_is_lossless_up_to_near_ties(B):
    """ESP loop on the bf16 path reproduces the same path's plain greedy decoding.  Row results
    do not depend on the number of rows in the GEMMs, but the attention sums run over a different
    key order in the two loops, so a token may differ only where the greedy margin is inside the
    bf16 band; the test stops comparing at the first such position."""
    from paper_2603_17942_amd import decode
    shape = small_shape(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=1280, vocab=4096, n_layers=2,
                        dtype="bf16", rope_theta=5.0e5)
    w = synth.make_weights(shape, seed=18)
    prompt = synth.make_prompt(100, shape.vocab, seed=19).tolist()
    n_new = 24
    ref = gpu_greedy(B, decode, shape, w, prompt, n_new + 6, cap=1024)
    params = B.tree_params(12, 2, 4, 0, True, False, B.LAYOUT_PER_NODE)
    dec = decode.EspDecoder(shape, w, params, 6, [1024], prefill_chunk=64)
    dec.prefill([prompt])
    M = dec.rows_per_seq
    dec.logits_dbg = torch.zeros((M, shape.vocab), dtype=torch.float32, device="cuda")
    out, step, accepted = [], 0, 0
    while len(out) < n_new:
        dec.step()
        got = dec.emitted()[0]
        want = ref[len(out):len(out) + len(got)]
        if got != want:
            lg = dec.logits_dbg.cpu().numpy()
            star = int(dec.star_row[0])
            # a divergence is only legitimate at a near-tie of some verified row
            rows = dec.accepted_row[0, :len(got)].tolist()
            assert any(not decisive(lg[r], 2e-2) for r in rows), (step, got, want)
            break
        out.extend(got)
        accepted += len(got) - 1
        step += 1
        if step % 2 == 1:
            tok, parent = planted(shape.vocab, ref[len(out):], 2, 200 + step)
            tok[0] = out[-1]
            dec.set_tree([tok], [parent])
    assert dec.eng.device_status() == 0
    assert len(out) >= 8 and accepted >= 2


def test_hip_graph_replay_matches_eager_steps(B):
    """A pair of steps captured into a HIP graph and replayed several times (with the program's
    own eager work and synchronisations in between) emits exactly the tokens of the same number
    of eager steps, and leaves the cache in the same state."""
    from paper_2603_17942_amd import decode
    shape = small_shape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=512, vocab=2048, n_layers=2,
                        dtype="bf16", rope_theta=5.0e5)
    w = synth.make_weights(shape, seed=41)
    prompt = synth.make_prompt(90, shape.vocab, seed=42).tolist()
    params = B.tree_params(10, 2, 3, 0, True, False, B.LAYOUT_PER_NODE)
    n_pairs = 4

    def run(use_graph):
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            dec = decode.EspDecoder(shape, w, params, 5, [1024], prefill_chunk=64)
            dec.prefill([prompt])
            toks = []
            for _ in range(2):                      # every launch site runs once before the capture
                dec.step()
                toks.append(dec.emitted()[0])
            g = dec.capture_step_pair(n_pairs, side) if use_graph else None
            # the captured pair has not advanced the cache: capture records, it does not run
            for _ in range(n_pairs):
                if use_graph:
                    g.replay()
                    toks.append(("pair", dec.emitted()[0]))          # eager work + sync between replays
                else:
                    dec.step()
                    dec.step()
                    toks.append(("pair", dec.emitted()[0]))
                _ = (dec.hidden.float().sum() + dec.kv.len.sum()).item()
            side.synchronize()
            state = (int(dec.kv.len[0]), dec.cur.tok[:dec.rows_per_seq].tolist(), dec.cur.parent[:dec.rows_per_seq].tolist())
            assert dec.eng.device_status() == 0
            k0, v0 = dec.eng.kv_load(dec.kv, 1, 0, 0, state[0])
            dec.eng.close()
        return toks, state, k0.float().cpu().numpy(), v0.float().cpu().numpy()

    eager, graph = run(False), run(True)
    assert graph[0] == eager[0]
    assert graph[1] == eager[1]
    assert np.array_equal(graph[2], eager[2]) and np.array_equal(graph[3], eager[3])


# ---------------------------------------------------------------------------------------------
# sample matching (temperature 1)
# ---------------------------------------------------------------------------------------------
def gpu_sampled_ar(B, decode, shape, w, prompt, n_new, seed, cap=512):
    """One-token-at-a-time sampling on the GPU path: a tree of the root alone, sampling on."""
    params = B.tree_params(1, 1, 1, 1, True, False, B.LAYOUT_ROOT_CHAIN)
    dec = decode.EspDecoder(shape, w, params, 1, [cap], prefill_chunk=64)
    dec.eng.set_sampling(True, seed)
    out = dec.generate([prompt], n_new)[0]
    assert dec.eng.device_status() == 0
    dec.eng.close()
    return out


@pytest.mark.parametrize("layout", [0, 1])
def test_config1_sampled_loop_is_lossless_and_matches_oracle(B, tiny_setup, layout):
    """Sample matching on the tiny fp32 model: (a) the GPU's one-token-at-a-time sampling draws the
    oracle's tokens (same counter-based noise); (b) the GPU ESP loop with sampling on emits that
    sequence token for token and agrees with the oracle's sampled ESP loop step by step, with
    planted continuations so that acceptance occurs."""
    decode, shape, w, prompt, m = tiny_setup
    n_new, k, K, kp, Bn, seed = 24, 3, 4, 6, 15, 1234
    ref_cpu = O.greedy_generate(m, prompt, n_new + 8, "f32", sample_seed=seed)
    ref_gpu = gpu_sampled_ar(B, decode, shape, w, prompt, n_new + 8, seed)
    assert ref_gpu == ref_cpu
    assert ref_cpu != O.greedy_generate(m, prompt, n_new + 8, "f32")
    params = B.tree_params(Bn, k, K, 1, True, False, layout)
    dec = make_decoder(B, decode, shape, w, params, kp)
    dec.eng.set_sampling(True, seed)
    dec.prefill([prompt])
    st = oracle_state_after_prefill(m, prompt, k, "f32")
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=1)
    out, step, accepted = [], 0, 0
    while len(out) < n_new:
        res = O.esp_step(m, st, op, layout, kp, "f32", sample_seed=seed)
        dec.step()
        got = dec.emitted()[0]
        assert got == res.emitted, (step, got, res.emitted)
        out.extend(got)
        accepted += len(got) - 1
        step += 1
        if step % 2 == 1:
            tok, parent = planted(shape.vocab, ref_gpu[len(out):], 3, 300 + step)
            tok[0] = out[-1]
            dec.set_tree([tok], [parent])
            st.tok, st.parent = np.asarray(tok), np.asarray(parent)
    assert dec.eng.device_status() == 0
    assert out[:n_new] == ref_gpu[:n_new]
    assert accepted >= 6
    dec.eng.close()


@pytest.mark.parametrize("n_nodes,k", [(12, 2), (40, 4), (160, 2)])
def test_bf16_sampled_loop_is_lossless_up_to_near_ties(B, n_nodes, k):
    """bf16 path (noise in the LM-head GEMM's arg-max epilogue; 36 rows = one pass over the LM head
    for all rows, 200 rows = gathered tree rows, 160 tree rows = the large-tile kernel's epilogue): the ESP loop with sampling on reproduces the same
    path's one-token-at-a-time sampling; a token may differ only where the margin of the noisy
    arg-max is inside the bf16 band."""
    from paper_2603_17942_amd import decode
    shape = small_shape(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=1280, vocab=4096, n_layers=2,
                        dtype="bf16", rope_theta=5.0e5)
    w = synth.make_weights(shape, seed=18)
    prompt = synth.make_prompt(100, shape.vocab, seed=19).tolist()
    n_new, seed = 20, 77
    ref = gpu_sampled_ar(B, decode, shape, w, prompt, n_new + 6, seed, cap=1024)
    params = B.tree_params(n_nodes, k, 4, 0, True, False, B.LAYOUT_PER_NODE)
    dec = decode.EspDecoder(shape, w, params, 6, [1024], prefill_chunk=64)
    dec.eng.set_sampling(True, seed)
    dec.prefill([prompt])
    M = dec.rows_per_seq
    # a second decoder on the same engine runs the debug path (logits of all rows written, noisy
    # arg-max taken by the stand-alone kernel); `dec` runs the fused epilogues
    dbg = decode.EspDecoder(shape, w, params, 6, [1024], prefill_chunk=64, engine=dec.eng)
    dbg.prefill([prompt])
    dbg.logits_dbg = torch.zeros((M, shape.vocab), dtype=torch.float32, device="cuda")
    out, step, accepted = [], 0, 0
    while len(out) < n_new:
        L0 = int(dec.kv.len[0])
        depth = dec.cur.depth[:M].tolist()
        dbg.step()
        dec.step()
        got = dec.emitted()[0]
        assert got == dbg.emitted()[0], step            # fused and stand-alone draws agree
        want = ref[len(out):len(out) + len(got)]
        if got != want:
            lg = dbg.logits_dbg.cpu().numpy()
            rows = dec.accepted_row[0, :len(got)].tolist()
            noisy = [lg[r].astype(np.float64) -
                     np.log(-np.log(O.counter_uniform(seed, L0 + depth[r] + 1, np.arange(shape.vocab)))) for r in rows]
            assert any(not decisive(x, 2e-2) for x in noisy), (step, got, want)
            break
        out.extend(got)
        accepted += len(got) - 1
        step += 1
        if step % 2 == 1:
            tok, parent = planted(shape.vocab, ref[len(out):], 2, 400 + step)
            tok[0] = out[-1]
            dec.set_tree([tok], [parent])
            dbg.set_tree([tok], [parent])
    assert dec.eng.device_status() == 0
    assert len(out) >= 8 and accepted >= 2
    dec.eng.close()
