"""Parity at the workload sizes, in the launch configuration bench.py times.

The oracle cannot run a 32-layer 8B-shaped decoder in test time, so each case keeps the full
widths (d_model, heads, d_ff, vocabulary, KV length, tree size, rows) and cuts the depth to two
layers; integer results are compared exactly where the oracle's margin exceeds the bf16 band.
The KV cache contents are synthetic N(0,1)-like values (stand-in for a prefilled prompt).
Long-context and ragged-batch attention are checked on sampled rows at full size."""
import numpy as np
import pytest
import torch

from util import O, identical_logits_leg, oracle_model, small_shape, synth, to_np

pytestmark = pytest.mark.gpu
TOL = 2e-2


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


def decisive(row, tol=TOL):
    top2 = np.sort(row)[-2:]
    return (top2[1] - top2[0]) > 2 * tol * np.max(np.abs(row))


@pytest.mark.parametrize("name,layout,n_nodes,k,K,kp,L", [
    ("llama3_8b", 0, 64, 4, 8, 10, 2048),     # configs[1], block complexity (k+1) N = 320 rows
    ("llama3_8b", 1, 64, 4, 8, 10, 2048),     # configs[1], root chain: 68 rows
    ("qwen3_8b", 0, 96, 5, 10, 12, 4096),     # configs[2] shape: QK-norm, 576 rows
])
def test_step_at_full_width_two_layer_cut(B, name, layout, n_nodes, k, K, kp, L):
    from paper_2603_17942_amd import decode
    print(f"full-width step {name} layout={layout} N={n_nodes} k={k} L={L}", flush=True)
    shape = synth.SHAPES[name].replace(n_layers=2)
    w = synth.make_weights(shape, seed=1, device="cuda")
    params = B.tree_params(n_nodes, k, K, 0, True, False, layout)
    dec = decode.EspDecoder(shape, w, params, kp, [L + 1024], prefill_chunk=64)
    kf, vf = synth.make_kv_fill(shape, L, seed=5, device="cuda")
    for l in range(shape.n_layers):
        dec.eng.kv_store(dec.kv, l, 0, 0, kf[l].contiguous(), vf[l].contiguous())
    dec.kv.set_len([L])
    tok, par = synth.make_random_tree(n_nodes, k, shape.vocab, seed=7)
    dec.set_tree([tok.tolist()], [par.tolist()])
    masks = synth.normal_like((k, shape.d_model), 0.02, 6, 0, "cuda", torch.bfloat16)
    dec.mask_embed.copy_(masks)
    R = dec.rows_per_seq
    dec.logits_dbg = torch.zeros((R, shape.vocab), dtype=torch.float32, device="cuda")
    dec.mask_logits = torch.zeros((1, k, shape.vocab), dtype=torch.float32, device="cuda")
    dec.step()
    assert dec.eng.device_status() == 0
    torch.cuda.synchronize()
    # identical-logits leg (unconditional): arg-max, accepted path, cache length, Top-K' ids and the
    # next tree, exactly, from the logits the GPU itself produced
    op = O.TreeParams(B=n_nodes, k=k, K=K, expand_width=0)
    info = identical_logits_leg(dec, 0, tok.numpy(), par.numpy(), k, layout, kp, op, L,
                                dec.logits_dbg.cpu().numpy(), dec.mask_logits[0].cpu().numpy())
    print(f"identical-logits leg: {info}", flush=True)
    # the same step without debug outputs (the configuration bench.py times) decides the same integers
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
    assert torch.equal(fused.cur.anc, dec.cur.anc)
    del fused
    print("gpu step done; oracle ...", flush=True)

    m = oracle_model(shape, w)
    blk = O.make_block(tok.numpy(), par.numpy(), k, layout)
    assert blk.n_rows == R
    kc = [to_np(kf[l]) for l in range(shape.n_layers)]
    vc = [to_np(vf[l]) for l in range(shape.n_layers)]
    _, hidden, k_new, v_new = O.tree_forward(m, blk, to_np(masks), kc, vc, L, want_logits_rows=[])
    print("oracle forward done", flush=True)
    # LM head at the tree rows -> verification
    node_logits = O.lm_head_logits(m, hidden[:n_nodes])
    lg = dec.logits_dbg[:n_nodes].cpu().numpy()
    assert rel_err_rows(lg, node_logits) <= TOL
    g = np.argmax(node_logits, axis=1)
    g_gpu = dec.node_argmax[:n_nodes].cpu().numpy()
    all_decisive = True
    for r in range(n_nodes):
        if decisive(node_logits[r]):
            assert g_gpu[r] == g[r], r
        else:
            all_decisive = False
    hid_gpu = to_np(dec.hidden[:R])
    assert rel_err_rows(hid_gpu, hidden) <= TOL
    print(f"tree rows whose oracle arg-max margin is inside the band: "
          f"{sum(not decisive(node_logits[r]) for r in range(n_nodes))} of {n_nodes}", flush=True)
    if all_decisive:
        n_star, accepted, emitted = O.verify_accept(blk.tok, blk.parent, g)
        ne = int(dec.n_emit[0])
        assert dec.emit_tok[0, :ne].tolist() == emitted
        assert int(dec.star_row[0]) == n_star
        assert int(dec.kv.len[0]) == L + ne
        a = len(accepted)
        rows = [blk.mask_row(n_star, j) for j in range(1, k + 1)] if layout == 0 else \
            [blk.mask_row(0, a + i) for i in range(1, k - a + 1)]
        mask_logits = O.lm_head_logits(m, hidden[rows])
        assert rel_err_rows(dec.logits_dbg[rows].cpu().numpy(), mask_logits) <= TOL
        ids_gpu = dec.topk_id[0].cpu().numpy()
        ps_gpu = dec.topk_p[0].cpu().numpy()
        same = True
        for i, r in enumerate(rows):
            ids, ps = O.softmax_topk(mask_logits[i], kp + 1)
            np.testing.assert_allclose(ps_gpu[i], ps[:kp], rtol=0.5)
            band = 2 * TOL * np.max(np.abs(mask_logits[i]))
            v = mask_logits[i][ids]
            for j in range(kp):
                up = j == 0 or (v[j - 1] - v[j]) > band
                down = (v[j] - v[j + 1]) > band
                if up and down:
                    assert ids_gpu[i, j] == ids[j], (i, j)
                elif ids_gpu[i, j] != ids[j]:
                    same = False
        # committed K/V of root + accepted rows
        keep = [0] + accepted
        for l in range(shape.n_layers):
            kk, vv = dec.eng.kv_load(dec.kv, l, 0, L, ne)
            assert rel_err_rows(to_np(kk).reshape(ne, -1), k_new[l][keep].reshape(ne, -1)) <= TOL
            assert rel_err_rows(to_np(vv).reshape(ne, -1), v_new[l][keep].reshape(ne, -1)) <= TOL
        # the next tree is valid: full budget, ancestor closed, root = bonus token
        nn = int(dec.cur.n_nodes[0])
        assert nn == n_nodes and int(dec.cur.tok[0]) == emitted[-1]
        par_next = dec.cur.parent[:nn].tolist()
        assert par_next[0] == -1 and all(0 <= par_next[i] < i for i in range(1, nn))
        if same:
            lists_id = [O.softmax_topk(mask_logits[i], kp)[0] for i in range(len(rows))]
            lists_p = [O.softmax_topk(mask_logits[i], kp)[1] for i in range(len(rows))]
            nt, npar, _ = O.build_prune_tree(O.TreeParams(B=n_nodes, k=k, K=K, expand_width=0), lists_id, lists_p,
                                             emitted[-1], n_depths=len(rows))
            # same candidate lists: the tree can only differ if two cumulative probabilities tie to
            # within the last bits of the two softmaxes
            assert dec.cur.tok[:nn].tolist() == nt.tolist()
            assert par_next == npar.tolist()
    dec.eng.close()


@pytest.mark.parametrize("name,layout,n_nodes,k,K,kp,L,lam", [
    ("qwen3_8b", 1, 96, 5, 10, 12, 4096, 0.1),     # configs[2] shape, root chain: 101 rows, EMA on
    ("llama3_8b", 0, 24, 4, 8, 10, 2048, 0.0),     # configs[1] shape, paper layout at block complexity 120
])
def test_four_rolling_steps_at_full_width(B, name, layout, n_nodes, k, K, kp, L, lam):
    """The first four steps of a generation at full width (2-layer cut): every step runs on what the step
    before left on the GPU -- the tree it built, the cache with the rows it committed, the mask vectors
    it updated -- and is checked against the oracle run on exactly that state: logits and hidden states
    of all rows, the integer chain (arg-max, accepted path, cache length, Top-K' ids, next tree) exactly
    on the GPU's own logits, the committed K/V rows against the oracle's rows of the accepted path, and
    the Eq. 5 update.  Before every step the true continuation is planted two levels deep (the token the
    model itself produces, read from a forward of the same block), so that steps commit several rows and
    the next step attends to them."""
    from paper_2603_17942_amd import decode
    print(f"rolling steps {name} layout={layout} N={n_nodes} k={k} L={L}", flush=True)
    shape = synth.SHAPES[name].replace(n_layers=2)
    w = synth.make_weights(shape, seed=1, device="cuda")
    m = oracle_model(shape, w)
    params = B.tree_params(n_nodes, k, K, 0, True, False, layout)
    op = O.TreeParams(B=n_nodes, k=k, K=K, expand_width=0)
    dec = decode.EspDecoder(shape, w, params, kp, [L + 1024], prefill_chunk=64, ema_lambda=lam)
    kf, vf = synth.make_kv_fill(shape, L, seed=5, device="cuda")
    for l in range(shape.n_layers):
        dec.eng.kv_store(dec.kv, l, 0, 0, kf[l].contiguous(), vf[l].contiguous())
    dec.kv.set_len([L])
    tok0, par0 = synth.make_random_tree(n_nodes, k, shape.vocab, seed=7)
    dec.set_tree([tok0.tolist()], [par0.tolist()])
    dec.mask_embed.copy_(synth.normal_like((k, shape.d_model), 0.02, 6, 0, "cuda", torch.bfloat16))
    R = dec.rows_per_seq
    dec.logits_dbg = torch.zeros((R, shape.vocab), dtype=torch.float32, device="cuda")
    dec.mask_logits = torch.zeros((1, k, shape.vocab), dtype=torch.float32, device="cuda")
    committed = 0
    for step in range(4):
        # plant the model's own continuation along one path, two levels deep (untimed forwards)
        n = int(dec.cur.n_nodes[0])
        tok = dec.cur.tok[:n].cpu().numpy().astype(np.int64)
        par = dec.cur.parent[:n].cpu().numpy().astype(np.int64)
        node = 0
        for _ in range(2):
            ch = [c for c in range(1, n) if par[c] == node]
            if not ch:
                break
            dec.eng.tree_forward(dec.cur, dec.mask_embed, dec.kv, dec.hidden, dec.node_argmax, None)
            g = int(dec.node_argmax[node])
            hit = [c for c in ch if tok[c] == g]
            c = hit[0] if hit else ch[0]
            dec.cur.tok[c] = g
            tok[c] = g
            node = c
        # the state the step starts from, as the oracle's input
        L_now = int(dec.kv.len[0])
        masks_in = to_np(dec.mask_embed)
        kc, vc = [], []
        for l in range(shape.n_layers):
            kk, vv = dec.eng.kv_load(dec.kv, l, 0, 0, L_now)
            kc.append(to_np(kk)); vc.append(to_np(vv))
        dec.step()
        assert dec.eng.device_status() == 0
        lg = dec.logits_dbg.cpu().numpy()
        info = identical_logits_leg(dec, 0, tok, par, k, layout, kp, op, L_now, lg, dec.mask_logits[0].cpu().numpy())
        blk = O.make_block(tok, par, k, layout)
        logits, hidden, k_new, v_new = O.tree_forward(m, blk, masks_in, kc, vc, L_now, want_logits_rows=list(range(n)))
        assert rel_err_rows(lg[:n], logits[:n]) <= TOL, step
        assert rel_err_rows(to_np(dec.hidden[:blk.n_rows]), hidden) <= TOL, step
        ne = int(dec.n_emit[0])
        keep = dec.accepted_row[0, :ne].tolist()
        for l in range(shape.n_layers):
            kk, vv = dec.eng.kv_load(dec.kv, l, 0, L_now, ne)
            assert rel_err_rows(to_np(kk).reshape(ne, -1), k_new[l][keep].reshape(ne, -1)) <= TOL, (step, l)
            assert rel_err_rows(to_np(vv).reshape(ne, -1), v_new[l][keep].reshape(ne, -1)) <= TOL, (step, l)
        if lam != 0.0:
            want_m = O.mask_ema_update(masks_in, to_np(w["embed"][int(dec.emit_tok[0, ne - 1])]), lam)
            assert rel_err_rows(to_np(dec.mask_embed), want_m) < 1e-2, step
        committed += ne
        print(f"  step {step}: L={L_now} nodes={n} {info}", flush=True)
    assert int(dec.kv.len[0]) == L + committed
    assert committed >= 8          # planted paths were accepted: at least two extra rows in most steps
    dec.eng.close()


def test_long_context_attention_sampled_rows(B):
    """configs[3]: L = 32768, tree 64 + 4 masks (68 rows) and the 320-row layout, one layer of the
    Llama shape; the oracle evaluates a sample of rows (all heads) one by one."""
    shape = synth.SHAPES["llama3_8b"].replace(n_layers=1, vocab=1024, d_ff=256)
    w = synth.make_weights(shape, seed=1, device="cuda")
    L = 32768
    eng = B.Engine(shape, w, 1, 320, L + 1024)
    kv = B.KvCache(shape, [L + 512])
    kf, vf = synth.make_kv_fill(shape, L + 320, seed=5, device="cuda")
    eng.kv_store(kv, 0, 0, 0, kf[0].contiguous(), vf[0].contiguous())
    kv.set_len([L])
    kn, vn = to_np(kf[0]), to_np(vf[0])
    for layout, rows in [(1, 68), (0, 320)]:
        print(f"long-context attention layout={layout}", flush=True)
        tok, par = synth.make_random_tree(64, 4, shape.vocab, seed=9)
        blk = B.BlockBuffers(1, rows, 4, layout)
        blk.upload_trees([tok.tolist()], [par.tolist()])
        eng.block_from_tree(blk)
        q = synth.normal_like((rows, shape.n_q_heads, shape.head_dim), 1.0, 3, layout, "cuda", torch.bfloat16)
        out = torch.zeros_like(q)
        eng.attn_tree(blk, kv, 0, q, out)
        assert eng.device_status() == 0
        ob = O.make_block(tok.numpy(), par.numpy(), 4, layout)
        sample = sorted(set([0, 1, 5, 37, 63, 64, 65, rows - 1]))
        want = O.tree_attention(to_np(q)[sample], kn[:L], vn[:L], kn[L:L + rows], vn[L:L + rows],
                                ob.visible[sample])
        got = to_np(out)[sample]
        assert rel_err_rows(got.reshape(-1, shape.head_dim), want.reshape(-1, shape.head_dim)) <= TOL
    eng.close()


def test_ragged_batch_attention_sampled_rows(B):
    """configs[4]: 16 sequences, KV lengths uniform in [512, 8192], trees of 32..128 nodes with 4
    mask tokens each (ragged pool); sampled rows of every sequence against the oracle."""
    shape = synth.SHAPES["llama3_8b"].replace(n_layers=1, vocab=1024, d_ff=256)
    w = synth.make_weights(shape, seed=1, device="cuda")
    batch, k, layout = 16, 4, 1
    lens = (512 + synth.uniform_ints(batch, 8192 - 512 + 1, 3, 0)).tolist()
    nodes = (32 + synth.uniform_ints(batch, 128 - 32 + 1, 4, 0)).tolist()
    rows = max(nodes) + k
    eng = B.Engine(shape, w, batch, rows, max(lens) + rows + 64)
    kv = B.KvCache(shape, [l + rows + 8 for l in lens])
    trees = [synth.make_random_tree(nodes[b], 4, shape.vocab, seed=20 + b) for b in range(batch)]
    blk = B.BlockBuffers(batch, rows, k, layout)
    blk.upload_trees([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    eng.block_from_tree(blk)
    fills = []
    for b in range(batch):
        kf, vf = synth.make_kv_fill(shape, lens[b] + nodes[b] + k, seed=40 + b, device="cuda")
        eng.kv_store(kv, 0, b, 0, kf[0].contiguous(), vf[0].contiguous())
        fills.append((to_np(kf[0]), to_np(vf[0])))
    kv.set_len(lens)
    q = synth.normal_like((batch * rows, shape.n_q_heads, shape.head_dim), 1.0, 3, 7, "cuda", torch.bfloat16)
    out = torch.zeros_like(q)
    eng.attn_tree(blk, kv, 0, q, out)
    assert eng.device_status() == 0
    qn, on = to_np(q).reshape(batch, rows, shape.n_q_heads, -1), to_np(out).reshape(batch, rows, shape.n_q_heads, -1)
    for b in range(batch):
        R, L = nodes[b] + k, lens[b]
        ob = O.make_block(trees[b][0].numpy(), trees[b][1].numpy(), k, layout)
        sample = sorted(set([0, 1, nodes[b] // 2, nodes[b] - 1, nodes[b], R - 1]))
        kn, vn = fills[b]
        want = O.tree_attention(qn[b][sample], kn[:L], vn[:L], kn[L:L + R], vn[L:L + R], ob.visible[sample])
        assert rel_err_rows(on[b][sample].reshape(-1, shape.head_dim), want.reshape(-1, shape.head_dim)) <= TOL
        assert np.all(on[b][R:] == 0)
    eng.close()


@pytest.mark.parametrize("Bn,nodes", [(24, [24, 9, 17]), (48, [48, 20, 33])])
def test_batched_step_against_oracle(B, Bn, nodes):
    """Three independent sequences of different cache lengths and tree sizes in one block: every
    entry point handles the batch dimension (small bf16 model, full oracle comparison).  The larger
    case has more than 128 tree rows, so the LM head runs on gathered rows through the large-tile
    GEMM.  Every sequence has mask vectors of its own (Sec. 3.1: Eq. 4 and Eq. 5 are per generation),
    and the Eq. 5 update after the step follows each sequence's own last token."""
    from paper_2603_17942_amd import decode
    shape = small_shape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=512, vocab=2048, n_layers=2,
                        dtype="bf16", rope_theta=5.0e5)
    w = synth.make_weights(shape, seed=28, unit_gains=False)
    m = oracle_model(shape, w)
    k, K, kp, layout = 3, 4, 6, 0
    lens = [300, 64, 1000]
    print(f"batched step B={Bn} nodes={nodes}", flush=True)
    params = B.tree_params(Bn, k, K, 0, True, False, layout)
    lam = 0.25
    dec = decode.EspDecoder(shape, w, params, kp, [l + 512 for l in lens], prefill_chunk=64, ema_lambda=lam)
    fills = []
    for b in range(3):
        kf, vf = synth.make_kv_fill(shape, lens[b], seed=30 + b, device="cuda")
        for l in range(shape.n_layers):
            dec.eng.kv_store(dec.kv, l, b, 0, kf[l].contiguous(), vf[l].contiguous())
        fills.append((kf, vf))
    dec.kv.set_len(lens)
    trees = [synth.make_random_tree(nodes[b], k, shape.vocab, seed=50 + b) for b in range(3)]
    dec.set_tree([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    masks = synth.normal_like((3, k, shape.d_model), 0.02, 12, 0, "cuda", torch.bfloat16)
    assert dec.mask_embed.shape == masks.shape
    dec.mask_embed.copy_(masks)
    R = dec.rows_per_seq
    dec.logits_dbg = torch.zeros((3 * R, shape.vocab), dtype=torch.float32, device="cuda")
    dec.mask_logits = torch.zeros((3, k, shape.vocab), dtype=torch.float32, device="cuda")
    dec.step()
    assert dec.eng.device_status() == 0
    lg = dec.logits_dbg.cpu().numpy()
    emitted = dec.emitted()
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=0)
    for b in range(3):     # identical-logits leg, unconditional, per sequence
        info = identical_logits_leg(dec, b, trees[b][0].numpy(), trees[b][1].numpy(), k, layout, kp, op, lens[b],
                                    lg[b * R:(b + 1) * R], dec.mask_logits[b].cpu().numpy())
        print(f"  seq {b}: {info}", flush=True)
    for b in range(3):
        kf, vf = fills[b]
        st = O.DecodeState([to_np(kf[l]) for l in range(shape.n_layers)], [to_np(vf[l]) for l in range(shape.n_layers)],
                           lens[b], trees[b][0].numpy().astype(np.int64), trees[b][1].numpy().astype(np.int64),
                           to_np(masks[b]))
        res = O.esp_step(m, st, O.TreeParams(B=Bn, k=k, K=K, expand_width=0), layout, kp, "bf16")
        rb = res.logits.shape[0]
        assert rel_err_rows(lg[b * R:b * R + rb], res.logits) <= TOL
        # Eq. 5 on this sequence's own vectors and its own last emitted token (the GPU's: exact inputs)
        want_m = O.mask_ema_update(to_np(masks[b]), to_np(w["embed"][emitted[b][-1]]), lam)
        assert rel_err_rows(to_np(dec.mask_embed[b]), want_m) < 1e-2        # one bf16 rounding
        if all(decisive(res.logits[r]) for r in range(nodes[b])):
            assert emitted[b] == res.emitted
            assert int(dec.star_row[b]) == res.n_star
            assert int(dec.kv.len[b]) == st.cache_len
            assert int(dec.cur.n_nodes[b]) == len(res.next_tok)
    dec.eng.close()


def test_qwen3_shape_256_token_generation_loop(B):
    """configs[2] at full depth: Qwen3-8B shape (36 layers, QK-norm, vocabulary 151936), cache of
    4096 prompt tokens (GPU prefill), k = 5 mask tokens, Top-K 10, trees of 96 nodes (576 rows per
    step), mask EMA on: 256 generated tokens.  The oracle cannot run this size; losslessness is
    checked against the same kernels' one-token-at-a-time decoding, kept in step with the ESP
    loop (it is fed the tokens the loop emits): every emitted token must be the greedy token of
    its prefix, or within the bf16 band of it (the two paths sum attention over a different key
    order, and with random weights over 151936 tokens near-ties are common).  The cache length
    always equals prompt + emitted tokens, and every third step the tree carries the true
    continuation (three tokens of look-ahead by the reference), so that multi-token acceptance
    and the KV commit are exercised at this size."""
    from paper_2603_17942_amd import decode
    shape = synth.SHAPES["qwen3_8b"]
    print("qwen3 loop: weights", flush=True)
    w = synth.make_weights(shape, seed=1, device="cuda")
    L0, n_new, k, K, kp, nodes = 4096, 256, 5, 10, 12, 96
    prompt = synth.make_prompt(L0 + 1, shape.vocab, seed=2).tolist()
    decode.EspDecoder.default_max_rows = nodes * (k + 1)
    ar = decode.EspDecoder(shape, w, B.tree_params(1, 1, 1, 1, True, False, B.LAYOUT_ROOT_CHAIN), 1,
                           [L0 + n_new + 1024], prefill_chunk=256)
    eng = ar.eng
    print("qwen3 loop: prefill", flush=True)
    ar.prefill([prompt])
    ar.logits_dbg = torch.zeros((ar.rows_per_seq, shape.vocab), dtype=torch.float32, device="cuda")
    params = B.tree_params(nodes, k, K, 0, True, False, B.LAYOUT_PER_NODE)
    dec = decode.EspDecoder(shape, w, params, kp, [L0 + n_new + 1024], prefill_chunk=256, ema_lambda=0.1, engine=eng)
    dec.prefill([prompt])

    def ar_feed(root_tok):
        """One reference forward with `root_tok` as the last token; returns the logits of its successor."""
        ar.set_tree([[int(root_tok)]], [[-1]])
        ar.step()
        return ar.logits_dbg[0]

    print("qwen3 loop: ESP loop", flush=True)
    out, step, accepted, exact, last = [], 0, 0, 0, prompt[-1]
    while len(out) < n_new:
        dec.step()
        got = dec.emitted()[0]
        assert 1 <= len(got) <= k + 1
        assert int(dec.kv.len[0]) == L0 + len(out) + len(got)
        for g in got:                                   # the reference follows, token by token
            lg = ar_feed(last)
            top = float(lg.max())
            exact += int(int(lg.argmax()) == g)
            assert float(lg[g]) >= top - 2 * TOL * float(lg.abs().max()), (len(out), g, int(lg.argmax()))
            out.append(g)
            last = g
        accepted += len(got) - 1
        step += 1
        if step % 3 == 1:
            # three tokens of look-ahead by the reference, then rewind it; plant them as a chain
            L_sync = int(ar.kv.len[0])
            cont, t = [], last
            for _ in range(3):
                t = int(ar_feed(t).argmax())
                cont.append(t)
            ar.kv.set_len([L_sync])
            dec.set_tree([[last] + cont], [[-1, 0, 1, 2]])
    assert eng.device_status() == 0
    print(f"qwen3 loop: {step} steps, {len(out)} tokens, {accepted} accepted draft tokens, "
          f"{exact} of {len(out)} tokens are the reference's arg-max exactly", flush=True)
    assert exact >= 0.85 * len(out)          # the rest sit inside the band (asserted above, token by token)
    assert accepted >= 60                # about a third of the steps carry three true tokens
    decode.EspDecoder.default_max_rows = 0
    eng.close()


def test_config5_batched_step_at_full_size(B):
    """configs[4] as a whole step: 16 independent sequences, KV lengths uniform in [512, 8192] and
    trees of 32..128 nodes (both seeded), k = 4 mask tokens per node (block complexity 5 N, up to 640
    rows per sequence, 10240-row block), Top-K 8, Llama-3-8B widths, depth cut to two layers.
    Every sequence: the integer chain of the step, exactly, on the GPU's own logits.  Two sampled
    sequences (the cheapest and the costliest for the oracle): logits, hidden states and committed
    K/V against the oracle's forward."""
    from paper_2603_17942_amd import decode
    shape = synth.SHAPES["llama3_8b"].replace(n_layers=2)
    batch, k, K, kp, layout, Bn = 16, 4, 8, 10, 0, 128
    lens = (512 + synth.uniform_ints(batch, 8192 - 512 + 1, 3, 0)).tolist()
    nodes = (32 + synth.uniform_ints(batch, 128 - 32 + 1, 4, 0)).tolist()
    print(f"config 5 step: lens={lens} nodes={nodes}", flush=True)
    w = synth.make_weights(shape, seed=1, device="cuda")
    params = B.tree_params(Bn, k, K, 0, True, False, layout)
    dec = decode.EspDecoder(shape, w, params, kp, [l + 640 + 64 for l in lens], prefill_chunk=64)
    R = dec.rows_per_seq
    assert R == 640
    cost = [lens[b] * nodes[b] for b in range(batch)]
    sampled = sorted({int(np.argmin(cost)), int(np.argmax(cost))})
    fills = {}
    for b in range(batch):
        kf, vf = synth.make_kv_fill(shape, lens[b], seed=40 + b, device="cuda")
        for l in range(shape.n_layers):
            dec.eng.kv_store(dec.kv, l, b, 0, kf[l].contiguous(), vf[l].contiguous())
        if b in sampled:
            fills[b] = (kf, vf)
    dec.kv.set_len(lens)
    trees = [synth.make_random_tree(nodes[b], k, shape.vocab, seed=60 + b) for b in range(batch)]
    dec.set_tree([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    masks = synth.normal_like((k, shape.d_model), 0.02, 6, 0, "cuda", torch.bfloat16)
    dec.mask_embed.copy_(masks)
    dec.logits_dbg = torch.zeros((batch * R, shape.vocab), dtype=torch.float32, device="cuda")
    dec.mask_logits = torch.zeros((batch, k, shape.vocab), dtype=torch.float32, device="cuda")
    dec.step()
    assert dec.eng.device_status() == 0
    torch.cuda.synchronize()
    print("gpu step done", flush=True)
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=0)
    total_acc = 0
    for b in range(batch):
        info = identical_logits_leg(dec, b, trees[b][0].numpy(), trees[b][1].numpy(), k, layout, kp, op, lens[b],
                                    dec.logits_dbg[b * R:(b + 1) * R].cpu().numpy(), dec.mask_logits[b].cpu().numpy())
        total_acc += info["accepted"]
    print(f"identical-logits leg green for all {batch} sequences", flush=True)
    # the configuration bench.py times (no debug outputs): same integers from the same state
    fused = decode.EspDecoder(shape, w, params, kp, [l + 640 + 64 for l in lens], prefill_chunk=64, engine=dec.eng)
    for b in range(batch):
        kf, vf = fills[b] if b in fills else synth.make_kv_fill(shape, lens[b], seed=40 + b, device="cuda")
        for l in range(shape.n_layers):
            fused.eng.kv_store(fused.kv, l, b, 0, kf[l].contiguous(), vf[l].contiguous())
    fused.kv.set_len(lens)
    fused.set_tree([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    fused.mask_embed.copy_(masks)
    fused.step()
    assert fused.eng.device_status() == 0
    assert fused.emitted() == dec.emitted()
    assert torch.equal(fused.star_row, dec.star_row) and torch.equal(fused.kv.len, dec.kv.len)
    assert torch.equal(fused.topk_id, dec.topk_id) and torch.equal(fused.topk_p, dec.topk_p)
    assert torch.equal(fused.cur.tok, dec.cur.tok) and torch.equal(fused.cur.parent, dec.cur.parent)
    for b in range(batch):
        assert torch.equal(fused.node_argmax[b * R:b * R + nodes[b]], dec.node_argmax[b * R:b * R + nodes[b]])
    del fused
    # oracle forward of the sampled sequences
    m = oracle_model(shape, w)
    for b in sampled:
        print(f"oracle forward of sequence {b}: L={lens[b]} nodes={nodes[b]}", flush=True)
        kf, vf = fills[b]
        kc = [to_np(kf[l]) for l in range(shape.n_layers)]
        vc = [to_np(vf[l]) for l in range(shape.n_layers)]
        blk = O.make_block(trees[b][0].numpy(), trees[b][1].numpy(), k, layout)
        rb = blk.n_rows
        _, hidden, k_new, v_new = O.tree_forward(m, blk, to_np(masks), kc, vc, lens[b], want_logits_rows=[])
        assert rel_err_rows(to_np(dec.hidden[b * R:b * R + rb]), hidden) <= TOL
        node_logits = O.lm_head_logits(m, hidden[:nodes[b]])
        assert rel_err_rows(dec.logits_dbg[b * R:b * R + nodes[b]].cpu().numpy(), node_logits) <= TOL
        g = np.argmax(node_logits, axis=1)
        g_gpu = dec.node_argmax[b * R:b * R + nodes[b]].cpu().numpy()
        banded = 0
        for r in range(nodes[b]):
            if decisive(node_logits[r]):
                assert g_gpu[r] == g[r], (b, r)
            else:
                banded += 1
        print(f"  tree rows inside the band: {banded} of {nodes[b]}", flush=True)
        ne = int(dec.n_emit[b])
        keep = dec.accepted_row[b, :ne].tolist()
        for l in range(shape.n_layers):
            kk, vv = dec.eng.kv_load(dec.kv, l, b, lens[b], ne)
            assert rel_err_rows(to_np(kk).reshape(ne, -1), k_new[l][keep].reshape(ne, -1)) <= TOL
            assert rel_err_rows(to_np(vv).reshape(ne, -1), v_new[l][keep].reshape(ne, -1)) <= TOL
        # rows past the sequence's block stay zero
        assert float(dec.hidden[b * R + rb:(b + 1) * R].float().abs().max()) == 0.0 if rb < R else True
    dec.eng.close()
