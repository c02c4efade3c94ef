"""Stage parity on the GPU: each C-ABI entry point against the oracle on the same seeded
inputs.  Integer / index work must be bit-exact; floating point within the stated tolerance
(row-wise max |diff| / max |oracle|: 2e-2 for bf16 inputs, 1e-4 for fp32)."""
import numpy as np
import pytest
import torch

from util import O, oracle_model, small_shape, synth, to_np

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


# ---------------------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (5, 96, 64), (68, 384, 512), (33, 128, 4096), (97, 2048, 1024),
                                   (200, 640, 1024), (320, 512, 4096), (130, 6144, 512), (64, 1056, 256),
                                   (200, 256, 64), (160, 96, 128), (129, 32, 192), (1344, 512, 256)])
def test_gemm_bf16(B, M, N, K):
    print(f"gemm bf16 M={M} N={N} K={K}", flush=True)
    a = synth.normal_like((M, K), 1.0, 11, 0, "cuda", torch.bfloat16)
    w = synth.normal_like((N, K), 0.05, 11, 1, "cuda", torch.bfloat16)
    got = B.gemm(a, w).cpu().numpy()
    got_packed = B.gemm(a, B.pack_weight(w), packed=True).cpu().numpy()
    assert np.array_equal(got, got_packed)   # the streaming layout only moves bytes
    want = to_np(a) @ to_np(w).T            # fp64 on the same bf16 values
    # products of bf16 values are exact in fp32; only the accumulation order differs
    assert rel_err_rows(got, want) < 1e-5
    # split-K must not make a row depend on the other rows of the block (the split count is a
    # function of (N, K) within the <= 128-row tile class)
    if 1 < M <= 128:
        got1 = B.gemm(a[:1].contiguous(), w).cpu().numpy()
        assert np.array_equal(got1[0], got[0])


@pytest.mark.parametrize("M,N,K", [(1, 512, 128), (68, 4096, 256), (128, 1056, 192), (129, 768, 256), (320, 4096, 512),
                                   (200, 2048, 128), (1344, 1280, 256), (700, 33 * 32, 192), (180, 512, 64)])
def test_gemm_argmax_epilogue(B, M, N, K):
    """Sec. 2 Eq. 3: the greedy choice per row, taken in the LM-head GEMM's epilogue (small-tile kernel up
    to 128 rows, large-tile kernel above).  Against the same GEMM's written logits the arg-max must be
    exact, lowest index on ties; planted exact ties (duplicated weight rows) make the tie rule visible,
    also across column tiles and across the waves of a workgroup."""
    print(f"gemm arg-max M={M} N={N} K={K}", flush=True)
    a = synth.normal_like((M, K), 1.0, 13, 0, "cuda", torch.bfloat16)
    w = synth.normal_like((N, K), 0.05, 13, 1, "cuda", torch.bfloat16)
    # duplicate the winning weight row of a few rows at a higher and a lower index
    logits0 = B.gemm(a, w)
    win = logits0.argmax(dim=1)
    for r in range(0, M, max(1, M // 7)):
        n = int(win[r])
        for other in ((n + 40) % N, (n + N - 300) % N, (n + 129) % N):
            w[other] = w[n]
    wp = B.pack_weight(w)
    logits = B.gemm(a, wp, packed=True).cpu().numpy()
    want = np.array([O.argmax_lowest(row) for row in logits], dtype=np.int32)
    got = B.gemm_argmax(a, wp).cpu().numpy()
    assert np.array_equal(got, want), np.nonzero(got != want)[0][:8]
    ties = int(sum((logits[i] == logits[i].max()).sum() > 1 for i in range(M)))
    assert ties >= 1


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (13, 4096, 256), (52, 688, 256), (52, 256, 688), (70, 130, 77)])
def test_gemm_f32(B, M, N, K):
    print(f"gemm f32 M={M} N={N} K={K}", flush=True)
    a = synth.normal_like((M, K), 1.0, 12, 0, "cuda", torch.float32)
    w = synth.normal_like((N, K), 0.05, 12, 1, "cuda", torch.float32)
    got = B.gemm(a, w).cpu().numpy()
    want = to_np(a) @ to_np(w).T
    assert rel_err_rows(got, want) < 1e-5


# ---------------------------------------------------------------------------------------- Top-K
def check_topk(ids, ps, logits, kp, tol):
    """Oracle comparison with the near-tie rule: position j must match where the oracle's gap
    between ranks j and j+1 exceeds the band; probabilities within tolerance everywhere."""
    for r in range(logits.shape[0]):
        want_ids, want_ps = O.softmax_topk(logits[r], kp + 1)
        np.testing.assert_allclose(ps[r], want_ps[:kp], rtol=1e-4, atol=1e-9)
        for j in range(kp):
            gap_ok = (want_ps[j] - want_ps[j + 1]) > tol * want_ps[j] if j + 1 < len(want_ps) else True
            prev_ok = j == 0 or (want_ps[j - 1] - want_ps[j]) > tol * want_ps[j - 1]
            if gap_ok and prev_ok:
                assert ids[r, j] == want_ids[j], (r, j)
        assert len(set(ids[r].tolist())) == kp


@pytest.mark.parametrize("rows,vocab,kp", [(1, 211, 5), (4, 4096, 6), (3, 128256, 10), (5, 2048, 32),
                                           (2, 151936, 12), (7, 2049, 4)])
def test_softmax_topk(B, rows, vocab, kp):
    print(f"topk rows={rows} vocab={vocab} kp={kp}", flush=True)
    logits = synth.normal_like((rows, vocab), 2.0, 21, rows, "cuda", torch.float32)
    ids, ps = B.softmax_topk(logits, kp)
    check_topk(ids.cpu().numpy(), ps.cpu().numpy(), to_np(logits), kp, 1e-6)


def test_softmax_topk_exact_ties_take_lowest_id(B):
    logits = torch.zeros((2, 5000), dtype=torch.float32)
    logits[0, [4000, 7, 2100]] = 3.0
    logits[0, [9, 4999]] = 1.5
    logits[1, :] = -2.0                      # all equal: ids 0..kp-1
    ids, ps = B.softmax_topk(logits.cuda(), 6)
    assert ids[0].tolist() == [7, 2100, 4000, 9, 4999, 0]
    assert ids[1].tolist() == [0, 1, 2, 3, 4, 5]
    want = O.softmax_topk(logits[0].numpy(), 6)
    assert ids[0].tolist() == want[0].tolist()
    np.testing.assert_allclose(ps[0].cpu().numpy(), want[1], rtol=1e-5)


def test_softmax_topk_adversarial_orders_and_masked_logits(B):
    """Rows that defeat the streaming kernel's shortcuts: strictly ascending values (every block
    raises the bound), descending values, -inf entries, fewer finite logits than Kp, Kp == vocab,
    and many rows (one wave per row, several segments per row for few rows)."""
    vocab, kp = 20000, 9
    asc = torch.arange(vocab, dtype=torch.float32) * 1e-3
    desc = asc.flip(0)
    holes = synth.normal_like((vocab,), 1.0, 31, 0, "cpu", torch.float32).clone()
    holes[::3] = float("-inf")
    few = torch.full((vocab,), float("-inf"))
    few[[5, 17000, 9999]] = torch.tensor([0.5, 2.0, -1.0])
    logits = torch.stack([asc, desc, holes, few]).cuda()
    ids, ps = B.softmax_topk(logits, kp)
    ids, ps = ids.cpu().numpy(), ps.cpu().numpy()
    for r in range(3):
        want_ids, want_ps = O.softmax_topk(logits[r].cpu().numpy(), kp)
        assert ids[r].tolist() == want_ids.tolist()
        np.testing.assert_allclose(ps[r], want_ps, rtol=1e-4)
    assert ids[3, :3].tolist() == [17000, 5, 9999] and np.all(ids[3, 3:] == -1) and np.all(ps[3, 3:] == 0)
    np.testing.assert_allclose(ps[3, :3].sum(), 1.0, rtol=1e-5)
    small = synth.normal_like((2, 8), 1.0, 32, 0, "cuda", torch.float32)
    ids, ps = B.softmax_topk(small, 8)
    for r in range(2):
        want_ids, want_ps = O.softmax_topk(to_np(small)[r], 8)
        assert ids[r].tolist() == want_ids.tolist()
        np.testing.assert_allclose(ps[r].cpu().numpy(), want_ps, rtol=1e-5)
    many = synth.normal_like((700, 4100), 2.0, 33, 0, "cuda", torch.float32)
    ids, ps = B.softmax_topk(many, 10)
    check_topk(ids.cpu().numpy(), ps.cpu().numpy(), to_np(many), 10, 1e-6)


# ---------------------------------------------------------------------------------------- engine fixture
@pytest.fixture(scope="module")
def tiny_engine(B):
    shape = small_shape(d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ff=176, vocab=517, n_layers=2)
    w = synth.make_weights(shape, seed=3, unit_gains=False)
    eng = B.Engine(shape, w, max_batch=3, max_rows_per_seq=640, max_kv_len=2048)
    yield shape, w, eng
    eng.close()


# ---------------------------------------------------------------------------------------- block descriptor
def bits_to_matrix(anc_row_words, n):
    out = np.zeros(n, dtype=bool)
    for c in range(n):
        out[c] = (int(anc_row_words[c // 64]) >> (c % 64)) & 1
    return out


def check_block(blk, b, tok, par, k, layout):
    ob = O.make_block(tok, par, k, layout)
    r0 = b * blk.rows_per_seq
    R = ob.n_rows
    assert int(blk.n_rows[b]) == R and int(blk.n_nodes[b]) == len(tok)
    sl = slice(r0, r0 + R)
    assert blk.depth[sl].tolist() == ob.depth.tolist()
    assert blk.mask_j[sl].tolist() == ob.mask_j.tolist()
    assert blk.attach[sl].tolist() == ob.attach.tolist()
    assert blk.tok[r0:r0 + len(tok)].tolist() == [int(t) for t in tok]
    assert all(t == -1 for t in blk.tok[r0 + len(tok):r0 + R].tolist())
    anc = blk.anc[sl].cpu().numpy().astype(np.uint64)
    for r in range(R):
        assert np.array_equal(bits_to_matrix(anc[r], R), ob.visible[r]), r
    return ob


@pytest.mark.parametrize("k,layout,n_nodes", [(0, 0, 7), (3, 0, 13), (4, 0, 64), (4, 1, 64), (5, 0, 96), (2, 1, 1),
                                              (1, 0, 1), (4, 0, 128)])
def test_block_from_tree(B, tiny_engine, k, layout, n_nodes):
    shape, w, eng = tiny_engine
    print(f"block_from_tree k={k} layout={layout} n={n_nodes}", flush=True)
    rows = n_nodes * (k + 1) if layout == 0 else n_nodes + k
    blk = B.BlockBuffers(2, min(rows + 3, 640), k, layout)
    t0, p0 = synth.make_random_tree(n_nodes, max(k, 1) if k else 6, shape.vocab, seed=30 + n_nodes)
    t1, p1 = synth.make_random_tree(max(1, n_nodes // 2), max(k, 1) if k else 6, shape.vocab, seed=31)
    blk.upload_trees([t0.tolist(), t1.tolist()], [p0.tolist(), p1.tolist()])
    eng.block_from_tree(blk)
    assert eng.device_status() == 0
    check_block(blk, 0, t0.numpy(), p0.numpy(), k, layout)
    check_block(blk, 1, t1.numpy(), p1.numpy(), k, layout)


def test_block_from_tree_rejects_malformed_tree(B, tiny_engine):
    shape, w, eng = tiny_engine
    blk = B.BlockBuffers(2, 24, 1, 0)
    blk.upload_trees([[1, 2, 3], [4, 5, 6, 7]], [[-1, 0, 2], [-1, 0, 1, 1]])   # seq 0: parent not before child
    eng.block_from_tree(blk)
    assert eng.device_status() & B.DEV_BAD_TREE
    assert int(blk.n_rows[0]) == 0 and int(blk.n_rows[1]) == 8
    assert eng.device_status() == 0   # sticky word was cleared by the read


# ---------------------------------------------------------------------------------------- tree builder
def random_lists(rng, k, kp, vocab):
    ids = np.zeros((k, kp), dtype=np.int32)
    ps = np.zeros((k, kp), dtype=np.float32)
    for i in range(k):
        ids[i] = rng.choice(vocab, size=kp, replace=False)
        ps[i] = np.sort(rng.dirichlet(np.ones(kp + 3))[:kp])[::-1].astype(np.float32)
    return ids, ps


@pytest.mark.parametrize("Bn,k,K,kp,width,layout,prune,static", [
    (15, 3, 4, 6, 1, 0, True, None),
    (64, 4, 8, 10, 0, 0, True, None),
    (64, 4, 8, 10, 0, 1, False, None),
    (96, 5, 10, 12, 0, 0, True, None),
    (10, 2, 100, 12, 1, 0, True, None),
    (30, 1, 100, 32, 1, 0, True, None),
    (2, 2, 3, 5, 1, 0, True, None),
    (20, 2, 15, 17, 1, 0, True, [15, 4]),
    (6, 2, 3, 5, 1, 1, True, [3, 2]),
    (32, 4, 8, 10, 3, 0, True, None),
])
def test_build_prune_tree_bit_exact(B, tiny_engine, Bn, k, K, kp, width, layout, prune, static):
    shape, w, eng = tiny_engine
    print(f"build_tree B={Bn} k={k} K={K} kp={kp} width={width} layout={layout} static={static}", flush=True)
    rng = np.random.default_rng(Bn * 100 + k)
    batch = 3
    vocab_small = 40          # small vocabulary: repeats with the parent's token do occur
    nodes = Bn if static is None else 1 + sum(static)
    rows = nodes * (k + 1) if layout == 0 else nodes + k
    nxt = B.BlockBuffers(batch, rows, k, layout)
    ids = np.zeros((batch, k, kp), dtype=np.int32)
    ps = np.zeros((batch, k, kp), dtype=np.float32)
    for b in range(batch):
        ids[b], ps[b] = random_lists(rng, k, kp, vocab_small)
    # exact probability ties across parents and a zero-probability tail in sequence 2
    ps[2, :, kp // 2:] = ps[2, :, kp // 2:kp // 2 + 1]
    n_lists = np.array([k, max(k - 1, 0), k], dtype=np.int32)
    n_emit = np.array([1, 2, 1], dtype=np.int32)
    emit = np.zeros((batch, B.MAX_MASKS + 1), dtype=np.int32)
    emit[0, 0] = ids[0, 0, 0]          # root token equals the best depth-1 candidate
    emit[1, 1] = 7
    emit[2, 0] = 3
    params = B.tree_params(Bn, k, K, width, prune, False, layout, static)
    dev = lambda a: torch.as_tensor(a).cuda()
    eng.build_prune_tree(params, dev(ids), dev(ps), kp, dev(n_lists), dev(n_emit), dev(emit), nxt)
    assert eng.device_status() == 0
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=width, prune_parent=prune, static_widths=static)
    for b in range(batch):
        root = int(emit[b, n_emit[b] - 1])
        tok, par, _ = O.build_prune_tree(op, ids[b], ps[b], root, n_depths=int(n_lists[b]))
        r0 = b * rows
        n = int(nxt.n_nodes[b])
        assert n == len(tok)
        assert nxt.tok[r0:r0 + n].tolist() == tok.tolist()
        assert nxt.parent[r0:r0 + n].tolist() == par.tolist()
        check_block(nxt, b, tok, par, k, layout)
    if static is None:
        return
    # Fixed tree, same block again (Sec. 4.3: its rows are built once; later calls only write tokens):
    # new lists and roots, every sequence with all k lists -- then a call in which a list of sequence
    # 1 runs out of entries, so that its tree is smaller and must be rebuilt in full -- then full lists
    # again.  Every call is checked against the oracle like the first one.
    for rnd in range(3):
        for b in range(batch):
            ids[b], ps[b] = random_lists(rng, k, kp, vocab_small)
        n_lists[:] = k
        if rnd == 1:
            ids[1, 0, 1:] = -1                       # depth 1 of sequence 1 has a single entry
            ps[1, 0, 1:] = 0.0
        emit[:, 0] = rng.integers(0, vocab_small, size=batch)
        n_emit[:] = 1
        eng.build_prune_tree(params, dev(ids), dev(ps), kp, dev(n_lists), dev(n_emit), dev(emit), nxt)
        assert eng.device_status() == 0
        for b in range(batch):
            # (a negative id ends a list on the device; the oracle is handed the list cut there)
            li = [ids[b, i][:1] if (rnd == 1 and b == 1 and i == 0) else ids[b, i] for i in range(k)]
            lp = [ps[b, i][:1] if (rnd == 1 and b == 1 and i == 0) else ps[b, i] for i in range(k)]
            tok, par, _ = O.build_prune_tree(op, li, lp, int(emit[b, 0]), n_depths=k)
            r0 = b * rows
            n = int(nxt.n_nodes[b])
            assert n == len(tok), (rnd, b, n, len(tok))
            assert nxt.tok[r0:r0 + n].tolist() == tok.tolist(), (rnd, b)
            assert nxt.parent[r0:r0 + n].tolist() == par.tolist(), (rnd, b)
            check_block(nxt, b, tok, par, k, layout)


def test_build_prune_tree_with_every_probability_tied(B, tiny_engine):
    """All list entries carry the same probability (a power of two, so the products are exact and
    equal per depth): every selection is decided by creation order alone, and the hundreds of
    candidates that share one probability defeat the histogram shortcut of the selection, so the
    full sort behind it runs.  Bit-exact against the oracle."""
    shape, w, eng = tiny_engine
    Bn, k, K, kp, layout = 96, 5, 10, 12, 0
    batch = 2
    rows = Bn * (k + 1)
    nxt = B.BlockBuffers(batch, rows, k, layout)
    rng = np.random.default_rng(77)
    ids = np.stack([np.stack([rng.permutation(500)[:kp] for _ in range(k)]) for _ in range(batch)]).astype(np.int32)
    ps = np.full((batch, k, kp), 0.0625, dtype=np.float32)
    ps[1, :, 0] = 0.125                                   # sequence 1: one better entry per list, ties below it
    n_lists = np.array([k, k], dtype=np.int32)
    n_emit = np.array([1, 1], dtype=np.int32)
    emit = np.zeros((batch, B.MAX_MASKS + 1), dtype=np.int32)
    emit[:, 0] = [501, 502]
    params = B.tree_params(Bn, k, K, 0, True, False, layout, None)
    dev = lambda a: torch.as_tensor(a).cuda()
    eng.build_prune_tree(params, dev(ids), dev(ps), kp, dev(n_lists), dev(n_emit), dev(emit), nxt)
    assert eng.device_status() == 0
    op = O.TreeParams(B=Bn, k=k, K=K, expand_width=0, prune_parent=True)
    for b in range(batch):
        tok, par, _ = O.build_prune_tree(op, ids[b], ps[b], int(emit[b, 0]), n_depths=k)
        r0 = b * rows
        n = int(nxt.n_nodes[b])
        assert n == len(tok)
        assert nxt.tok[r0:r0 + n].tolist() == tok.tolist()
        assert nxt.parent[r0:r0 + n].tolist() == par.tolist()


# ---------------------------------------------------------------------------------------- verify + KV commit
def test_verify_accept_and_kv_commit(B, tiny_engine):
    shape, w, eng = tiny_engine
    rng = np.random.default_rng(5)
    k, layout, batch = 3, 0, 3
    trees = []
    for b in range(batch):
        t, p = synth.make_random_tree(20 + 5 * b, 3, 6, seed=40 + b, max_children=4)   # tokens in 0..5
        trees.append((t.numpy().copy(), p.numpy().copy()))
    rows = 35 * (k + 1)
    blk = B.BlockBuffers(batch, rows, k, layout)
    blk.upload_trees([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    eng.block_from_tree(blk)
    kv = B.KvCache(shape, [512, 300, 700])
    L0 = [100, 37, 250]
    kv.set_len(L0)
    # fill the block's scratch slots with recognisable rows
    krows, vrows = [], []
    for b in range(batch):
        n = int(blk.n_rows[b])
        kr = synth.normal_like((shape.n_layers, n, shape.n_kv_heads, shape.head_dim), 1.0, 50 + b, 0, "cuda")
        vr = synth.normal_like((shape.n_layers, n, shape.n_kv_heads, shape.head_dim), 1.0, 50 + b, 1, "cuda")
        for l in range(shape.n_layers):
            eng.kv_store(kv, l, b, L0[b], kr[l].contiguous(), vr[l].contiguous())
        krows.append(kr.cpu().numpy()); vrows.append(vr.cpu().numpy())
    g = rng.integers(0, 6, size=batch * rows).astype(np.int32)
    # make sequence 0 accept a full root-to-depth-3 path
    t0, p0 = trees[0]
    d3 = [i for i in range(len(t0)) if O.make_block(t0, p0, 0, 0).depth[i] == 3]
    if d3:
        c = d3[0]
        while p0[c] >= 0:
            g[p0[c]] = t0[c]
            c = p0[c]
    i32 = dict(dtype=torch.int32, device="cuda")
    n_emit = torch.zeros(batch, **i32)
    emit = torch.zeros((batch, B.MAX_MASKS + 1), **i32)
    acc = torch.zeros((batch, B.MAX_MASKS + 1), **i32)
    star = torch.zeros(batch, **i32)
    eng.verify_accept(blk, torch.as_tensor(g).cuda(), kv, n_emit, emit, acc, star)
    assert eng.device_status() == 0
    total_acc = 0
    for b in range(batch):
        tok, par = trees[b]
        n_star, accepted, emitted = O.verify_accept(tok, par, g[b * rows:b * rows + len(tok)])
        ne = int(n_emit[b])
        assert ne == len(emitted)
        assert emit[b, :ne].tolist() == emitted
        assert acc[b, :ne].tolist() == [0] + accepted
        assert int(star[b]) == n_star
        assert int(kv.len[b]) == L0[b] + ne
        total_acc += len(accepted)
        for l in range(shape.n_layers):
            kk, vv = eng.kv_load(kv, l, b, L0[b], ne)
            want_rows = [0] + accepted
            assert np.array_equal(kk.cpu().numpy(), krows[b][l][want_rows])
            assert np.array_equal(vv.cpu().numpy(), vrows[b][l][want_rows])
    assert total_acc >= 3


# ---------------------------------------------------------------------------------------- attention
def run_attention_case(B, shape, eng, n_nodes, k, layout, cache_lens, seed):
    batch = len(cache_lens)
    if k == 0:   # prefill-like chain block: row i sees rows 0..i
        trees = [(torch.arange(n_nodes - 3 * b, dtype=torch.int32) % shape.vocab,
                  torch.arange(-1, n_nodes - 3 * b - 1, dtype=torch.int32)) for b in range(batch)]
    else:
        trees = [synth.make_random_tree(n_nodes - 3 * b, max(k, 2), shape.vocab, seed=seed + b)
                 for b in range(batch)]
    rows = n_nodes * (k + 1) if layout == 0 else n_nodes + k
    blk = B.BlockBuffers(batch, rows, k, layout)
    blk.upload_trees([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    eng.block_from_tree(blk)
    kv = B.KvCache(shape, [L + rows + 5 for L in cache_lens])
    kv.set_len(cache_lens)
    dt = eng.dt
    hq, hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    layer = shape.n_layers - 1
    q = synth.normal_like((batch * rows, hq, hd), 1.0, seed, 7, "cuda", dt)
    oracle_in = []
    for b in range(batch):
        R = int(blk.n_rows[b])
        L = cache_lens[b]
        kf = synth.normal_like((L + R, hkv, hd), 1.0, seed + b, 8, "cuda", dt)
        vf = synth.normal_like((L + R, hkv, hd), 1.0, seed + b, 9, "cuda", dt)
        eng.kv_store(kv, layer, b, 0, kf, vf)
        oracle_in.append((to_np(kf), to_np(vf), R, L))
    out = torch.zeros_like(q)
    eng.attn_tree(blk, kv, layer, q, out)
    assert eng.device_status() == 0
    got = to_np(out).reshape(batch, rows, hq, hd)
    qn = to_np(q).reshape(batch, rows, hq, hd)
    worst = 0.0
    for b in range(batch):
        kf, vf, R, L = oracle_in[b]
        ob = O.make_block(trees[b][0].numpy(), trees[b][1].numpy(), k, layout)
        want = O.tree_attention(qn[b, :R], kf[:L], vf[:L], kf[L:], vf[L:], ob.visible)
        worst = max(worst, rel_err_rows(got[b, :R].reshape(R * hq, hd), want.reshape(R * hq, hd)))
        assert np.all(got[b, R:] == 0)
    return worst


@pytest.mark.parametrize("n_nodes,k,layout,cache_lens", [
    (13, 3, 0, [128]), (5, 2, 1, [0, 3]), (20, 2, 0, [700, 64, 1]), (64, 0, 0, [190])])
def test_attn_tree_f32(B, tiny_engine, n_nodes, k, layout, cache_lens):
    shape, w, eng = tiny_engine
    print(f"attn f32 n={n_nodes} k={k} layout={layout} L={cache_lens}", flush=True)
    err = run_attention_case(B, shape, eng, n_nodes, k, layout, cache_lens, seed=60)
    assert err < 1e-4


@pytest.fixture(scope="module")
def bf16_engine(B):
    shape = small_shape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=384, vocab=1024, n_layers=2,
                        dtype="bf16", qk_norm=True, rope_theta=1.0e6, rms_eps=1e-6)
    w = synth.make_weights(shape, seed=4, unit_gains=False)
    eng = B.Engine(shape, w, max_batch=3, max_rows_per_seq=640, max_kv_len=5000)
    yield shape, w, eng
    eng.close()


@pytest.mark.parametrize("n_nodes,k,layout,cache_lens", [
    (13, 3, 0, [128]), (5, 2, 1, [0, 3]), (64, 4, 0, [2048]), (64, 4, 1, [2048, 777, 63]),
    (17, 4, 0, [4100, 64, 1]), (128, 4, 0, [300]), (200, 0, 0, [129])])
def test_attn_tree_bf16_mfma(B, bf16_engine, n_nodes, k, layout, cache_lens):
    shape, w, eng = bf16_engine
    print(f"attn bf16 n={n_nodes} k={k} layout={layout} L={cache_lens}", flush=True)
    err = run_attention_case(B, shape, eng, n_nodes, k, layout, cache_lens, seed=70)
    assert err < 2e-2


# ------------------------------------------------------------------------- mask initialisations
@pytest.mark.parametrize("hq,hkv,n_nodes,k,layout,cache_lens", [
    (2, 2, 40, 3, 0, [515]),            # no grouping: one query head per kv head
    (8, 1, 30, 4, 0, [260, 31]),        # eight query heads share one kv head: 1200 query columns per kv head
    (16, 2, 9, 2, 1, [70]),             # G = 8, few rows
    (4, 4, 120, 4, 1, [1000, 64, 129, 5]),
])
def test_attn_tree_bf16_other_head_groupings(B, hq, hkv, n_nodes, k, layout, cache_lens):
    """The MFMA attention kernel at other ratios of query to kv heads than the 4 of the two 8B shapes
    (query columns of a kv head = block rows x group size: from 124 to 1200 here, i.e. one to four
    workgroups per kv head and split, with and without paired waves)."""
    shape = small_shape(d_model=max(hq * 16, 128), n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=256, vocab=512, n_layers=1,
                        dtype="bf16", qk_norm=False, rope_theta=1.0e4)
    w = synth.make_weights(shape, seed=5)
    rows = n_nodes * (k + 1) if layout == 0 else n_nodes + k
    eng = B.Engine(shape, w, max_batch=len(cache_lens), max_rows_per_seq=rows, max_kv_len=max(cache_lens) + rows + 64)
    print(f"attn bf16 hq={hq} hkv={hkv} n={n_nodes} k={k} layout={layout} L={cache_lens}", flush=True)
    err = run_attention_case(B, shape, eng, n_nodes, k, layout, cache_lens, seed=90)
    eng.close()
    assert err < 2e-2


@pytest.mark.parametrize("which", ["tiny", "bf16"])
def test_mask_last_k_and_gaussian_inits(B, tiny_engine, bf16_engine, which):
    """Sec. 4 mask-design variants a (last k prompt tokens) and b (Gaussian fit of the embedding
    table), and the mu + 5 sigma / mu + 10 sigma rows of the appendix, against the oracle."""
    shape, w, eng = tiny_engine if which == "tiny" else bf16_engine
    print(f"mask inits {which}", flush=True)
    m = oracle_model(shape, w)
    k = 3
    dt = torch.float32 if shape.dtype == "f32" else torch.bfloat16
    tol = 1e-4 if shape.dtype == "f32" else 2e-2
    out = torch.zeros((k, shape.d_model), dtype=dt, device="cuda")
    prompt = [5, 9, 2, 7, 11]
    eng.mask_last_k(torch.tensor(prompt, dtype=torch.int32, device="cuda"), k, out)
    assert np.array_equal(to_np(out), O.mask_last_k_init(m, prompt, k))     # a copy of table rows: exact
    z = synth.normal_like((k, shape.d_model), 1.0, 41, 0, "cuda", torch.float32)
    for zz, shift in [(z, 0.0), (None, 5.0), (None, 10.0), (z, -1.5)]:
        eng.mask_gaussian(zz, shift, k, out)
        want = O.mask_gaussian_init(m, k, None if zz is None else zz.cpu().numpy(), shift)
        assert rel_err_rows(to_np(out), want) <= tol
    with pytest.raises(RuntimeError):
        eng.mask_last_k(torch.tensor([1, 2], dtype=torch.int32, device="cuda"), 3, out)
