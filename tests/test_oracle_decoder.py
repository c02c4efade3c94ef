"""Pins of the oracle's decoder forward, block layout and tree mask (CPU only).

The pins are things other than the oracle itself: the transformers library's Llama and
Qwen3 decoders (a textbook implementation the oracle's special cases must reduce to),
the complex-number form of the rotary embedding, path-by-path sequential decoding
(Sec. 2; App. C: a tree row conditions only on the cache and its root-to-node path),
and brute-force visibility on every small tree.
"""
import itertools

import numpy as np
import pytest
import torch

from util import O, oracle_model, small_shape, synth


def hf_model(shape, weights):
    """Library decoder holding the same weights, float64, eager attention."""
    from transformers import LlamaConfig, LlamaForCausalLM, Qwen3Config, Qwen3ForCausalLM
    common = dict(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ff,
                  num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                  num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                  rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta, attention_bias=False,
                  tie_word_embeddings=False, max_position_embeddings=4096,
                  attn_implementation="eager")
    if shape.qk_norm:
        cfg = Qwen3Config(**common, use_sliding_window=False)
        net = Qwen3ForCausalLM(cfg)
    else:
        cfg = LlamaConfig(**common, mlp_bias=False)
        net = LlamaForCausalLM(cfg)
    net = net.double().eval()
    sd = {"model.embed_tokens.weight": weights["embed"], "lm_head.weight": weights["lm_head"],
          "model.norm.weight": weights["final_norm"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj",
             "w_down": "mlp.down_proj", "norm_attn": "input_layernorm",
             "norm_mlp": "post_attention_layernorm"}
    if shape.qk_norm:
        names.update({"q_norm": "self_attn.q_norm", "k_norm": "self_attn.k_norm"})
    for l, lw in enumerate(weights["layers"]):
        for ours, theirs in names.items():
            sd[f"model.layers.{l}.{theirs}.weight"] = lw[ours]
    missing = net.load_state_dict({k: v.double() for k, v in sd.items()}, strict=True)
    assert not missing.missing_keys and not missing.unexpected_keys
    return net


def hf_logits(net, embeds, positions, allowed):
    """Run the library decoder on explicit embeddings, position ids and a boolean
    [T, T] 'may attend' matrix (passed as an additive 4-D mask)."""
    T = embeds.shape[0]
    add = torch.zeros(1, 1, T, T, dtype=torch.float64)
    add.masked_fill_(~torch.as_tensor(allowed)[None, None], torch.finfo(torch.float64).min)
    with torch.no_grad():
        out = net(inputs_embeds=torch.as_tensor(embeds)[None], attention_mask=add,
                  position_ids=torch.as_tensor(positions, dtype=torch.long)[None], use_cache=False)
    return out.logits[0].numpy()


@pytest.mark.parametrize("qk_norm", [False, True])
def test_chain_equals_library_decoder(qk_norm):
    shape = small_shape(qk_norm=qk_norm, rope_theta=5.0e5 if not qk_norm else 1.0e6)
    w = synth.make_weights(shape, seed=3, unit_gains=False)
    m = oracle_model(shape, w)
    net = hf_model(shape, w)
    toks = synth.make_prompt(11, shape.vocab, seed=4).numpy()
    T = len(toks)
    blk = O.make_block(toks, [-1] + list(range(T - 1)), 0, O.LAYOUT_PER_NODE)
    empty = [np.zeros((0, shape.n_kv_heads, shape.head_dim))] * shape.n_layers
    ours, _, _, _ = O.tree_forward(m, blk, np.zeros((0, shape.d_model)), empty, empty, 0)
    emb = m.weights["embed"][toks]
    theirs = hf_logits(net, emb, np.arange(T), np.tril(np.ones((T, T), dtype=bool)))
    # the library builds its rotary cos/sin tables in float32: agreement to ~1e-7
    np.testing.assert_allclose(ours, theirs, rtol=0, atol=1e-6)


@pytest.mark.parametrize("qk_norm,layout", [(False, O.LAYOUT_PER_NODE), (True, O.LAYOUT_PER_NODE),
                                            (False, O.LAYOUT_ROOT_CHAIN)])
def test_tree_block_with_cache_equals_library_decoder(qk_norm, layout):
    """Cache + tree rows + mask rows in one block equals the library decoder run on
    [prompt, block rows] with the same visibility and positions (Fig. 3, Fig. 7)."""
    shape = small_shape(qk_norm=qk_norm)
    w = synth.make_weights(shape, seed=5, unit_gains=False)
    m = oracle_model(shape, w)
    net = hf_model(shape, w)
    prompt = synth.make_prompt(9, shape.vocab, seed=6).numpy()
    k = 2
    kc, vc, L = O.prefill(m, prompt)
    assert L == len(prompt) - 1
    tok, par = synth.make_random_tree(7, 3, shape.vocab, seed=8)
    tok = tok.numpy().copy()
    tok[0] = prompt[-1]
    blk = O.make_block(tok, par.numpy(), k, layout)
    masks = O.mask_mean_init(m, prompt, k) + 0.01 * np.arange(k)[:, None]  # distinct vectors
    ours, _, _, _ = O.tree_forward(m, blk, masks, kc, vc, L)
    R = blk.n_rows
    emb = np.concatenate([m.weights["embed"][prompt[:-1]], O.block_inputs(m, blk, masks)])
    pos = np.concatenate([np.arange(L), L + blk.depth])
    allowed = np.zeros((L + R, L + R), dtype=bool)
    allowed[:L, :L] = np.tril(np.ones((L, L), dtype=bool))
    allowed[L:, :L] = True
    allowed[L:, L:] = blk.visible
    theirs = hf_logits(net, emb, pos, allowed)[L:]
    # the library builds its rotary cos/sin tables in float32: agreement to ~1e-7
    np.testing.assert_allclose(ours, theirs, rtol=0, atol=1e-6)


def test_rope_against_complex_rotation_and_invariants():
    rng = np.random.default_rng(0)
    hd, theta = 16, 5.0e5
    x = rng.standard_normal((5, 3, hd))
    pos = np.array([0, 1, 7, 100, 2047])
    y = O.rope(x, pos, theta)
    half = hd // 2
    z = x[..., :half] + 1j * x[..., half:]
    w = np.exp(1j * pos[:, None, None] * theta ** (-2.0 * np.arange(half) / hd))
    zr = z * w
    np.testing.assert_allclose(y[..., :half], zr.real, atol=1e-12)
    np.testing.assert_allclose(y[..., half:], zr.imag, atol=1e-12)
    np.testing.assert_allclose(y[0], x[0], atol=0)                        # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    q, kk = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    d1 = O.rope(q, [13], theta)[0, 0] @ O.rope(kk, [5], theta)[0, 0]
    d2 = O.rope(q, [1013], theta)[0, 0] @ O.rope(kk, [1005], theta)[0, 0]
    assert abs(d1 - d2) < 1e-10                                           # relative positions only


def _paths(parent):
    n = len(parent)
    out = []
    for leaf in range(n):
        p, c = [], leaf
        while c >= 0:
            p.append(c)
            c = parent[c]
        out.append(p[::-1])
    return out


@pytest.mark.parametrize("layout", [O.LAYOUT_PER_NODE, O.LAYOUT_ROOT_CHAIN])
def test_tree_forward_equals_sequential_decoding_of_each_path(layout):
    """Every node row's logits (and every mask row's) equal ordinary causal decoding of
    the row's own path: cache, root..node, then masks 1..j (Sec. 2 Eq. 2; App. C)."""
    shape = small_shape()
    w = synth.make_weights(shape, seed=11, unit_gains=False)
    m = oracle_model(shape, w)
    prompt = synth.make_prompt(6, shape.vocab, seed=12).numpy()
    k = 3
    kc, vc, L = O.prefill(m, prompt)
    tok, par = synth.make_random_tree(9, 3, shape.vocab, seed=13)
    tok, par = tok.numpy(), par.numpy()
    blk = O.make_block(tok, par, k, layout)
    masks = O.mask_mean_init(m, prompt, k) * (1.0 + 0.1 * np.arange(k)[:, None])
    logits, _, k_new, v_new = O.tree_forward(m, blk, masks, kc, vc, L)
    emb = m.weights["embed"]
    for node, path in enumerate(_paths(par)):
        owns_masks = layout == O.LAYOUT_PER_NODE or node == 0
        seq = [emb[tok[c]] for c in path] + ([masks[j] for j in range(k)] if owns_masks else [])
        pos = [L + i for i in range(len(seq))]
        ref, k_rows, _ = O.sequence_forward(m, np.stack(seq), pos, kc, vc, L)
        rows = list(path) + ([blk.mask_row(node, j) for j in range(1, k + 1)] if owns_masks else [])
        np.testing.assert_allclose(logits[rows], ref, rtol=0, atol=1e-10)
        np.testing.assert_allclose(k_new[:, rows], k_rows, rtol=0, atol=1e-11)


def _all_parent_arrays(n):
    for combo in itertools.product(*[range(i) for i in range(1, n)]):
        yield [-1] + list(combo)


def test_visibility_and_positions_brute_force_small_trees():
    """Definition check on every rooted tree with <= 6 nodes in topological numbering:
    row r sees block row c iff c lies on r's own chain (root..node, then its masks up to
    itself); position offset = number of rows seen minus one."""
    for n in range(1, 7):
        for parent in _all_parent_arrays(n):
            depth = [0] * n
            for i in range(1, n):
                depth[i] = depth[parent[i]] + 1
            if any(depth[i] < depth[i - 1] for i in range(1, n)):
                continue   # rows must be in depth order
            for k, layout in [(0, 0), (1, 0), (2, 0), (2, 1)]:
                blk = O.make_block(list(range(n)), parent, k, layout)
                owners = range(n) if layout == 0 else [0]
                chains = {}
                for a in (owners if k else []):
                    for j in range(1, k + 1):
                        chains[blk.mask_row(a, j)] = (a, j)
                assert blk.n_rows == n + len(chains)
                assert sorted(chains) == list(range(n, blk.n_rows))
                for r in range(blk.n_rows):
                    a, j = chains.get(r, (r, 0))
                    anc = set()
                    c = a
                    while c >= 0:
                        anc.add(c)
                        c = parent[c]
                    want = set(anc) | {blk.mask_row(a, jj) for jj in range(1, j + 1)}
                    got = set(np.nonzero(blk.visible[r])[0].tolist())
                    assert got == want
                    assert blk.depth[r] == len(want) - 1


def test_static_structure_is_independent_of_cache_length():
    """App. E: between steps the mask structure is unchanged (only fully visible cache
    columns are added) and positions shift uniformly by the number of emitted tokens."""
    shape = small_shape(n_layers=1)
    w = synth.make_weights(shape, seed=21)
    m = oracle_model(shape, w)
    tok, par = synth.make_random_tree(6, 2, shape.vocab, seed=22)
    blk = O.make_block(tok.numpy(), par.numpy(), 2, O.LAYOUT_PER_NODE)
    kf, vf = synth.make_kv_fill(shape, 12, seed=23)
    kf, vf = kf.double().numpy(), vf.double().numpy()
    masks = np.ones((2, shape.d_model)) * 0.01
    # same cache content, but shifted two slots later with two extra leading entries:
    # every row's attention set grows by the same two columns and positions shift by 2.
    l1, _, k1, _ = O.tree_forward(m, blk, masks, kf, vf, 10)
    l2, _, k2, _ = O.tree_forward(m, blk, masks, kf, vf, 12)
    assert not np.allclose(l1, l2)
    # keys are rotated by exactly two more positions: un-rotating gives the same vectors
    back = O.rope(k2[0], -2 * np.ones(blk.n_rows), shape.rope_theta)
    np.testing.assert_allclose(back, k1[0], atol=1e-10)


def test_mask_mean_and_ema_closed_forms():
    shape = small_shape(n_layers=1)
    w = synth.make_weights(shape, seed=31)
    m = oracle_model(shape, w)
    prompt = [3, 5, 5, 9]
    mm = O.mask_mean_init(m, prompt, 3)
    want = (m.weights["embed"][3] + 2 * m.weights["embed"][5] + m.weights["embed"][9]) / 4
    for i in range(3):
        np.testing.assert_allclose(mm[i], want, atol=1e-15)
    # Eq. 5 unrolled: after s updates with a constant e, m = e + (1-lam)^s (m0 - e)
    lam, e = 0.1, m.weights["embed"][7]
    cur = mm
    for _ in range(5):
        cur = O.mask_ema_update(cur, e, lam)
    np.testing.assert_allclose(cur[0], e + (1 - lam) ** 5 * (want - e), atol=1e-14)


def test_mask_last_k_and_gaussian_inits_on_tables_with_known_statistics():
    """Sec. 4 mask-design variants a and b, and the out-of-distribution rows of the appendix table."""
    shape = small_shape(n_layers=1)
    w = synth.make_weights(shape, seed=32)
    m = oracle_model(shape, w)
    emb = m.weights["embed"]
    # a. the last k prompt tokens, in prompt order
    lk = O.mask_last_k_init(m, [3, 5, 6, 9], 2)
    np.testing.assert_array_equal(lk[0], np.asarray(emb[6], np.float64))
    np.testing.assert_array_equal(lk[1], np.asarray(emb[9], np.float64))
    with pytest.raises(ValueError):
        O.mask_last_k_init(m, [3], 2)
    # b. a table built to have mean a_d in dimension d and every entry exactly b away from it
    V, d = emb.shape
    a = np.linspace(-0.5, 0.75, d)
    sign = np.where(np.arange(V - V % 2) % 2 == 0, 1.0, -1.0)  # an even number of rows: the signs cancel
    m.weights["embed"] = a[None, :] + 0.125 * sign[:, None]
    mu, sigma = O.embed_table_stats(m)
    np.testing.assert_allclose(mu, a, atol=1e-15)
    assert abs(sigma - 0.125) < 1e-15
    np.testing.assert_allclose(O.mask_gaussian_init(m, 3, None, 5.0), np.tile(a + 0.625, (3, 1)), atol=1e-14)
    np.testing.assert_allclose(O.mask_gaussian_init(m, 3, None, 10.0), np.tile(a + 1.25, (3, 1)), atol=1e-14)
    z = np.random.default_rng(5).standard_normal((3, d))
    g = O.mask_gaussian_init(m, 3, z)
    np.testing.assert_allclose((g - a[None, :]) / 0.125, z, atol=1e-12)
    # the seeded N(0, 0.02^2) table: the fit recovers the generator's parameters, and masks drawn
    # from the fit have the table's own first two moments
    m.weights["embed"] = emb
    mu, sigma = O.embed_table_stats(m)
    assert np.max(np.abs(mu)) < 5 * 0.02 / np.sqrt(V)
    assert abs(sigma / 0.02 - 1) < 0.02
    big = O.mask_gaussian_init(m, 64, np.random.default_rng(6).standard_normal((64, d)))
    assert abs(big.std() / np.asarray(emb, np.float64).std() - 1) < 0.05
