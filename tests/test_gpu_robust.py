"""Error paths, determinism and memory discipline of the HIP path, all driven from the host with
every kernel exiting normally: conditions only the device can see must set the sticky status
word and skip the offending work (nothing is read or written out of bounds), the same inputs must
give bit-identical outputs, and no kernel may write outside the workspace it was given."""
import numpy as np
import pytest
import torch

from util import small_shape, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_17942_amd import binding
    binding.load_library()
    assert torch.cuda.is_available(), "GPU tests need a GPU; there is no fallback path"
    return binding


def small_bf16():
    return small_shape(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=512, vocab=2048, n_layers=2,
                       dtype="bf16", rope_theta=5.0e5)


def make_batch_decoder(B, shape, w, lens, nodes, k=3, kp=6, Bn=24, engine=None, guard_bytes=0):
    from paper_2603_17942_amd import decode
    params = B.tree_params(Bn, k, 4, 0, True, False, B.LAYOUT_PER_NODE)
    if engine is None and guard_bytes:
        engine = B.Engine(shape, w, len(lens), Bn * (k + 1), max(lens) + 512, guard_bytes=guard_bytes)
    dec = decode.EspDecoder(shape, w, params, kp, [l + 512 for l in lens], prefill_chunk=64, engine=engine)
    for b in range(len(lens)):
        kf, vf = synth.make_kv_fill(shape, lens[b], seed=30 + b, device="cuda")
        for l in range(shape.n_layers):
            dec.eng.kv_store(dec.kv, l, b, 0, kf[l].contiguous(), vf[l].contiguous())
    dec.kv.set_len(lens)
    trees = [synth.make_random_tree(nodes[b], k, shape.vocab, seed=50 + b) for b in range(len(lens))]
    dec.set_tree([t.tolist() for t, _ in trees], [p.tolist() for _, p in trees])
    dec.mask_embed.copy_(synth.normal_like((k, shape.d_model), 0.02, 12, 0, "cuda", torch.bfloat16))
    return dec, trees


def snapshot(dec):
    torch.cuda.synchronize()
    return {"hidden": dec.hidden.clone(), "argmax": dec.node_argmax.clone(), "n_emit": dec.n_emit.clone(),
            "emit": dec.emit_tok.clone(), "star": dec.star_row.clone(), "ids": dec.topk_id.clone(),
            "p": dec.topk_p.clone(), "len": dec.kv.len.clone(), "tok": dec.cur.tok.clone(),
            "parent": dec.cur.parent.clone(), "anc": dec.cur.anc.clone(), "n_nodes": dec.cur.n_nodes.clone()}


def test_length_over_bound_sets_status_and_skips_only_that_sequence(B):
    """ESP_DEV_LEN_OVER_BOUND: sequence 1's device-side length exceeds the bound the host passed
    (the bound sizes the attention launch).  The status bit is set, the sequence's rows are zero,
    it emits nothing and its cache length stays; the other sequences are computed as if it were
    absent.  Reading the status clears it and the next valid step runs clean."""
    shape = small_bf16()
    w = synth.make_weights(shape, seed=28)
    lens, nodes = [300, 200, 90], [24, 9, 17]
    good, _ = make_batch_decoder(B, shape, w, lens, nodes)
    good.step()
    assert good.eng.device_status() == 0
    ref = snapshot(good)
    bad, _ = make_batch_decoder(B, shape, w, lens, nodes, engine=good.eng)
    bad.kv.len[1] = 450            # device value; the host's bound stays max(lens) = 300
    assert bad.kv.len_bound == 300
    bad.step()
    st = bad.eng.device_status()
    assert st & B.DEV_LEN_OVER_BOUND, st
    got = snapshot(bad)
    R = bad.rows_per_seq
    assert float(got["hidden"][R:2 * R].float().abs().max()) == 0.0
    assert int(got["n_emit"][1]) == 0 and int(got["len"][1]) == 450 and int(got["n_nodes"][1]) == 0
    for b in (0, 2):
        assert torch.equal(got["hidden"][b * R:(b + 1) * R], ref["hidden"][b * R:(b + 1) * R])
        assert int(got["n_emit"][b]) == int(ref["n_emit"][b]) and torch.equal(got["emit"][b], ref["emit"][b])
        assert torch.equal(got["ids"][b], ref["ids"][b]) and torch.equal(got["tok"][b * R:(b + 1) * R], ref["tok"][b * R:(b + 1) * R])
    assert bad.eng.device_status() == 0        # sticky until read, then cleared
    # capacity: length + rows beyond the sequence's slot range is the same condition
    cap, _ = make_batch_decoder(B, shape, w, lens, nodes, engine=good.eng)
    cap.kv.seq_cap[2] = 100        # 90 + 68 rows > 100
    cap.step()
    assert cap.eng.device_status() & B.DEV_LEN_OVER_BOUND
    assert int(cap.n_emit[2]) == 0 and int(cap.kv.len[2]) == 90
    # a clean step afterwards on the same context
    again, _ = make_batch_decoder(B, shape, w, lens, nodes, engine=good.eng)
    again.step()
    assert again.eng.device_status() == 0
    now = snapshot(again)
    for key in ref:
        assert torch.equal(now[key], ref[key]), key
    good.eng.close()


def test_bad_token_and_bad_tree_set_status(B):
    """ESP_DEV_BAD_TOKEN: a token id outside the vocabulary reads nothing (its embedding row is
    zero) and sets the bit.  ESP_DEV_BAD_TREE: a parent that does not precede its child empties
    the sequence's block."""
    shape = small_bf16()
    w = synth.make_weights(shape, seed=28)
    lens, nodes = [120, 64], [10, 12]
    dec, trees = make_batch_decoder(B, shape, w, lens, nodes)
    R = dec.rows_per_seq
    dec.cur.tok[R + 3] = shape.vocab + 5          # sequence 1, node row 3
    dec.step()
    st = dec.eng.device_status()
    assert st == B.DEV_BAD_TOKEN, st
    assert int(dec.n_emit[0]) >= 1 and int(dec.n_emit[1]) >= 1          # both sequences still ran
    neg, _ = make_batch_decoder(B, shape, w, lens, nodes, engine=dec.eng)
    neg.cur.tok[2] = -7
    neg.step()
    assert neg.eng.device_status() == B.DEV_BAD_TOKEN
    tr, _ = make_batch_decoder(B, shape, w, lens, nodes, engine=dec.eng)
    toks = [t.tolist() for t, _ in trees]
    pars = [p.tolist() for _, p in trees]
    pars[0][4] = 7                                 # parent after child
    tr.cur.upload_trees(toks, pars)
    tr.eng.block_from_tree(tr.cur)
    st = tr.eng.device_status()
    assert st == B.DEV_BAD_TREE, st
    assert int(tr.cur.n_rows[0]) == 0 and int(tr.cur.n_rows[1]) == nodes[1] * 4
    tr.step()                                       # the emptied sequence is skipped, the other one runs
    assert int(tr.n_emit[0]) == 0 and int(tr.n_emit[1]) >= 1
    assert tr.eng.device_status() & B.DEV_BAD_TREE   # the tree builder reports the skipped sequence
    dec.eng.close()


@pytest.mark.parametrize("layout,n_nodes,k", [(0, 40, 4), (1, 64, 4)])
def test_step_is_deterministic_run_to_run(B, layout, n_nodes, k):
    """The same step from the same state twice (fresh buffers each time, other work in between):
    every output is bit-identical -- split-K and split-KV partials are reduced in a fixed order,
    there are no floating-point atomics."""
    from paper_2603_17942_amd import decode
    shape = small_shape(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=1280, vocab=4096, n_layers=3,
                        dtype="bf16", qk_norm=True, rope_theta=5.0e5)
    w = synth.make_weights(shape, seed=8, unit_gains=False)
    L, kp = 700, 8
    params = B.tree_params(n_nodes, k, 6, 0, True, False, layout)
    kf, vf = synth.make_kv_fill(shape, L, seed=9, device="cuda")
    tok, par = synth.make_random_tree(n_nodes, k, shape.vocab, seed=10)
    masks = synth.normal_like((k, shape.d_model), 0.02, 12, 0, "cuda", torch.bfloat16)
    eng, snaps = None, []
    for rep in range(3):
        dec = decode.EspDecoder(shape, w, params, kp, [L + 1024], prefill_chunk=64, engine=eng)
        eng = dec.eng
        for l in range(shape.n_layers):
            eng.kv_store(dec.kv, l, 0, 0, kf[l].contiguous(), vf[l].contiguous())
        dec.kv.set_len([L])
        dec.set_tree([tok.tolist()], [par.tolist()])
        dec.mask_embed.copy_(masks)
        dec.step()
        dec.step()                                  # the second step runs on the tree the first one built
        assert eng.device_status() == 0
        s = snapshot(dec)
        s["k1"], s["v1"] = eng.kv_load(dec.kv, 1, 0, 0, int(dec.kv.len[0]))
        snaps.append(s)
        _ = torch.randn(1 << 20, device="cuda").sum().item()      # unrelated work between the repetitions
    for s in snaps[1:]:
        for key in snaps[0]:
            assert torch.equal(s[key], snaps[0][key]), key
    eng.close()


def test_no_write_outside_the_workspace(B):
    """Canaries: the workspace handed to esp_create sits between two guard regions filled with a
    byte pattern; after prefill-sized and step-sized forwards, Top-K', tree building and the mask
    kernels every guard byte is intact, and so are guards around the caller-owned outputs."""
    shape = small_bf16()
    w = synth.make_weights(shape, seed=28)
    lens, nodes = [300, 64, 513], [24, 9, 17]
    dec, _ = make_batch_decoder(B, shape, w, lens, nodes, guard_bytes=1 << 20)
    assert dec.eng.guards_intact()
    R, M = dec.rows_per_seq, 3 * dec.rows_per_seq
    # caller-owned outputs with their own guards: [guard | payload | guard] in one allocation
    pad = 4096
    hid = torch.full((M + 2 * pad // shape.d_model + 2, shape.d_model), 7.0, dtype=torch.bfloat16, device="cuda")
    lo = pad // shape.d_model + 1
    dec.hidden = hid[lo:lo + M]
    for _ in range(3):
        dec.step()
    assert dec.eng.device_status() == 0
    torch.cuda.synchronize()
    assert dec.eng.guards_intact()
    assert float((hid[:lo].float() - 7.0).abs().max()) == 0.0 and float((hid[lo + M:].float() - 7.0).abs().max()) == 0.0
    # the largest row count the context was created for, as a chain block (prefill shape)
    prompt = synth.make_prompt(200, shape.vocab, seed=2).tolist()
    dec2 = make_batch_decoder(B, shape, w, lens, nodes, engine=dec.eng)[0]
    dec2.prefill([prompt, prompt[:50], prompt[:131]])
    dec2.step()
    assert dec.eng.device_status() == 0
    torch.cuda.synchronize()
    assert dec.eng.guards_intact()
    dec.eng.close()
