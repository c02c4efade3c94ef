"""Pins of the oracle's verification and of the whole-loop losslessness (CPU only)."""
import itertools
import os

import numpy as np
import pytest

from util import O, oracle_model, read_golden, small_shape, synth


def _brute_force_accept(tok, parent, g):
    """Enumerate every root-to-node path; a path is valid when each edge's child token
    equals g at the edge's parent; the answer is the longest valid path."""
    n = len(tok)
    best = [0]
    for node in range(n):
        path, c = [], node
        while c >= 0:
            path.append(c)
            c = parent[c]
        path = path[::-1]
        if all(tok[path[i + 1]] == g[path[i]] for i in range(len(path) - 1)):
            if len(path) > len(best):
                best = path
    return best


def test_verify_equals_brute_force_on_random_small_trees():
    rng = np.random.default_rng(1)
    for trial in range(400):
        n = int(rng.integers(1, 9))
        parent = [-1] + [int(rng.integers(0, i)) for i in range(1, n)]
        tok = [int(t) for t in rng.integers(0, 4, size=n)]
        # sibling tokens must be distinct (they come from distinct list entries)
        seen = set()
        ok = True
        for i in range(1, n):
            if (parent[i], tok[i]) in seen:
                ok = False
            seen.add((parent[i], tok[i]))
        if not ok:
            continue
        g = [int(t) for t in rng.integers(0, 4, size=n)]
        n_star, acc, emitted = O.verify_accept(tok, parent, g)
        best = _brute_force_accept(tok, parent, g)
        assert [0] + acc == best
        assert n_star == best[-1]
        assert emitted == [tok[c] for c in best[1:]] + [g[best[-1]]]


def test_tau_accounting_matches_paper_tables(golden_dir):
    rows = read_golden(os.path.join(golden_dir, "tau_model_calls.txt"))
    assert len(rows) == 8
    for _, _, tau, red in rows:
        assert abs(O.calls_reduction_percent(float(tau)) - float(red)) < 0.006
    # one step that accepts a tokens emits a+1 (the bonus token counts, Sec. 4)
    _, acc, emitted = O.verify_accept([5, 6, 7], [-1, 0, 1], [6, 7, 9])
    assert len(acc) == 2 and emitted == [6, 7, 9]


def _planted_tree(vocab, continuation, depth, k_noise, rng):
    """Tree whose spine is the true greedy continuation, plus noise siblings."""
    tok, parent = [None], [-1]
    prev = 0
    levels = []
    for d in range(depth):
        level = []
        tok.append(continuation[d]); parent.append(prev); level.append(len(tok) - 1)
        used = {continuation[d]}
        for _ in range(k_noise):
            t = int(rng.integers(0, vocab))
            if t in used:
                continue
            used.add(t)
            tok.append(t); parent.append(prev); level.append(len(tok) - 1)
        prev = level[0]
        levels.append(level)
    return tok, parent


@pytest.mark.parametrize("layout", [O.LAYOUT_PER_NODE, O.LAYOUT_ROOT_CHAIN])
def test_planted_continuation_is_accepted_exactly(layout):
    """If the draft tree contains the base model's own greedy continuation down to depth
    d (and the next true token is not below it), exactly d tokens are accepted and the
    step emits the first d+1 greedy tokens (Sec. 2: accepted iff exact match)."""
    shape = small_shape()
    w = synth.make_weights(shape, seed=41, unit_gains=False)
    m = oracle_model(shape, w)
    prompt = synth.make_prompt(7, shape.vocab, seed=42).numpy()
    ref = O.greedy_generate(m, prompt, 6)
    rng = np.random.default_rng(2)
    for d in range(0, 4):
        kc, vc, L = O.prefill(m, prompt)
        tok, parent = _planted_tree(shape.vocab, ref, d, 2, rng)
        tok[0] = int(prompt[-1])
        st = O.DecodeState(kc, vc, L, np.asarray(tok), np.asarray(parent),
                           O.mask_mean_init(m, prompt, 3))
        res = O.esp_step(m, st, O.TreeParams(B=8, k=3, K=3), layout, 5)
        assert len(res.accepted) == d
        assert res.emitted == ref[:d + 1]
        assert st.cache_len == L + d + 1
        assert int(st.tok[0]) == ref[d]


@pytest.mark.parametrize("layout,prune,width", [(O.LAYOUT_PER_NODE, True, 1),
                                                (O.LAYOUT_PER_NODE, False, 0),
                                                (O.LAYOUT_ROOT_CHAIN, True, 0)])
def test_esp_loop_reproduces_plain_greedy_decoding(layout, prune, width):
    """Losslessness: the ESP loop emits the base model's greedy decode token for token,
    whatever the tree holds.  Every other step the freshly built tree is replaced by one
    that carries the true continuation, so that multi-token acceptance really occurs."""
    shape = small_shape()
    w = synth.make_weights(shape, seed=51, unit_gains=False)
    m = oracle_model(shape, w)
    prompt = synth.make_prompt(8, shape.vocab, seed=52).numpy()
    n_new = 14
    ref = O.greedy_generate(m, prompt, n_new + 6)
    params = O.TreeParams(B=7, k=2, K=3, expand_width=width, prune_parent=prune)
    kc, vc, L = O.prefill(m, prompt)
    st = O.DecodeState(kc, vc, L, np.asarray([prompt[-1]]), np.asarray([-1]),
                       O.mask_mean_init(m, prompt, params.k))
    out, accepted_total, step = [], 0, 0
    rng = np.random.default_rng(3)
    while len(out) < n_new:
        res = O.esp_step(m, st, params, layout, 5, ema_lambda=0.1)
        out.extend(res.emitted)
        accepted_total += len(res.accepted)
        step += 1
        if step % 2 == 1:
            tok, parent = _planted_tree(shape.vocab, ref[len(out):], 2, 1, rng)
            tok[0] = int(st.tok[0])
            st.tok, st.parent = np.asarray(tok), np.asarray(parent)
    assert out[:n_new] == ref[:n_new]
    assert accepted_total >= 4            # the planted steps did accept


def test_generate_wrapper_equals_greedy():
    shape = small_shape(n_layers=1)
    w = synth.make_weights(shape, seed=61)
    m = oracle_model(shape, w)
    prompt = synth.make_prompt(5, shape.vocab, seed=62).numpy()
    out, steps = O.esp_generate(m, prompt, 8, O.TreeParams(B=6, k=2, K=4, prune_parent=False),
                                O.LAYOUT_PER_NODE, 6)
    assert out == O.greedy_generate(m, prompt, 8)
    assert sum(len(s.emitted) for s in steps) >= 8


# ---------------------------------------------------------------------------------------------
# sample matching (temperature 1)
# ---------------------------------------------------------------------------------------------
def test_counter_uniform_is_a_uniform_stream_in_the_open_interval():
    u = O.counter_uniform(7, 3, np.arange(200000))
    assert u.min() > 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / len(u))
    hist = np.histogram(u, bins=16, range=(0, 1))[0] / len(u)
    assert np.all(np.abs(hist - 1 / 16) < 5 * np.sqrt((1 / 16) * (15 / 16) / len(u)))
    # the three counters all matter
    assert not np.array_equal(u[:64], O.counter_uniform(8, 3, np.arange(64)))
    assert not np.array_equal(u[:64], O.counter_uniform(7, 4, np.arange(64)))
    # lag-1 correlation over consecutive ids is that of independent draws
    c = np.corrcoef(u[:-1], u[1:])[0, 1]
    assert abs(c) < 5 / np.sqrt(len(u))


def test_sample_token_follows_the_softmax_distribution():
    """The arg-max of logit + standard Gumbel noise is a draw from softmax(logits): frequencies
    over many positions against the closed form (a wrong sign, a missing logarithm or a
    temperature other than 1 all fail)."""
    logits = np.array([1.5, -0.3, 0.0, 2.2, -4.0, 0.9])
    p = O.softmax(logits)
    n = 60000
    draws = np.array([O.sample_token(logits, 11, pos) for pos in range(n)])
    freq = np.bincount(draws, minlength=len(logits)) / n
    assert np.all(np.abs(freq - p) < 4.5 * np.sqrt(p * (1 - p) / n))
    # a draw is a function of (seed, position) only
    assert O.sample_token(logits, 11, 123) == draws[123]


@pytest.mark.parametrize("layout,width", [(O.LAYOUT_PER_NODE, 1), (O.LAYOUT_ROOT_CHAIN, 0)])
def test_sampled_esp_loop_reproduces_plain_sampled_decoding(layout, width):
    """Losslessness under sample matching: with the draw of every position fixed by
    (seed, position), the ESP loop emits the token sequence of one-token-at-a-time sampling,
    including steps whose tree carries the true continuation."""
    shape = small_shape()
    w = synth.make_weights(shape, seed=71, unit_gains=False)
    m = oracle_model(shape, w)
    prompt = synth.make_prompt(8, shape.vocab, seed=72).numpy()
    n_new, seed = 14, 5
    ref = O.greedy_generate(m, prompt, n_new + 6, sample_seed=seed)
    assert ref != O.greedy_generate(m, prompt, n_new + 6)            # it really samples
    params = O.TreeParams(B=7, k=2, K=3, expand_width=width)
    kc, vc, L = O.prefill(m, prompt)
    st = O.DecodeState(kc, vc, L, np.asarray([prompt[-1]]), np.asarray([-1]),
                       O.mask_mean_init(m, prompt, params.k))
    out, accepted_total, step = [], 0, 0
    rng = np.random.default_rng(4)
    while len(out) < n_new:
        res = O.esp_step(m, st, params, layout, 5, sample_seed=seed)
        out.extend(res.emitted)
        accepted_total += len(res.accepted)
        step += 1
        if step % 2 == 1:
            tok, parent = _planted_tree(shape.vocab, ref[len(out):], 2, 1, rng)
            tok[0] = int(st.tok[0])
            st.tok, st.parent = np.asarray(tok), np.asarray(parent)
    assert out[:n_new] == ref[:n_new]
    assert accepted_total >= 4


def test_round_like_bf16_is_round_to_nearest_even():
    """Storage rounding of the KV cache and mask vectors (bf16 workloads) pinned to the IEEE rule
    through torch's own float32 -> bfloat16 conversion and through hand-built cases: bf16 keeps the
    top 16 bits of a float32, a value exactly half way between two neighbours goes to the one whose
    last kept bit is 0, everything else to the nearer one.  Truncation, round-half-up and
    round-half-away all fail one of the hand-built cases."""
    import torch

    def f32_from_bits(bits):
        return np.asarray(bits, dtype=np.uint32).view(np.float32)

    base = 0x3F800000                    # 1.0; bf16 neighbours are 0x10000 apart in float32 bits
    cases_bits = [
        base + 0x8000,                   # half way, kept bit 0 -> down to 1.0
        base + 0x18000,                  # half way, kept bit 1 -> up (round to even)
        base + 0x7FFF,                   # just below half -> down
        base + 0x8001,                   # just above half -> up
        base + 0x28000,                  # half way, kept bit 0 -> down
        0xBF800000 + 0x8000,             # negative half way, kept bit 0 -> towards zero (-1.0)
        0xBF800000 + 0x18000,            # negative half way, kept bit 1 -> away from zero
        0x3F7F8000,                      # half way below 1.0 with kept bit 1 -> carries into the exponent: 1.0
        0x00008000, 0x00018000,          # subnormal float32 inputs
        0x7F7F7FFF,                      # largest value that stays finite
        0x00000000, 0x80000000,
    ]
    want_bits = [base, base + 0x20000, base, base + 0x10000, base + 0x20000,
                 0xBF800000, 0xBF800000 + 0x20000, 0x3F800000, 0x00000000, 0x00020000, 0x7F7F0000,
                 0x00000000, 0x80000000]
    x = f32_from_bits(cases_bits)
    got = O.round_like(x, "bf16")
    assert got.dtype == np.float64
    assert np.array_equal(got.astype(np.float32).view(np.uint32), np.asarray(want_bits, dtype=np.uint32))
    # library conversion on the same cases and on a seeded sweep (weights-like and cache-like scales)
    lib = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.astype(np.float32).view(np.uint32), lib.view(np.uint32))
    for std, seed in [(0.02, 3), (1.0, 4), (300.0, 5)]:
        v = synth.normal_like((50000,), std, seed, 0, "cpu", torch.float32)
        lib = v.to(torch.bfloat16).to(torch.float64).numpy()
        assert np.array_equal(O.round_like(v.numpy(), "bf16"), lib)
    # float64 inputs are first rounded to float32 (the GPU holds these values in fp32 before the store)
    y = np.asarray([1.0 + 2.0 ** -8 + 2.0 ** -40, 1.0 + 2.0 ** -8 - 2.0 ** -40])
    assert O.round_like(y, "bf16").tolist() == [1.0, 1.0]          # both collapse to the fp32 tie 1 + 2^-8 -> even
    # the other storage types
    z = np.asarray([1.0 + 2.0 ** -30, np.pi])
    assert np.array_equal(O.round_like(z, "f32"), z.astype(np.float32).astype(np.float64))
    assert np.array_equal(O.round_like(z, "f64"), z)
    with pytest.raises(ValueError):
        O.round_like(z, "fp8")
