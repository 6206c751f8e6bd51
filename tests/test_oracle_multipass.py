"""Pins for the multi-pass draft (block regeneration used as a left-to-right multi-pass schedule).

 * n_passes = 1 is the one-pass draft, bit for bit; the fixed positions after each pass are ceil(k s / n).
 * Exactness of the acceptance rule with a drafter whose later positions are conditioned on earlier drafts, by
   exact enumeration on tabular models; the enumeration REJECTS the planted mistake of testing a token against
   the first pass's law although it was drawn from a later pass's.
 * On the Tiny pair: a pass over a partially filled block equals the drafter's plain forward pass over the same
   rows (the definition, computed without the pair's bookkeeping); T = 0 decoding stays equal to greedy decoding;
   the drafter cache ends in the same state as after a one-pass draft."""
import functools

import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from test_oracle_acceptance import _law_of_first_tokens, _logs, _pair, _tables, _target_law, greedy_truth  # noqa: F401


def test_bounds():
    assert O.multipass_bounds(8, 1) == [0, 8]
    assert O.multipass_bounds(8, 2) == [0, 4, 8]
    assert O.multipass_bounds(8, 3) == [0, 3, 6, 8]
    assert O.multipass_bounds(2, 4) == [0, 1, 1, 2, 2]


@pytest.mark.parametrize("V,k,n", [(2, 2, 2), (3, 2, 2), (2, 3, 3), (2, 3, 2)])
def test_sequence_level_theorem_exact_with_multipass_draft(V, k, n):
    P, Q = _tables(V, k, 500 + 10 * V + k)
    got = _law_of_first_tokens(V, k, 3, P, Q, iteration=functools.partial(O.deer_iteration_tabular, n_draft_passes=n))
    want = _target_law(V, 3, P)
    assert abs(sum(got.values()) - 1.0) < 1e-12
    for s, pr in want.items():
        assert abs(got.get(s, 0.0) - pr) < 1e-12


def test_enumeration_detects_stale_first_pass_law():
    V, k = 3, 2
    P, Q = _tables(V, k, 139)

    def it(prefix, k, target_logp, drafter_logq, rng):
        j = len(prefix)
        first = np.stack([drafter_logq(prefix, i + 1) for i in range(k)])      # pass 1: all positions masked
        y1 = rng.categorical(first[0], j, O.TAG_DRAFT)
        second = drafter_logq(list(prefix) + [y1], 1)                           # pass 2: position 2 given y1
        y2 = rng.categorical(second, j + 1, O.TAG_DRAFT)
        logp = np.stack([target_logp(list(prefix)), target_logp(list(prefix) + [y1])])
        a, c = O.accept_block_sampling(logp, first, [y1, y2], rng, j)           # mistake: q_2 of pass 1
        return [y1, y2][:a] + ([] if c is None else [c]), a

    got = _law_of_first_tokens(V, k, 3, P, Q, iteration=it)
    want = _target_law(V, 3, P)
    assert max(abs(got.get(s, 0.0) - pr) for s, pr in want.items()) > 1e-3


def test_one_pass_is_the_plain_draft(tiny, tiny_weights):
    prompt = di.prompt_ids(tiny["target"].vocab, 40, seq=3)
    a, b = _pair(tiny, tiny_weights), _pair(tiny, tiny_weights)
    a.prefill(prompt)
    b.prefill(prompt)
    k = 8
    z = a.draft_logits(k)
    y, zz = O.draft_block_multipass(b, k, 0.0, None, 1)
    assert np.array_equal(z, zz) and y == [O.argmax_lowest(z[i]) for i in range(k)]


def test_partially_filled_pass_equals_a_plain_forward_pass(tiny, tiny_weights):
    """Pass 2 of a 2-pass draft: rows [y_1..y_4, MASK x 4] at positions j..j+7, every row seeing the cache and
    the whole block - evaluated here directly with the decoder, on a cache built by a plain prefill."""
    t, d = tiny["target"], tiny["drafter"]
    prompt = di.prompt_ids(t.vocab, 40, seq=3)
    k, j = 8, 40
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    y, z = O.draft_block_multipass(pair, k, 0.0, None, 2)
    assert pair.dc.n == j                                   # block rows were never appended to the cache
    dec = O.Decoder(d, tiny_weights[1])
    cache = O.KVCache(d, 160, dec.dtype)
    dec.forward(list(prompt), np.arange(j), cache, O.causal_mask(j), j, logits_rows=[])
    mask_id = di.mask_token_id(t.vocab)
    z1 = dec.forward([mask_id] * k, np.arange(j, j + k), cache, np.ones((k, k), dtype=bool), 0)
    assert np.allclose(z[:4], z1[:4], atol=1e-9)
    y1 = [O.argmax_lowest(z1[i]) for i in range(4)]
    assert y[:4] == y1
    z2 = dec.forward(y1 + [mask_id] * 4, np.arange(j, j + k), cache, np.ones((k, k), dtype=bool), 0)
    assert np.allclose(z[4:], z2[4:], atol=1e-9)
    assert y[4:] == [O.argmax_lowest(z2[i]) for i in range(4, 8)]
    assert not np.allclose(z1[4:], z2[4:], atol=1e-3)       # the second pass does see the fixed tokens


@pytest.mark.parametrize("n", [2, 8])
def test_t0_lossless_with_multipass_draft(tiny, tiny_weights, greedy_truth, n):
    prompt, truth = greedy_truth
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    out = []
    while len(out) < 40:
        res = O.deer_iteration(pair, 8, 0.0, O.CounterRng(0), n_draft_passes=n)
        out += res["committed"]
        assert pair.dc.n == len(pair.prefix()) - len(res["committed"])   # only committed rows were ingested
    assert out[:40] == truth[:40]
