"""Pins for the bonus-token variant of the acceptance loop (k drafts verified by k+1 target rows; a
(k+1)-th target token is committed when all k drafts are accepted).

 * Sequence-level exactness by exact enumeration on tabular models (the Appendix Theorem's induction
   step with one more draw from p): the law of the first tokens equals the target's own law.  The same
   enumeration REJECTS two planted mistakes (bonus drawn from the previous row's p; bonus drawn although
   a draft was rejected).
 * T = 0 on the Tiny pair: output equals greedy decoding token for token; a perfect drafter commits
   k+1 tokens per pass; EOS cuts a commit that includes the bonus token.
 * A block with a rejection commits exactly what the variant without bonus commits."""
import functools

import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from test_oracle_acceptance import _law_of_first_tokens, _logs, _pair, _tables, _target_law, enumerate_outcomes, greedy_truth  # noqa: F401


@pytest.mark.parametrize("V,k,n_tok", [(2, 1, 3), (2, 2, 4), (3, 2, 3)])
def test_sequence_level_theorem_exact_with_bonus(V, k, n_tok):
    P, Q = _tables(V, k, 300 + 10 * V + k)
    got = _law_of_first_tokens(V, k, n_tok, P, Q, iteration=functools.partial(O.deer_iteration_tabular, bonus=True))
    want = _target_law(V, n_tok, P)
    assert abs(sum(got.values()) - 1.0) < 1e-12
    for s, pr in want.items():
        assert abs(got.get(s, 0.0) - pr) < 1e-12


def test_bonus_commits_k_plus_one_with_its_exact_probability():
    """P[k+1 tokens committed] = prod_i gamma-like accept probabilities along the accepted path, summed over paths
    = sum over draft blocks of prod_i min(q_i(y_i), p(y_i | ...)); checked by enumeration for k = 2."""
    V, k = 3, 2
    P, Q = _tables(V, k, 77)
    full = 0.0
    for (toks, a), pr in enumerate_outcomes(lambda rng: O.deer_iteration_tabular(
            [0], k, lambda pre: _logs(P[pre[-1]]), lambda pre, i: _logs(Q[pre[-1], i - 1]), rng, bonus=True)):
        assert len(toks) == a + 1
        full += pr * (a == k)
    want = sum(min(Q[0, 0, y1], P[0, y1]) * min(Q[0, 1, y2], P[y1, y2]) for y1 in range(V) for y2 in range(V))
    assert abs(full - want) < 1e-13


def _planted(kind):
    def it(prefix, k, target_logp, drafter_logq, rng):
        j = len(prefix)
        logq = np.stack([drafter_logq(prefix, i + 1) for i in range(k)])
        yhat = [rng.categorical(logq[i], j + i, O.TAG_DRAFT) for i in range(k)]
        logp = np.stack([target_logp(list(prefix) + yhat[:i]) for i in range(k + 1)])
        out = []
        for i in range(k):
            if rng.accept(O.log_alpha(logp[i, yhat[i]], logq[i, yhat[i]]), j + i):
                out.append(yhat[i])
                continue
            out.append(rng.categorical(O.residual_logweights(logp[i], logq[i]), j + i, O.TAG_RESID))
            if kind == "bonus_after_reject":     # row k was conditioned on the rejected drafts
                out.append(rng.categorical(logp[k], j + k, O.TAG_RESID))
            return out, i
        out.append(rng.categorical(logp[k - 1 if kind == "bonus_from_previous_row" else k], j + k, O.TAG_RESID))
        return out, k

    return it


@pytest.mark.parametrize("kind", ["bonus_from_previous_row", "bonus_after_reject"])
def test_enumeration_detects_planted_bonus_mistakes(kind):
    V, k = 3, 2
    P, Q = _tables(V, k, 139)
    got = _law_of_first_tokens(V, k, 3, P, Q, iteration=_planted(kind))
    want = _target_law(V, 3, P)
    assert max(abs(got.get(s, 0.0) - pr) for s, pr in want.items()) > 1e-3


@pytest.mark.parametrize("k", [1, 2, 7])
def test_t0_lossless_with_bonus(tiny, tiny_weights, greedy_truth, k):
    prompt, truth = greedy_truth
    out, accepts = O.deer_decode(_pair(tiny, tiny_weights), prompt, k, 0.0, 64, O.CounterRng(0), bonus=True)
    assert out == truth
    assert all(0 <= a <= k for a in accepts)


def test_t0_perfect_drafter_commits_k_plus_one(tiny, tiny_weights, greedy_truth):
    prompt, truth = greedy_truth
    k = 7
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    out, n_iter = [], 0
    while len(out) < 64:
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=truth[len(out): len(out) + k], bonus=True)
        assert res["accept_len"] == k and len(res["committed"]) == k + 1
        assert res["target_logits"].shape[0] == k + 1
        out += res["committed"]
        n_iter += 1
        assert pair.tc.n == len(prompt) + len(out) - 1
    assert out == truth and n_iter == 8


def test_rejected_block_commits_the_same_with_and_without_bonus(tiny, tiny_weights, greedy_truth):
    prompt, truth = greedy_truth
    k, V = 8, tiny["target"].vocab
    blk = list(truth[:3]) + [(truth[3] + 1) % V] + list(truth[4:8])
    outs = []
    for bonus in (False, True):
        pair = _pair(tiny, tiny_weights)
        pair.prefill(prompt)
        outs.append(O.deer_iteration(pair, k, 0.0, None, draft_override=blk, bonus=bonus))
    assert outs[0]["accept_len"] == outs[1]["accept_len"] == 3
    assert outs[0]["committed"] == outs[1]["committed"] == truth[:4]
    assert np.allclose(outs[0]["target_logits"], outs[1]["target_logits"][:k], atol=1e-6, rtol=0)   # row count changes BLAS blocking


def test_eos_cuts_a_commit_with_bonus(tiny, tiny_weights, greedy_truth):
    prompt, truth = greedy_truth
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    k = 4
    eos = truth[k]                     # the bonus token itself is EOS (unless it occurred earlier)
    res = O.deer_iteration(pair, k, 0.0, None, eos_id=eos, draft_override=truth[:k], bonus=True)
    first = truth.index(eos)
    assert res["committed"] == truth[: first + 1]
    assert pair.tc.n == len(prompt) + first + 1 - 1


def test_sampling_bonus_uses_the_residual_stream_at_position_j_plus_k():
    """The bonus draw is the generator's categorical draw with the residual tag at position j+k (what the device
    path must reproduce): forced acceptance (p == q) of k = 2 drafts, then the third token."""
    V, k, j = 5, 2, 11
    g = np.random.default_rng(3)
    logq = _logs(g.dirichlet(np.ones(V), size=k))
    logp = np.concatenate([logq, _logs(g.dirichlet(np.ones(V), size=1))])
    rng = O.CounterRng(9)
    yhat = [rng.categorical(logq[i], j + i, O.TAG_DRAFT) for i in range(k)]
    a, c = O.accept_block_sampling(logp, logq, yhat, rng, j, bonus=True)
    assert a == k
    assert c == O.CounterRng(9).categorical(logp[k], j + k, O.TAG_RESID)
