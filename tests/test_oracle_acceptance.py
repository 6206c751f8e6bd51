"""Pins for the acceptance rule and the decoding loop.

 * T=0: draft-verify output equals plain greedy decoding of the target, token for token
   (Appendix, Theorem, specialised to one-hot distributions), for several block sizes, for an
   adversarial and for a perfect drafter.
 * One-step Lemma by exact enumeration: the emitted token's law is p, and P[reject] = 1 - gamma.
 * Sequence-level Theorem by exact enumeration of the loop on tabular models; the same
   enumeration REJECTS two planted mistakes (continuing after a rejection; resampling from p
   instead of the residual).
 * Closed-form acceptance rate gamma_1 and first-token law on the Tiny transformer pair."""
import itertools

import numpy as np
import pytest
from scipy.stats import binomtest, chisquare

import deer_inputs as di
from oracle import deer_oracle as O


# ----------------------------------------------------------------------------------------------
# an "rng" that enumerates every outcome of the loop with its exact probability
# ----------------------------------------------------------------------------------------------
class EnumRng:
    """Replays a fixed path of choices and records how many alternatives each choice had."""

    def __init__(self, path):
        self.path, self.i, self.prob, self.arity = path, 0, 1.0, []

    def _choose(self, probs):
        c = self.path[self.i] if self.i < len(self.path) else 0
        self.i += 1
        self.arity.append(len(probs))
        self.prob *= float(probs[c])
        return c

    def accept(self, log_alpha, pos):
        a = float(np.exp(log_alpha))
        return self._choose([a, 1.0 - a]) == 0

    def categorical(self, logw, pos, tag):
        w = np.exp(np.asarray(logw, dtype=np.float64) - np.max(logw))
        return self._choose(w / w.sum())


def enumerate_outcomes(run):
    """Depth-first walk over every choice path of run(rng) -> outcome; yields (outcome, prob)."""
    path = []
    while True:
        rng = EnumRng(path)
        out = run(rng)
        yield out, rng.prob
        taken = (list(path) + [0] * len(rng.arity))[: len(rng.arity)]
        i = len(taken) - 1
        while i >= 0 and taken[i] + 1 >= rng.arity[i]:
            i -= 1
        if i < 0:
            return
        path = taken[:i] + [taken[i] + 1]


def _logs(p):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(p, dtype=np.float64))


ONE_STEP_CASES = [
    ([0.5, 0.5], [0.5, 0.5]),
    ([0.9, 0.1], [0.2, 0.8]),
    ([0.0, 1.0], [0.5, 0.5]),                    # zero in p
    ([0.2, 0.0, 0.8], [0.1, 0.6, 0.3]),
    ([0.25, 0.25, 0.25, 0.25], [0.7, 0.1, 0.1, 0.1]),
    ([0.05, 0.15, 0.3, 0.1, 0.4], [0.3, 0.3, 0.2, 0.1, 0.1]),
    ([0.3, 0.0, 0.1, 0.0, 0.2, 0.4], [0.1, 0.2, 0.1, 0.3, 0.2, 0.1]),
]


@pytest.mark.parametrize("p,q", ONE_STEP_CASES)
def test_one_step_lemma_exact(p, q):
    p, q = np.array(p), np.array(q)
    law = np.zeros(len(p))
    reject = 0.0

    def run(rng):
        toks, a = O.deer_iteration_tabular([0], 1, lambda pre: _logs(p), lambda pre, i: _logs(q), rng)
        return toks[0], a

    for (tok, a), pr in enumerate_outcomes(run):
        law[tok] += pr
        reject += pr * (a == 0)
    assert np.allclose(law, p, atol=1e-14)
    gamma = np.minimum(p, q).sum()
    assert abs(reject - (1.0 - gamma)) < 1e-14
    if gamma < 1:
        assert np.allclose(O.residual_distribution(_logs(p), _logs(q)), (p - np.minimum(p, q)) / (1 - gamma), atol=1e-14)


def test_one_step_lemma_random_tables():
    g = np.random.default_rng(5)
    for V in (2, 3, 4, 5, 6):
        for _ in range(10):
            p = g.dirichlet(np.ones(V) * 0.7)
            q = g.dirichlet(np.ones(V) * 0.7)
            law = np.zeros(V)

            def run(rng):
                return O.deer_iteration_tabular([0], 1, lambda pre: _logs(p), lambda pre, i: _logs(q), rng)[0][0]

            for tok, pr in enumerate_outcomes(run):
                law[tok] += pr
            assert np.allclose(law, p, atol=1e-13)


def test_alpha_identities():
    assert O.log_alpha(np.log(0.3), np.log(0.6)) == pytest.approx(np.log(0.5))
    assert O.log_alpha(np.log(0.6), np.log(0.3)) == 0.0           # ratio above 1 is clipped
    assert O.log_alpha(-np.inf, np.log(0.3)) == -np.inf          # p(y) = 0: never accepted


# ----------------------------------------------------------------------------------------------
# sequence level: first-order tabular target, per-position tabular drafter
# ----------------------------------------------------------------------------------------------
def test_empty_residual_falls_back_to_the_target_law():
    """gamma = 1 (p <= q everywhere): the residual of Eq. "resample" is empty and the Appendix leaves the draw free; the
    oracle draws from p.  With p = q the branch is unreachable (alpha = 1, every draft accepted, any uniforms); it is
    reached here with an un-normalised q = e^c p > p, where rejections do occur."""
    rng0 = np.random.default_rng(3)
    V, k = 7, 3
    logp = O.log_softmax(rng0.normal(size=(k, V)))
    assert np.array_equal(O.residual_logweights(logp[0], logp[0]), logp[0])
    assert np.allclose(O.residual_distribution(logp[0], logp[0]), np.exp(logp[0]), atol=1e-15)
    for seed in range(50):      # p = q: nothing is ever rejected
        a, c = O.accept_block_sampling(logp, logp, [1, 2, 3], O.CounterRng(seed), 10)
        assert (a, c) == (k, None)
    logq = logp + 0.7           # p < q everywhere: alpha = e^-0.7 and an empty residual
    rejected = 0
    for seed in range(200):
        rng = O.CounterRng(seed)
        a, c = O.accept_block_sampling(logp, logq, [1, 2, 3], rng, 10)
        if a < k:
            rejected += 1
            assert c == O.CounterRng(seed).categorical(logp[a], 10 + a, O.TAG_RESID)   # a draw from p at the rejected position
    assert rejected > 100


def _tables(V, k, seed):
    g = np.random.default_rng(seed)
    P = g.dirichlet(np.ones(V), size=V)            # p(x_t | x_{t-1})
    Q = g.dirichlet(np.ones(V), size=(V, k))       # q_i(. | x_j): depends on the LAST prefix token only
    return P, Q


def _law_of_first_tokens(V, k, n_tok, P, Q, iteration=O.deer_iteration_tabular):
    def run(rng):
        x = [0]
        while len(x) - 1 < n_tok:
            toks, _ = iteration(x, k, lambda pre: _logs(P[pre[-1]]), lambda pre, i: _logs(Q[pre[-1], i - 1]), rng)
            x = x + toks
        return tuple(x[1: 1 + n_tok])

    law = {}
    for out, pr in enumerate_outcomes(run):
        law[out] = law.get(out, 0.0) + pr
    return law


def _target_law(V, n_tok, P):
    law = {}
    for seq in itertools.product(range(V), repeat=n_tok):
        pr, prev = 1.0, 0
        for t in seq:
            pr *= P[prev, t]
            prev = t
        law[seq] = pr
    return law


@pytest.mark.parametrize("V,k", [(2, 2), (2, 3), (3, 2)])
def test_sequence_level_theorem_exact(V, k):
    P, Q = _tables(V, k, 100 + 10 * V + k)
    got = _law_of_first_tokens(V, k, 3, P, Q)
    want = _target_law(V, 3, P)
    assert abs(sum(got.values()) - 1.0) < 1e-12
    for s, pr in want.items():
        assert abs(got.get(s, 0.0) - pr) < 1e-12


def _planted_iteration(kind):
    """The oracle's iteration with one deliberate mistake (planted here, on the CPU)."""

    def it(prefix, k, target_logp, drafter_logq, rng):
        j = len(prefix)
        logq = np.stack([drafter_logq(prefix, i + 1) for i in range(k)])
        yhat = [rng.categorical(logq[i], j + i, O.TAG_DRAFT) for i in range(k)]
        logp = np.stack([target_logp(list(prefix) + yhat[:i]) for i in range(k)])
        out = []
        for i in range(k):
            if rng.accept(O.log_alpha(logp[i, yhat[i]], logq[i, yhat[i]]), j + i):
                out.append(yhat[i])
                continue
            if kind == "resample_from_p":
                out.append(rng.categorical(logp[i], j + i, O.TAG_RESID))
                return out, i
            out.append(rng.categorical(O.residual_logweights(logp[i], logq[i]), j + i, O.TAG_RESID))
            # kind == "continue_after_reject": keep testing later drafts against stale p_i
        return out, k

    return it


@pytest.mark.parametrize("kind", ["continue_after_reject", "resample_from_p"])
def test_enumeration_detects_planted_mistakes(kind):
    V, k = 3, 2
    P, Q = _tables(V, k, 139)
    got = _law_of_first_tokens(V, k, 3, P, Q, iteration=_planted_iteration(kind))
    want = _target_law(V, 3, P)
    assert max(abs(got.get(s, 0.0) - pr) for s, pr in want.items()) > 1e-3


# ----------------------------------------------------------------------------------------------
# T = 0 on the Tiny transformer pair
# ----------------------------------------------------------------------------------------------
def _pair(tiny, tiny_weights, cap=160):
    wt, wd = tiny_weights
    return O.TransformerPair(O.Decoder(tiny["target"], wt), O.Decoder(tiny["drafter"], wd),
                             di.mask_token_id(tiny["target"].vocab), cap)


@pytest.fixture(scope="module")
def greedy_truth(tiny, tiny_weights):
    prompt = di.prompt_ids(tiny["target"].vocab, tiny["prefix"])
    return prompt, O.ar_decode(O.Decoder(tiny["target"], tiny_weights[0]), prompt, 64)


@pytest.mark.parametrize("k", [1, 2, 8])
def test_t0_lossless_own_drafter(tiny, tiny_weights, greedy_truth, k):
    prompt, truth = greedy_truth
    out, accepts = O.deer_decode(_pair(tiny, tiny_weights), prompt, k, 0.0, 64, O.CounterRng(0))
    assert out == truth
    assert all(0 <= a <= k for a in accepts)


def test_t0_lossless_adversarial_and_perfect_drafter(tiny, tiny_weights, greedy_truth):
    prompt, truth = greedy_truth
    V, k = tiny["target"].vocab, 8
    g = np.random.default_rng(7)
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    out = []
    while len(out) < 64:                      # random drafts: almost always a = 0, one token per pass
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=g.integers(0, V, k))
        out += res["committed"]
    assert out[:64] == truth
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    out, n_iter = [], 0
    while len(out) < 64:                      # perfect drafts: a = k every pass, k tokens per pass, no bonus
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=truth[len(out): len(out) + k])
        assert res["accept_len"] == k and len(res["committed"]) == k
        out += res["committed"]
        n_iter += 1
    assert out == truth and n_iter == 8


def test_eos_truncates_commit(tiny, tiny_weights, greedy_truth):
    prompt, truth = greedy_truth
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    eos = truth[2]
    res = O.deer_iteration(pair, 8, 0.0, None, eos_id=eos, draft_override=truth[:8])
    first = truth.index(eos)
    assert res["committed"] == truth[: first + 1]
    assert pair.tc.n == len(prompt) + first + 1 - 1


# ----------------------------------------------------------------------------------------------
# T = 1 on the Tiny pair: closed forms at position 1
# ----------------------------------------------------------------------------------------------
def test_accept_rate_and_first_token_law_match_closed_forms(tiny, tiny_weights):
    prompt = di.prompt_ids(tiny["target"].vocab, 32, seq=2)
    V, k, T, j = tiny["target"].vocab, 8, 1.0, 32
    base = _pair(tiny, tiny_weights)
    base.prefill(prompt)
    zd = base.draft_logits(k)
    logq = O.log_softmax(zd / T)
    # p_1 does not depend on the draft; later p_i do, so they are recomputed per draft below only
    # through the oracle's own accept routine on position 1 (k = 1 slice)
    zt1 = base.verify_logits([0])
    base.tc.truncate(j - 1)
    logp1 = O.log_softmax(zt1[:1] / T)
    gamma1 = np.minimum(np.exp(logp1[0]), np.exp(logq[0])).sum()
    n = 4000
    acc, first = 0, np.zeros(V)
    for s in range(n):
        rng = O.CounterRng(1000 + s)
        y1 = rng.categorical(zd[0] / T, j, O.TAG_DRAFT)
        a, c = O.accept_block_sampling(logp1, logq[:1], [y1], rng, j)
        acc += a
        first[y1 if a == 1 else c] += 1
    assert binomtest(acc, n, gamma1).pvalue > 1e-3
    buckets = (np.arange(V) * 2654435761 % 2**32) % 16
    obs = np.bincount(buckets, weights=first, minlength=16)
    exp = np.bincount(buckets, weights=np.exp(logp1[0]), minlength=16) * n
    assert chisquare(obs, exp).pvalue > 1e-3
