"""GPU parity at T > 0 on the Tiny workload: Gumbel-max drafting, the log-space acceptance test and
the residual resample against the oracle, which implements the same counter-based generator.

Tokens are compared exactly wherever the oracle's decision is not within 1e-3 of a tie (perturbed
top-2 margin of the draft and residual draws, distance of log u from log alpha); the laws are compared
with chi-square / binomial tests at p > 0.01 (accept-length histogram, first committed token against
the exact p_1, P[a >= 1] against gamma_1)."""
import numpy as np
import pytest
from scipy.stats import binomtest, chi2_contingency, chisquare

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]
T = 1.0


@pytest.fixture(scope="module")
def setup():
    import torch
    t, d = CFG["target"], CFG["drafter"]
    wt = StoredWeights(t, di.TARGET_SEED, "bf16")
    wd = StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, max_batch=1, max_seq=256, max_k=8)
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=5)
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    yield eng, pair, prompt, torch
    eng.close()


def _reset(eng, pair, prompt):
    n = len(prompt)
    pair.x = [int(v) for v in prompt]
    pair.tc.truncate(min(pair.tc.n, n - 1))
    pair.dc.truncate(min(pair.dc.n, n))
    eng.set_prefilled([n], [int(prompt[-1])])


def _oracle_iteration(pair, k, seed, zd, rollback=True):
    """The oracle's iteration with the decision slacks needed to know where exact agreement is due."""
    rng = O.CounterRng(seed, 0, np.float64)
    j = len(pair.prefix())
    pert = [zd[i] / T + rng._gumbel(O.TAG_DRAFT, j + i, zd.shape[1]) for i in range(k)]
    yhat = [O.argmax_lowest(p) for p in pert]
    draft_margin = min(float(np.partition(p, -2)[-1] - np.partition(p, -2)[-2]) for p in pert)
    zt = pair.verify_logits(yhat)
    logp, logq = O.log_softmax(zt / T), O.log_softmax(zd / T)
    slack = np.inf
    a, c = k, None
    for i in range(k):
        la = O.log_alpha(logp[i, yhat[i]], logq[i, yhat[i]])
        lu = float(np.log(O.uniforms(O.row_key(seed, O.TAG_ACCEPT, 0, j + i), 0)))
        slack = min(slack, abs(lu - la) if la < 0 else np.inf)
        if not (lu <= la):
            a = i
            w = O.residual_logweights(logp[i], logq[i]) + rng._gumbel(O.TAG_RESID, j + i, zd.shape[1])
            c = O.argmax_lowest(w)
            fin = np.sort(w[np.isfinite(w)])
            slack = min(slack, float(fin[-1] - fin[-2]))
            break
    if rollback:
        pair.tc.truncate(j - 1)
    return dict(draft=yhat, draft_margin=draft_margin, a=a, c=c, slack=slack, zt=zt, logp1=logp[0], logq1=logq[0])


def test_sampling_iteration_matches_oracle_and_laws(setup):
    eng, pair, prompt, torch = setup
    k, V, n = CFG["k"], CFG["target"].vocab, 1200
    _reset(eng, pair, prompt)
    zd = pair.draft_logits(k)
    hist_g, hist_o = np.zeros(k + 1), np.zeros(k + 1)
    first_g = np.zeros(V)
    exact_checked = exact_draft_checked = acc1 = 0
    logp1 = None
    for seed in range(n):
        _reset(eng, pair, prompt)
        ref = _oracle_iteration(pair, k, seed, zd)
        gd = eng.draft_block(k, T, seed).cpu().numpy()[0].tolist()
        if seed == 0:
            assert np.abs(eng.debug_get_logits(1, k)[0] - zd).max() < 2e-3
        if ref["draft_margin"] > 1e-3:
            assert gd == ref["draft"], seed
            exact_draft_checked += 1
        # verify the oracle's draft on the GPU so that both sides judge the same block
        eng.verify_block(k, T, torch.tensor([ref["draft"]], dtype=torch.int32, device="cuda"))
        if seed == 0:
            assert np.abs(eng.debug_get_logits(0, k)[0] - ref["zt"]).max() < 2e-3
        acc, com, ncom = eng.accept_and_commit(k, T, seed)
        want = ref["draft"][: ref["a"]] + ([] if ref["c"] is None else [ref["c"]])
        if ref["slack"] > 1e-3:
            assert acc[0] == ref["a"] and com[0] == want, (seed, acc, com, ref["a"], want)
            exact_checked += 1
        assert ncom[0] == min(acc[0] + 1, k)
        hist_g[acc[0]] += 1
        hist_o[ref["a"]] += 1
        first_g[com[0][0]] += 1
        acc1 += acc[0] >= 1
        logp1, logq1 = ref["logp1"], ref["logq1"]
    assert exact_checked > 0.9 * n and exact_draft_checked > 0.9 * n
    # (i) accept-length histogram, GPU vs oracle, two-sample chi-square over the occupied bins
    keep = (hist_g + hist_o) > 0
    assert chi2_contingency(np.stack([hist_g[keep], hist_o[keep]]) + 1e-9)[1] > 0.01
    # (ii) first committed token against the exact target law p_1, 16 hashed buckets
    buckets = (np.arange(V) * 2654435761 % 2 ** 32) % 16
    obs = np.bincount(buckets, weights=first_g, minlength=16)
    exp = np.bincount(buckets, weights=np.exp(logp1), minlength=16) * n
    assert chisquare(obs, exp).pvalue > 0.01
    # (iii) P[a >= 1] against gamma_1 = sum_v min(p_1, q_1)
    gamma1 = float(np.minimum(np.exp(logp1), np.exp(logq1)).sum())
    assert binomtest(int(acc1), n, gamma1).pvalue > 0.01
    assert hist_g[1:].sum() > 0.5 * n          # real accepts do occur at T = 1 (near-uniform laws overlap)


def test_free_running_sampling_keeps_state_consistent(setup):
    """Run 12 iterations end to end at T = 1 with ragged accepts; the engine's committed text must equal
    what the oracle commits from the same seeds wherever no decision was near a tie."""
    eng, pair, prompt, torch = setup
    k = CFG["k"]
    _reset(eng, pair, prompt)
    for it in range(12):
        seed = 5000 + it
        zd = pair.draft_logits(k)
        ref = _oracle_iteration(pair, k, seed, zd, rollback=False)
        eng.draft_block(k, T, seed)
        eng.verify_block(k, T, torch.tensor([ref["draft"]], dtype=torch.int32, device="cuda"))
        acc, com, ncom = eng.accept_and_commit(k, T, seed)
        want = ref["draft"][: ref["a"]] + ([] if ref["c"] is None else [ref["c"]])
        if ref["slack"] <= 1e-3 or ref["draft_margin"] <= 1e-3:
            break
        assert com[0] == want, (it, com, want)
        pair.commit(want)
        assert eng.get_lengths()[0] == len(pair.prefix())
    assert it >= 3
