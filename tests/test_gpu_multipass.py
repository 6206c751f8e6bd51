"""GPU parity of the multi-pass draft (a block filled in from the left over several drafter passes) on the Tiny
workload against the oracle's draft_block_multipass: tokens, the per-position logits kept for acceptance (each
from the pass that fixed the position), acceptance at T = 1 with those laws, and the drafter cache state."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]
TOL_STORED = 2e-3


@pytest.fixture(scope="module")
def setup():
    import torch
    t, d = CFG["target"], CFG["drafter"]
    wt = StoredWeights(t, di.TARGET_SEED, "bf16")
    wd = StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, max_batch=2, max_seq=256, max_k=8)
    yield eng, wt, wd, torch
    eng.close()


@pytest.mark.parametrize("n_passes", [1, 2, 3, 8])
def test_t0_multipass_lockstep(setup, n_passes):
    """Several iterations with commits of different lengths (so the first pass also ingests 1..k rows)."""
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    prompt = di.prompt_ids(t.vocab, 50, seq=6)
    truth = O.ar_decode(O.Decoder(t, wt.as_f32, np.float64, "bf16"), prompt, 40 + k)
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    out = []
    for a_want in [3, 0, 8, 5]:
        yhat, zd = O.draft_block_multipass(pair, k, 0.0, None, n_passes)
        gd = eng.draft_block_multipass(k, 0.0, 0, n_passes).cpu().numpy()[0]
        gzd = eng.debug_get_logits(1, k)[0]
        assert np.abs(gzd - zd).max() < TOL_STORED
        if top2_margin(zd).min() > 1e-2:
            assert gd.tolist() == yhat
        assert eng.get_lengths()[0] == len(pair.prefix())
        # both sides verify the same injected block so that the commit lengths are the wanted ones
        block = list(truth[len(out): len(out) + k])
        if a_want < k:
            block[a_want] = (block[a_want] + 1) % t.vocab
        zt = pair.verify_logits(block)
        a, c = O.accept_block_greedy([O.argmax_lowest(zt[i]) for i in range(k)], block)
        com_o = block[:a] + ([] if c is None else [c])
        pair.commit(com_o)
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        acc, com, _ = eng.accept_and_commit(k, 0.0, 0)
        assert acc[0] == a == a_want and com[0] == com_o
        out += com_o


def test_sampling_multipass_uses_each_positions_own_law(setup):
    """T = 1, 3 passes: drafts and accept decisions equal the oracle's wherever no decision is within 1e-3 of a
    tie; the residual at a rejected position is formed with the law of the pass that fixed that position."""
    eng, wt, wd, torch = setup
    t, d, k, T, n_passes = CFG["target"], CFG["drafter"], CFG["k"], 1.0, 3
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=5)
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    j, V = len(prompt), t.vocab
    exact = late = 0
    n = 150
    for seed in range(n):
        eng.set_prefilled([j], [int(prompt[-1])])
        rng = O.CounterRng(seed, 0, np.float64)
        yhat, zd = O.draft_block_multipass(pair, k, T, rng, n_passes)
        margin = min(float(np.diff(np.partition(zd[i] / T + rng._gumbel(O.TAG_DRAFT, j + i, V), -2)[-2:])[0]) for i in range(k))
        gd = eng.draft_block_multipass(k, T, seed, n_passes).cpu().numpy()[0].tolist()
        if seed == 0:
            assert np.abs(eng.debug_get_logits(1, k)[0] - zd).max() < TOL_STORED
        if margin <= 1e-3:
            continue                       # a near-tie in a draw changes every later pass: nothing to compare
        assert gd == yhat, seed
        zt = pair.verify_logits(yhat)
        pair.tc.truncate(j - 1)
        logp, logq = O.log_softmax(zt / T), O.log_softmax(zd / T)
        a, c = O.accept_block_sampling(logp, logq, yhat, O.CounterRng(seed, 0, np.float64), j)
        slack = np.inf
        for i in range(min(a + 1, k)):
            la = O.log_alpha(logp[i, yhat[i]], logq[i, yhat[i]])
            lu = float(np.log(O.uniforms(O.row_key(seed, O.TAG_ACCEPT, 0, j + i), 0)))
            slack = min(slack, abs(lu - la) if la < 0 else np.inf)
        if a < k:
            w = O.residual_logweights(logp[a], logq[a]) + rng._gumbel(O.TAG_RESID, j + a, V)
            fin = np.sort(w[np.isfinite(w)])
            slack = min(slack, float(fin[-1] - fin[-2]))
        eng.verify_block(k, T, torch.tensor([yhat], dtype=torch.int32, device="cuda"))
        acc, com, _ = eng.accept_and_commit(k, T, seed)
        if slack > 1e-3:
            assert acc[0] == a and com[0] == yhat[:a] + ([] if c is None else [c]), (seed, acc, com, a, c)
            exact += 1
            late += a >= 3                 # the rejected position was fixed by a later pass than the first
    assert exact > 0.8 * n and late >= 10


def test_multipass_batch_and_argument_errors(setup):
    from paper_2512_15176_amd import DeerError
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    prompts = [di.prompt_ids(t.vocab, 37, seq=1), di.prompt_ids(t.vocab, 70, seq=2)]
    eng.prefill(prompts)
    with pytest.raises(DeerError) as e:
        eng.draft_block_multipass(k, 0.0, 0, 0)
    assert e.value.status == -1
    with pytest.raises(DeerError) as e:
        eng.draft_block_multipass(k, 0.0, 0, k + 1)
    assert e.value.status == -1
    gd = eng.draft_block_multipass(k, 0.0, 0, 2).cpu().numpy()
    gz = eng.debug_get_logits(1, k)
    for b, prompt in enumerate(prompts):
        pair = make_pair(t, d, wt, wd, 256)
        pair.prefill(prompt)
        yhat, zd = O.draft_block_multipass(pair, k, 0.0, None, 2)
        assert np.abs(gz[b] - zd).max() < TOL_STORED
        if top2_margin(zd).min() > 1e-2:
            assert gd[b].tolist() == yhat
    eng.verify_block(k, 0.0, torch.tensor(gd, dtype=torch.int32, device="cuda"))
    eng.accept_and_commit(k, 0.0, 0)
