"""GPU parity of the bonus-token variant (k drafts verified by k+1 target rows; after k accepted drafts one
more target token is committed) on the Tiny workload, against the oracle's variant of the same name."""
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
    eng = make_engine(t, d, wt, wd, max_batch=1, max_seq=256, max_k=32)
    eng.set_bonus_token(True)
    yield eng, wt, wd, torch
    eng.close()


def test_t0_lockstep_forced_accept_lengths_with_bonus(setup):
    """Every accepted length 0..k occurs; a == k commits k+1 tokens; logits of all k+1 target rows match."""
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=1)
    truth = O.ar_decode(O.Decoder(t, wt.as_f32, np.float64, "bf16"), prompt, 80 + k)
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    out, it, full = [], 0, 0
    wanted = [8, 0, 8, 3, 1, 8, 5, 2, 7, 4, 6, 0, 8, 8, 1]
    while len(out) < 72:
        a_want = wanted[it % len(wanted)]
        block = list(truth[len(out): len(out) + k])
        if a_want < k:
            block[a_want] = (block[a_want] + 1) % t.vocab
        eng.draft_block(k, 0.0, 0)
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=block, bonus=True)
        assert np.abs(eng.debug_get_logits(1, k)[0] - res["draft_logits"]).max() < TOL_STORED
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k + 1)[0]
        assert res["target_logits"].shape[0] == k + 1
        assert np.abs(gzt - res["target_logits"]).max() < TOL_STORED
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        assert res["accept_len"] == a_want
        assert acc[0] == a_want and com[0] == res["committed"], (it, acc, com, res["committed"])
        assert ncom[0] == a_want + 1
        full += a_want == k
        out += com[0]
        it += 1
        assert eng.get_lengths()[0] == len(pair.prefix())
    assert out[:72] == truth[:72] and full >= 3


def test_t0_free_running_with_bonus_equals_greedy_ar(setup):
    eng, wt, wd, torch = setup
    t, k = CFG["target"], CFG["k"]
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=2)
    dec = O.Decoder(t, wt.as_f32, np.float64, "bf16")
    truth = O.ar_decode(dec, prompt, 40)
    eng.prefill([prompt])
    out = []
    while len(out) < 40:
        dr = eng.draft_block(k, 0.0, 0)
        eng.verify_block(k, 0.0, dr)
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        assert 0 <= acc[0] <= k and ncom[0] == acc[0] + 1
        out += com[0]
    cache = O.KVCache(t, 256, np.float64)
    x = list(prompt)
    z = dec.forward(x, np.arange(len(x)), cache, O.causal_mask(len(x)), len(x), logits_rows=[len(x) - 1])[0]
    compared = 0
    for i in range(40):
        if out[i] != truth[i]:
            assert top2_margin(z[None])[0] < 1e-2, (i, out[i], truth[i])
            break
        compared += 1
        z = dec.forward([truth[i]], [len(x)], cache, O.causal_mask(1), 1)[0]
        x.append(truth[i])
    assert compared >= 20


def _oracle_sampling_iteration(pair, k, seed, zd, T):
    """The oracle's bonus-variant iteration, with the decision slacks that say where exact agreement is due."""
    rng = O.CounterRng(seed, 0, np.float64)
    j = len(pair.prefix())
    V = zd.shape[1]
    pert = [zd[i] / T + rng._gumbel(O.TAG_DRAFT, j + i, V) for i in range(k)]
    yhat = [O.argmax_lowest(p) for p in pert]
    zt = pair.verify_logits(yhat, bonus=True)
    logp, logq = O.log_softmax(zt / T), O.log_softmax(zd / T)
    a, c = O.accept_block_sampling(logp, logq, yhat, O.CounterRng(seed, 0, np.float64), j, bonus=True)
    slack = np.inf
    for i in range(min(a + 1, k)):
        la = O.log_alpha(logp[i, yhat[i]], logq[i, yhat[i]])
        lu = float(np.log(O.uniforms(O.row_key(seed, O.TAG_ACCEPT, 0, j + i), 0)))
        slack = min(slack, abs(lu - la) if la < 0 else np.inf)
    w = (O.residual_logweights(logp[a], logq[a]) if a < k else logp[k]) + rng._gumbel(O.TAG_RESID, j + a, V)
    assert O.argmax_lowest(w) == c
    fin = np.sort(w[np.isfinite(w)])
    slack = min(slack, float(fin[-1] - fin[-2]))
    pair.tc.truncate(j - 1)
    return dict(draft=yhat, a=a, c=c, slack=slack, zt=zt)


def test_sampling_with_bonus_matches_oracle(setup):
    eng, wt, wd, torch = setup
    t, d, k, T = CFG["target"], CFG["drafter"], CFG["k"], 1.0
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=5)
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    zd = pair.draft_logits(k)
    n, exact, full = 400, 0, 0
    for seed in range(n):
        eng.set_prefilled([len(prompt)], [int(prompt[-1])])
        ref = _oracle_sampling_iteration(pair, k, seed, zd, T)
        eng.draft_block(k, T, seed)
        eng.verify_block(k, T, torch.tensor([ref["draft"]], dtype=torch.int32, device="cuda"))
        if seed == 0:
            assert np.abs(eng.debug_get_logits(0, k + 1)[0] - ref["zt"]).max() < TOL_STORED
        acc, com, ncom = eng.accept_and_commit(k, T, seed)
        assert ncom[0] == acc[0] + 1
        if ref["slack"] > 1e-3:
            assert acc[0] == ref["a"] and com[0] == ref["draft"][: ref["a"]] + [ref["c"]], (seed, acc, com, ref["a"], ref["c"])
            exact += 1
            full += ref["a"] == k
    assert exact > 0.9 * n
    assert full >= 20          # k acceptances followed by the extra draw do occur (near-uniform laws overlap)


def test_bonus_argument_and_state_errors(setup):
    from paper_2512_15176_amd import DeerError
    eng, _, _, torch = setup
    eng.prefill([di.prompt_ids(CFG["target"].vocab, 16)])
    with pytest.raises(DeerError) as e:
        eng.draft_block(32, 0.0, 0)          # 33 rows do not fit one tile
    assert e.value.status == -1
    dr = eng.draft_block(31, 0.0, 0)
    with pytest.raises(DeerError) as e:
        eng.set_bonus_token(False)           # not inside an iteration
    assert e.value.status == -2
    eng.verify_block(31, 0.0, dr)
    acc, com, ncom = eng.accept_and_commit(31, 0.0, 0)
    assert ncom[0] == acc[0] + 1
    eng.set_bonus_token(False)
    dr = eng.draft_block(32, 0.0, 0)
    eng.verify_block(32, 0.0, dr)
    acc, com, ncom = eng.accept_and_commit(32, 0.0, 0)
    assert ncom[0] == min(acc[0] + 1, 32)
    eng.set_bonus_token(True)
