"""GPU regression test of the sampling acceptance kernel when every draft of a block is accepted (T > 0, no bonus
token) in a batch large enough that the kernel's workgroups cannot all be resident at once.

Iteration 1: the oracle picks, position by position, the draft y^_i = argmax_v (log p_i(v) - log q_i(v)); then
p_i(y^_i) >= q_i(y^_i), alpha_i = 1 (Sec. 3.2, Eq. "accept") and all k drafts are accepted whatever the uniforms
are.  Iterations 2 and 3 are ordinary sampled iterations: accepted lengths and residual tokens must equal the
oracle's wherever no decision is within 1e-3 of a tie.  (A kernel in which one workgroup commits while others of
the same sequence have not yet read the sequence's length fails the later iterations: they find a stale arrival
count.)"""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]
T = 1.0
B = 32


def _always_accepted_block(pair, k, zd):
    """Drafts with alpha_i = 1 for every i: chosen left to right, since p_i depends on the earlier drafts."""
    j = len(pair.prefix())
    logq = O.log_softmax(zd / T)
    yhat = []
    for i in range(k):
        zt = pair.verify_logits(yhat + [0] * (k - i))   # block-causal: row i depends on the drafts before it only
        pair.tc.truncate(j - 1)
        yhat.append(O.argmax_lowest(O.log_softmax(zt[i] / T) - logq[i]))
    return yhat


def _sampled_iteration(pair, k, seed, seq, zd):
    """The oracle's sampled iteration with the slack of every decision it took."""
    rng = O.CounterRng(seed, seq, np.float64)
    j = len(pair.prefix())
    V = zd.shape[1]
    pert = [zd[i] / T + rng._gumbel(O.TAG_DRAFT, j + i, V) for i in range(k)]
    yhat = [O.argmax_lowest(p) for p in pert]
    margin = min(float(np.partition(p, -2)[-1] - np.partition(p, -2)[-2]) for p in pert)
    zt = pair.verify_logits(yhat)
    logp, logq = O.log_softmax(zt / T), O.log_softmax(zd / T)
    slack, a, c = np.inf, k, None
    for i in range(k):
        la = O.log_alpha(logp[i, yhat[i]], logq[i, yhat[i]])
        lu = float(np.log(O.uniforms(O.row_key(seed, O.TAG_ACCEPT, seq, j + i), 0)))
        slack = min(slack, abs(lu - la) if la < 0 else np.inf)
        if not (lu <= la):
            a = i
            w = O.residual_logweights(logp[i], logq[i]) + rng._gumbel(O.TAG_RESID, j + i, V)
            c = O.argmax_lowest(w)
            fin = np.sort(w[np.isfinite(w)])
            slack = min(slack, float(fin[-1] - fin[-2]))
            break
    return dict(draft=yhat, margin=margin, a=a, c=c, slack=slack)


def test_all_accepted_blocks_then_sampled_iterations_batch_32():
    import torch
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    wt = StoredWeights(t, di.TARGET_SEED, "bf16")
    wd = StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, max_batch=B, max_seq=256, max_k=k)
    prompts = [di.prompt_ids(t.vocab, 40 + (7 * b) % 23, seq=100 + b) for b in range(B)]
    pairs = []
    for b in range(B):
        p = make_pair(t, d, wt, wd, 256)
        p.prefill(prompts[b])
        pairs.append(p)
    eng.prefill(prompts)

    # iteration 1: every draft accepted in every sequence
    blocks = [_always_accepted_block(pairs[b], k, pairs[b].draft_logits(k)) for b in range(B)]
    eng.draft_block(k, T, 11)
    eng.verify_block(k, T, torch.tensor(blocks, dtype=torch.int32, device="cuda"))
    acc, com, ncom = eng.accept_and_commit(k, T, 11)
    assert acc.tolist() == [k] * B and ncom.tolist() == [k] * B
    assert com == blocks
    for b in range(B):
        pairs[b].verify_logits(blocks[b])    # the target cache takes the block's rows, as on the device
        pairs[b].commit(blocks[b])

    # iterations 2 and 3: ordinary sampled iterations from the state iteration 1 left
    checked = 0
    alive = [True] * B
    for it, seed in enumerate((12, 13)):
        refs = []
        for b in range(B):
            refs.append(_sampled_iteration(pairs[b], k, seed, b, pairs[b].draft_logits(k)))
        gd = eng.draft_block(k, T, seed).cpu().numpy()
        for b in range(B):
            if alive[b] and refs[b]["margin"] > 1e-3:
                assert gd[b].tolist() == refs[b]["draft"], (it, b)
        eng.verify_block(k, T, torch.tensor([r["draft"] for r in refs], dtype=torch.int32, device="cuda"))
        acc, com, ncom = eng.accept_and_commit(k, T, seed)
        for b in range(B):
            r = refs[b]
            want = r["draft"][: r["a"]] + ([] if r["c"] is None else [r["c"]])
            if alive[b] and r["slack"] > 1e-3:
                assert acc[b] == r["a"] and com[b] == want, (it, b, acc[b], com[b], r["a"], want)
                checked += 1
            elif com[b] != want:
                alive[b] = False      # a near-tie went the other way: this sequence's texts differ from here on
            pairs[b].commit(want)
        assert eng.get_lengths().tolist() == [len(p.prefix()) if alive[b] else eng.get_lengths()[b] for b, p in enumerate(pairs)]
    assert checked >= 2 * B - 8
    eng.close()
