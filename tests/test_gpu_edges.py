"""GPU edge cases on the Tiny workload, against the oracle: a one-token prompt (empty target cache), block size 1
(an autoregressive step), EOS inside a block (cut commit, finished sequence stays finished, also beside a live
sequence in a batch), and a sequence that runs up to the cache capacity."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]
TOL = 2e-3


@pytest.fixture(scope="module")
def weights():
    t, d = CFG["target"], CFG["drafter"]
    return StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")


def _lockstep(eng, pair, k, blocks, torch, eos=-1):
    """Runs the given injected blocks on both sides; returns the committed tokens of both."""
    got, want = [], []
    for block in blocks:
        eng.draft_block(k, 0.0, 0)
        res = O.deer_iteration(pair, k, 0.0, None, eos_id=eos, draft_override=block)
        assert np.abs(eng.debug_get_logits(1, k)[0] - res["draft_logits"]).max() < TOL
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        assert np.abs(eng.debug_get_logits(0, k)[0] - res["target_logits"]).max() < TOL
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        assert acc[0] == res["accept_len"] and com[0] == res["committed"], (acc, com, res["accept_len"], res["committed"])
        got += com[0]
        want += res["committed"]
        assert eng.get_lengths()[0] == len(pair.prefix())
    return got, want


def test_one_token_prompt_and_block_size_one(weights):
    import torch
    t, d = CFG["target"], CFG["drafter"]
    wt, wd = weights
    eng = make_engine(t, d, wt, wd, 1, 128, 8)
    prompt = [int(di.prompt_ids(t.vocab, 4, seq=11)[2])]
    truth = O.ar_decode(O.Decoder(t, wt.as_f32, np.float64, "bf16"), prompt, 24)
    pair = make_pair(t, d, wt, wd, 128)
    pair.prefill(prompt)
    eng.prefill([prompt])          # the target cache stays empty: x_1 is the pending token
    assert eng.get_lengths()[0] == 1
    # k = 1: every iteration is one autoregressive step of the target (a wrong draft is replaced by its token)
    got, want = _lockstep(eng, pair, 1, [[(truth[i] + 1) % t.vocab] for i in range(4)], torch)
    assert got == want == truth[:4]
    # then blocks of 8 with accepted lengths 8 and 2
    blk = list(truth[4:12])
    blk2 = list(truth[12:20])
    blk2[2] = (blk2[2] + 1) % t.vocab
    got, want = _lockstep(eng, pair, 8, [blk, blk2], torch)
    assert got == want == truth[4:15]
    eng.close()


def test_eos_cuts_the_commit_and_finishes_the_sequence(weights):
    import torch
    t, d, k = CFG["target"], CFG["drafter"], 8
    wt, wd = weights
    dec = O.Decoder(t, wt.as_f32, np.float64, "bf16")
    for seq in range(12, 40):                            # a continuation whose token k+3 has not occurred before
        prompt = di.prompt_ids(t.vocab, 30, seq=seq)
        truth = O.ar_decode(dec, prompt, 3 * k)
        if truth[k + 3] not in truth[: k + 3]:
            break
    eos = truth[k + 3]                                   # appears inside the second block
    assert eos not in truth[: k + 3]
    eng = make_engine(t, d, wt, wd, 2, 128, k, eos=eos)
    pair = make_pair(t, d, wt, wd, 128)
    pair.prefill(prompt)
    other = di.prompt_ids(t.vocab, 21, seq=13)           # a second, live sequence beside it
    eng.prefill([prompt, other])
    for it in range(3):
        block = list(truth[it * k: (it + 1) * k])
        dr = eng.draft_block(k, 0.0, 0).clone()
        dr[0] = torch.tensor(block, dtype=torch.int32, device="cuda")
        eng.verify_block(k, 0.0, dr)
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        if it == 0:
            res = O.deer_iteration(pair, k, 0.0, None, eos_id=eos, draft_override=block)
            assert com[0] == res["committed"] == truth[:k]
        elif it == 1:
            res = O.deer_iteration(pair, k, 0.0, None, eos_id=eos, draft_override=block)
            assert com[0] == res["committed"] == truth[k: k + 4] and com[0][-1] == eos   # cut at EOS
        else:
            assert ncom[0] == 0 and com[0] == []             # finished: nothing more is committed
        assert ncom[1] >= 1                                  # the other sequence keeps going
    assert eng.get_lengths()[0] == len(prompt) + k + 4
    eng.close()


def test_sequence_runs_up_to_the_cache_capacity(weights):
    import torch
    from paper_2512_15176_amd import DeerError
    t, d, k = CFG["target"], CFG["drafter"], 8
    wt, wd = weights
    eng = make_engine(t, d, wt, wd, 1, 64, k)            # max_seq 64
    prompt = di.prompt_ids(t.vocab, 40, seq=14)
    truth = O.ar_decode(O.Decoder(t, wt.as_f32, np.float64, "bf16"), prompt, 24)
    pair = make_pair(t, d, wt, wd, 64 + k)
    pair.prefill(prompt)
    eng.prefill([prompt])
    got, want = _lockstep(eng, pair, k, [list(truth[0:8]), list(truth[8:16])], torch)     # length 40 -> 56
    assert got == want == truth[:16]
    assert eng.get_lengths()[0] == 56                    # 56 + 8 = 64: one more block fits exactly
    blk = list(truth[16:24])
    blk[1] = (blk[1] + 1) % t.vocab
    got, want = _lockstep(eng, pair, k, [blk], torch)
    assert got == want == truth[16:18]
    with pytest.raises(DeerError) as e:                  # 58 + 8 > 64
        eng.draft_block(k, 0.0, 0)
    assert e.value.status == -3
    got, want = _lockstep(eng, pair, 4, [list(truth[18:22])], torch)   # a shorter block still fits (58 + 4 <= 64)
    assert got == want == truth[18:22]
    eng.close()
