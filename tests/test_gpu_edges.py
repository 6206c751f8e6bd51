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


def test_finished_sequence_beside_a_sampling_one(weights):
    """T > 0 with one sequence already ended by EOS: it commits nothing more and keeps its length, while the live
    sequence's acceptance tests and residual draws (its own generator stream, sequence index 1) follow the oracle."""
    import torch
    t, d, k, T = CFG["target"], CFG["drafter"], 8, 1.0
    wt, wd = weights
    dec = O.Decoder(t, wt.as_f32, np.float64, "bf16")
    prompt = di.prompt_ids(t.vocab, 30, seq=12)
    truth = O.ar_decode(dec, prompt, k)
    eos = truth[2]
    if eos in truth[:2]:
        pytest.skip("the chosen continuation repeats its third token")
    eng = make_engine(t, d, wt, wd, 2, 128, k, eos=eos)
    other = di.prompt_ids(t.vocab, 21, seq=13)
    live = make_pair(t, d, wt, wd, 128)
    live.prefill(other)
    eng.prefill([prompt, other])
    # one greedy iteration: sequence 0 accepts its own continuation and is cut at the EOS token
    dr = eng.draft_block(k, 0.0, 0).clone()
    dr[0] = torch.tensor(truth[:k], dtype=torch.int32, device="cuda")
    eng.verify_block(k, 0.0, dr)
    acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
    assert com[0] == truth[:3] and ncom[1] >= 1
    live.draft_logits(k)                                  # the oracle's caches take the same rows as the engine's
    live.verify_logits(dr[1].tolist())
    live.commit(com[1])
    len0 = int(eng.get_lengths()[0])
    checked = 0
    for it in range(4):
        seed = 700 + it
        eng.draft_block(k, T, seed)
        rng = O.CounterRng(seed, 1)
        j = len(live.prefix())
        zd = live.draft_logits(k)
        pert = [zd[i] / T + rng._gumbel(O.TAG_DRAFT, j + i, t.vocab) for i in range(k)]
        y = [O.argmax_lowest(p) for p in pert]
        eng.verify_block(k, T, torch.tensor([[0] * k, y], dtype=torch.int32, device="cuda"))
        acc, com, ncom = eng.accept_and_commit(k, T, seed)
        assert ncom[0] == 0 and com[0] == [] and int(eng.get_lengths()[0]) == len0
        zt = live.verify_logits(y)
        a, c = O.accept_block_sampling(O.log_softmax(zt / T), O.log_softmax(zd / T), y, rng, j)
        want = y[:a] + ([] if c is None else [c])
        if eos in want:
            want = want[: want.index(eos) + 1]
        if com[1] != want:
            break           # a decision within rounding of a tie: the texts part here
        live.commit(want)
        checked += 1
        if eos in want:
            break
    assert checked >= 2
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


def test_read_rate_probe_runs_and_checks_its_arguments(weights):
    """deer_debug_stream_read: a measurement aid that reads a caller's buffer; it must time something, refuse sizes
    and alignments its kernel does not handle, and refuse to run while launch timing uses the same events."""
    import torch
    from paper_2512_15176_amd import DeerError
    t, d = CFG["target"], CFG["drafter"]
    wt, wd = weights
    eng = make_engine(t, d, wt, wd, 1, 64, 4)
    buf = torch.ones(8 << 20, dtype=torch.uint8, device="cuda")
    for nt in (0, 1):
        ms = eng.debug_stream_read(buf, 8 << 20, 256, nt, 3)
        assert 0.0 < ms < 50.0
    assert eng.debug_stream_read(buf, 16, 1, 0, 1) > 0.0            # one vector, ragged against the grid
    with pytest.raises(DeerError):
        eng.debug_stream_read(buf, (8 << 20) - 8, 256, 0, 3)        # not a multiple of 16
    with pytest.raises(DeerError):
        eng.debug_stream_read(buf[8:], 1 << 20, 256, 0, 3)          # not 16-byte aligned
    with pytest.raises(ValueError):
        eng.debug_stream_read(buf, (8 << 20) + 16, 256, 0, 3)       # beyond the tensor
    with pytest.raises(DeerError):
        eng.debug_stream_read(buf, 1 << 20, 0, 0, 3)
    eng.debug_profile(True)
    with pytest.raises(DeerError):
        eng.debug_stream_read(buf, 1 << 20, 256, 0, 3)
    eng.debug_profile(False)
    eng.close()
