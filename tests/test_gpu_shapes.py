"""GPU parity at the real layer widths (8B-, 4B- and drafter-shaped layers, 2 layers each so the
fp32 oracle finishes in seconds): prefixes that span several 32-row tiles with a ragged tail, block
sizes 32 and 16, forced accepted lengths so the drafter ingests 1, k and a middling number of rows; the
bonus-token variant at k = 31 (32 target rows, up to 32 committed tokens).

Lock-step protocol: the device's logits say what its acceptance kernel must decide.  Where that equals the
oracle's commit the acceptance call runs and is compared exactly; where the two differ, the first differing row
must have an oracle top-2 margin below 1e-2 (the only legitimate cause), and the acceptance call is replaced by a
forced commit of the oracle's tokens (deer_debug_force_commit) so that the comparison goes on from a common state."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, lockstep_commit, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

TOL = 2e-2   # logits, max abs (the stated bar); observed errors are far smaller and are printed


CASES = {
    "8b_layers": dict(target=di.scaled(di.CONFIGS["qwen3_8b"]["target"], n_layers=2, vocab=16384),
                      drafter=di.scaled(di.DRAFTER_05B, n_layers=2, vocab=16384), prefix=203, k=32,
                      forced=[0, 32, 7]),
    "4b_layers_full_vocab": dict(target=di.scaled(di.CONFIGS["qwen3_4b"]["target"], n_layers=2),
                                 drafter=di.scaled(di.DRAFTER_05B, n_layers=1), prefix=613, k=16,   # two prefill chunks: 512 + 101 rows
                                 forced=[16, 3]),
}
CASES["8b_layers_bonus"] = dict(CASES["8b_layers"], k=31, forced=[31, 0, 9, 31], bonus=True)


@pytest.mark.parametrize("name", list(CASES))
def test_lockstep_at_real_widths(name):
    import torch
    case = CASES[name]
    t, d, k, n = case["target"], case["drafter"], case["k"], case["prefix"]
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    bonus = bool(case.get("bonus"))
    eng = make_engine(t, d, wt, wd, 1, 1024, k)
    eng.set_bonus_token(bonus)
    pair = make_pair(t, d, wt, wd, 1024, dtype=np.float32)
    prompt = di.prompt_ids(t.vocab, n)
    pair.prefill(prompt)
    eng.prefill([prompt])
    dec = O.Decoder(t, wt.as_f32, np.float32, "bf16")
    worst_d = worst_t = 0.0
    exact = 0
    for a_want in case["forced"]:
        truth = O.ar_decode(dec, pair.prefix(), k)
        block = list(truth)
        n_want = a_want + 1 if (bonus or a_want < k) else k
        if a_want < k:
            block[a_want] = (block[a_want] + 1) % t.vocab
        gd = eng.draft_block(k, 0.0, 0).cpu().numpy()[0]
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=block, bonus=bonus)
        zd = res["draft_logits"]
        ed = float(np.abs(eng.debug_get_logits(1, k)[0] - zd).max())
        ok = top2_margin(zd) > 1e-2
        assert np.array_equal(gd[ok], np.argmax(zd, -1)[ok])
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k + bonus)[0]
        et = float(np.abs(gzt - res["target_logits"]).max())
        worst_d, worst_t = max(worst_d, ed), max(worst_t, et)
        assert ed < TOL and et < TOL, (ed, et)
        if lockstep_commit(eng, k, [gzt], [res], [block], bonus):
            assert res["accept_len"] == a_want and len(res["committed"]) == n_want
            exact += 1
        assert eng.get_lengths()[0] == len(pair.prefix())
    print(f"\n[{name}] max |logit error|: drafter {worst_d:.2e}, target {worst_t:.2e}; exact commits {exact}/{len(case['forced'])}")
    assert exact >= len(case["forced"]) - 1
    eng.close()


def test_two_sequences_at_8b_widths():
    """Two sequences (two 32-row tiles per pass) at the 8B layer widths: the launches in which row tiles get
    workgroups of their own (QKV, O) and those that take them in pairs (gate/up, down) against the oracle."""
    import torch
    case = CASES["8b_layers"]
    t, d, k = case["target"], case["drafter"], 32
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, 2, 512, k)
    lens = [203, 77]
    prompts = [di.prompt_ids(t.vocab, n, seq=40 + b) for b, n in enumerate(lens)]
    pairs = [make_pair(t, d, wt, wd, 512, dtype=np.float32) for _ in lens]
    for p, pr in zip(pairs, prompts):
        p.prefill(pr)
    eng.prefill(prompts)
    dec = O.Decoder(t, wt.as_f32, np.float32, "bf16")
    exact = 0
    for it, wants in enumerate([[5, 32], [0, 17]]):
        blocks = []
        for b, pair in enumerate(pairs):
            truth = O.ar_decode(dec, pair.prefix(), k)
            blk = list(truth)
            if wants[b] < k:
                blk[wants[b]] = (blk[wants[b]] + 1) % t.vocab
            blocks.append(blk)
        eng.draft_block(k, 0.0, 0)
        gzd = eng.debug_get_logits(1, k)
        eng.verify_block(k, 0.0, torch.tensor(blocks, dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k)
        results = [O.deer_iteration(pair, k, 0.0, None, draft_override=blocks[b]) for b, pair in enumerate(pairs)]
        for b, res in enumerate(results):
            ed = float(np.abs(gzd[b] - res["draft_logits"]).max())
            et = float(np.abs(gzt[b] - res["target_logits"]).max())
            assert ed < TOL and et < TOL, (it, b, ed, et)
        if lockstep_commit(eng, k, gzt, results, blocks):
            assert [res["accept_len"] for res in results] == wants
            exact += 1
        assert eng.get_lengths().tolist() == [len(p.prefix()) for p in pairs]
    assert exact >= 1
    eng.close()
