"""GPU parity on the Tiny workload (2-layer target, 1-layer drafter, d=128, vocab 1024, prefix 64,
k=8): every call of the C ABI against the oracle, element by element."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]
TOL_STORED = 2e-3     # oracle given the same stored bf16 weights and a bf16 cache
TOL_NORTH_STAR = 2e-2  # logits, bf16 path vs the fp32-weight oracle


@pytest.fixture(scope="module")
def setup():
    import torch
    t, d = CFG["target"], CFG["drafter"]
    wt = StoredWeights(t, di.TARGET_SEED, "bf16")
    wd = StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, max_batch=1, max_seq=256, max_k=8)
    yield eng, wt, wd, torch
    eng.close()


def test_prefill_draft_verify_logits_and_tokens(setup):
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    prompt = di.prompt_ids(t.vocab, CFG["prefix"])
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    # draft
    zd = pair.draft_logits(k)
    pair.dc.truncate(len(prompt))
    draft = eng.draft_block(k, 0.0, 0)
    gzd = eng.debug_get_logits(1, k)[0]
    assert np.abs(gzd - zd).max() < TOL_STORED
    ok = top2_margin(zd) > 1e-2
    gd = draft.cpu().numpy()[0]
    assert np.array_equal(gd[ok], np.argmax(zd, -1)[ok])
    # verify the oracle's own draft on both sides
    yhat = [O.argmax_lowest(zd[i]) for i in range(k)]
    zt = pair.verify_logits(yhat)
    eng.verify_block(k, 0.0, torch.tensor([yhat], dtype=torch.int32, device="cuda"))
    gzt = eng.debug_get_logits(0, k)[0]
    assert np.abs(gzt - zt).max() < TOL_STORED
    a, c = O.accept_block_greedy([O.argmax_lowest(zt[i]) for i in range(k)], yhat)
    acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
    if top2_margin(zt)[: a + 1].min() > 1e-2:
        assert acc[0] == a
        assert com[0] == yhat[:a] + ([] if c is None else [c])


def test_north_star_tolerance_against_fp32_weight_oracle(setup):
    """The workload states fp32 weights; the library stores bf16.  Logits within 2e-2."""
    eng, _, _, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    wt32 = StoredWeights(t, di.TARGET_SEED, "f32")
    wd32 = StoredWeights(d, di.DRAFTER_SEED, "f32")
    eng32 = make_engine(t, d, wt32, wd32, 1, 256, 8)
    prompt = di.prompt_ids(t.vocab, CFG["prefix"])
    pair = make_pair(t, d, wt32, wd32, 256, kv_storage=None)
    pair.prefill(prompt)
    eng32.prefill([prompt])
    zd = pair.draft_logits(k)
    eng32.draft_block(k, 0.0, 0)
    assert np.abs(eng32.debug_get_logits(1, k)[0] - zd).max() < TOL_NORTH_STAR
    yhat = [O.argmax_lowest(zd[i]) for i in range(k)]
    zt = pair.verify_logits(yhat)
    eng32.verify_block(k, 0.0, torch.tensor([yhat], dtype=torch.int32, device="cuda"))
    assert np.abs(eng32.debug_get_logits(0, k)[0] - zt).max() < TOL_NORTH_STAR
    eng32.close()


def test_t0_lockstep_64_tokens_forced_accept_lengths(setup):
    """Generate 64 tokens; each iteration injects the target's own greedy continuation corrupted at
    a chosen position, so every accepted length 0..k occurs; states must stay identical."""
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=1)
    truth = O.ar_decode(O.Decoder(t, wt.as_f32, np.float64, "bf16"), prompt, 64 + k)
    pair = make_pair(t, d, wt, wd, 256)
    pair.prefill(prompt)
    eng.prefill([prompt])
    out, it = [], 0
    wanted = [0, 8, 3, 1, 8, 5, 2, 7, 4, 6, 0, 8, 8, 1]
    while len(out) < 64:
        a_want = wanted[it % len(wanted)]
        block = list(truth[len(out): len(out) + k])
        if a_want < k:
            block[a_want] = (block[a_want] + 1) % t.vocab
        gdraft = eng.draft_block(k, 0.0, 0)          # the drafter still runs (ingests the last commit)
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=block)
        assert np.abs(eng.debug_get_logits(1, k)[0] - res["draft_logits"]).max() < TOL_STORED
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        assert np.abs(eng.debug_get_logits(0, k)[0] - res["target_logits"]).max() < TOL_STORED
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        assert res["accept_len"] == a_want
        assert acc[0] == a_want and com[0] == res["committed"], (it, acc, com, res["committed"])
        out += com[0]
        it += 1
        assert eng.get_lengths()[0] == len(pair.prefix())
    assert out[:64] == truth[:64]


def test_t0_free_running_equals_greedy_ar(setup):
    """Losslessness end to end on the GPU: its own drafts, its own accepts; output = greedy decoding."""
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    prompt = di.prompt_ids(t.vocab, CFG["prefix"], seq=2)
    dec = O.Decoder(t, wt.as_f32, np.float64, "bf16")
    truth = O.ar_decode(dec, prompt, 40)
    eng.prefill([prompt])
    out = []
    while len(out) < 40:
        dr = eng.draft_block(k, 0.0, 0)
        eng.verify_block(k, 0.0, dr)
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        assert 0 <= acc[0] <= k and ncom[0] == min(acc[0] + 1, k)
        out += com[0]
    # token for token; a difference is tolerated only where the oracle's top-2 margin is below 1e-2
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


def test_call_order_and_argument_errors(setup):
    from paper_2512_15176_amd import DeerError
    eng, _, _, torch = setup
    prompt = di.prompt_ids(CFG["target"].vocab, 16)
    eng.prefill([prompt])
    buf = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(DeerError) as e:
        eng.verify_block(8, 0.0, buf)
    assert e.value.status == -2
    with pytest.raises(DeerError) as e:
        eng.accept_and_commit(8, 0.0, 0)
    assert e.value.status == -2
    with pytest.raises(DeerError) as e:
        eng.draft_block(9, 0.0, 0)          # k > max_k
    assert e.value.status == -1
    with pytest.raises(DeerError) as e:
        eng.draft_block(8, -1.0, 0)
    assert e.value.status == -1
    dr = eng.draft_block(8, 0.0, 0)
    with pytest.raises(DeerError) as e:
        eng.draft_block(8, 0.0, 0)
    assert e.value.status == -2
    with pytest.raises(DeerError) as e:
        eng.verify_block(4, 0.0, dr)        # k differs from the draft call
    assert e.value.status == -1
    eng.verify_block(8, 0.0, dr)
    eng.accept_and_commit(8, 0.0, 0)
    with pytest.raises(DeerError) as e:
        eng.prefill([di.prompt_ids(CFG["target"].vocab, 250)])   # 250 + 8 > max_seq 256
    assert e.value.status == -3


def test_recomputing_both_caches_every_iteration_gives_the_same_text(setup):
    """The setting of the paper's batch experiment (no KV cache kept between iterations): a prefill of every
    committed token before each iteration must lead to the same logits and commits as the kept caches."""
    eng, wt, wd, torch = setup
    t, k = CFG["target"], CFG["k"]
    prompt = [int(v) for v in di.prompt_ids(t.vocab, 45, seq=4)]

    def run(recompute):
        text, logs = list(prompt), []
        eng.prefill([text])
        for _ in range(6):
            if recompute:
                eng.prefill([text])
            dr = eng.draft_block(k, 0.0, 0)
            zd = eng.debug_get_logits(1, k)[0]
            eng.verify_block(k, 0.0, dr)
            zt = eng.debug_get_logits(0, k)[0]
            acc, com, _ = eng.accept_and_commit(k, 0.0, 0)
            logs.append((zd, zt, int(acc[0]), com[0]))
            text += com[0]
        return logs

    kept, redone = run(False), run(True)
    for it, ((zd0, zt0, a0, c0), (zd1, zt1, a1, c1)) in enumerate(zip(kept, redone)):
        assert np.abs(zd0 - zd1).max() < TOL_STORED and np.abs(zt0 - zt1).max() < TOL_STORED, it
        if (a0, c0) != (a1, c1):     # only a near-tie may decide differently; the texts part ways there
            assert min(top2_margin(zt0).min(), top2_margin(zd0).min()) < 1e-2, (it, a0, c0, a1, c1)
            break
    assert it >= 2


def test_gemm_stamps_are_ordered(setup):
    """deer_debug_gemm_stamps: every workgroup of the chosen launch records start <= multiplied <= stored, and in
    a split launch exactly one workgroup per column group records the finish."""
    eng, wt, wd, torch = setup
    k = CFG["k"]
    from paper_2512_15176_amd import binding
    eng.prefill([di.prompt_ids(CFG["target"].vocab, 40, seq=3)])
    for launch in (0, 1, 3):                      # QKV, O and down projection of the target's first layer
        eng.debug_gemm_stamps(binding.DEER_TARGET, launch)
        dr = eng.draft_block(k, 0.0, 0)
        eng.verify_block(k, 0.0, dr)
        eng.accept_and_commit(k, 0.0, 0)
        st = eng.debug_gemm_stamps(binding.DEER_TARGET, -1)
        assert st is not None and st.shape[1] == 8
        st = st[: st.shape[0] // 2]                 # the chosen launch (the second half holds the launch after it)
        st = st[st[:, 0] > 0]                       # rows of the workgroups that ran
        assert st.shape[0] >= 1
        assert (st[:, 0] > 0).all() and (st[:, 1] >= st[:, 0]).all() and (st[:, 2] >= st[:, 1]).all()
        split = (st[:, 3] > 0).any()
        if split:
            assert (st[:, 3] >= st[:, 2]).all() and 1 <= (st[:, 4] > 0).sum() <= st.shape[0]
    assert eng.debug_gemm_stamps(binding.DEER_TARGET, -1) is None      # recording is off again
