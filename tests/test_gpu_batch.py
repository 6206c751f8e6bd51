"""GPU parity with several sequences decoded together: ragged prompt lengths, ragged accepted lengths
with per-sequence rollback, per-sequence random streams, and caches filled with seeded stand-in
contents (the mechanism used for 32k-token prefixes, where a real prefill is too costly)."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]
TOL = 2e-3


@pytest.fixture(scope="module")
def setup():
    import torch
    t, d = CFG["target"], CFG["drafter"]
    wt = StoredWeights(t, di.TARGET_SEED, "bf16")
    wd = StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, max_batch=4, max_seq=256, max_k=8)
    yield eng, wt, wd, torch
    eng.close()


def test_ragged_batch_t0_lockstep(setup):
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    lens = [40, 64, 17, 33]
    prompts = [di.prompt_ids(t.vocab, n, seq=10 + b) for b, n in enumerate(lens)]
    pairs = [make_pair(t, d, wt, wd, 256) for _ in lens]
    for p, pr in zip(pairs, prompts):
        p.prefill(pr)
    eng.prefill(prompts)
    dec = O.Decoder(t, wt.as_f32, np.float64, "bf16")
    wanted = [[0, 8, 3, 5], [8, 1, 8, 0], [2, 2, 7, 8], [5, 0, 1, 8], [8, 8, 4, 6]]
    for a_want in wanted:
        blocks, refs = [], []
        eng.draft_block(k, 0.0, 0)
        gzd = eng.debug_get_logits(1, k)
        for b, pair in enumerate(pairs):
            truth = O.ar_decode(dec, pair.prefix(), k)
            blk = list(truth)
            if a_want[b] < k:
                blk[a_want[b]] = (blk[a_want[b]] + 1) % t.vocab
            blocks.append(blk)
            refs.append(O.deer_iteration(pair, k, 0.0, None, draft_override=blk))
            assert np.abs(gzd[b] - refs[b]["draft_logits"]).max() < TOL
        eng.verify_block(k, 0.0, torch.tensor(blocks, dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k)
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        for b in range(len(pairs)):
            assert np.abs(gzt[b] - refs[b]["target_logits"]).max() < TOL
            assert acc[b] == a_want[b] == refs[b]["accept_len"]
            assert com[b] == refs[b]["committed"]
        assert eng.get_lengths().tolist() == [len(p.prefix()) for p in pairs]


def test_batch_sampling_uses_per_sequence_streams(setup):
    eng, wt, wd, torch = setup
    t, d, k, T = CFG["target"], CFG["drafter"], CFG["k"], 1.0
    lens = [24, 50, 31]
    prompts = [di.prompt_ids(t.vocab, n, seq=20 + b) for b, n in enumerate(lens)]
    pairs = [make_pair(t, d, wt, wd, 256) for _ in lens]
    for p, pr in zip(pairs, prompts):
        p.prefill(pr)
    eng.prefill(prompts)
    checked = 0
    for it in range(6):
        seed = 900 + it
        gd = eng.draft_block(k, T, seed).cpu().numpy()
        gzd = eng.debug_get_logits(1, k)
        drafts, infos = [], []
        for b, pair in enumerate(pairs):
            rng = O.CounterRng(seed, b)
            j = len(pair.prefix())
            zd = pair.draft_logits(k)
            assert np.abs(gzd[b] - zd).max() < TOL
            pert = [zd[i] / T + rng._gumbel(O.TAG_DRAFT, j + i, t.vocab) for i in range(k)]
            y = [O.argmax_lowest(p) for p in pert]
            if min(top2_margin(np.stack(pert))) > 1e-3:
                assert gd[b].tolist() == y
            drafts.append(y)
            infos.append((rng, j, zd))
        eng.verify_block(k, T, torch.tensor(drafts, dtype=torch.int32, device="cuda"))
        acc, com, ncom = eng.accept_and_commit(k, T, seed)
        ok = True
        for b, pair in enumerate(pairs):
            rng, j, zd = infos[b]
            zt = pair.verify_logits(drafts[b])
            logp, logq = O.log_softmax(zt / T), O.log_softmax(zd / T)
            a, c = O.accept_block_sampling(logp, logq, drafts[b], rng, j)
            want = drafts[b][:a] + ([] if c is None else [c])
            if com[b] != want:
                ok = False      # a decision within rounding of a tie: stop comparing this run
                break
            pair.commit(want)
            checked += 1
        if not ok:
            break
    assert checked >= 9
    # ragged accepts did occur and the two sides agree on every length
    assert eng.get_lengths().tolist()[: len(pairs)] == [len(p.prefix()) for p in pairs] or not ok


def _fill_engine_cache(eng, torch, model, shape, lens):
    for l in range(shape.n_layers):
        for b, n in enumerate(lens):
            kb = torch.from_numpy(di.kv_fill_bits(shape, "k", l, b, n).view(np.int16)).cuda()
            vb = torch.from_numpy(di.kv_fill_bits(shape, "v", l, b, n).view(np.int16)).cuda()
            eng.debug_load_kv(model, l, b, 0, kb, vb)
    torch.cuda.synchronize()


def test_seeded_cache_contents_and_set_prefilled(setup):
    eng, wt, wd, torch = setup
    t, d, k = CFG["target"], CFG["drafter"], CFG["k"]
    lens = [130, 77]
    last = [5, 900]
    _fill_engine_cache(eng, torch, 0, t, [n - 1 for n in lens])
    _fill_engine_cache(eng, torch, 1, d, lens)
    eng.set_prefilled(lens, last)
    pairs = []
    for b, n in enumerate(lens):
        pair = make_pair(t, d, wt, wd, 256)
        pair.x = [0] * (n - 1) + [last[b]]
        for l in range(t.n_layers):
            pair.tc.K[l, : n - 1] = di.bf16_bits_to_f32(di.kv_fill_bits(t, "k", l, b, n - 1))
            pair.tc.V[l, : n - 1] = di.bf16_bits_to_f32(di.kv_fill_bits(t, "v", l, b, n - 1))
        for l in range(d.n_layers):
            pair.dc.K[l, :n] = di.bf16_bits_to_f32(di.kv_fill_bits(d, "k", l, b, n))
            pair.dc.V[l, :n] = di.bf16_bits_to_f32(di.kv_fill_bits(d, "v", l, b, n))
        pair.tc.n, pair.dc.n = n - 1, n
        pairs.append(pair)
    for it in range(2):
        gd = eng.draft_block(k, 0.0, 0).cpu().numpy()
        gzd = eng.debug_get_logits(1, k)
        drafts = []
        for b, pair in enumerate(pairs):
            zd = pair.draft_logits(k)
            assert np.abs(gzd[b] - zd).max() < TOL
            drafts.append([O.argmax_lowest(zd[i]) for i in range(k)])
        eng.verify_block(k, 0.0, torch.tensor(drafts, dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k)
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        for b, pair in enumerate(pairs):
            zt = pair.verify_logits(drafts[b])
            assert np.abs(gzt[b] - zt).max() < TOL
            a, c = O.accept_block_greedy([O.argmax_lowest(zt[i]) for i in range(k)], drafts[b])
            want = drafts[b][:a] + ([] if c is None else [c])
            if top2_margin(zt)[: a + 1].min() > 1e-2:
                assert acc[b] == a and com[b] == want
            pair.commit(com[b])
