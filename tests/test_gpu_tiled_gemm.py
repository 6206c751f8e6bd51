"""GPU parity of the LDS-tiled GEMM (passes with at least 256 rows): prefill through it against the oracle and
against the weight-streaming kernels, at Tiny widths (ragged row and column blocks) and at 8B layer widths."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, gpu_available, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]


def _logits_after_prefill(eng, prompt, k, torch):
    eng.prefill([prompt])
    dr = eng.draft_block(k, 0.0, 0)
    zd = eng.debug_get_logits(1, k)[0]
    eng.verify_block(k, 0.0, dr)
    zt = eng.debug_get_logits(0, k)[0]
    eng.accept_and_commit(k, 0.0, 0)
    return zd, zt, dr.cpu().numpy()[0]


@pytest.mark.parametrize("n_prompt", [256, 300, 700])
def test_tiny_prefill_through_tiled_gemm(n_prompt):
    """300 = 9 row tiles + 12 rows (a ragged second row block); 700 spans three row blocks."""
    import torch
    cfg = di.CONFIGS["tiny"]
    t, d, k = cfg["target"], cfg["drafter"], cfg["k"]
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, 1, 1024, k)
    prompt = di.prompt_ids(t.vocab, n_prompt, seq=9)
    eng.debug_gemm_tiled(0)
    zd0, zt0, _ = _logits_after_prefill(eng, prompt, k, torch)
    eng.debug_gemm_tiled(1)
    zd1, zt1, dr1 = _logits_after_prefill(eng, prompt, k, torch)
    assert np.abs(zd0 - zd1).max() < 2e-3 and np.abs(zt0 - zt1).max() < 2e-3
    pair = make_pair(t, d, wt, wd, 1024)
    pair.prefill(prompt)
    zd = pair.draft_logits(k)
    assert np.abs(zd1 - zd).max() < 2e-3
    zt = pair.verify_logits([int(v) for v in dr1])
    assert np.abs(zt1 - zt).max() < 2e-3
    eng.close()


def test_8b_layer_widths_prefill_through_tiled_gemm():
    import torch
    t = di.scaled(di.CONFIGS["qwen3_8b"]["target"], n_layers=2, vocab=16384)
    d = di.scaled(di.DRAFTER_05B, n_layers=2, vocab=16384)      # d = 896: an odd number of column groups
    k, n = 32, 613
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, 1, 1024, k)
    eng.debug_gemm_tiled(1)
    prompt = di.prompt_ids(t.vocab, n)
    zd1, zt1, dr1 = _logits_after_prefill(eng, prompt, k, torch)
    pair = make_pair(t, d, wt, wd, 1024, dtype=np.float32)
    pair.prefill(prompt)
    zd = pair.draft_logits(k)
    ed = float(np.abs(zd1 - zd).max())
    zt = pair.verify_logits([int(v) for v in dr1])
    et = float(np.abs(zt1 - zt).max())
    print(f"\n[tiled prefill, 8B layer widths] max |logit error|: drafter {ed:.2e}, target {et:.2e}")
    assert ed < 2e-2 and et < 2e-2
    eng.close()


def test_batch_of_64_sequences_through_tiled_gemm():
    """64 sequences make 2048-row verify passes and 4096-row draft passes (ingest + MASK tiles, LM head on every
    second tile): every GEMM of both passes, the LM heads included, runs through the tiled kernel."""
    import torch
    cfg = di.CONFIGS["tiny"]
    t, d, k, B = cfg["target"], cfg["drafter"], cfg["k"], 64
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, B, 128, k)
    eng.debug_gemm_tiled(1)
    prompts = [di.prompt_ids(t.vocab, 20 + (7 * b) % 41, seq=100 + b) for b in range(B)]
    eng.prefill(prompts)
    g = np.random.default_rng(4)
    check = [0, 1, 17, 40, 63]
    pairs = {}
    for b in check:
        pairs[b] = make_pair(t, d, wt, wd, 128)
        pairs[b].prefill(prompts[b])
    for it in range(2):                                  # the second iteration ingests the first one's commits
        dr = eng.draft_block(k, 0.0, 0)
        gzd = eng.debug_get_logits(1, k)
        blocks = g.integers(0, t.vocab, (B, k)).astype(np.int32)
        for b in check:                                  # forced accepted lengths 0..k on the checked sequences
            truth = O.ar_decode(O.Decoder(t, wt.as_f32, np.float64, "bf16"), pairs[b].prefix(), k)
            a_want = (b + 3 * it) % (k + 1)
            blocks[b] = truth
            if a_want < k:
                blocks[b, a_want] = (truth[a_want] + 1) % t.vocab
        eng.verify_block(k, 0.0, torch.tensor(blocks, device="cuda"))
        gzt = eng.debug_get_logits(0, k)
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        for b in check:
            res = O.deer_iteration(pairs[b], k, 0.0, None, draft_override=[int(v) for v in blocks[b]])
            assert np.abs(gzd[b] - res["draft_logits"]).max() < 2e-3, (it, b)
            assert np.abs(gzt[b] - res["target_logits"]).max() < 2e-3, (it, b)
            assert acc[b] == res["accept_len"] and com[b] == res["committed"], (it, b)
    eng.close()
