"""GPU parity for a mixture-of-experts target (softmax router, top-k of E, renormalised weights,
grouped expert GEMMs): a small mixture, and one layer at the 30B-A3B layer widths with all 128 experts."""
import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from gpu_common import StoredWeights, fill_seeded_cache, gpu_available, lockstep_commit, make_engine, make_pair, top2_margin

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CASES = {
    "small_mixture": dict(
        target=di.ModelShape(2, 256, 4, 2, 64, 0, 1024, n_experts=16, top_k=4, d_ff_expert=128, rope_base=1e4),
        drafter=di.CONFIGS["tiny"]["drafter"], prefix=45, k=8, forced=[8, 0, 3], tol=2e-3),
    "a3b_layer_widths": dict(
        target=di.scaled(di.CONFIGS["qwen3_30b_a3b"]["target"], n_layers=1, vocab=4096),
        drafter=di.scaled(di.DRAFTER_05B, n_layers=1, vocab=4096), prefix=70, k=32, forced=[5, 32], tol=2e-2),
}


@pytest.mark.parametrize("name", list(CASES))
def test_moe_lockstep(name):
    import torch
    case = CASES[name]
    t, d, k, n = case["target"], case["drafter"], case["k"], case["prefix"]
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, 1, 256, k)
    dtype = np.float64 if name == "small_mixture" else np.float32
    pair = make_pair(t, d, wt, wd, 256, dtype=dtype)
    prompt = di.prompt_ids(t.vocab, n)
    pair.prefill(prompt)
    eng.prefill([prompt])
    dec = O.Decoder(t, wt.as_f32, dtype, "bf16")
    worst = 0.0
    eng.debug_experts_streamed()      # reset: count the verify passes only
    for a_want in case["forced"]:
        truth = O.ar_decode(dec, pair.prefix(), k)
        block = list(truth)
        if a_want < k:
            block[a_want] = (block[a_want] + 1) % t.vocab
        eng.draft_block(k, 0.0, 0)
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=block)
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k)[0]
        err = float(np.abs(gzt - res["target_logits"]).max())
        worst = max(worst, err)
        assert err < case["tol"], err
        if lockstep_commit(eng, k, [gzt], [res], [block]):
            assert res["accept_len"] == a_want
        assert eng.get_lengths()[0] == len(pair.prefix())
    per_pass = eng.debug_experts_streamed() / (len(case["forced"]) * t.n_layers)
    print(f"\n[{name}] max |target logit error| {worst:.2e}; experts streamed per layer and verify pass: {per_pass:.1f} of {t.n_experts}")
    assert per_pass > t.top_k      # the rows of a block do go to different experts (the grouped path is exercised)
    eng.close()


def test_a3b_twelve_layers_all_experts_full_vocab_prefix_2048():
    """The mixture workload deeper: 12 of the 48 layers at the real widths (d = 2048, 32 q / 4 kv heads, 128 experts of
    width 768, top-8), the full 151936-entry vocabulary, a 2048-token prefix (seeded stand-in cache contents on both
    sides: a real prefill of it on the CPU oracle would take minutes), k = 32, T = 0; two iterations, the second after
    a commit (the drafter ingests, the target cache has grown)."""
    import torch
    cfg = di.CONFIGS["qwen3_30b_a3b"]
    t, d, k, n = di.scaled(cfg["target"], n_layers=12), di.scaled(cfg["drafter"], n_layers=2), cfg["k"], cfg["prefix"]
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, 1, n + 128, k)
    pair = make_pair(t, d, wt, wd, n + 128, dtype=np.float32)
    last = 4242
    pair.x = [0] * (n - 1) + [last]
    fill_seeded_cache(eng, torch, 0, t, 0, n - 1, pair.tc)
    fill_seeded_cache(eng, torch, 1, d, 0, n, pair.dc)
    eng.set_prefilled([n], [last])
    eng.debug_experts_streamed()
    worst_d = worst_t = 0.0
    rng = np.random.default_rng(7)
    for it in range(2):
        gd = eng.draft_block(k, 0.0, 0).cpu().numpy()[0]
        zd = pair.draft_logits(k)
        ed = float(np.abs(eng.debug_get_logits(1, k)[0] - zd).max())
        ok = top2_margin(zd) > 1e-2
        assert np.array_equal(gd[ok], np.argmax(zd, -1)[ok])
        block = [int(v) for v in rng.integers(0, t.vocab, size=k)]
        res = O.deer_iteration(pair, k, 0.0, None, draft_override=block)
        eng.verify_block(k, 0.0, torch.tensor([block], dtype=torch.int32, device="cuda"))
        gzt = eng.debug_get_logits(0, k)[0]
        et = float(np.abs(gzt - res["target_logits"]).max())
        worst_d, worst_t = max(worst_d, ed), max(worst_t, et)
        assert ed < 2e-2 and et < 2e-2, (it, ed, et)
        okt = top2_margin(res["target_logits"]) > 1e-2
        assert np.array_equal(np.argmax(gzt, -1)[okt], np.argmax(res["target_logits"], -1)[okt])
        lockstep_commit(eng, k, [gzt], [res], [block])
        assert eng.get_lengths()[0] == len(pair.prefix())
    per_pass = eng.debug_experts_streamed() / (2 * t.n_layers)
    print(f"\n[30B-A3B widths, 12 layers, 128 experts, full vocab, prefix {n}] max |logit error|: drafter {worst_d:.2e}, "
          f"target {worst_t:.2e}; experts streamed per layer and pass: {per_pass:.1f}")
    eng.close()


def test_uniform_routing_stand_in_spreads_the_rows():
    """The benchmarking aid: with deer_debug_route_spread a block of 32 rows touches about
    n (1 - (1 - top_k / n)^32) experts per layer, whatever the (random-init) router would choose."""
    import torch
    t = di.scaled(di.CONFIGS["qwen3_30b_a3b"]["target"], n_layers=3, vocab=4096)
    d = di.scaled(di.DRAFTER_05B, n_layers=1, vocab=4096)
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, 1, 256, 32)
    eng.prefill([di.prompt_ids(t.vocab, 40)])
    eng.debug_route_spread(True)
    eng.debug_experts_streamed()
    dr = eng.draft_block(32, 0.0, 0)
    eng.verify_block(32, 0.0, dr)
    per_layer = eng.debug_experts_streamed() / t.n_layers
    expected = t.n_experts * (1.0 - (1.0 - t.top_k / t.n_experts) ** 32)
    assert abs(per_layer - expected) < 8, (per_layer, expected)
    acc, com, ncom = eng.accept_and_commit(32, 0.0, 0)
    assert 0 <= acc[0] <= 32 and ncom[0] >= 1
    logits_finite = np.isfinite(eng.debug_get_logits(0, 32)).all()
    assert logits_finite
    eng.close()
