"""Pins for the oracle's two transformers and cache handling.

 * whole-model forward against an independent library implementation (a randomly initialised
   Llama-architecture decoder and a Mixtral-architecture mixture decoder from `transformers`,
   weights copied in) - fails on a transposed projection, wrong RoPE pairing, wrong GQA head
   mapping, a missing residual, wrong expert weighting;
 * k=1 verify == ordinary autoregressive step; one k-row block-causal pass == k sequential
   steps; state after ragged commits == fresh prefill of the committed text;
 * GQA and mixture-of-experts reductions; RoPE shift invariance of a whole forward."""
import dataclasses

import numpy as np
import pytest

import deer_inputs as di
from oracle import deer_oracle as O
from conftest import SeededWeights

SMALL = di.ModelShape(2, 32, 4, 2, 8, 48, 64, rope_base=10000.0)
SMALL_MOE = di.ModelShape(2, 32, 4, 2, 8, 0, 64, n_experts=8, top_k=2, d_ff_expert=16, rope_base=10000.0)


def scaled_weights(shape, seed, gain=12.0):
    """N(0,0.02) weights scaled up so that attention and routing are far from uniform."""
    base = SeededWeights(shape, seed)
    return lambda name, layer=-1, expert=-1: base(name, layer, expert) * gain


def _hf_llama(shape, w):
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    cfg = tf.LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ff,
                         num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                         num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
                         rope_theta=shape.rope_base, tie_word_embeddings=False, attention_bias=False,
                         mlp_bias=False, max_position_embeddings=512)
    m = tf.LlamaForCausalLM(cfg).double().eval()
    sd = m.state_dict()
    T = lambda a: torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.float64).T))
    sd["model.embed_tokens.weight"].copy_(torch.from_numpy(np.asarray(w("embed"), dtype=np.float64)))
    sd["lm_head.weight"].copy_(T(w("lm_head")))
    sd["model.norm.weight"].fill_(1.0)
    for l in range(shape.n_layers):
        p = f"model.layers.{l}."
        for ours, theirs in (("wq", "self_attn.q_proj"), ("wk", "self_attn.k_proj"), ("wv", "self_attn.v_proj"),
                             ("wo", "self_attn.o_proj"), ("wg", "mlp.gate_proj"), ("wu", "mlp.up_proj"),
                             ("wd", "mlp.down_proj")):
            sd[p + theirs + ".weight"].copy_(T(w(ours, l)))
        sd[p + "input_layernorm.weight"].fill_(1.0)
        sd[p + "post_attention_layernorm.weight"].fill_(1.0)
    return m, torch


def test_dense_forward_matches_library_llama():
    w = scaled_weights(SMALL, 11)
    m, torch = _hf_llama(SMALL, w)
    ids = di.prompt_ids(SMALL.vocab, 13, seq=1)
    dec = O.Decoder(SMALL, w)
    cache = O.KVCache(SMALL, 32, np.float64)
    z = dec.forward(ids, np.arange(13), cache, O.causal_mask(13), 13)
    with torch.no_grad():
        ref = m(torch.from_numpy(ids.astype(np.int64))[None]).logits[0].numpy()
    assert np.abs(ref).max() > 0.5          # the comparison is not vacuous
    assert np.allclose(z, ref, atol=5e-6)   # the library evaluates RoPE angles in fp32
    # continuing from the cache (3 more rows, causal) equals the library's full pass on 16 tokens
    more = di.prompt_ids(SMALL.vocab, 3, seq=2)
    z2 = dec.forward(more, np.arange(13, 16), cache, O.causal_mask(3), 3)
    with torch.no_grad():
        ref2 = m(torch.from_numpy(np.concatenate([ids, more]).astype(np.int64))[None]).logits[0].numpy()
    assert np.allclose(z2, ref2[13:], atol=5e-6)


def test_moe_forward_matches_library_mixtral():
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    s = SMALL_MOE
    w = scaled_weights(s, 12, gain=20.0)
    cfg = tf.MixtralConfig(vocab_size=s.vocab, hidden_size=s.d_model, intermediate_size=s.d_ff_expert,
                           num_hidden_layers=s.n_layers, num_attention_heads=s.n_q_heads,
                           num_key_value_heads=s.n_kv_heads, head_dim=s.head_dim, num_local_experts=s.n_experts,
                           num_experts_per_tok=s.top_k, rms_norm_eps=s.rms_eps, rope_theta=s.rope_base,
                           tie_word_embeddings=False, sliding_window=None, max_position_embeddings=512,
                           experts_implementation="eager")
    m = tf.MixtralForCausalLM(cfg).double().eval()
    sd = m.state_dict()
    T = lambda a: torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.float64).T))
    sd["model.embed_tokens.weight"].copy_(torch.from_numpy(np.asarray(w("embed"), dtype=np.float64)))
    sd["lm_head.weight"].copy_(T(w("lm_head")))
    sd["model.norm.weight"].fill_(1.0)
    for l in range(s.n_layers):
        p = f"model.layers.{l}."
        for ours, theirs in (("wq", "self_attn.q_proj"), ("wk", "self_attn.k_proj"), ("wv", "self_attn.v_proj"),
                             ("wo", "self_attn.o_proj")):
            sd[p + theirs + ".weight"].copy_(T(w(ours, l)))
        sd[p + "input_layernorm.weight"].fill_(1.0)
        sd[p + "post_attention_layernorm.weight"].fill_(1.0)
        sd[p + "mlp.gate.weight"].copy_(T(w("router", l)))
        gu = sd[p + "mlp.experts.gate_up_proj"]
        dn = sd[p + "mlp.experts.down_proj"]
        assert tuple(gu.shape) == (s.n_experts, 2 * s.d_ff_expert, s.d_model)
        for e in range(s.n_experts):
            gu[e, : s.d_ff_expert].copy_(T(w("wg", l, e)))
            gu[e, s.d_ff_expert:].copy_(T(w("wu", l, e)))
            dn[e].copy_(T(w("wd", l, e)))
    ids = di.prompt_ids(s.vocab, 11, seq=3)
    z = O.Decoder(s, w).forward(ids, np.arange(11), O.KVCache(s, 16, np.float64), O.causal_mask(11), 11)
    with torch.no_grad():
        ref = m(torch.from_numpy(ids.astype(np.int64))[None]).logits[0].numpy()
    assert np.abs(ref).max() > 0.5
    assert np.allclose(z, ref, atol=5e-6)


def test_moe_reduces_to_dense_when_experts_are_identical():
    s = SMALL_MOE
    dense = dataclasses.replace(s, n_experts=0, top_k=0, d_ff=s.d_ff_expert, d_ff_expert=0)
    base = scaled_weights(s, 13)

    def w_moe(name, layer=-1, expert=-1):
        return base(name, layer, 0 if expert >= 0 else -1)     # every expert = expert 0

    def w_dense(name, layer=-1, expert=-1):
        return base(name, layer, 0 if name in ("wg", "wu", "wd") else -1)

    ids = di.prompt_ids(s.vocab, 9, seq=4)
    z1 = O.Decoder(s, w_moe).forward(ids, np.arange(9), O.KVCache(s, 9, np.float64), O.causal_mask(9), 9)
    z2 = O.Decoder(dense, w_dense).forward(ids, np.arange(9), O.KVCache(dense, 9, np.float64), O.causal_mask(9), 9)
    assert np.allclose(z1, z2, atol=1e-12)


def test_gqa_equals_mha_with_replicated_kv_weights():
    s = SMALL
    mha = dataclasses.replace(s, n_kv_heads=s.n_q_heads)
    base = scaled_weights(s, 14)
    g = s.n_q_heads // s.n_kv_heads

    def w_mha(name, layer=-1, expert=-1):
        w = base(name, layer, expert)
        if name in ("wk", "wv"):
            w = w.reshape(s.d_model, s.n_kv_heads, s.head_dim)
            w = np.repeat(w, g, axis=1).reshape(s.d_model, -1)   # q head h <- kv head h // g
        return w

    ids = di.prompt_ids(s.vocab, 10, seq=5)
    z1 = O.Decoder(s, base).forward(ids, np.arange(10), O.KVCache(s, 10, np.float64), O.causal_mask(10), 10)
    z2 = O.Decoder(mha, w_mha).forward(ids, np.arange(10), O.KVCache(mha, 10, np.float64), O.causal_mask(10), 10)
    assert np.allclose(z1, z2, atol=1e-12)


def test_forward_invariant_under_constant_position_shift():
    w = scaled_weights(SMALL, 15)
    ids = di.prompt_ids(SMALL.vocab, 8, seq=6)
    dec = O.Decoder(SMALL, w)
    z0 = dec.forward(ids, np.arange(8), O.KVCache(SMALL, 8, np.float64), O.causal_mask(8), 8)
    z1 = dec.forward(ids, np.arange(8) + 1000, O.KVCache(SMALL, 8, np.float64), O.causal_mask(8), 8)
    assert np.allclose(z0, z1, atol=1e-9)


def _pair(tiny, tiny_weights, cap=160, kv_storage=None):
    wt, wd = tiny_weights
    return O.TransformerPair(O.Decoder(tiny["target"], wt, kv_storage=kv_storage), O.Decoder(tiny["drafter"], wd, kv_storage=kv_storage),
                             di.mask_token_id(tiny["target"].vocab), cap)


# The three properties below hold for a cache kept in the compute precision and, unchanged, for a cache that stores
# bf16 rows - provided a pass rounds its new K,V rows BEFORE it attends to them, so that a row is seen with the same
# value by its own pass and by every later one (rounding only at the cache write would break the block-verify and
# k = 1 identities: the in-pass rows would be unrounded, the cached ones rounded).
KV_STORAGES = [None, "bf16"]


def _is_bf16(x):
    return np.array_equal(O.round_to_bf16(x), x)


@pytest.mark.parametrize("kv_storage", KV_STORAGES)
def test_k1_verify_is_an_ordinary_ar_step(tiny, tiny_weights, kv_storage):
    prompt = di.prompt_ids(tiny["target"].vocab, 20)
    pair = _pair(tiny, tiny_weights, kv_storage=kv_storage)
    pair.prefill(prompt)
    z = pair.verify_logits([5])          # k = 1: the single row is the pending token x_j
    dec = O.Decoder(tiny["target"], tiny_weights[0], kv_storage=kv_storage)
    cache = O.KVCache(tiny["target"], 32, np.float64)
    ref = dec.forward(prompt, np.arange(20), cache, O.causal_mask(20), 20)   # plain full causal pass
    assert np.allclose(z[0], ref[-1], atol=1e-12)
    assert np.allclose(pair.tc.K[:, :20], cache.K[:, :20], atol=1e-13)
    assert np.allclose(pair.tc.V[:, :20], cache.V[:, :20], atol=1e-13)
    assert _is_bf16(pair.tc.K[:, :20]) == (kv_storage == "bf16") and _is_bf16(pair.tc.V[:, :20]) == (kv_storage == "bf16")


def test_bf16_cache_storage_changes_the_logits_measurably(tiny, tiny_weights):
    """The storage branch is not a no-op: the same pass with rounded rows differs from the unrounded one by about
    the rounding step of the rows (2^-9 relative), far above the 1e-12 of the identities above."""
    prompt = di.prompt_ids(tiny["target"].vocab, 20)
    zs = []
    for kv_storage in KV_STORAGES:
        pair = _pair(tiny, tiny_weights, kv_storage=kv_storage)
        pair.prefill(prompt)
        zs.append(pair.verify_logits([5, 6, 7]))
    diff = np.abs(zs[0] - zs[1]).max()
    assert 1e-7 < diff < 1e-2


@pytest.mark.parametrize("kv_storage", KV_STORAGES)
def test_block_verify_equals_sequential_steps(tiny, tiny_weights, kv_storage):
    prompt = di.prompt_ids(tiny["target"].vocab, 24)
    yhat = [int(t) for t in di.prompt_ids(tiny["target"].vocab, 8, seq=9)]
    pair = _pair(tiny, tiny_weights, kv_storage=kv_storage)
    pair.prefill(prompt)
    zb = pair.verify_logits(yhat)
    dec = O.Decoder(tiny["target"], tiny_weights[0], kv_storage=kv_storage)
    cache = O.KVCache(tiny["target"], 64, np.float64)
    dec.forward(prompt[:-1], np.arange(23), cache, O.causal_mask(23), 23, logits_rows=[])
    rows = [int(prompt[-1])] + yhat[:-1]
    for i, t in enumerate(rows):          # p_i = p_AR(. | x_{1:j}, y^_{1:i-1}) one step at a time
        zi = dec.forward([t], [23 + i], cache, O.causal_mask(1), 1)[0]
        assert np.allclose(zb[i], zi, atol=1e-12)


class _RoundsAtCacheWriteOnly(O.Decoder):
    """A planted mistake: rows are stored as bf16 but the pass that produces them attends to the unrounded values."""

    def forward(self, ids, pos, cache, allowed_new, keep, logits_rows=None):
        n_old = cache.n
        z = super().forward(ids, pos, cache, allowed_new, keep, logits_rows)
        cache.K[:, n_old:cache.n] = O.round_to_bf16(cache.K[:, n_old:cache.n])
        cache.V[:, n_old:cache.n] = O.round_to_bf16(cache.V[:, n_old:cache.n])
        return z


def test_block_verify_identity_rejects_rounding_at_cache_write_only(tiny, tiny_weights):
    prompt = di.prompt_ids(tiny["target"].vocab, 24)
    yhat = [int(t) for t in di.prompt_ids(tiny["target"].vocab, 8, seq=9)]
    dec = _RoundsAtCacheWriteOnly(tiny["target"], tiny_weights[0])
    block_cache, step_cache = O.KVCache(tiny["target"], 64, np.float64), O.KVCache(tiny["target"], 64, np.float64)
    for c in (block_cache, step_cache):
        dec.forward(prompt[:-1], np.arange(23), c, O.causal_mask(23), 23, logits_rows=[])
    rows = [int(prompt[-1])] + yhat[:-1]
    zb = dec.forward(rows, np.arange(23, 31), block_cache, O.causal_mask(8), 8)
    worst = 0.0
    for i, t in enumerate(rows):
        zi = dec.forward([t], [23 + i], step_cache, O.causal_mask(1), 1)[0]
        worst = max(worst, float(np.abs(zb[i] - zi).max()))
    assert worst > 1e-7      # one k-row pass is no longer k single steps


@pytest.mark.parametrize("kv_storage", KV_STORAGES)
def test_state_after_ragged_commits_equals_fresh_prefill(tiny, tiny_weights, kv_storage):
    V = tiny["target"].vocab
    prompt = di.prompt_ids(V, 16)
    pair = _pair(tiny, tiny_weights, kv_storage=kv_storage)
    pair.prefill(prompt)
    rng = O.CounterRng(4)
    dec_t = O.Decoder(tiny["target"], tiny_weights[0], kv_storage=kv_storage)
    forced = [0, 3, 8, 1, 5]             # accepted lengths to force at T=0 via injected drafts
    for it, a_want in enumerate(forced):
        truth = O.ar_decode(dec_t, pair.prefix(), 8)        # the target's own greedy continuation
        block = list(truth)
        if a_want < 8:
            block[a_want] = (block[a_want] + 1) % V          # corrupt position a_want
        res = O.deer_iteration(pair, 8, 0.0, rng, draft_override=block)
        assert res["accept_len"] == a_want
        assert res["committed"] == truth[: min(a_want + 1, 8)]
    fresh = _pair(tiny, tiny_weights, kv_storage=kv_storage)
    fresh.prefill(pair.prefix())
    n = len(pair.prefix())
    assert pair.tc.n == fresh.tc.n == n - 1
    assert np.allclose(pair.tc.K[:, : n - 1], fresh.tc.K[:, : n - 1], atol=1e-12)
    assert np.allclose(pair.tc.V[:, : n - 1], fresh.tc.V[:, : n - 1], atol=1e-12)
    # the drafter has not yet ingested the last commit; its next draft must equal the fresh one
    za, zb = pair.draft_logits(8), fresh.draft_logits(8)
    assert np.allclose(za, zb, atol=1e-12)
    assert pair.dc.n == fresh.dc.n == n
    assert np.allclose(pair.dc.K[:, :n], fresh.dc.K[:, :n], atol=1e-12)
    yb = [1, 2, 3, 4, 5, 6, 7, 8]
    assert np.allclose(pair.verify_logits(yb), fresh.verify_logits(yb), atol=1e-12)


def test_drafter_marginals_do_not_depend_on_sampled_tokens(tiny, tiny_weights):
    prompt = di.prompt_ids(tiny["target"].vocab, 12)
    outs = []
    for seed in (1, 2):
        pair = _pair(tiny, tiny_weights)
        pair.prefill(prompt)
        outs.append(O.deer_iteration(pair, 8, 1.0, O.CounterRng(seed)))
    assert outs[0]["draft"] != outs[1]["draft"]                       # different samples ...
    assert np.array_equal(outs[0]["draft_logits"], outs[1]["draft_logits"])   # ... same q_i
    # MASK rows are bidirectional: q_1 changes with the block size (it sees more MASK rows)
    pair = _pair(tiny, tiny_weights)
    pair.prefill(prompt)
    z8 = pair.draft_logits(8)
    pair2 = _pair(tiny, tiny_weights)
    pair2.prefill(prompt)
    z4 = pair2.draft_logits(4)
    assert np.abs(z8[0] - z4[0]).max() > 1e-6
