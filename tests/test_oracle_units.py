"""Pins for the oracle's elementary routines against closed forms and library routines.

Each check is chosen so that a plausible slip (dropped term, wrong sign, transposed operand,
wrong head mapping) fails it.  None of them re-types the oracle's own formula."""
import numpy as np
import pytest
import scipy.special as sp

import deer_inputs as di
from oracle import deer_oracle as O


def test_log_softmax_matches_scipy():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(5, 37)) * 7
    assert np.allclose(O.log_softmax(z), sp.log_softmax(z, axis=-1), atol=1e-13)
    assert np.allclose(O.softmax(z).sum(-1), 1.0, atol=1e-14)
    big = np.array([[1e4, 1e4 - 1.0, -1e4]])
    assert np.allclose(O.log_softmax(big), sp.log_softmax(big, axis=-1), atol=1e-12)


def test_silu_matches_expit_form():
    x = np.linspace(-20, 20, 401)
    assert np.allclose(O.silu(x), x * sp.expit(x), atol=1e-14)
    assert O.silu(np.array([0.0]))[0] == 0.0


def test_rmsnorm_closed_forms():
    # a constant vector normalises to +-1 (up to eps); scaling the input leaves the output unchanged
    x = np.full((1, 16), -3.0)
    assert np.allclose(O.rmsnorm(x, np.ones(16), 0.0), -1.0)
    rng = np.random.default_rng(1)
    v = rng.normal(size=(4, 64))
    g = rng.normal(size=64)
    y = O.rmsnorm(v, g, 0.0)
    assert np.allclose(O.rmsnorm(7.5 * v, g, 0.0), y)
    assert np.allclose(np.sqrt(np.mean((y / g) ** 2, axis=-1)), 1.0)
    # eps enters under the root, added to the mean square: x = (2,2), eps = 5 -> 2/sqrt(4+5)
    assert np.allclose(O.rmsnorm(np.array([[2.0, 2.0]]), np.ones(2), 5.0), 2.0 / 3.0)


def test_argmax_ties_lowest_index():
    assert O.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0, 3.0])) == 1
    assert O.argmax_lowest(np.array([5.0, 5.0])) == 0


def test_rope_is_a_rotation_by_pos_times_theta():
    # head_dim 2: a single pair (0,1), theta_0 = 1: (1,0) at position p -> (cos p, sin p)
    x = np.array([[[1.0, 0.0]]])
    for p in (0, 1, 5):
        y = O.rope(x, [p], 10000.0)
        assert np.allclose(y[0, 0], [np.cos(p), np.sin(p)])
    # head_dim 4: pairs are (0,2) and (1,3); theta_1 = base^(-2/4)
    x = np.array([[[1.0, 2.0, 0.0, 0.0]]])
    y = O.rope(x, [3], 100.0)
    t1 = 100.0 ** (-0.5)
    assert np.allclose(y[0, 0], [np.cos(3.0), 2 * np.cos(3 * t1), np.sin(3.0), 2 * np.sin(3 * t1)])


def test_rope_norm_preserving_and_relative():
    rng = np.random.default_rng(2)
    q = rng.normal(size=(6, 3, 16))
    k = rng.normal(size=(6, 3, 16))
    pos = np.array([0, 1, 2, 10, 11, 400])
    qr, kr = O.rope(q, pos, 1e4), O.rope(k, pos, 1e4)
    assert np.allclose(np.linalg.norm(qr, axis=-1), np.linalg.norm(q, axis=-1))
    # scores depend on position differences only
    qs, ks = O.rope(q, pos + 77, 1e4), O.rope(k, pos + 77, 1e4)
    s0 = np.einsum("rhd,chd->hrc", qr, kr)
    s1 = np.einsum("rhd,chd->hrc", qs, ks)
    assert np.allclose(s0, s1, atol=1e-10)


def test_gqa_attention_matches_torch_sdpa():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    R, C, Hq, Hkv, hd = 5, 9, 6, 2, 8
    q = rng.normal(size=(R, Hq, hd))
    k = rng.normal(size=(C, Hkv, hd))
    v = rng.normal(size=(C, Hkv, hd))
    allowed = rng.random((R, C)) < 0.6
    allowed[:, 0] = True
    o = O.gqa_attention(q, k, v, allowed)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    # library routine with explicitly repeated K/V heads: head h uses kv head h // (Hq/Hkv)
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(allowed))
    assert np.allclose(o, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_drafter_block_mask_structure():
    a = O.drafter_block_mask(3, 4)
    assert a.shape == (7, 7)
    assert (a[:3, :3] == np.tril(np.ones((3, 3), bool))).all()   # committed rows causal
    assert not a[:3, 3:].any()                                     # committed rows never see MASK rows
    assert a[3:, :].all()                                          # MASK rows see everything
    assert (O.causal_mask(4) == np.tril(np.ones((4, 4), bool))).all()


def test_counter_rng_uniformity_and_range():
    key = O.row_key(1234, O.TAG_DRAFT, 0, 17)
    u = O.uniforms(key, np.arange(200000))
    assert u.min() > 0.0 and u.max() < 1.0
    # exactly representable in fp32: (r + 0.5) / 2^23 with r < 2^23
    assert np.all(u.astype(np.float32).astype(np.float64) == u)
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = ((hist - len(u) / 64) ** 2 / (len(u) / 64)).sum()
    from scipy.stats import chi2 as chi2dist
    assert chi2dist.sf(chi2, 63) > 1e-3
    # distinct streams for distinct (tag, seq, pos)
    keys = {int(O.row_key(1234, t, s, p)) for t in (1, 2, 3) for s in (0, 1) for p in range(50)}
    assert len(keys) == 300


def test_mix64_known_values():
    # splitmix64 reference stream for seed 0 (tests/golden/splitmix64_seed0.txt): output i = mix64((i + 1) * golden)
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "splitmix64_seed0.txt")
    want = [int(l, 16) for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(want) >= 3
    for i, w in enumerate(want):
        state = ((i + 1) * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
        assert int(O.mix64(np.uint64(state))) == w


def _published_splitmix64():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "splitmix64_seed0.txt")
    return [int(l, 16) for l in open(path) if l.strip() and not l.startswith("#")]


def test_uniforms_of_key_zero_are_the_published_splitmix64_stream():
    # uniforms(key, idx) takes the top 23 bits of finaliser(key + (idx + 1) * golden): with key 0 that is output
    # idx of the published seed-0 stream, so index offset, increment and bit selection are pinned from outside
    want = _published_splitmix64()
    u = O.uniforms(0, np.arange(len(want)))
    for i, w in enumerate(want):
        assert u[i] == ((w >> 41) + 0.5) / 2 ** 23


def test_row_key_of_seed_zero_starts_from_the_published_stream():
    # row_key(seed, tag, seq, pos) = finaliser(finaliser(seed + golden * tag) xor ((seq << 40) + pos)): with seed 0 the
    # inner value is output tag - 1 of the published stream; the outer step is done here with Python integers
    M = (1 << 64) - 1

    def fin(z):
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        return z ^ (z >> 31)

    want = _published_splitmix64()
    for tag in (1, 2, 3):
        assert int(O.row_key(0, tag, 0, 0)) == fin(want[tag - 1])
        assert int(O.row_key(0, tag, 5, 77)) == fin(want[tag - 1] ^ ((5 << 40) + 77))


def test_counter_rng_golden_values():
    """Keys and 23-bit draws at stored points (tests/golden/counter_rng_golden.txt, written by the script beside it
    from the oracle alone): a changed shift, constant, tag or index offset fails here."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "counter_rng_golden.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 8
    for seed, tag, seq, pos, idx, key_hex, r in rows:
        key = O.row_key(int(seed), int(tag), int(seq), int(pos))
        assert int(key) == int(key_hex, 16)
        assert float(O.uniforms(key, int(idx))) == (int(r) + 0.5) / 2 ** 23


def test_gumbel_max_samples_the_categorical():
    from scipy.stats import chisquare
    w = np.array([0.5, 0.0, 0.2, 0.25, 0.05])
    with np.errstate(divide="ignore"):
        logw = np.log(w)
    n = 20000
    counts = np.zeros(5)
    for s in range(n):
        counts[O.CounterRng(s).categorical(logw, 3, O.TAG_RESID)] += 1
    assert counts[1] == 0
    keep = w > 0
    assert chisquare(counts[keep], n * w[keep]).pvalue > 1e-3


def test_bf16_roundtrip_plumbing():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -9, -0.3, 3.14159, 1e-3], dtype=np.float32)
    b = di.f32_to_bf16_bits(x)
    y = di.bf16_bits_to_f32(b)
    assert y[0] == 1.0
    assert y[1] == 1.0            # exactly halfway, ties to even (mantissa 0)
    assert y[2] == np.float32(1.0 + 2 ** -7)  # halfway between 1+2^-8... rounds to even mantissa 2
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    try:
        import torch
        t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert (t == b).all()
    except ImportError:
        pass


def test_round_to_bf16_matches_torch_cast():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(9)
    x = np.concatenate([rng.normal(size=5000) * 3, [1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -1.0 - 2 ** -8, 0.0]]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_to_bf16(x), ref)
    assert O.round_to_bf16(x.astype(np.float64)).dtype == np.float64
