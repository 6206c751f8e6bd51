"""Helpers for the GPU parity tests: build an engine and an oracle over the same seeded inputs."""
import numpy as np

import deer_inputs as di
from oracle import deer_oracle as O


def gpu_available():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


class StoredWeights:
    """Seeded weights as the model stores them.  as_f32(): exact values for the oracle;
    for_engine(): what the library loads (fp32 values, or bf16 bit patterns)."""

    def __init__(self, shape, seed, weight_dtype):
        self.shape, self.seed, self.weight_dtype = shape, seed, weight_dtype
        self._cache = {}

    def raw(self, name, layer=-1, expert=-1):
        key = (name, layer, expert)
        if key not in self._cache:
            w = di.weight_f32(self.shape, self.seed, name, layer, expert)
            self._cache[key] = di.f32_to_bf16_bits(w) if self.weight_dtype == "bf16" else w
        return self._cache[key]

    def as_f32(self, name, layer=-1, expert=-1):
        r = self.raw(name, layer, expert)
        return di.bf16_bits_to_f32(r) if r.dtype == np.uint16 else r

    def for_engine(self, name, layer=-1, expert=-1):
        return self.raw(name, layer, expert)


def make_engine(target, drafter, wt, wd, max_batch, max_seq, max_k, keep_logits=True, eos=-1):
    from paper_2512_15176_amd import DeerEngine, binding
    eng = DeerEngine(target, drafter, max_batch, max_seq, max_k, di.mask_token_id(target.vocab), eos, keep_logits)
    eng.load_model(binding.DEER_TARGET, target, wt.for_engine)
    eng.load_model(binding.DEER_DRAFTER, drafter, wd.for_engine)
    return eng


def make_pair(target, drafter, wt, wd, capacity, dtype=np.float64, kv_storage="bf16"):
    return O.TransformerPair(O.Decoder(target, wt.as_f32, dtype, kv_storage), O.Decoder(drafter, wd.as_f32, dtype, kv_storage),
                             di.mask_token_id(target.vocab), capacity)


def top2_margin(z):
    """Per row: gap between the largest and second largest logit."""
    part = np.partition(z, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def greedy_commit(z, block, bonus=False):
    """(accepted length, committed tokens) that the T = 0 rule gives for the target logits z and the draft block."""
    a, c = O.accept_block_greedy([O.argmax_lowest(z[i]) for i in range(len(z))], block, bonus)
    return a, list(block[:a]) + ([] if c is None else [c])


def lockstep_commit(eng, k, gzt, results, blocks, bonus=False):
    """T = 0 lock-step commit of one iteration for every sequence of the batch.  gzt[b]: the device's target logits,
    results[b]: the oracle's iteration (deer_iteration) on the same block blocks[b].  The device's own logits say what
    its acceptance kernel must decide; where that equals the oracle's commit for every sequence, the acceptance call
    runs and is compared exactly (returns True).  Otherwise the first differing row must have an oracle top-2 margin
    below 1e-2 (the only legitimate cause), and the oracle's commits are forced into the device state
    (deer_debug_force_commit) so that the comparison goes on from a common state (returns False)."""
    agree = True
    for b, res in enumerate(results):
        a_dev, com_dev = greedy_commit(gzt[b], blocks[b], bonus)
        if (a_dev, com_dev) != (res["accept_len"], res["committed"]):
            first = min(a_dev, res["accept_len"])
            assert top2_margin(res["target_logits"])[first] < 1e-2, (b, a_dev, res["accept_len"])
            agree = False
    if agree:
        acc, com, ncom = eng.accept_and_commit(k, 0.0, 0)
        for b, res in enumerate(results):
            assert acc[b] == res["accept_len"] and com[b] == res["committed"], (b, acc[b], com[b], res["accept_len"], res["committed"])
        return True
    eng.debug_force_commit([res["committed"] for res in results])
    return False


def fill_seeded_cache(eng, torch, model, shape, b, n, cache=None, threads=16):
    """The same seeded stand-in K,V rows (slots 0 .. n-1 of sequence slot b) into the engine's cache and, if given,
    the oracle's KVCache."""
    for l in range(shape.n_layers):
        kb = di.kv_fill_bits(shape, "k", l, b, n, threads=threads)
        vb = di.kv_fill_bits(shape, "v", l, b, n, threads=threads)
        eng.debug_load_kv(model, l, b, 0, torch.from_numpy(kb.view(np.int16)).cuda(), torch.from_numpy(vb.view(np.int16)).cuda())
        if cache is not None:
            cache.K[l, :n] = di.bf16_bits_to_f32(kb)
            cache.V[l, :n] = di.bf16_bits_to_f32(vb)
    torch.cuda.synchronize()
    if cache is not None:
        cache.n = n
