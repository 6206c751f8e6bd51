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
