"""pytest configuration: markers, import path, and small seeded-model helpers."""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import deer_inputs as di  # noqa: E402


class SeededWeights:
    """Callable weight provider over the seeded generator, with a small cache."""

    def __init__(self, shape, seed, weight_dtype="f32", cache=True):
        self.shape, self.seed, self.weight_dtype = shape, seed, weight_dtype
        self._cache = {} if cache else None

    def __call__(self, name, layer=-1, expert=-1):
        key = (name, layer, expert)
        if self._cache is not None and key in self._cache:
            return self._cache[key]
        w = di.weight_as_f32(self.shape, self.seed, name, layer, expert, self.weight_dtype)
        if self._cache is not None:
            self._cache[key] = w
        return w


@pytest.fixture(scope="session")
def tiny():
    return di.CONFIGS["tiny"]


@pytest.fixture(scope="session")
def tiny_weights(tiny):
    return (SeededWeights(tiny["target"], di.TARGET_SEED), SeededWeights(tiny["drafter"], di.DRAFTER_SEED))
