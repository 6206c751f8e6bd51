"""The C ABI without a GPU: the library loads, exports every function include/deer.h declares (and the binding
knows each of them), and its host-only entry points validate their arguments.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

import deer_inputs as di
from paper_2512_15176_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_15176_amd import build
        build.build_library()
    return binding.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "deer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(deer_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_function_is_exported_and_bound(lib):
    names = _declared()
    assert len(names) >= 20 and "deer_init_models" in names and "deer_accept_and_commit" in names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/deer.h but not exported by libdeer.so"
    assert sorted(binding.EXPORTS) == names


def test_query_sizes_is_host_only_and_scales(lib):
    cfg = di.CONFIGS["qwen3_8b"]
    t, d = cfg["target"], cfg["drafter"]
    s1 = binding.query_sizes(binding.init_params(t, d, 1, 4096 + 64, 32, di.mask_token_id(t.vocab)))
    s16 = binding.query_sizes(binding.init_params(t, d, 16, 4096 + 64, 32, di.mask_token_id(t.vocab)))
    layer = t.d_model * (t.n_q_heads + 2 * t.n_kv_heads) * t.head_dim + t.n_q_heads * t.head_dim * t.d_model + 3 * t.d_model * t.d_ff
    params = t.n_layers * layer + 2 * t.vocab * t.d_model
    assert params * 2 <= s1.weights[0] < params * 2 * 1.01           # bf16, small alignment padding only
    kv = 2 * t.n_layers * t.n_kv_heads * t.head_dim * (4096 + 64) * 2
    assert kv <= s1.kv[0] < kv * 1.01 and s16.kv[0] == pytest.approx(16 * s1.kv[0], rel=1e-3)
    assert s16.weights[0] == s1.weights[0] and s16.workspace > s1.workspace and s1.staging == 0


def _rc(lib, p):
    s = binding.Sizes()
    return lib.deer_query_sizes(C.byref(p), C.byref(s))


def test_argument_validation_on_the_host(lib):
    cfg = di.CONFIGS["tiny"]
    t, d = cfg["target"], cfg["drafter"]
    mk = lambda **kw: binding.init_params(kw.get("t", t), kw.get("d", d), kw.get("b", 1), kw.get("s", 256), kw.get("k", 8),
                                          kw.get("mask", di.mask_token_id(t.vocab)))
    assert _rc(lib, mk()) == 0
    assert _rc(lib, mk(k=33)) == -1                      # a block has at most 32 rows
    assert _rc(lib, mk(k=0)) == -1
    assert _rc(lib, mk(s=100)) == -1                     # max_seq must be a multiple of 64
    assert _rc(lib, mk(b=0)) == -1
    assert _rc(lib, mk(mask=t.vocab)) == -1              # MASK id outside the vocabulary
    assert _rc(lib, mk(t=di.scaled(t, head_dim=48))) == -1
    assert _rc(lib, mk(d=di.scaled(d, vocab=t.vocab * 2))) == -1     # the two models share the vocabulary
    assert b"vocabulary" in lib.deer_last_error(None)
    bad = mk()
    bad.struct_size += 8                                 # a caller built against another header
    assert _rc(lib, bad) == -5
    bad = mk()
    bad.abi_version = 99
    assert _rc(lib, bad) == -5
    # init with missing buffers fails before any device call
    ctx = C.c_void_p()
    p, bufs, sizes = mk(), binding.Buffers(), binding.Sizes()
    assert lib.deer_init_models(C.byref(p), C.byref(bufs), C.byref(sizes), C.byref(ctx)) == -1 and not ctx.value
    # entry points refuse a null context
    assert lib.deer_draft_block(None, 8, C.c_float(0.0), 0, None) == -1
    assert lib.deer_destroy(None) == -1
