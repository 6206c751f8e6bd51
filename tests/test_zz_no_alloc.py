"""GPU test of deer_accept_and_commit_static, the acceptance entry point that allocates nothing (its sampling kernel's
scratch is a static device array inside the library), against deer_accept_and_commit on the same inputs: two engines
with the same weights and prompts run the same draft and verify passes; one commits through the existing entry point,
the other through the new one.  Two calls in a row, the second on a smaller batch and block, so that the static array
still holds the first call's candidates.  Integer outputs: compared exactly."""
import numpy as np
import pytest

import deer_inputs as di
from gpu_common import StoredWeights, gpu_available, make_engine

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not gpu_available(), reason="needs a GPU")]

CFG = di.CONFIGS["tiny"]


def test_static_scratch_entry_point_matches_the_workspace_one():
    t, d = CFG["target"], CFG["drafter"]
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    engines = [make_engine(t, d, wt, wd, max_batch=5, max_seq=256, max_k=8) for _ in range(2)]
    T = 1.0
    for call, (B, k, seed) in enumerate([(5, 8, 21), (2, 5, 22)]):
        prompts = [di.prompt_ids(t.vocab, 33 + 9 * b + call, seq=300 + 10 * call + b) for b in range(B)]
        outs = []
        for e, eng in enumerate(engines):
            eng.prefill(prompts)
            for it in range(3):      # a few iterations from the same state: ragged accepts, residual draws
                dr = eng.draft_block(k, T, seed + 100 * it)
                eng.verify_block(k, T, dr)
                acc, com, ncom = eng.accept_and_commit(k, T, seed + 100 * it, static=(e == 1))
                outs.append((e, it, acc.tolist(), com, ncom.tolist()))
        ref = [o[2:] for o in outs if o[0] == 0]
        new = [o[2:] for o in outs if o[0] == 1]
        assert ref == new, (call, ref, new)
        assert any(a < k for r in ref for a in r[0]) and all(len(c) >= 1 for r in ref for c in r[1])
        assert engines[0].get_lengths().tolist() == engines[1].get_lengths().tolist()
    # T = 0 goes through the same entry point (no scratch in use)
    for e, eng in enumerate(engines):
        dr = eng.draft_block(5, 0.0, 0)
        eng.verify_block(5, 0.0, dr)
        res = eng.accept_and_commit(5, 0.0, 0, static=(e == 1))
        if e == 0:
            first = res
        else:
            assert first[0].tolist() == res[0].tolist() and first[1] == res[1]
    for eng in engines:
        eng.close()


def test_static_scratch_entry_point_rejects_a_batch_beyond_its_limit():
    from paper_2512_15176_amd import binding
    t, d = CFG["target"], CFG["drafter"]
    wt, wd = StoredWeights(t, di.TARGET_SEED, "bf16"), StoredWeights(d, di.DRAFTER_SEED, "bf16")
    eng = make_engine(t, d, wt, wd, max_batch=65, max_seq=128, max_k=4)
    eng.prefill([di.prompt_ids(t.vocab, 20, seq=b) for b in range(65)])
    dr = eng.draft_block(4, 1.0, 1)
    eng.verify_block(4, 1.0, dr)
    with pytest.raises(binding.DeerError) as ei:
        eng.accept_and_commit(4, 1.0, 1, static=True)
    assert ei.value.status == -3          # DEER_ECAPACITY, nothing changed: the ordinary entry point still works
    acc, com, ncom = eng.accept_and_commit(4, 1.0, 1)
    assert len(com) == 65
    eng.close()
