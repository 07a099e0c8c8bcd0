"""GPU check of quasar_lmhead_verify_static (the entry point that allocates nothing) against
quasar_lmhead_verify on the same inputs: two calls in a row, the second on a smaller vocabulary
and fewer positions, so that whatever the first call left in the library's device array must
not show in the second; then the first size once more."""
import numpy as np
import pytest
import torch

from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, f32_to_dev, i32_to_dev

pytestmark = pytest.mark.gpu


def test_static_scratch_verify_matches_workspace_verify():
    assert torch.cuda.is_available()
    from paper_2603_01399_amd import binding as qb
    K = 1024
    cases = []
    for idx, (M, V) in enumerate(((8, 40000), (5, 4112), (8, 40000), (32, 2048), (1, 16))):
        h = synth.activations_bf16(M, K, seed=synth.seed_for(12, idx, 0))
        w = synth.normal_weights(V, K, seed=synth.seed_for(12, idx, 1))
        t = synth.distinct_targets(M, V, seed=synth.seed_for(12, idx, 2))
        synth.plant_targets(w, h, t)
        wq, sc = qb.quantize_weights(f32_to_dev(w))
        d = i32_to_dev(synth.draft_with_matches(t, min(2, M - 1), V, M - 1)) if M > 1 else None
        ws = qb.make_workspace(M, V, K)
        cases.append((M, V, bf16_to_dev(h), wq, sc, d, ws, t,
                      torch.full((M,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda")))
    torch.cuda.synchronize()
    for M, V, h, wq, sc, d, ws, t, out_am, out_acc in cases:
        print("static verify", M, V, flush=True)
        before = torch.cuda.memory_allocated()
        qb.lmhead_verify_static(h, wq, sc, V, d, out_am, out_acc)
        assert torch.cuda.memory_allocated() == before
        am, acc = qb.lmhead_verify(h, wq, sc, V, d, ws)
        torch.cuda.synchronize()
        assert torch.equal(out_am, am) and torch.equal(out_acc, acc)
        assert np.array_equal(out_am.cpu().numpy(), t)
        assert int(out_acc.cpu()[0]) == min(2, M - 1)
    # sizes beyond the array's (more than 32 positions) are refused before anything runs
    M, V, h, wq, sc, d, ws, t, out_am, out_acc = cases[3]
    big = torch.zeros((33, K), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.lmhead_verify_static(big, wq, sc, V, None, torch.zeros(33, dtype=torch.int32, device="cuda"), out_acc)
