"""The closed loop draft -> verify -> accept with the pieces of the library on a toy model whose
greedy continuation is known: the n-gram drafter proposes, the fused vocabulary kernel verifies
gamma + 1 positions at once, the accepted candidates plus the token at the first mismatch (or the
bonus token) are appended.  Checked: the generated sequence is EXACTLY the one plain greedy
decoding produces (verification is lossless, Sec. 3.1), every step emits at least one token, and
on text that repeats the mean number of tokens per step is well above one (the quantity L of the
paper's tables; its value here says nothing about real text).

The toy model has no layers: the hidden state of a position is the embedding of its token, and the
vocabulary matrix is planted so that the argmax after token t is a fixed successor s(t) whose
orbits revisit the same phrases."""
import numpy as np
import pytest
import torch

from oracle import quasar_drafter_ref as dr
from oracle import quasar_ref as ref
from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, f32_to_dev, i32_to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_01399_amd import binding
    return binding


def toy_model(V=2048, K=128, phrase=32, seed=5):
    r = np.random.Generator(np.random.Philox(seed))
    emb = synth.to_bf16_bits(r.standard_normal((V, K)).astype(np.float32))
    e = ref.bf16_bits_to_f64(emb)
    # successor (a permutation of the vocabulary): walk through a phrase of `phrase` consecutive ids, then
    # jump to the start of another phrase; phrases 0 -> 3 -> 1 -> 0, so the text cycles through three phrases
    assert V % phrase == 0
    nphr = V // phrase
    jump = {0: 3, 3: 1, 1: 0, 2: 4, nphr - 1: 2}
    succ = np.zeros(V, dtype=np.int64)
    for t in range(V):
        ph, off = divmod(t, phrase)
        succ[t] = t + 1 if off + 1 < phrase else jump.get(ph, ph + 1) * phrase
    assert sorted(succ.tolist()) == list(range(V))
    w = (r.standard_normal((V, K)) * 0.02).astype(np.float32)
    for t in range(V):
        w[succ[t]] += (16.0 / float(e[t] @ e[t]) * e[t]).astype(np.float32)
    return emb, succ, w


@pytest.mark.parametrize("gamma", [3, 7])
def test_speculative_loop_is_lossless_and_accepts_on_repetitive_text(qb, gamma):
    print("closed loop, gamma", gamma, flush=True)
    V, K = 2048, 128
    emb, succ, w = toy_model(V, K)
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    emb_dev = bf16_to_dev(emb)
    ws = qb.make_workspace(gamma + 1, V, K)
    # the quantised head still realises the successor map (checked on the tokens the text visits)
    q_ref, s_ref = ref.quantize_weights(w)
    visit = np.concatenate([np.arange(0, 32), np.arange(96, 128), np.arange(32, 64)])
    res = ref.lmhead_verify(emb[visit], q_ref, s_ref, [])
    assert np.array_equal(res["argmax"], succ[visit]) and np.all(res["top1"] - res["top2"] > 2.0)

    n_new = 400
    start = [5]
    want = list(start)
    while len(want) < len(start) + n_new:
        want.append(int(succ[want[-1]]))

    ctx = list(start)
    drafter = qb.Drafter(1, 4, capacity_hint=1024)
    drafter.append(ctx)
    steps, per_step, len_before = 0, [], []
    while len(ctx) < len(start) + n_new:
        draft, k = drafter.propose(gamma)
        assert (draft, k) == dr.propose(ctx, gamma)                       # the native drafter is the oracle's
        inputs = [ctx[-1]] + draft                                        # position i predicts the token after inputs[i]
        hidden = emb_dev[torch.tensor(inputs, device="cuda")]
        am, acc = qb.lmhead_verify(hidden, wq, sc, V, i32_to_dev(draft) if draft else None, ws)
        n_acc = int(acc.cpu()[0])
        assert 0 <= n_acc <= len(draft)
        new = draft[:n_acc] + [int(am.cpu()[n_acc])]
        len_before.append(len(ctx))
        ctx += new
        drafter.append(new)
        per_step.append(len(new))
        steps += 1
    ctx = ctx[:len(want)]
    assert ctx == want                                                    # lossless: plain greedy decoding's sequence
    mean_len = sum(per_step) / steps
    print("   steps", steps, "mean tokens per step", round(mean_len, 2), flush=True)
    # the first pass through the three phrases (96 tokens) cannot be drafted: one token per step; once the text
    # repeats, every candidate and the bonus token are accepted in every step
    steady = [n for n, before in zip(per_step, len_before) if before > 100]
    assert steady and all(n == gamma + 1 for n in steady)
    assert steps <= 100 + (n_new - 96) // (gamma + 1) + 2
