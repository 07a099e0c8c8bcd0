"""GPU parity for stochastic verification (temperature T > 0) through the C-ABI against the CPU
oracle.  The GPU takes the softmax and the prefix sums in fp32, the oracle in fp64, so the
probabilities are held to a relative 1e-3; the accepted length is required exact (every
acceptance test below is built at least 2e-3 of the probability away from its threshold); the
drawn token must be one whose interval of the oracle's cumulative sum lies within 1e-4 of the
total mass of the drawn point (fp32 summation over the vocabulary can move the point that
much), and must equal the oracle's token whenever the oracle's own margin exceeds that."""
import numpy as np
import pytest
import torch

from oracle import quasar_ref as ref
from oracle import quasar_sampling_ref as sp
from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, f32_to_dev, i32_to_dev

pytestmark = pytest.mark.gpu
P_TOL = 1e-3
DRAW_MARGIN = 1e-4


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2603_01399_amd import binding
    return binding


def say(*a):
    print(*a, flush=True)


def case(qb, M, V, K, seed, scale=0.05):
    """Hidden states and an int8 vocabulary matrix whose logits have a few nats of spread."""
    h = synth.activations_bf16(M, K, seed=synth.seed_for(7, 0, seed))
    w = synth.normal_weights(V, K, seed=synth.seed_for(7, 1, seed)) * np.float32(scale / 0.02)
    q_ref, s_ref = ref.quantize_weights(w)
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    logits = ref.w8_linear(h, q_ref, s_ref)                  # fp64, unrounded
    return h, wq, sc, logits


def check_draw(tok, mass, u, want_tok, want_margin):
    """tok is a valid draw for the uniform number u; identical to the oracle's when that is clear."""
    c = np.cumsum(np.asarray(mass, dtype=np.float64))
    total = c[-1]
    assert 0 <= tok < len(mass) and mass[tok] > 0
    lo = c[tok - 1] if tok > 0 else 0.0
    assert lo - DRAW_MARGIN * total <= u * total < c[tok] + DRAW_MARGIN * total, (tok, want_tok, want_margin)
    if want_margin > DRAW_MARGIN:
        assert tok == want_tok, (tok, want_tok, want_margin)


def run(qb, h, wq, sc, V, draft, T, ua, us):
    acc, tok, pd = qb.lmhead_verify_sample(bf16_to_dev(h), wq, sc, V, None if len(draft) == 0 else i32_to_dev(draft),
                                           T, None if len(draft) == 0 else f32_to_dev(ua), f32_to_dev(us))
    torch.cuda.synchronize()
    return int(acc.cpu()[0]), int(tok.cpu()[0]), pd.cpu().numpy()


@pytest.mark.parametrize("M,V,K,T,seed", [(8, 4096, 512, 1.0, 1), (5, 16 * 333, 192, 0.7, 2), (16, 8192, 1024, 1.3, 3),
                                         (32, 2048, 256, 1.0, 4), (2, 16, 64, 0.5, 5)])
def test_accept_reject_and_draw(qb, M, V, K, T, seed):
    say("sample verify", M, V, K, T, seed)
    h, wq, sc, logits = case(qb, M, V, K, seed)
    p = sp.softmax(logits, T)
    rng = np.random.Generator(np.random.Philox(100 + seed))
    n_draft = M - 1
    # candidates: a mix of likely and unlikely tokens
    draft = np.array([int(np.argsort(p[i])[-1 - (i % 3)]) for i in range(n_draft)], dtype=np.int32)
    pd = p[np.arange(n_draft), draft]
    for j in sorted({0, n_draft // 2, n_draft}):                 # first rejected position (n_draft: none)
        ua = (pd * 0.5).astype(np.float32)
        if j < n_draft:
            ua[j] = np.float32(min(0.999, pd[j] + 0.5 * (1.0 - pd[j])))
        us = np.zeros(M, dtype=np.float32)
        us[j] = np.float32(rng.random() * 0.999)
        want = sp.speculative_verify(logits, draft, T, ua.astype(np.float64), us.astype(np.float64))
        assert want["n_acc"] == j and np.all(want["accept_margin"][:j + 1] > 2 * P_TOL * pd[:j + 1])
        n_acc, tok, pd_gpu = run(qb, h, wq, sc, V, draft, T, ua, us)
        assert np.allclose(pd_gpu, pd, rtol=P_TOL, atol=1e-9), np.abs(pd_gpu / pd - 1).max()
        assert n_acc == j
        mass = p[j].copy()
        if j < n_draft:
            mass[draft[j]] = 0.0
            assert tok != draft[j]                               # the rejected token is never drawn again
        check_draw(tok, mass, float(us[j]), want["token"], want["sample_margin"])


def test_no_candidates_is_plain_sampling_and_is_repeatable(qb):
    say("sample verify, no candidates")
    M, V, K, T = 1, 4096, 256, 0.9
    h, wq, sc, logits = case(qb, M, V, K, 9)
    p = sp.softmax(logits, T)[0]
    rng = np.random.Generator(np.random.Philox(9))
    seen = set()
    for _ in range(12):
        us = np.array([rng.random() * 0.999], dtype=np.float32)
        n_acc, tok, _ = run(qb, h, wq, sc, V, np.zeros(0, np.int32), T, None, us)
        assert n_acc == 0
        check_draw(tok, p, float(us[0]), *sp.inverse_cdf(p, float(us[0])))
        assert run(qb, h, wq, sc, V, np.zeros(0, np.int32), T, None, us)[1] == tok
        seen.add(tok)
    assert len(seen) > 3                                         # it does sample


def test_low_temperature_agrees_with_greedy_verification(qb):
    say("sample verify, low temperature")
    M, V, K = 8, 4096, 512
    h = synth.activations_bf16(M, K, seed=synth.seed_for(7, 0, 11))
    w = synth.normal_weights(V, K, seed=synth.seed_for(7, 1, 11))
    am = synth.distinct_targets(M, V, seed=synth.seed_for(7, 2, 11))
    synth.plant_targets(w, h, am)                                # clear winners
    q_ref, s_ref = ref.quantize_weights(w)
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    logits = ref.w8_linear(h, q_ref, s_ref)
    srt = np.sort(logits, axis=1)
    assert np.array_equal(logits.argmax(axis=1), am) and np.all(srt[:, -1] - srt[:, -2] > 1.0)
    draft = am[:M - 1].astype(np.int32).copy()
    draft[3] = (draft[3] + 1) % V
    ua = np.full(M - 1, 0.5, dtype=np.float32)
    us = np.full(M, 0.5, dtype=np.float32)
    n_acc, tok, _ = run(qb, h, wq, sc, V, draft, 1e-2, ua, us)
    ws = qb.make_workspace(M, V, K)
    g_am, g_acc = qb.lmhead_verify(bf16_to_dev(h), wq, sc, V, i32_to_dev(draft), ws)
    assert n_acc == int(g_acc.cpu()[0]) == 3 and tok == int(g_am.cpu()[3]) == am[3]


def test_out_of_vocabulary_candidate_is_rejected(qb):
    say("sample verify, out-of-vocabulary candidate")
    M, V, K, T = 4, 1024, 128, 1.0
    h, wq, sc, logits = case(qb, M, V, K, 13)
    p = sp.softmax(logits, T)
    draft = np.array([int(p[0].argmax()), V + 7, int(p[2].argmax())], dtype=np.int32)
    ua = np.array([p[0].max() * 0.5, 1e-6, 0.0], dtype=np.float32)
    us = np.array([0, 0.4321, 0, 0], dtype=np.float32)
    n_acc, tok, pd = run(qb, h, wq, sc, V, draft, T, ua, us)
    assert n_acc == 1 and pd[1] == 0.0
    check_draw(tok, p[1], float(us[1]), *sp.inverse_cdf(p[1], float(us[1])))   # nothing to remove: the full distribution


def test_sample_argument_errors(qb):
    say("sample verify, argument errors")
    h = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    wq = torch.zeros(64 * 128, dtype=torch.int8, device="cuda")
    sc = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    u4 = torch.zeros(4, dtype=torch.float32, device="cuda")
    d4 = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.lmhead_verify_sample(h, wq, sc, 64, d4, 1.0, u4, u4)            # no position left for the bonus token
    with pytest.raises(qb.QuasarError):
        qb.lmhead_verify_sample(h, wq, sc, 64, d4[:3], 0.0, u4, u4)        # temperature must be positive
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(qb.QuasarError):
        qb.lmhead_verify_sample(h, wq, sc, 64, d4[:3], 1.0, u4, u4, workspace=small)
