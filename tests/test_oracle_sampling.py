"""Pins for the stochastic-verification oracle: closed forms, the lossless property of the
accept/resample rule (checked by exact integration over the uniform numbers), invariances and
edge cases.  No GPU."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quasar_sampling_ref as sp


def test_softmax_closed_forms():
    p = sp.softmax(np.zeros((2, 5)), 0.7)
    assert np.allclose(p, 0.2, rtol=0, atol=1e-15)
    # two tokens: p0 = 1 / (1 + exp(-(a - b) / T))
    a, b, T = 1.25, -0.5, 0.8
    p = sp.softmax(np.array([[a, b]]), T)
    assert abs(p[0, 0] - 1.0 / (1.0 + np.exp(-(a - b) / T))) < 1e-15
    # shift invariance, and (logits, T) -> (c logits, c T)
    r = np.random.Generator(np.random.Philox(1))
    lg = r.standard_normal((3, 50)) * 4
    assert np.allclose(sp.softmax(lg + 123.0, 1.3), sp.softmax(lg, 1.3), atol=1e-14)
    assert np.allclose(sp.softmax(lg * 2.5, 1.3 * 2.5), sp.softmax(lg, 1.3), atol=1e-14)
    # huge logits do not overflow; T -> 0 concentrates on the argmax
    big = np.array([[1e4, 1e4 - 1.0, -1e4]])
    p = sp.softmax(big, 1.0)
    assert np.isfinite(p).all() and abs(p[0, 0] - 1 / (1 + np.exp(-1.0))) < 1e-12
    assert sp.softmax(lg, 1e-3).argmax(axis=1).tolist() == lg.argmax(axis=1).tolist()
    assert np.all(sp.softmax(lg, 1e-3).max(axis=1) > 0.99)
    with pytest.raises(ValueError):
        sp.softmax(lg, 0.0)


def test_inverse_cdf_worked_example():
    mass = [0.5, 0.0, 0.25, 0.25]
    want = {0.0: 0, 0.49: 0, 0.5: 2, 0.74: 2, 0.75: 3, 0.999: 3}
    for u, tok in want.items():
        assert sp.inverse_cdf(mass, u)[0] == tok, u
    # unnormalised masses give the same draw; zero-mass entries are never drawn
    assert all(sp.inverse_cdf(np.array(mass) * 7.0, u)[0] == tok for u, tok in want.items())
    assert sp.inverse_cdf([0.0, 0.0, 3.0], 0.0)[0] == 2
    # margin: distance to the nearer boundary of the token's interval
    tok, mg = sp.inverse_cdf(mass, 0.6)
    assert tok == 2 and abs(mg - 0.1) < 1e-15
    with pytest.raises(ValueError):
        sp.inverse_cdf([0.0, 0.0], 0.3)
    with pytest.raises(ValueError):
        sp.inverse_cdf([0.2, 0.8], 1.0)


def test_inverse_cdf_interval_lengths_are_the_probabilities():
    r = np.random.Generator(np.random.Philox(2))
    mass = r.random(9)
    mass[4] = 0
    grid = (np.arange(200000) + 0.5) / 200000
    toks = np.array([sp.inverse_cdf(mass, u)[0] for u in grid[::40]])
    freq = np.bincount(toks, minlength=9) / toks.size
    assert np.abs(freq - mass / mass.sum()).max() < 2e-3
    assert freq[4] == 0


def _outcome_distribution(logits, draft_tok, T, grid=400):
    """Exact (up to the u-grid) distribution of the emitted token for ONE candidate position
    followed by a bonus position: integrate the rule over (u_accept, u_sample)."""
    V = logits.shape[1]
    out = np.zeros(V)
    us = (np.arange(grid) + 0.5) / grid
    for ua in us:
        for ub in us[:: max(1, grid // 50)]:
            res = sp.speculative_verify(logits, [draft_tok], T, [ua], [ub, ub])
            tok = draft_tok if res["n_acc"] == 1 else res["token"]
            out[tok] += 1
    return out / out.sum()


def test_accept_or_resample_reproduces_the_target_distribution():
    """The lossless guarantee of the accept/resample rule: whatever token the deterministic drafter
    proposes, the token emitted at that position is distributed exactly as p.  A wrong residual
    (e.g. keeping the rejected token's mass) or a wrong acceptance probability fails this."""
    r = np.random.Generator(np.random.Philox(3))
    logits = r.standard_normal((2, 6)) * 1.5
    p = sp.softmax(logits, 0.9)[0]
    for draft_tok in (int(np.argmax(p)), int(np.argmin(p)), 2):
        dist = _outcome_distribution(logits, draft_tok, 0.9)
        assert np.abs(dist - p).max() < 1.5e-2, (draft_tok, dist, p)
    # analytically, with exact rationals on a two-token vocabulary:
    # P(emit x~) = p(x~); P(emit other) = (1 - p(x~)) * 1 = 1 - p(x~)
    pa = Fraction(3, 10)
    lg = np.log(np.array([[float(pa), float(1 - pa)], [0.5, 0.5]]))
    acc = sum(sp.speculative_verify(lg, [0], 1.0, [(k + 0.5) / 1000], [0.3, 0.3])["n_acc"] for k in range(1000))
    assert acc == 300
    for k in (5, 299, 300, 500, 995):
        res = sp.speculative_verify(lg, [0], 1.0, [(k + 0.5) / 1000], [0.3, 0.3])
        if k < 300:
            assert res["n_acc"] == 1                       # accepted: the bonus token comes from position 1
        else:
            assert (res["n_acc"], res["token"]) == (0, 1)  # rejected: the only other token


def test_verification_stops_at_first_rejection_and_bonus_token():
    r = np.random.Generator(np.random.Philox(4))
    M, V = 6, 40
    logits = r.standard_normal((M, V)) * 3
    p = sp.softmax(logits, 1.0)
    draft = p.argmax(axis=1)[:5]
    pd = p[np.arange(5), draft]
    # accept everything: u just below p; bonus token drawn from position 5
    res = sp.speculative_verify(logits, draft, 1.0, pd * 0.5, np.full(M, 0.37))
    assert res["n_acc"] == 5 and res["token"] == sp.inverse_cdf(p[5], 0.37)[0]
    assert np.allclose(res["p_draft"], pd)
    # reject at position 2: later uniforms are irrelevant, the rejected token is never re-drawn
    ua = pd * 0.5
    ua[2] = min(0.999999, pd[2] + 0.5 * (1 - pd[2]))
    for us in (0.0, 0.25, 0.5, 0.75, 0.999):
        res = sp.speculative_verify(logits, draft, 1.0, ua, np.full(M, us))
        assert res["n_acc"] == 2 and res["token"] != draft[2]
        m = p[2].copy()
        m[draft[2]] = 0
        assert res["token"] == sp.inverse_cdf(m, us)[0]
    ua2 = ua.copy()
    ua2[4] = 0.0
    assert sp.speculative_verify(logits, draft, 1.0, ua2, np.full(M, 0.5))["n_acc"] == 2
    # u == p is a rejection (strict inequality), u = 0 always accepts a token with positive mass
    ue = pd.copy()
    assert sp.speculative_verify(logits, draft, 1.0, ue, np.full(M, 0.5))["n_acc"] == 0
    assert sp.speculative_verify(logits, draft, 1.0, np.zeros(5), np.full(M, 0.5))["n_acc"] == 5
    # no room for the bonus token
    with pytest.raises(ValueError):
        sp.speculative_verify(logits[:5], draft, 1.0, np.zeros(5), np.zeros(5))
    # out-of-vocabulary candidate: probability 0, rejected
    bad = draft.copy()
    bad[1] = V + 3
    assert sp.speculative_verify(logits, bad, 1.0, np.full(5, 1e-9), np.full(M, 0.5))["n_acc"] == 1


def test_low_temperature_limit_is_greedy_acceptance():
    r = np.random.Generator(np.random.Philox(5))
    M, V = 5, 30
    logits = r.standard_normal((M, V)) * 2
    am = logits.argmax(axis=1)
    draft = am[:4].copy()
    draft[2] = (draft[2] + 1) % V
    res = sp.speculative_verify(logits, draft, 1e-4, np.full(4, 0.5), np.full(M, 0.5))
    assert res["n_acc"] == 2 and res["token"] == am[2]
