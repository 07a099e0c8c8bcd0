"""The native prompt-lookup drafter (host code of the library, called through the C-ABI) against
the brute-force oracle, token for token: random text over small and large alphabets, repetitive
text, incremental growth with a proposal after every appended token, growth past the initial
index size, the lookup ranges of the paper's sensitivity study, argument errors.  Needs no GPU."""
import numpy as np
import pytest

from oracle import quasar_drafter_ref as dr


@pytest.fixture(scope="module")
def qb():
    from paper_2603_01399_amd import binding
    return binding


def repetitive_text(r, n, vocab, phrase_len=17, noise=0.15):
    phrases = [r.integers(0, vocab, size=phrase_len).tolist() for _ in range(5)]
    out = []
    while len(out) < n:
        ph = list(phrases[int(r.integers(0, len(phrases)))])
        for i in range(len(ph)):
            if r.random() < noise:
                ph[i] = int(r.integers(0, vocab))
        out += ph
    return out[:n]


@pytest.mark.parametrize("vocab,n,seed", [(2, 120, 1), (4, 400, 2), (50, 600, 3), (151936, 600, 4)])
@pytest.mark.parametrize("k_range", [(1, 4), (1, 3), (2, 4), (3, 5), (1, 1)])
def test_every_prefix_matches_oracle(qb, vocab, n, seed, k_range):
    r = np.random.Generator(np.random.Philox(100 + seed))
    text = repetitive_text(r, n, vocab) if seed % 2 else r.integers(0, vocab, size=n).tolist()
    d = qb.Drafter(k_range[0], k_range[1], capacity_hint=0)
    assert d.propose(4) == ([], 0)
    for i, tok in enumerate(text):
        d.append([tok])
        assert len(d) == i + 1
        for gamma in (1, 7):
            assert d.propose(gamma) == dr.propose(text[:i + 1], gamma, *k_range), (i, gamma)
    d.close()


def test_bulk_append_growth_and_hint(qb):
    r = np.random.Generator(np.random.Philox(7))
    text = repetitive_text(r, 30000, 151936, phrase_len=40, noise=0.05)     # grows the index several times
    a, b = qb.Drafter(1, 4, capacity_hint=0), qb.Drafter(1, 4, capacity_hint=40000)
    a.append(text[:1000])
    b.append(text[:1000])
    for lo in range(1000, 30000, 2900):
        a.append(text[lo:lo + 2900])
        b.append(text[lo:lo + 2900])
        want = dr.propose(text[:lo + 2900], 7)
        assert a.propose(7) == want and b.propose(7) == want
    assert len(a) == len(b) == 30000


def test_drafter_argument_errors(qb):
    for bad in ((0, 4), (3, 2), (1, 65)):
        with pytest.raises(qb.QuasarError):
            qb.Drafter(*bad)
    d = qb.Drafter()
    with pytest.raises(qb.QuasarError):
        d.propose(0)
    d.append([])
    assert len(d) == 0 and d.propose(3) == ([], 0)
    assert qb.lib().quasar_drafter_length(None) == -1
