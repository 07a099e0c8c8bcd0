"""Pins for the prompt-lookup drafter oracle: hand-worked cases (longest lookup first, most recent
match, overlap with the pattern, cut at the end of the context, nothing to find) and agreement
with a library routine (bytes.rfind on the byte-encoded context) on random sequences.  No GPU."""
import numpy as np
import pytest

from oracle import quasar_drafter_ref as dr


def test_worked_examples():
    # k = 4 finds nothing, k = 3 finds (1,2,3) at 0: the draft is what followed it
    assert dr.propose([1, 2, 3, 4, 1, 2, 3], 3) == ([4, 1, 2], 3)
    # two earlier (5,6): the most recent one (start 3) wins, its continuation is cut at the end
    assert dr.propose([5, 6, 7, 5, 6, 8, 5, 6], 3) == ([8, 5, 6], 2)
    assert dr.propose([5, 6, 7, 5, 6, 8, 5, 6], 1) == ([8], 2)
    # the longest lookup that matches is used even if a shorter one has a more recent match
    assert dr.propose([1, 2, 9, 3, 2, 7, 1, 2], 2) == ([9, 3], 2)
    assert dr.propose([1, 2, 9, 3, 2, 7, 1, 2], 2, k_min=1, k_max=1) == ([7, 1], 1)
    # a match may overlap the pattern: (7,7,7,7) at start 0 is followed by one more token
    assert dr.propose([7, 7, 7, 7, 7], 4) == ([7], 4)
    # nothing repeats / context too short / lookup range excludes the only match
    assert dr.propose([1, 2, 3, 4, 5], 4) == ([], 0)
    assert dr.propose([4], 4) == ([], 0) and dr.propose([], 4) == ([], 0)
    assert dr.propose([4, 4], 4) == ([4], 1)
    assert dr.propose([1, 2, 3, 1], 5) == ([2, 3, 1], 1)
    assert dr.propose([1, 2, 3, 1], 5, k_min=2, k_max=4) == ([], 0)
    with pytest.raises(ValueError):
        dr.propose([1, 2], 0)
    with pytest.raises(ValueError):
        dr.propose([1, 2], 2, k_min=3, k_max=2)


@pytest.mark.parametrize("alphabet,n,seed", [(2, 40, 1), (3, 200, 2), (5, 300, 3), (30, 500, 4)])
def test_agrees_with_bytes_rfind(alphabet, n, seed):
    r = np.random.Generator(np.random.Philox(seed))
    c = r.integers(0, alphabet, size=n).astype(np.uint8)
    raw = c.tobytes()
    for end in range(0, n + 1, 7):
        ctx = c[:end].tolist()
        for (k_min, k_max) in ((1, 4), (2, 3), (1, 1)):
            for gamma in (1, 5):
                want = ([], 0)
                for k in range(k_max, k_min - 1, -1):
                    if end < k + 1:
                        continue
                    # the highest start whose k tokens lie inside c[0 : end-1] and equal the last k
                    s = raw.rfind(raw[end - k:end], 0, end - 1)
                    if s >= 0:
                        want = (list(raw[s + k:min(s + k + gamma, end)]), k)
                        break
                assert dr.propose(ctx, gamma, k_min, k_max) == want, (end, k_min, k_max, gamma)


def test_draft_is_a_true_continuation_on_repetitive_text():
    r = np.random.Generator(np.random.Philox(9))
    phrase = r.integers(0, 1000, size=23).tolist()
    ctx = []
    for rep in range(6):
        ctx += phrase + r.integers(1000, 2000, size=3).tolist()
    ctx += phrase[:10]
    draft, k = dr.propose(ctx, 7)
    assert k == 4 and draft == phrase[10:17]                  # inside the repeated phrase: the next tokens
