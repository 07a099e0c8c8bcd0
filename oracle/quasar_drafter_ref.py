"""CPU oracle for the prompt-lookup n-gram drafter (TEST INFRASTRUCTURE ONLY).

Plain Python, brute force.  Nothing in the product path imports this file and this file imports
nothing from the product path.

The paper drafts with prompt-lookup decoding (Sec. 2 "n-gram matching against the pre-generated
context"; Sec. 4 "Implementation Details": the lookup length is adjusted dynamically between a
minimum of 1 and a maximum of 4; Sec. 4.4: lookup range (K_min, K_max) and gamma speculative
tokens).  It does not spell the search out.  Reading:

  * the context is every token so far (prompt + accepted tokens), n of them;
  * lookup lengths are tried from K_max down to K_min; for a length k (needing n >= k + 1) the
    pattern is the last k tokens, and a match is an EARLIER start s < n - k with
    c[s : s + k] == c[n - k : n] (it may overlap the pattern);
  * among the matches of the first length that has any, the most recent one (largest s) is
    taken - recent context is the most likely to repeat;
  * the draft is the tokens that followed it, c[s + k : s + k + gamma], cut at the end of the
    context (so at least one token, at most gamma);
  * no match at any length: no draft.
"""
from __future__ import annotations


def propose(context, gamma: int, k_min: int = 1, k_max: int = 4):
    """Returns (draft tokens as a list, lookup length used or 0)."""
    c = [int(t) for t in context]
    n = len(c)
    if not (1 <= k_min <= k_max) or gamma < 1:
        raise ValueError("need 1 <= k_min <= k_max and gamma >= 1")
    for k in range(k_max, k_min - 1, -1):
        if n < k + 1:
            continue
        pattern = c[n - k:]
        for s in range(n - k - 1, -1, -1):          # most recent earlier start first
            if c[s:s + k] == pattern:
                return c[s + k:min(s + k + gamma, n)], k
    return [], 0
