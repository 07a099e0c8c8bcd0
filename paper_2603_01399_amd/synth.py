"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only draws numbers and arranges them; it contains none of the
method's arithmetic (no quantiser, no matmul, no argmax).  The shapes stand in
for the Qwen3-8B / Qwen3-32B checkpoints the paper evaluates (Sec. 4,
"Experimental Setup"): only the published layer dimensions are used, the values
are random.

Recipe: weights fp32 ~ N(0, 0.02^2); activations ~ N(0, 1) rounded once to bf16
(round-to-nearest-even, torch's conversion) and handed out as uint16 bit
patterns so every consumer sees the same bits; generator = numpy Philox keyed by
``seed_for(config, layer, linear)``.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20260301

# (name, d_in K, d_out N) for one decoder layer; attention itself is not part of the path
QWEN3_8B_LAYER = (
    ("q_proj", 4096, 4096),
    ("k_proj", 4096, 1024),
    ("v_proj", 4096, 1024),
    ("o_proj", 4096, 4096),
    ("gate_proj", 4096, 12288),
    ("up_proj", 4096, 12288),
    ("down_proj", 12288, 4096),
)
QWEN3_8B_LAYERS = 36
QWEN3_8B_HIDDEN = 4096
QWEN3_VOCAB = 151936

QWEN3_32B_LAYER = (
    ("q_proj", 5120, 8192),
    ("k_proj", 5120, 1024),
    ("v_proj", 5120, 1024),
    ("o_proj", 8192, 5120),
    ("gate_proj", 5120, 25600),
    ("up_proj", 5120, 25600),
    ("down_proj", 25600, 5120),
)
QWEN3_32B_LAYERS = 64


def seed_for(config: int, layer: int = 0, linear: int = 0) -> int:
    return BASE_SEED + 1000 * config + 100 * layer + linear


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def to_bf16_bits(a32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns via torch's own conversion (input preparation only)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def normal_weights(N: int, K: int, seed: int, std: float = 0.02) -> np.ndarray:
    w = _rng(seed).standard_normal((N, K), dtype=np.float32)
    w *= np.float32(std)
    return w


def activations_bf16(M: int, K: int, seed: int) -> np.ndarray:
    return to_bf16_bits(_rng(seed).standard_normal((M, K), dtype=np.float32))


def integer_case(M: int, N: int, K: int, seed: int, xmax: int = 8, row_exponents=False):
    """Integer-valued activations and weights whose products and sums are exact.

    x in [-xmax, xmax]; W rows integer in [-127, 127] with one entry forced to
    +-127 so the row step size is exactly 1 (times 2**e when row_exponents).
    Returns (x_bits uint16 [M,K], W fp32 [N,K], W_int int64 [N,K], exps int64 [N]).
    """
    r = _rng(seed)
    xi = r.integers(-xmax, xmax + 1, size=(M, K))
    wi = r.integers(-127, 128, size=(N, K))
    cols = r.integers(0, K, size=N)
    signs = r.integers(0, 2, size=N) * 2 - 1
    wi[np.arange(N), cols] = 127 * signs
    exps = r.integers(-6, 4, size=N) if row_exponents else np.zeros(N, dtype=np.int64)
    w = (wi.astype(np.float64) * np.exp2(exps.astype(np.float64))[:, None]).astype(np.float32)
    return to_bf16_bits(xi.astype(np.float32)), w, wi.astype(np.int64), exps.astype(np.int64)


def plant_targets(w: np.ndarray, h_bits: np.ndarray, targets, boost: float = 16.0) -> None:
    """Make row targets[i] of w the clear winner for position i (in place).

    Adds (boost / |h_i|^2) * h_i to that row, which raises position i's logit for
    that row by `boost` while natural logits are ~N(0, (0.02*sqrt(K))^2).
    """
    import torch
    h = torch.from_numpy(h_bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    for i, t in enumerate(targets):
        hi = h[i]
        w[int(t)] += (boost / float(hi @ hi) * hi).astype(np.float32)


def distinct_targets(M: int, V: int, seed: int) -> np.ndarray:
    return _rng(seed).choice(V, size=M, replace=False).astype(np.int64)


def draft_with_matches(targets, j: int, V: int, n_draft: int) -> np.ndarray:
    """Draft ids equal to targets for the first j positions, wrong from position j on."""
    d = np.array([int(t) for t in targets[:n_draft]], dtype=np.int32)
    for i in range(j, n_draft):
        d[i] = (int(targets[i]) + 1 + i) % V
    return d
