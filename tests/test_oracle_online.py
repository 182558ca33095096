"""Pins for the oracle's online part: the annealed schedule (Eq. 4), the budget loop and the
decode loop of Algorithm 1."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle


def test_annealed_schedule_retained_fractions_at_the_paper_defaults():
    """r = 0.8, 0.6, 0.4, 0.2, 0 (Eq. 4 with r_init 0.8, delta 0.2, Sec. 6.1).  A round with merge
    fraction r removes r/2 of the tokens, so the retained fraction after each round is the running
    product of (1 - r/2): 0.6, 0.42, 0.336, 0.3024, and then nothing more is removed."""
    rs = [oracle.annealed_ratio(j, 0.8, 0.2) for j in range(6)]
    assert np.allclose(rs, [0.8, 0.6, 0.4, 0.2, 0.0, 0.0], atol=1e-7)
    s, c = 10 * 1000, 1000                     # chunk of 1000: |A| = 500, r*|A| is an integer for all r
    lens = oracle.round_lengths(s, c, rs[:5])
    assert lens == [10000, 6000, 4200, 3360, 3024, 3024]


def test_rounds_to_budget_follows_the_while_loop():
    assert oracle.rounds_to_budget(10000, 1000, 10000, 0.8, 0.2) == []                  # already within budget
    assert np.allclose(oracle.rounds_to_budget(10000, 1000, 6000, 0.8, 0.2), [0.8])
    assert np.allclose(oracle.rounds_to_budget(10000, 1000, 5999, 0.8, 0.2), [0.8, 0.6])
    assert np.allclose(oracle.rounds_to_budget(10000, 1000, 3024, 0.8, 0.2), [0.8, 0.6, 0.4, 0.2])
    with pytest.raises(ValueError):            # as printed, the defaults never reach 25%
        oracle.rounds_to_budget(10000, 1000, 2500, 0.8, 0.2)
    got = oracle.rounds_to_budget(10000, 1000, 2500, 0.8, 0.2, r_floor=0.2)
    assert np.allclose(got, [0.8, 0.6, 0.4, 0.2, 0.2, 0.2])
    # sinks and recents are never removed: the same budget needs more rounds
    assert len(oracle.rounds_to_budget(4096, 256, 2500, 1.0, 0.0)) == 1
    assert len(oracle.rounds_to_budget(4096, 256, 2500, 1.0, 0.0, n_sink=500, n_recent=500)) == 2


def _runs(rng, n_tokens, run, d):
    """Tokens in runs of `run` identical vectors."""
    base = rng.standard_normal((-(-n_tokens // run), d))
    return np.repeat(base, run, axis=0)[:n_tokens]


def _vanilla(q, K, V, G):
    """Eq. 1 with a library softmax: one query per head over the whole history."""
    d = K.shape[-1]
    out = np.zeros_like(q)
    for h in range(q.shape[0]):
        w = softmax(K[h // G] @ q[h] / np.sqrt(d))
        out[h] = w @ V[h // G]
    return out


@pytest.mark.parametrize("n_sink,n_recent", [(0, 0), (3, 5)])
def test_decode_loop_is_exact_on_runs_of_identical_tokens(n_sink, n_recent):
    """Clusters whose members are identical make Eq. 3 exact, so Algorithm 1's outputs must equal
    plain attention over the ENTIRE uncompressed history at every step, through several
    clustering rounds.  With r = 0.5 only the best half of each chunk's edges merge, and on runs
    of 16 identical tokens those all have similarity 1 (lossless)."""
    rng = np.random.default_rng(3)
    Hkv, G, d, n, steps, c = 2, 2, 16, 256, 200, 32
    Kall = np.stack([_runs(rng, n + steps, 16, d) for _ in range(Hkv)])
    Vall = np.stack([np.repeat(rng.standard_normal((-(-(n + steps) // 16), d)), 16, axis=0)[:n + steps]
                     for _ in range(Hkv)])
    qs = rng.standard_normal((steps, Hkv * G, d))
    deg0 = np.ones((Hkv, n), dtype=np.int64)
    ks = [Kall[:, n + i] for i in range(steps)]
    vs = [Vall[:, n + i] for i in range(steps)]
    budget, g = 256, 64
    outs, K, V, deg, ran = oracle.alg1_decode(Kall[:, :n], Vall[:, :n], deg0, qs, ks, vs, c, budget, g, [0.5],
                                              "f32", n_sink, n_recent)
    assert len(ran) >= 2 and ran[0] == g - 1          # first round when s reaches budget + g
    assert K.shape[1] < n + steps
    assert np.array_equal(deg.sum(axis=1), np.full(Hkv, n + steps))
    for i in range(steps):
        ref = _vanilla(qs[i], Kall[:, :n + i + 1], Vall[:, :n + i + 1], G)
        assert np.max(np.abs(outs[i] - ref)) < 1e-6, i     # fp32 storage of the (identical) centroids


def test_decode_loop_without_clustering_is_plain_attention_and_triggers_on_time():
    rng = np.random.default_rng(4)
    Hkv, G, d, n, steps = 1, 4, 8, 40, 30
    Kall, Vall = rng.standard_normal((Hkv, n + steps, d)), rng.standard_normal((Hkv, n + steps, d))
    qs = rng.standard_normal((steps, Hkv * G, d))
    ks, vs = [Kall[:, n + i] for i in range(steps)], [Vall[:, n + i] for i in range(steps)]
    deg0 = np.ones((Hkv, n), dtype=np.int64)
    outs, K, V, deg, ran = oracle.alg1_decode(Kall[:, :n], Vall[:, :n], deg0, qs, ks, vs, 8, 1000, 8, [1.0], "f32")
    assert ran == [] and K.shape[1] == n + steps and np.array_equal(K, Kall)
    for i in range(steps):
        assert np.allclose(outs[i], _vanilla(qs[i], Kall[:, :n + i + 1], Vall[:, :n + i + 1], G), atol=1e-12)
    # r = 1, chunk dividing the length, budget 40, g = 8: a round whenever s reaches 48, halving it to 24;
    # s then grows by one per step: rounds at steps 7, 31, 55 (0-based)
    steps = 60
    Kall, Vall = rng.standard_normal((Hkv, n + steps, d)), rng.standard_normal((Hkv, n + steps, d))
    qs = rng.standard_normal((steps, Hkv * G, d))
    ks, vs = [Kall[:, n + i] for i in range(steps)], [Vall[:, n + i] for i in range(steps)]
    outs, K, V, deg, ran = oracle.alg1_decode(Kall[:, :n], Vall[:, :n], deg0, qs, ks, vs, 8, 40, 8, [1.0], "f32")
    assert ran == [7, 31, 55]
    assert K.shape[1] == 24 + 4 and deg.sum() == n + steps
