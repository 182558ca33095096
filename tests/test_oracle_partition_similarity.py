"""Pins for the oracle's partition, similarity and storage rounding (CPU only)."""
import itertools
import math

import numpy as np
import torch

from oracle import (alternating_partition, chunk_bounds, cosine_similarity, round_to_storage)
from synth import ar1_keys_host


# ---- alternating partition: Theorem A.1 -----------------------------------
def _cross_sum(A, B, f):
    return sum(f[abs(x - y)] for x in A for y in B)


def test_theorem_a1_bruteforce():
    """Among all balanced partitions of [2n], the alternating one maximises
    sum f(|x-y|) over cross pairs for convex decreasing f (Theorem A.1)."""
    rng = np.random.default_rng(1)
    for n in (1, 2, 3, 4, 5):
        a_off, b_off = alternating_partition(2 * n)
        for _ in range(4):
            # f(1)-f(2) >= f(2)-f(3) >= ... >= 0: cumulate sorted non-negative decrements
            dec = np.sort(rng.random(2 * n))[::-1]
            f = {i + 1: float(-np.sum(dec[:i])) for i in range(2 * n)}
            best = max(_cross_sum(A, [x for x in range(2 * n) if x not in A], f)
                       for A in itertools.combinations(range(2 * n), n))
            got = _cross_sum(list(a_off), list(b_off), f)
            assert got >= best - 1e-12


def _c_closed_form(n, l):
    """c_{2n,l} as printed in the proof of Theorem A.1 (the two-case cubic)."""
    if l % 2 == 0:
        return -l ** 3 / 12 + (2 * n - 1) * l ** 2 / 4 + (6 * n - 1) * l / 6
    return -l ** 3 / 12 + (2 * n - 1) * l ** 2 / 4 + (12 * n - 5) * l / 12 + (2 * n - 1) / 4


def test_partition_matches_closed_form_of_the_proof():
    """For the alternating partition, sum_{i<=l} (l+1-i) |D_i| (cross pairs at
    distance i) equals the printed c_{2n,l}; a partition with A and B laid out
    any other way gives a different distance histogram."""
    for n in range(1, 9):
        a_off, b_off = alternating_partition(2 * n)
        assert list(a_off) == list(range(0, 2 * n, 2))      # 1st, 3rd, ... token
        assert list(b_off) == list(range(1, 2 * n, 2))
        D = np.zeros(2 * n + 1, dtype=int)
        for x in a_off:
            for y in b_off:
                D[abs(int(x) - int(y))] += 1
        for l in range(1, 2 * n):
            lhs = sum((l + 1 - i) * D[i] for i in range(1, l + 1))
            assert abs(lhs - _c_closed_form(n, l)) < 1e-9


def test_partition_odd_and_tiny():
    a, b = alternating_partition(5)
    assert list(a) == [0, 2, 4] and list(b) == [1, 3]
    a, b = alternating_partition(1)
    assert list(a) == [0] and len(b) == 0
    assert chunk_bounds(10, 4) == [(0, 4), (4, 8), (8, 10)]
    assert chunk_bounds(8, 4) == [(0, 4), (4, 8)]


# ---- cosine similarity: Eq. 2 ---------------------------------------------
def test_self_and_scaled_cosine():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((7, 16))
    S = cosine_similarity(X, X)
    assert np.allclose(np.diag(S), 1.0, atol=1e-14)
    assert np.allclose(cosine_similarity(X, 3.5 * X).diagonal(), 1.0, atol=1e-14)
    assert np.allclose(cosine_similarity(X, -0.25 * X).diagonal(), -1.0, atol=1e-14)
    assert np.all(np.abs(S) <= 1 + 1e-14)


def test_cosine_against_library_routine():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((9, 32))
    B = rng.standard_normal((5, 32))
    ref = torch.nn.functional.cosine_similarity(
        torch.from_numpy(A)[:, None, :], torch.from_numpy(B)[None, :, :], dim=-1).numpy()
    S = cosine_similarity(A, B)
    assert S.shape == (9, 5)                      # rows = first operand (a transposed result fails)
    assert np.allclose(S, ref, atol=1e-13)
    # hand value: cos((1,0),(1,1)) = 1/sqrt(2)
    assert abs(cosine_similarity(np.array([[1.0, 0.0]]), np.array([[1.0, 1.0]]))[0, 0]
               - 1 / math.sqrt(2)) < 1e-15


def test_zero_key_has_zero_similarity():
    S = cosine_similarity(np.zeros((1, 4)), np.array([[1.0, 2, 3, 4]]))
    assert S[0, 0] == 0.0


def test_ar1_keys_decay_like_alpha_power():
    """Generator sanity: mean cosine at distance delta is close to alpha**delta."""
    rng = np.random.Generator(np.random.PCG64(5))
    K = ar1_keys_host(rng, 4096, 64, 0.9)
    for delta in (1, 2, 4, 8):
        S = np.einsum("td,td->t", K[:-delta], K[delta:]) / (
            np.linalg.norm(K[:-delta], axis=1) * np.linalg.norm(K[delta:], axis=1))
        assert abs(S.mean() - 0.9 ** delta) < 0.03


# ---- storage rounding ------------------------------------------------------
def test_bf16_rounding_matches_torch_on_fp32_inputs():
    rng = np.random.default_rng(4)
    x32 = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    ref = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_to_storage(x32.astype(np.float64), "bf16"), ref)


def test_bf16_rounding_ties_and_single_step():
    # bf16 spacing in [1, 2) is 2**-7: 1 + 2**-8 is a tie -> even (1.0); 1 + 3*2**-8 -> 1 + 2**-6
    assert round_to_storage(np.array([1 + 2.0 ** -8]), "bf16")[0] == 1.0
    assert round_to_storage(np.array([1 + 3 * 2.0 ** -8]), "bf16")[0] == 1 + 2.0 ** -6
    # just above a tie must round up even though fp32 would first collapse it onto the tie
    x = 1 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(x) == np.float32(1 + 2.0 ** -8)
    assert round_to_storage(np.array([x]), "bf16")[0] == 1 + 2.0 ** -7
    assert round_to_storage(np.array([-x]), "bf16")[0] == -(1 + 2.0 ** -7)
    assert round_to_storage(np.array([0.0]), "bf16")[0] == 0.0
    # every bf16 value is a fixed point
    v = torch.arange(-300, 300, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_to_storage(v, "bf16"), v)


def test_f32_rounding():
    x = np.array([1 + 2.0 ** -30, math.pi])
    assert np.array_equal(round_to_storage(x, "f32"), x.astype(np.float32).astype(np.float64))
