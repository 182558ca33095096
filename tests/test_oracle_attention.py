"""Pins for the oracle's attention over centroids, Eq. 3 (CPU only)."""
import math

import numpy as np
import torch

from oracle import app_attn, compress, csm_round
from synth import ar1_keys_host


def _case(seed, Hkv, G, L, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((Hkv * G, d)), rng.standard_normal((Hkv, L, d)),
            rng.standard_normal((Hkv, L, d)))


def test_degree_one_is_textbook_attention():
    q, K, V = _case(0, 2, 4, 37, 16)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).reshape(2, 4, 1, 16).reshape(8, 1, 16)[None],
        torch.from_numpy(K).repeat_interleave(4, dim=0)[None],
        torch.from_numpy(V).repeat_interleave(4, dim=0)[None])[0, :, 0].numpy()
    assert np.allclose(app_attn(q, K, V), ref, atol=1e-13)
    assert np.allclose(app_attn(q, K, V, np.ones((2, 37), dtype=np.int64)), ref, atol=1e-13)


def test_gqa_head_mapping_and_length():
    q, K, V = _case(1, 2, 2, 10, 8)
    o = app_attn(q, K, V, length=6)
    for h in range(4):
        z = K[h // 2, :6] @ q[h] / math.sqrt(8)
        p = np.exp(z - z.max())
        assert np.allclose(o[h], (p / p.sum()) @ V[h // 2, :6], atol=1e-14)
    assert np.array_equal(app_attn(q, K, V, length=0), np.zeros((4, 8)))


def test_zero_query_returns_the_mean_of_the_original_values():
    """With q = 0 the weights are the degrees, so for ANY clustering the output
    is the plain mean of the original values: pins the log N term."""
    rng = np.random.Generator(np.random.PCG64(3))
    K = ar1_keys_host(rng, 256, 16, 0.9)
    V = rng.standard_normal((256, 16))
    out = compress(K, V, 32, [1.0, 0.5], "f32")
    o = app_attn(np.zeros((1, 16)), out["K"][None], out["V"][None], out["deg"][None])
    assert np.allclose(o[0], V.mean(0), atol=1e-6)
    # without the degrees the answer is different
    o_wrong = app_attn(np.zeros((1, 16)), out["K"][None], out["V"][None])
    assert not np.allclose(o_wrong[0], V.mean(0), atol=1e-3)


def test_duplicate_key_clusters_are_exact():
    """When all keys of a cluster are equal the approximation of Eq. 3 is an
    equality: attention over centroids == attention over the full cache."""
    rng = np.random.default_rng(4)
    d, c = 8, 8
    protos = rng.standard_normal((6, d))
    K = np.repeat(protos, c, axis=0)                   # each chunk = one repeated key
    V = rng.standard_normal((6 * c, d))
    res = csm_round(K, V, np.ones(6 * c, dtype=np.int64), c, 1.0, "f32")
    q = rng.standard_normal((3, d))
    full = app_attn(q, K[None], V[None])
    comp = app_attn(q, res["K"][None], res["V_exact"][None], res["deg"][None])
    assert len(res["K"]) == 6 * c // 2
    assert np.allclose(full, comp, atol=1e-13)


def test_log_degree_equals_repeating_tokens():
    q, K, V = _case(5, 1, 2, 9, 8)
    deg = np.array([[1, 3, 2, 1, 1, 4, 1, 2, 1]])
    rep = np.repeat(np.arange(9), deg[0])
    assert np.allclose(app_attn(q, K, V, deg), app_attn(q, K[:, rep], V[:, rep]), atol=1e-13)


def test_permutation_invariance_and_scale():
    q, K, V = _case(6, 1, 1, 20, 8)
    deg = np.random.default_rng(0).integers(1, 4, (1, 20))
    p = np.random.default_rng(1).permutation(20)
    assert np.allclose(app_attn(q, K, V, deg), app_attn(q, K[:, p], V[:, p], deg[:, p]), atol=1e-13)
    assert np.allclose(app_attn(q, K, V, deg, scale=1 / math.sqrt(8)), app_attn(q, K, V, deg), atol=1e-15)
