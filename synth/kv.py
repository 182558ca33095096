"""Seeded generators for sequence-correlated keys, i.i.d. values and queries.

Keys follow a first-order autoregressive process along the sequence, one
independent process per channel:  k_0 ~ N(0,1),  k_t = alpha*k_{t-1} +
sqrt(1-alpha^2)*N(0,1).  Neighbouring keys are then highly similar and the
expected cosine similarity decays convexly with distance (about alpha**dist),
which is the structure the clustering method relies on.  A few "outlier"
channels can be scaled up after the recursion, as real key caches show.
Values and queries are i.i.d. N(0,1).

Two back ends produce the same process (not the same random stream):
  * host: numpy PCG64, literal recursion, for sizes an fp64 CPU check can take;
  * device: torch's generator on the GPU, recursion unrolled into log2(W)
    shift-and-add passes (the impulse response alpha**j is below 1e-9 after W
    steps, so W warm-up samples are drawn and dropped), for multi-GiB caches.
Everything returned is already rounded to the storage dtype.
"""
from __future__ import annotations

import math

import numpy as np
import torch
from scipy.signal import lfilter

_DTYPES = {"f32": torch.float32, "bf16": torch.bfloat16}


def head_seed(seed: int, layer: int, head: int) -> int:
    """A 63-bit seed for one (layer, KV head) stream."""
    ss = np.random.SeedSequence([int(seed), int(layer), int(head)])
    return int(ss.generate_state(1, dtype=np.uint64)[0] >> np.uint64(1))


def to_storage(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float64 numpy -> torch tensor in the storage dtype (round-to-nearest-even)."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(_DTYPES[dtype])


def ar1_keys_host(rng: np.random.Generator, s: int, d: int, alpha: float,
                  n_outlier: int = 0, outlier_scale: float = 10.0) -> np.ndarray:
    """[s, d] float64 keys.  Draw order: k_0 (d), noise (s-1, d) row-major,
    then the outlier channel indices (if any)."""
    k0 = rng.standard_normal(d)
    noise = rng.standard_normal((max(s - 1, 0), d))
    x = np.concatenate([k0[None, :], math.sqrt(1.0 - alpha * alpha) * noise], axis=0)
    k = lfilter([1.0], [1.0, -alpha], x, axis=0)      # k[t] = x[t] + alpha*k[t-1]
    if n_outlier:
        ch = rng.choice(d, size=n_outlier, replace=False)
        k[:, ch] *= outlier_scale
    return k


def kv_host(seed: int, heads: int, s: int, d: int, dtype: str, alpha: float = 0.9,
            n_outlier: int = 0, layer: int = 0, single_stream: bool = False):
    """K, V as torch CPU tensors [1, heads, s, d] in the storage dtype.

    single_stream=True draws everything from one PCG64(seed) stream (keys, then
    values), and returns that generator so a query can be drawn next from it;
    otherwise every head has its own stream seeded by head_seed().
    """
    K = np.empty((1, heads, s, d))
    V = np.empty((1, heads, s, d))
    rng = np.random.Generator(np.random.PCG64(seed)) if single_stream else None
    for h in range(heads):
        g = rng if single_stream else np.random.Generator(np.random.PCG64(head_seed(seed, layer, h)))
        K[0, h] = ar1_keys_host(g, s, d, alpha, n_outlier)
        V[0, h] = g.standard_normal((s, d))
    return to_storage(K, dtype), to_storage(V, dtype), rng


def prototype_kv_host(seed: int, heads: int, s: int, d: int, dtype: str, n_proto: int, noise: float = 0.02):
    """K, V as torch CPU tensors [1, heads, s, d]: every key is one of n_proto random directions
    (drawn per head) plus a little noise, so that many tokens pick the same partner and clusters
    grow long.  Draw order per head: the directions (n_proto, d), the choice per token (s), the
    key noise (s, d), the values (s, d)."""
    K = np.empty((1, heads, s, d))
    V = np.empty((1, heads, s, d))
    for h in range(heads):
        g = np.random.Generator(np.random.PCG64(head_seed(seed, 0, h)))
        proto = g.standard_normal((n_proto, d))
        pick = g.integers(0, n_proto, s)
        K[0, h] = proto[pick] + noise * g.standard_normal((s, d))
        V[0, h] = g.standard_normal((s, d))
    return to_storage(K, dtype), to_storage(V, dtype)


def query_host(rng_or_seed, batch: int, q_heads: int, d: int, dtype: str) -> torch.Tensor:
    """[batch, q_heads, d] i.i.d. N(0,1) queries in the storage dtype."""
    g = rng_or_seed if isinstance(rng_or_seed, np.random.Generator) else \
        np.random.Generator(np.random.PCG64(int(rng_or_seed)))
    return to_storage(g.standard_normal((batch, q_heads, d)), dtype)


def _warmup(alpha: float) -> int:
    need = math.log(1e-9) / math.log(alpha)
    return 1 << max(1, math.ceil(math.log2(need)))


def kv_device(seed: int, heads: int, s: int, d: int, dtype: str, alpha: float = 0.9,
              n_outlier: int = 0, layer: int = 0, device: str = "cuda",
              out_k: torch.Tensor | None = None, out_v: torch.Tensor | None = None):
    """K, V on `device`, [heads, s, d] in the storage dtype (one layer).

    Per (layer, head) the stream is torch's device generator seeded with
    head_seed().  If out_k / out_v are given the result is written there.
    """
    tdt = _DTYPES[dtype]
    K = out_k if out_k is not None else torch.empty((heads, s, d), dtype=tdt, device=device)
    V = out_v if out_v is not None else torch.empty((heads, s, d), dtype=tdt, device=device)
    W = _warmup(alpha)
    sigma = math.sqrt(1.0 - alpha * alpha)
    gen = torch.Generator(device=device)
    for h in range(heads):
        gen.manual_seed(head_seed(seed, layer, h))
        x = torch.randn((W + s, d), generator=gen, device=device, dtype=torch.float32) * sigma
        step = 1
        while step < W:                      # x_t <- sum_{j < 2*step} alpha^j e_{t-j}
            y = x.clone()
            y[step:] += (alpha ** step) * x[:-step]
            x = y
            step *= 2
        x = x[W:]
        if n_outlier:
            ch = torch.randperm(d, generator=gen, device=device)[:n_outlier]
            x[:, ch] *= 10.0
        K[h].copy_(x)
        V[h].copy_(torch.randn((s, d), generator=gen, device=device, dtype=torch.float32))
    return K, V
