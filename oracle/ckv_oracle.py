"""CPU oracle for CentroidKV's hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the path computes, written from the
paper (arXiv 2506.11418): one clustering round of Chunked Soft Matching
(Sec. 5.2) with the degree-weighted merge (Sec. 5.3, centroid equation), the
multi-round loop that compresses until the budget is met (Algorithm 1, prefill
part), and approximate attention over centroids (Eq. 3).  Nothing here is
tiled, fused or reordered, it shares no code with the HIP library and imports
nothing from it; only tests, the smoke check and the benchmark's cpu_baseline
leg may call it.  The product path never does.

The method is a greedy heuristic, so the oracle is the algorithm itself taken
step by step; only attention has a closed definition, and it is that
definition.  Readings where the paper is silent (tie-breaks, floor of the merge
count, output order, per-chunk selection, schedule for a retain ratio) are
stated where they are taken; each function names the passage it follows.

Pins (tests/test_oracle_*.py): Theorem A.1 by brute force and the closed form
c_{2n,l} printed in its proof (partition); unit self-similarity, scale
invariance and a normalise-then-matmul library check (similarity); exhaustive
enumeration on chunks of <= 8 tokens (matching + selection); mass
conservation, lossless merge of duplicated keys and scatter-mean from the
assignment map (merge); textbook softmax attention at degree 1, the q = 0 mean
and exactness on duplicate-key clusters (attention); the paper's KV-cache size
column (budget arithmetic); sink / recent tokens bit-identical, the middle equal
to a round on the slice alone (sinks and recents); the retained fractions
0.6, 0.42, 0.336, 0.3024 of the annealed schedule at its defaults, and
Algorithm 1's decode loop against plain attention over the whole uncompressed
history on caches made of runs of identical tokens (online loop).  Parity
unpinned: the POLICY that picks r for a decode-time clustering call and the
floor that lets the annealed loop reach its budget are readings, not facts of
the paper (the arithmetic for a given r is pinned).  Selection over all chunks
of a sequence (scope "head") is pinned by exhaustive search over merge sets on
tiny inputs, by its agreement with the per-chunk rule at r = 1 and on a single
chunk, and by the dominance of every kept edge over every dropped one.
"""
from __future__ import annotations

import math

import numpy as np

TAU = 1e-5          # score gaps below this are reported as near-ties


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the cache's storage type, nearest-even, in ONE
    rounding step (no detour through fp32 for bf16).  Returns fp64 holding
    exactly representable values.  bf16: 8 significant bits, fp32 exponent range.
    """
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype != "bf16":
        raise ValueError(dtype)
    _, e = np.frexp(x)                       # x = m * 2**e, 0.5 <= |m| < 1
    q = np.maximum(e - 1, -126) - 7          # exponent of one unit in the last place
    y = np.ldexp(np.rint(np.ldexp(x, -q)), q)   # np.rint rounds half to even
    return np.where(np.isfinite(x), y, x)


# --------------------------------------------------------------------------
# Sec. 5.2: chunking, alternating partition, similarity, matching
# --------------------------------------------------------------------------
def chunk_bounds(s: int, c: int):
    """Chunks of c consecutive tokens; the last one may be shorter (Sec. 5.2)."""
    return [(g0, min(g0 + c, s)) for g0 in range(0, s, c)]


def alternating_partition(L: int):
    """Offsets of set A (1st, 3rd, 5th ... token) and set B (2nd, 4th, ...) in a
    chunk of L tokens: Theorem A.1's (A_0, B_0), written 0-based (Sec. 5.2)."""
    return np.arange(0, L, 2), np.arange(1, L, 2)


def cosine_similarity(KA: np.ndarray, KB: np.ndarray) -> np.ndarray:
    """S[i, j] = k_i . k_j / (|k_i| |k_j|)  (Eq. 2).  A zero key has similarity 0."""
    na = np.sqrt(np.sum(KA * KA, axis=1))
    nb = np.sqrt(np.sum(KB * KB, axis=1))
    inv_a = 1.0 / np.maximum(na, 1e-30)
    inv_b = 1.0 / np.maximum(nb, 1e-30)
    return (KA @ KB.T) * inv_a[:, None] * inv_b[None, :]


def match(K: np.ndarray, c: int, tau: float = TAU):
    """For every A token draw the edge to its most similar B token of the same
    chunk (Sec. 5.2, the soft-matching step).  Lowest B index wins ties.

    Returns, over all A tokens of the sequence in ascending position:
      src[i]  position of the A token,  dst[i] position of its B partner (-1 if
      the chunk has no B token),  score[i] the similarity of that edge,
      near_tie[i]  True when best and second-best differ by less than tau.
    """
    src, dst, score, near = [], [], [], []
    if K.shape[0] == 0:
        e = np.zeros(0, dtype=np.int64)
        return e, e.copy(), np.zeros(0), np.zeros(0, dtype=bool)
    for g0, g1 in chunk_bounds(K.shape[0], c):
        a_off, b_off = alternating_partition(g1 - g0)
        if len(b_off) == 0:
            src.append(g0 + a_off)
            dst.append(np.full(len(a_off), -1))
            score.append(np.zeros(len(a_off)))
            near.append(np.zeros(len(a_off), dtype=bool))
            continue
        S = cosine_similarity(K[g0 + a_off], K[g0 + b_off])
        j = np.argmax(S, axis=1)                       # first maximum = lowest index
        best = S[np.arange(len(a_off)), j]
        if S.shape[1] > 1:
            S2 = S.copy()
            S2[np.arange(len(a_off)), j] = -np.inf
            gap = best - S2.max(axis=1)
        else:
            gap = np.full(len(a_off), np.inf)
        src.append(g0 + a_off)
        dst.append(g0 + b_off[j])
        score.append(best)
        near.append(gap < tau)
    return (np.concatenate(src), np.concatenate(dst), np.concatenate(score), np.concatenate(near))


def merge_count(r: float, n_a: int) -> int:
    """Number of edges merged in a chunk with n_a candidate edges: floor(r*n_a).
    r is carried as float32 (as the C interface does) and widened; the 1e-9
    guard makes products such as 0.5*512 exact (Sec. 5.3, top-r)."""
    return int(math.floor(float(np.float32(r)) * n_a + 1e-9))


def select(src, dst, score, s: int, c: int, r: float, tau: float = TAU):
    """Keep, per chunk, the m = floor(r * |A|) highest-scoring edges; ties go to
    the lower A index (Sec. 5.3, top-r selection).  Returns the
    keep mask and the list of chunks whose cut falls inside a near-tie."""
    keep = np.zeros(len(src), dtype=bool)
    cut_ties = []
    chunk_of = src // c
    for g, (g0, g1) in enumerate(chunk_bounds(s, c)):
        idx = np.nonzero(chunk_of == g)[0]
        if len(idx) == 0 or dst[idx[0]] < 0:
            continue
        m = merge_count(r, len(idx))
        order = idx[np.lexsort((idx, -score[idx]))]    # score descending, index ascending
        keep[order[:m]] = True
        if 0 < m < len(idx) and score[order[m - 1]] - score[order[m]] < tau:
            cut_ties.append(g)
    return keep, cut_ties


def select_global(src, dst, score, r: float, tau: float = TAU):
    """The other reading of Sec. 5.2-5.3 (edges collected over all chunks, one ranking): the
    edges of ALL chunks of the sequence are ranked together and the
    m = floor(r * number of edges) best are merged; ties go to the lower A position.  Returns the
    keep mask and (cut score, True when the first dropped edge is within tau of it)."""
    keep = np.zeros(len(src), dtype=bool)
    idx = np.nonzero(np.asarray(dst) >= 0)[0]
    m = merge_count(r, len(idx))
    if m == 0:
        return keep, (np.inf, False)
    order = idx[np.lexsort((idx, -score[idx]))]        # score descending, position ascending
    keep[order[:m]] = True
    cut = float(score[order[m - 1]])
    near = m < len(idx) and cut - float(score[order[m]]) < tau
    return keep, (cut, bool(near))


# --------------------------------------------------------------------------
# Sec. 5.3: degree-weighted merge, order-preserving output
# --------------------------------------------------------------------------
def merge(K, V, deg, src, dst, keep, dtype: str):
    """Merge every kept A token into its B partner with degree weights
    (centroid equation of Sec. 5.3; values with the same weights), leave the rest
    unchanged, and emit the retained tokens in their original order.

    Returns K', V' (rounded to the storage type, as fp64), deg', the round's
    assignment map (input position -> output index) and the unrounded K', V'.
    """
    s = K.shape[0]
    wK = K * deg[:, None].astype(np.float64)
    wV = V * deg[:, None].astype(np.float64)
    new_deg = deg.astype(np.int64).copy()
    merged_away = np.zeros(s, dtype=bool)
    for i in np.nonzero(keep)[0]:                      # ascending A position
        a, b = src[i], dst[i]
        wK[b] += K[a] * float(deg[a])
        wV[b] += V[a] * float(deg[a])
        new_deg[b] += deg[a]
        merged_away[a] = True
    retained = np.nonzero(~merged_away)[0]
    out_index = np.cumsum(~merged_away) - 1            # valid on retained positions
    assign = out_index.copy()
    for i in np.nonzero(keep)[0]:
        assign[src[i]] = out_index[dst[i]]
    Kc = wK[retained] / new_deg[retained, None]
    Vc = wV[retained] / new_deg[retained, None]
    # tokens that took part in no merge are passed through bit-for-bit
    untouched = new_deg[retained] == deg[retained]
    Kc[untouched] = K[retained][untouched]
    Vc[untouched] = V[retained][untouched]
    return (round_to_storage(Kc, dtype), round_to_storage(Vc, dtype),
            new_deg[retained].astype(np.int64), assign.astype(np.int64), Kc, Vc)


def clusterable_range(s: int, n_sink: int, n_recent: int):
    """The first n_sink and the last n_recent tokens are kept out of the clustering (Sec. 5.2:
    sinks and recent tokens are set aside before partitioning); chunks start right after the
    sinks.  A cache no longer than n_sink + n_recent has nothing to cluster."""
    if s <= n_sink + n_recent:
        return 0, 0
    return n_sink, s - n_recent


def csm_round(K, V, deg, c: int, r: float, dtype: str, tau: float = TAU, n_sink: int = 0, n_recent: int = 0,
              scope: str = "chunk"):
    """One clustering round on one (layer, KV head) sequence: set sinks / recents aside, chunk
    the rest, alternating partition, cosine similarity, per-A argmax edge, top-r (per chunk, or
    over all chunks of the sequence when scope == "head"), merge, and put the result back
    between the untouched sinks and recents (Sec. 5.2 + 5.3).
    K, V: [s, d] fp64 holding storage-type values.  cut_ties: the chunks whose cut falls in a
    near-tie (scope "chunk"), or (cut score, near-tie flag) of the one cut (scope "head")."""
    lo, hi = clusterable_range(K.shape[0], n_sink, n_recent)
    src, dst, score, near = match(K[lo:hi], c, tau)
    if scope == "head":
        keep, cut_ties = select_global(src, dst, score, r, tau)
    elif scope == "chunk":
        keep, cut_ties = select(src, dst, score, hi - lo, c, r, tau)
    else:
        raise ValueError(scope)
    src = src + lo
    dst = np.where(dst >= 0, dst + lo, dst)
    Ko, Vo, dego, assign, Kx, Vx = merge(K, V, deg, src, dst, keep, dtype)
    return dict(K=Ko, V=Vo, deg=dego, assign=assign, src=src, dst=dst, score=score,
                keep=keep, near_tie=near, cut_ties=cut_ties, K_exact=Kx, V_exact=Vx)


# --------------------------------------------------------------------------
# Algorithm 1 (prefill part): rounds until the budget is met
# --------------------------------------------------------------------------
def direct_schedule(retain_ratio: float):
    """Per-round merge fractions that land exactly on a retained fraction rho.
    A round removes at most half (Sec. 5.1), so J = ceil(log2(1/rho)) rounds are
    needed: J-1 full rounds (r = 1) and a last one with r = 2(1 - rho*2^(J-1))."""
    rho = float(np.float32(retain_ratio))
    if not (0.0 < rho <= 1.0):
        raise ValueError("retain_ratio must be in (0, 1]")
    J = 0
    while 0.5 ** J > rho * (1.0 + 1e-6):
        J += 1
    if J == 0:
        return []
    return [1.0] * (J - 1) + [2.0 * (1.0 - rho * 2.0 ** (J - 1))]


def round_lengths(s: int, c: int, rounds, n_sink: int = 0, n_recent: int = 0, scope: str = "chunk"):
    """Sequence length after each round (pure integer arithmetic)."""
    out = [s]
    for r in rounds:
        lo, hi = clusterable_range(out[-1], n_sink, n_recent)
        n = out[-1] - (hi - lo)
        edges = 0
        for g0, g1 in chunk_bounds(hi - lo, c):
            L = g1 - g0
            n_a, n_b = (L + 1) // 2, L // 2
            if scope == "chunk":
                n += L - (merge_count(r, n_a) if n_b > 0 else 0)
            else:
                n += L
                edges += n_a if n_b > 0 else 0
        if scope != "chunk":
            n -= merge_count(r, edges)
        out.append(n)
    return out


def compress(K, V, c: int, rounds, dtype: str, deg=None, tau: float = TAU, n_sink: int = 0, n_recent: int = 0,
             scope: str = "chunk"):
    """Repeat csm_round on the CURRENT cache with the same chunk size
    (Algorithm 1, the while-loop after prefill).  Degrees start at 1 and
    accumulate; the assignment maps compose.  Each round's rounded output is
    the next round's input."""
    s = K.shape[0]
    deg = np.ones(s, dtype=np.int64) if deg is None else np.asarray(deg, dtype=np.int64)
    assign = np.arange(s, dtype=np.int64)
    per_round = []
    for r in rounds:
        res = csm_round(K, V, deg, c, r, dtype, tau, n_sink, n_recent, scope)
        K, V, deg = res["K"], res["V"], res["deg"]
        assign = res["assign"][assign]
        per_round.append(res)
    return dict(K=K, V=V, deg=deg, assign=assign, rounds=per_round)


# --------------------------------------------------------------------------
# Eq. 3: attention over centroids
# --------------------------------------------------------------------------
def app_attn(q, K, V, deg=None, length=None, scale=None):
    """o_h = softmax(q_h K^T / sqrt(d) + log N) V  per query head (Eq. 3;
    Algorithm 1's decode line).  q: [Hq, d]; K, V: [Hkv, L, d]; deg: [Hkv, L]
    or None (all ones: Eq. 1).  Query head h reads KV head h // (Hq // Hkv).
    Only the first `length` tokens are attended; length 0 gives zeros."""
    q = np.asarray(q, dtype=np.float64)
    Hq, d = q.shape
    Hkv, L, _ = K.shape
    G = Hq // Hkv
    n = L if length is None else int(length)
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    o = np.zeros((Hq, d))
    if n == 0:
        return o
    for h in range(Hq):
        kv = h // G
        z = (K[kv, :n] @ q[h]) * scale
        if deg is not None:
            z = z + np.log(deg[kv, :n].astype(np.float64))
        p = np.exp(z - z.max())
        o[h] = (p @ V[kv, :n]) / p.sum()
    return o


# --------------------------------------------------------------------------
# Eq. 4 and Algorithm 1: annealed schedule, budget loop, online decoding
# --------------------------------------------------------------------------
def annealed_ratio(j: int, r_init: float, delta_r: float, r_floor: float = 0.0) -> float:
    """Merge fraction of clustering round j (Eq. 4): r_init - j*delta_r, never
    below r_floor (the paper gives no floor; 0 reproduces the formula as
    printed).  Returned as the float32 value the parameters carry."""
    return float(np.float32(max(r_init - j * delta_r, r_floor)))


def rounds_to_budget(s: int, c: int, budget: int, r_init: float, delta_r: float, r_floor: float = 0.0,
                     n_sink: int = 0, n_recent: int = 0, max_rounds: int = 8):
    """The loop after prefill of Algorithm 1 on lengths alone: cluster with
    r_0, r_1, ... (Eq. 4) while the cache is longer than the budget.  Returns
    the list of merge fractions used.  Raises when a round removes nothing
    while s > budget (the schedule has run dry) or max_rounds is exceeded."""
    rounds = []
    while s > budget:
        if len(rounds) == max_rounds:
            raise ValueError("budget not reached within max_rounds")
        r = annealed_ratio(len(rounds), r_init, delta_r, r_floor)
        nxt = round_lengths(s, c, [r], n_sink, n_recent)[-1]
        if nxt == s:
            raise ValueError("the schedule stalls above the budget")
        rounds.append(r)
        s = nxt
    return rounds


def alg1_decode(K, V, deg, qs, ks, vs, c: int, budget: int, g: int, r_calls, dtype: str,
                n_sink: int = 0, n_recent: int = 0, tau: float = TAU):
    """Decoding part of Algorithm 1 for one layer.  K, V: [Hkv, s, d] and deg:
    [Hkv, s], the cache after prefill (and its first clustering); step i
    appends (ks[i], vs[i]) with degree 1 to every KV head, attends with
    qs[i] over the whole cache (Eq. 3), then, if the cache has reached
    budget + g tokens, runs ONE clustering round with the next merge
    fraction of r_calls (a list, consumed in order; the last entry repeats).
    Returns (outputs [steps, Hq, d], K, V, deg, steps at which a round ran)."""
    K = [np.array(K[h], dtype=np.float64) for h in range(len(K))]
    V = [np.array(V[h], dtype=np.float64) for h in range(len(V))]
    deg = [np.array(deg[h], dtype=np.int64) for h in range(len(deg))]
    outs, ran = [], []
    for i in range(len(qs)):
        for h in range(len(K)):
            K[h] = np.concatenate([K[h], np.asarray(ks[i][h], dtype=np.float64)[None]], axis=0)
            V[h] = np.concatenate([V[h], np.asarray(vs[i][h], dtype=np.float64)[None]], axis=0)
            deg[h] = np.concatenate([deg[h], np.ones(1, dtype=np.int64)])
        outs.append(app_attn(qs[i], np.stack(K), np.stack(V), np.stack(deg)))
        if K[0].shape[0] >= budget + g:
            r = r_calls[min(len(ran), len(r_calls) - 1)]
            for h in range(len(K)):
                res = csm_round(K[h], V[h], deg[h], c, r, dtype, tau, n_sink, n_recent)
                K[h], V[h], deg[h] = res["K"], res["V"], res["deg"]
            ran.append(i)
    return np.stack(outs), np.stack(K), np.stack(V), np.stack(deg), ran
