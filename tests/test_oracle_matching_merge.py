"""Pins for the oracle's matching, top-r selection, merge and rounds driver (CPU only)."""
import itertools

import numpy as np
import torch

from oracle import (compress, csm_round, direct_schedule, match, merge_count, round_lengths, select)
from synth import ar1_keys_host


def _kv(seed, s, d, alpha=0.9):
    rng = np.random.Generator(np.random.PCG64(seed))
    return ar1_keys_host(rng, s, d, alpha), rng.standard_normal((s, d))


def _cos(a, b):
    return float(np.dot(a, b) / (np.linalg.norm(a) * np.linalg.norm(b)))


# ---- exhaustive enumeration on tiny chunks --------------------------------
def test_matching_is_the_exhaustive_optimum_on_tiny_chunks():
    """Over every subset of m A-tokens and every map of that subset into B, the
    total similarity is maximal for the oracle's (kept set, partners), and the
    maximiser is unique when nothing is flagged as a near-tie."""
    checked = 0
    for L in (2, 3, 4, 5, 6, 7, 8):
        for r in (1.0, 0.75, 0.5, 0.25):
            for seed in range(6):
                K, V = _kv(100 * L + seed, L, 8)
                res = csm_round(K, V, np.ones(L, dtype=np.int64), L, r, "f32")
                A = list(range(0, L, 2))
                B = list(range(1, L, 2))
                m = merge_count(r, len(A))
                assert res["keep"].sum() == m
                S = {(a, b): _cos(K[a], K[b]) for a in A for b in B}
                best, arg, n_best = -np.inf, None, 0
                for T in itertools.combinations(A, m):
                    for phi in itertools.product(B, repeat=m):
                        tot = sum(S[(a, b)] for a, b in zip(T, phi))
                        if tot > best + 1e-12:
                            best, arg, n_best = tot, (T, phi), 1
                        elif abs(tot - best) <= 1e-12:
                            n_best += 1
                kept = np.nonzero(res["keep"])[0]
                got_T = tuple(int(res["src"][i]) for i in kept)
                got_phi = tuple(int(res["dst"][i]) for i in kept)
                got = sum(S[(a, b)] for a, b in zip(got_T, got_phi))
                assert abs(got - best) < 1e-12
                if not res["near_tie"].any() and not res["cut_ties"] and n_best == 1:
                    assert (got_T, got_phi) == arg
                    checked += 1
    assert checked > 100


def test_every_a_token_points_to_its_most_similar_b_token_of_its_own_chunk():
    K, _ = _kv(7, 50, 16)
    c = 12                                           # 4 full chunks + a tail of 2
    src, dst, score, near = match(K, c)
    assert list(src) == [t for t in range(50) if (t % c) % 2 == 0]
    for a, b, sc in zip(src, dst, score):
        g0 = (a // c) * c
        cand = [t for t in range(g0, min(g0 + c, 50)) if (t - g0) % 2 == 1]
        sims = [_cos(K[a], K[t]) for t in cand]
        assert b == cand[int(np.argmax(sims))]
        assert abs(sc - max(sims)) < 1e-13


def test_ties_go_to_the_lowest_index():
    K = np.tile(np.array([[1.0, 2.0, -1.0, 0.5]]), (8, 1))          # all keys identical
    V = np.arange(32, dtype=np.float64).reshape(8, 4)
    res = csm_round(K, V, np.ones(8, dtype=np.int64), 8, 0.5, "f32")
    assert np.all(res["dst"] == 1)                                   # first B token
    assert list(np.nonzero(res["keep"])[0]) == [0, 1]                # lowest A indices kept
    assert res["near_tie"].all() and res["cut_ties"] == [0]


# ---- counts ----------------------------------------------------------------
def test_retained_count_per_chunk_and_half_bound():
    for s, c, r in [(64, 16, 1.0), (64, 16, 0.5), (70, 16, 0.3), (33, 8, 0.8), (5, 8, 1.0), (1, 4, 1.0)]:
        K, V = _kv(s + c, s, 8)
        res = csm_round(K, V, np.ones(s, dtype=np.int64), c, r, "f32")
        exp = 0
        for g0 in range(0, s, c):
            L = min(c, s - g0)
            n_a, n_b = (L + 1) // 2, L // 2
            m = merge_count(r, n_a) if n_b else 0
            exp += L - m
            in_chunk = (res["src"] // c) == (g0 // c)
            assert res["keep"][in_chunk].sum() == m
            assert L - n_a <= L - m <= L                              # at most half removed
        assert len(res["K"]) == exp == round_lengths(s, c, [r])[1]


def test_merge_count_floor():
    assert merge_count(0.5, 512) == 256 and merge_count(0.25, 512) == 128
    assert merge_count(1.0, 7) == 7 and merge_count(0.0, 7) == 0
    assert merge_count(0.8, 32) == 25 and merge_count(0.3, 5) == 1


# ---- merge: conservation, duplicates, identity -----------------------------
def test_mass_conservation_and_degree_sum():
    s, c = 96, 32
    K, V = _kv(11, s, 16)
    deg = np.random.default_rng(0).integers(1, 5, s)
    res = csm_round(K, V, deg, c, 0.75, "f32")
    for g0 in range(0, s, c):
        sel_in = slice(g0, g0 + c)
        out_idx = np.unique(res["assign"][sel_in])
        assert np.allclose((res["K_exact"][out_idx] * res["deg"][out_idx, None]).sum(0),
                           (K[sel_in] * deg[sel_in, None]).sum(0), atol=1e-11)
        assert np.allclose((res["V_exact"][out_idx] * res["deg"][out_idx, None]).sum(0),
                           (V[sel_in] * deg[sel_in, None]).sum(0), atol=1e-11)
        assert res["deg"][out_idx].sum() == deg[sel_in].sum()


def test_duplicate_keys_merge_losslessly():
    k = np.array([0.5, -1.25, 2.0, 0.75])
    K = np.tile(k, (16, 1))
    V = np.random.default_rng(1).standard_normal((16, 4))
    res = csm_round(K, V, np.ones(16, dtype=np.int64), 8, 1.0, "f32")
    assert np.array_equal(res["K"], np.tile(k, (len(res["K"]), 1)))   # every centroid key == the key
    # per chunk all four A tokens join the first B token: degrees 5,1,1,1
    assert list(res["deg"]) == [5, 1, 1, 1, 5, 1, 1, 1]
    assert np.allclose(res["V_exact"][0], V[[0, 1, 2, 4, 6]].mean(0), atol=1e-14)


def test_r_zero_is_identity():
    K, V = _kv(3, 40, 8)
    K = K.astype(np.float32).astype(np.float64)
    V = V.astype(np.float32).astype(np.float64)
    res = csm_round(K, V, np.ones(40, dtype=np.int64), 16, 0.0, "f32")
    assert np.array_equal(res["K"], K) and np.array_equal(res["V"], V)
    assert list(res["assign"]) == list(range(40))


def test_degree_weights_hand_example():
    # chunk of 2 tokens: A = token 0 (degree 3), B = token 1 (degree 1), merged at r = 1
    K = np.array([[2.0, 0.0], [4.0, 0.0]])
    V = np.array([[1.0, 1.0], [5.0, -3.0]])
    res = csm_round(K, V, np.array([3, 1]), 2, 1.0, "f32")
    assert np.array_equal(res["K"], [[(3 * 2 + 4) / 4, 0.0]])
    assert np.array_equal(res["V"], [[(3 * 1 + 5) / 4, (3 * 1 - 3) / 4]])
    assert list(res["deg"]) == [4] and list(res["assign"]) == [0, 0]


# ---- assignment map --------------------------------------------------------
def test_assign_properties_and_scatter_mean():
    s, c = 128, 32
    K, V = _kv(21, s, 16)
    K = K.astype(np.float32).astype(np.float64)
    res = csm_round(K, V, np.ones(s, dtype=np.int64), c, 0.5, "f32")
    a, n_out = res["assign"], len(res["K"])
    assert a.min() == 0 and a.max() == n_out - 1
    assert np.array_equal(np.bincount(a, minlength=n_out), res["deg"])
    merged = np.zeros(s, dtype=bool)
    merged[res["src"][res["keep"]]] = True
    assert np.all(np.diff(a[~merged]) == 1)          # retained tokens keep their order
    # centroids are the plain mean of their members (degree-1 inputs)
    for t in range(n_out):
        assert np.allclose(res["K_exact"][t], K[a == t].mean(0), atol=1e-13)
        assert np.allclose(res["V_exact"][t], V[a == t].mean(0), atol=1e-13)
    # B tokens are always retained; a merged A token shares its partner's slot
    for i in np.nonzero(res["keep"])[0]:
        assert a[res["src"][i]] == a[res["dst"][i]]


def test_two_rounds_compose_to_the_plain_mean():
    s, c = 256, 32
    K, V = _kv(22, s, 16)
    out = compress(K, V, c, [1.0, 0.5], "f32")
    a = out["assign"]
    assert len(out["K"]) == round_lengths(s, c, [1.0, 0.5])[-1] == 96
    assert np.array_equal(np.bincount(a), out["deg"])
    for t in range(len(out["K"])):
        # degree-weighted means of means = mean over all members (up to fp32 storage of round 0)
        assert np.allclose(out["V"][t], V[a == t].mean(0), atol=2e-6)
    # round 1 re-chunks the CURRENT cache: its chunk g covers round-0 outputs [32g, 32g+32)
    r1 = out["rounds"][1]
    assert np.all(r1["src"] // c == r1["dst"] // c)


# ---- whole-sequence chunk = plain bipartite soft matching -------------------
def test_chunk_covering_the_sequence_equals_plain_bsm():
    """With c >= s one round is bipartite soft matching over the whole sequence
    (the 'w/o chunk' ablation).  Cross-check against an independent formulation
    built from library ops (normalise, matmul, max, sort, index_add)."""
    s, d, r = 60, 16, 0.6
    K, V = _kv(31, s, d)
    res = csm_round(K, V, np.ones(s, dtype=np.int64), 4096, r, "f32")
    Kt, Vt = torch.from_numpy(K), torch.from_numpy(V)
    a, b = Kt[0::2], Kt[1::2]
    sim = torch.nn.functional.normalize(a, dim=-1) @ torch.nn.functional.normalize(b, dim=-1).T
    best, node = sim.max(dim=-1)
    order = torch.argsort(best, descending=True, stable=True)
    m = int(r * a.shape[0] + 1e-9)
    merged_src = order[:m]
    sumK, sumV, cnt = b.clone(), Vt[1::2].clone(), torch.ones(b.shape[0], dtype=torch.float64)
    sumK.index_add_(0, node[merged_src], a[merged_src])
    sumV.index_add_(0, node[merged_src], Vt[0::2][merged_src])
    cnt.index_add_(0, node[merged_src], torch.ones(m, dtype=torch.float64))
    keepA = torch.ones(a.shape[0], dtype=torch.bool)
    keepA[merged_src] = False
    pos = torch.cat([torch.arange(0, s, 2)[keepA], torch.arange(1, s, 2)])
    rows = torch.cat([a[keepA], sumK / cnt[:, None]])
    rowsV = torch.cat([Vt[0::2][keepA], sumV / cnt[:, None]])
    o = torch.argsort(pos)                            # the oracle keeps sequence order
    assert np.allclose(res["K_exact"], rows[o].numpy(), atol=1e-13)
    assert np.allclose(res["V_exact"], rowsV[o].numpy(), atol=1e-13)


# ---- schedule and budget arithmetic ----------------------------------------
def test_direct_schedule():
    assert direct_schedule(1.0) == []
    assert direct_schedule(0.5) == [1.0]
    assert direct_schedule(0.25) == [1.0, 1.0]
    assert direct_schedule(0.75) == [0.5]
    assert direct_schedule(0.375) == [1.0, 0.5]
    assert direct_schedule(0.125) == [1.0, 1.0, 1.0]
    for rho, s, c in [(0.75, 4096, 256), (0.375, 4096, 256), (0.25, 32768, 1024), (0.3, 5120, 512)]:
        got = round_lengths(s, c, direct_schedule(rho))[-1]
        assert abs(got - rho * s) <= s // c + 1       # floor per chunk


def test_budget_reproduces_the_papers_kv_cache_column(golden_dir):
    """B = R*n (Algorithm 1): with the 25% budget the compressed cache plus 1K
    decoded tokens has the size the paper's table prints."""
    per_token = 32 * 8 * 128 * 2 * 2                  # layers x kv heads x dim x (K,V) x bf16
    for line in open(f"{golden_dir}/kv_cache_gib.txt"):
        if line.startswith("#") or not line.strip():
            continue
        n, full, comp = line.split()
        n = int(n)
        out = round_lengths(n, 256, direct_schedule(0.25))[-1]
        assert out == n // 4
        assert abs((n + 1024) * per_token / 2 ** 30 - float(full)) < 0.01           # printed to two decimals
        assert abs((out + 1024) * per_token / 2 ** 30 - float(comp)) < 0.01           # printed to two decimals


# ---- attention sinks and recent tokens (Sec. 5.2 / 5.3) --------------------------------------
def test_sinks_and_recents_bypass_the_clustering():
    s, c, n1, n2 = 200, 32, 5, 11
    K, V = _kv(41, s, 16)
    K = K.astype(np.float32).astype(np.float64)
    V = V.astype(np.float32).astype(np.float64)
    deg = np.random.default_rng(2).integers(1, 4, s)
    res = csm_round(K, V, deg, c, 0.75, "f32", n_sink=n1, n_recent=n2)
    n_out = len(res["K"])
    # sinks first, recents last, bit for bit, degrees untouched
    assert np.array_equal(res["K"][:n1], K[:n1]) and np.array_equal(res["V"][:n1], V[:n1])
    assert np.array_equal(res["K"][n_out - n2:], K[s - n2:]) and np.array_equal(res["V"][n_out - n2:], V[s - n2:])
    assert np.array_equal(res["deg"][:n1], deg[:n1]) and np.array_equal(res["deg"][n_out - n2:], deg[s - n2:])
    assert list(res["assign"][:n1]) == list(range(n1))
    assert list(res["assign"][s - n2:]) == list(range(n_out - n2, n_out))
    # no edge touches a sink or a recent token; chunks start right after the sinks
    assert res["src"].min() >= n1 and res["src"].max() < s - n2
    assert res["dst"].min() >= n1 and res["dst"].max() < s - n2
    assert np.all((res["src"] - n1) // c == (res["dst"] - n1) // c)
    assert res["src"][0] == n1 and (res["src"][0] - n1) % 2 == 0
    # the middle is exactly a plain round on the slice alone
    mid = csm_round(K[n1:s - n2], V[n1:s - n2], deg[n1:s - n2], c, 0.75, "f32")
    assert np.array_equal(res["K"][n1:n_out - n2], mid["K"]) and np.array_equal(res["deg"][n1:n_out - n2], mid["deg"])
    assert n_out == n1 + n2 + len(mid["K"]) == round_lengths(s, c, [0.75], n1, n2)[1]


def test_sinks_and_recents_over_rounds_and_short_caches():
    s, c, n1, n2 = 300, 64, 16, 64
    K, V = _kv(42, s, 8)
    out = compress(K, V, c, [1.0, 1.0], "f32", n_sink=n1, n_recent=n2)
    lens = round_lengths(s, c, [1.0, 1.0], n1, n2)
    assert len(out["K"]) == lens[-1] == n1 + n2 + (s - n1 - n2) // 4
    assert np.array_equal(np.bincount(out["assign"]), out["deg"])
    assert np.all(out["deg"][:n1] == 1) and np.all(out["deg"][-n2:] == 1)
    # a cache no longer than sinks + recents is returned unchanged
    short = compress(K[:70], V[:70], c, [1.0], "f32", n_sink=n1, n_recent=n2)
    assert np.array_equal(short["K"], K[:70].astype(np.float32).astype(np.float64))
    assert list(short["assign"]) == list(range(70))


# ---- selection over all chunks of a sequence (scope "head") --------------------------------
def test_global_selection_is_the_exhaustive_optimum_on_tiny_sequences():
    """Two or three tiny chunks: over every set of m A-tokens (from any chunk) and every map of
    each into a B token of ITS OWN chunk, the total similarity is maximal for the oracle's
    choice (scope "head"), uniquely so when nothing is flagged as a near-tie."""
    checked = 0
    for c, s in ((4, 8), (4, 10), (2, 6), (4, 11)):
        for r in (1.0, 0.6, 0.34):
            for seed in range(5):
                K, V = _kv(7000 + 10 * s + seed, s, 8)
                res = csm_round(K, V, np.ones(s, dtype=np.int64), c, r, "f32", scope="head")
                bounds = [(g, min(g + c, s)) for g in range(0, s, c)]
                cand = []                                     # (a, [its chunk's B tokens])
                for g0, g1 in bounds:
                    Bs = list(range(g0 + 1, g1, 2))
                    if Bs:
                        cand += [(a, Bs) for a in range(g0, g1, 2)]
                m = merge_count(r, len(cand))
                assert res["keep"].sum() == m
                best, arg, n_best = -np.inf, None, 0
                for T in itertools.combinations(cand, m):
                    for phi in itertools.product(*[Bs for _, Bs in T]):
                        tot = sum(_cos(K[a], K[b]) for (a, _), b in zip(T, phi))
                        if tot > best + 1e-12:
                            best, arg, n_best = tot, (tuple(a for a, _ in T), phi), 1
                        elif abs(tot - best) <= 1e-12:
                            n_best += 1
                kept = np.nonzero(res["keep"])[0]
                got_T = tuple(int(res["src"][i]) for i in kept)
                got_phi = tuple(int(res["dst"][i]) for i in kept)
                got = sum(_cos(K[a], K[b]) for a, b in zip(got_T, got_phi))
                assert abs(got - best) < 1e-12
                if not res["near_tie"].any() and not res["cut_ties"][1] and n_best == 1:
                    assert (got_T, got_phi) == arg
                    checked += 1
    assert checked > 40


def test_global_selection_properties():
    K, V = _kv(77, 1000, 16)
    deg = np.ones(1000, dtype=np.int64)
    # r = 1 merges every edge under both rules; one chunk covering the sequence: the rules coincide
    for c, r in ((64, 1.0), (1000, 0.4)):
        a = csm_round(K, V, deg, c, r, "f32")
        b = csm_round(K, V, deg, c, r, "f32", scope="head")
        assert np.array_equal(a["keep"], b["keep"]) and np.array_equal(a["K"], b["K"])
    # every kept edge scores at least as high as every dropped one; the count is floor(r * edges)
    res = csm_round(K, V, deg, 64, 0.3, "f32", scope="head")
    has_b = res["dst"] >= 0
    assert res["keep"].sum() == merge_count(0.3, int(has_b.sum()))
    assert res["score"][res["keep"]].min() >= res["score"][has_b & ~res["keep"]].max()
    assert res["K"].shape[0] == round_lengths(1000, 64, [0.3], scope="head")[-1] == 1000 - 150
    # per-chunk counts now differ from chunk to chunk (that is the point of the global rule)
    per_chunk = np.bincount(res["src"][res["keep"]] // 64, minlength=16)
    assert per_chunk.min() < per_chunk.max()
    # exact ties across chunks go to the lower position: identical chunks repeated
    Kt = np.tile(K[:8], (4, 1))
    res = csm_round(Kt, Kt.copy(), np.ones(32, dtype=np.int64), 8, 0.5, "f32", scope="head")
    kept_pos = res["src"][res["keep"]]
    assert len(kept_pos) == 8
    best_in_chunk = np.argsort(-res["score"][:4], kind="stable")          # chunk 0's edges, best first
    # all four copies of the best edge, then of the second best: 8 edges
    expect = sorted(int(8 * g + 2 * best_in_chunk[k]) for k in range(2) for g in range(4))
    assert sorted(kept_pos.tolist()) == expect
    # a tail chunk of a single token has no edge and is never counted
    assert round_lengths(9, 4, [1.0], scope="head") == [9, 5]
    # with sinks / recents only the middle's edges are ranked
    K = K.astype(np.float32).astype(np.float64)
    res = csm_round(K, V, deg, 64, 0.3, "f32", n_sink=10, n_recent=20, scope="head")
    assert res["K"].shape[0] == round_lengths(1000, 64, [0.3], 10, 20, scope="head")[-1]
    assert np.array_equal(res["K"][:10], K[:10]) and np.array_equal(res["K"][-20:], K[-20:])
