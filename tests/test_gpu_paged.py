"""GPU parity for block-paged caches: attention reading the pool in place, gather / scatter, and
in-place compression with block release.  Paging is pure indexing, so the expected values are the
oracle's (or the strided entry points') results on the same tokens laid out contiguously; the
test packs the pool with torch indexing."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from parity_util import ATTN_TOL, assert_rows_close, f64, i64
from synth import kv_host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def _pack(K, V, deg, lens, bs, n_blocks, seed):
    """Put [B,H,S,D] caches into a pool through a random block table (unused entries = -1, unused
    pool blocks filled with NaN so that any stray read shows)."""
    B, H, S, D = K.shape
    max_blocks = -(-S // bs) + 2
    g = torch.Generator().manual_seed(seed)
    perm = torch.randperm(n_blocks, generator=g)
    table = torch.full((B, max_blocks), -1, dtype=torch.int32)
    K_pool = torch.full((n_blocks, H, bs, D), float("nan"), dtype=K.dtype)
    V_pool = torch.full((n_blocks, H, bs, D), float("nan"), dtype=K.dtype)
    deg_pool = torch.full((n_blocks, H, bs), -7, dtype=torch.int32)
    nxt = 0
    for b in range(B):
        for i in range(-(-int(lens[b]) // bs)):
            blk = int(perm[nxt]); nxt += 1
            table[b, i] = blk
            t0, t1 = i * bs, min((i + 1) * bs, int(lens[b]))
            K_pool[blk, :, :t1 - t0] = K[b, :, t0:t1]
            V_pool[blk, :, :t1 - t0] = V[b, :, t0:t1]
            deg_pool[blk, :, :t1 - t0] = deg[b, :, t0:t1]
    return K_pool.to(DEV), V_pool.to(DEV), deg_pool.to(DEV), table.to(DEV)


@pytest.mark.parametrize("dtype,B,H,G,S,D,bs", [
    ("bf16", 3, 2, 4, 1500, 128, 16),
    ("bf16", 2, 8, 4, 4096, 128, 32),
    ("bf16", 1, 1, 8, 300, 64, 1),
    ("f32", 2, 2, 2, 700, 64, 128),
])
def test_paged_decode_attention(dtype, B, H, G, S, D, bs):
    _say(f"paged attention {dtype} B={B} H={H} G={G} S={S} D={D} block={bs}")
    K, V, _ = kv_host(91, B * H, S, D, dtype, alpha=0.9, n_outlier=4 if D == 128 else 0)
    K, V = K.reshape(B, H, S, D), V.reshape(B, H, S, D)
    rng = np.random.default_rng(5)
    deg = torch.from_numpy(rng.integers(1, 9, size=(B, H, S)).astype(np.int32))
    lens = torch.tensor([S, max(S // 3, 1), 1][:B], dtype=torch.int32)
    n_blocks = B * (-(-S // bs)) + 5
    K_pool, V_pool, deg_pool, table = _pack(K, V, deg, lens, bs, n_blocks, 17)
    q = torch.randn((B, H * G, D), generator=torch.Generator().manual_seed(3)).to(K.dtype)
    o = ckv.paged_decode_attn(q.to(DEV), K_pool, V_pool, deg_pool, table, lens.to(DEV), max_len=S,
                              out_dtype=torch.float32)
    o1 = ckv.paged_decode_attn(q.to(DEV), K_pool, V_pool, None, table, lens.to(DEV), max_len=S,
                               out_dtype=torch.float32)               # degrees NULL: plain attention
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o).all())
    for b in range(B):
        ref = oracle.app_attn(f64(q[b]), f64(K[b]), f64(V[b]), i64(deg[b]), int(lens[b]))
        assert_rows_close(f64(o[b]), ref, ATTN_TOL, f"paged b{b}")
        ref1 = oracle.app_attn(f64(q[b]), f64(K[b]), f64(V[b]), None, int(lens[b]))
        assert_rows_close(f64(o1[b]), ref1, ATTN_TOL, f"paged, no degrees, b{b}")
    # the strided entry point on the same tokens gives the same bits (same kernel arithmetic and split)
    o2 = ckv.decode_attn(q.to(DEV), K.to(DEV), V.to(DEV), lens=lens.to(DEV), deg=deg.to(DEV), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(o, o2)


def test_paged_attention_masks_table_entries_outside_the_pool():
    B, H, G, S, D, bs = 1, 2, 4, 256, 128, 16
    K, V, _ = kv_host(92, H, S, D, "bf16", alpha=0.9, n_outlier=4)
    deg = torch.ones((B, H, S), dtype=torch.int32)
    lens = torch.tensor([S], dtype=torch.int32)
    K_pool, V_pool, deg_pool, table = _pack(K, V, deg, lens, bs, 40, 1)
    table[0, 3] = 1 << 20                       # tokens 48..63 point outside the pool
    table[0, 5] = -1
    q = torch.randn((B, H * G, D), generator=torch.Generator().manual_seed(4)).to(torch.bfloat16)
    o = ckv.paged_decode_attn(q.to(DEV), K_pool, V_pool, deg_pool, table, lens.to(DEV), max_len=S, out_dtype=torch.float32)
    torch.cuda.synchronize()
    keep = np.ones(S, dtype=bool)
    keep[48:64] = False
    keep[80:96] = False
    ref = oracle.app_attn(f64(q[0]), f64(K[0][:, keep]), f64(V[0][:, keep]))
    assert_rows_close(f64(o[0]), ref, ATTN_TOL, "masked blocks")


@pytest.mark.parametrize("dtype,B,H,S,D,bs", [("bf16", 2, 4, 1000, 128, 16), ("f32", 1, 2, 333, 64, 8)])
def test_gather_and_scatter_round_trip_and_release(dtype, B, H, S, D, bs):
    _say(f"paged gather/scatter {dtype} B={B} H={H} S={S} D={D} block={bs}")
    K, V, _ = kv_host(93, B * H, S, D, dtype, alpha=0.9)
    K, V = K.reshape(B, H, S, D), V.reshape(B, H, S, D)
    deg = torch.from_numpy(np.random.default_rng(6).integers(1, 50, size=(B, H, S)).astype(np.int32))
    lens = torch.full((B,), S, dtype=torch.int32)
    n_blocks = B * (-(-S // bs)) + 3
    K_pool, V_pool, deg_pool, table = _pack(K, V, deg, lens, bs, n_blocks, 23)
    gK, gV, gdeg = ckv.paged_gather(K_pool, V_pool, deg_pool, table, S)
    torch.cuda.synchronize()
    assert torch.equal(gK.cpu(), K) and torch.equal(gV.cpu(), V) and torch.equal(gdeg.cpu(), deg)
    # write a shorter, different cache back: the sequence keeps its first blocks, the rest are released
    new = S // 3
    nK, nV = (K[:, :, :new] * 2).contiguous().to(DEV), (V[:, :, :new] * 0.5).contiguous().to(DEV)
    ndeg = (deg[:, :, :new] + 1).contiguous().to(DEV)
    table_before = table.clone()
    lens_d = lens.to(DEV)
    freed = ckv.paged_scatter(nK, nV, ndeg, K_pool, V_pool, deg_pool, table, S, lens=lens_d)
    torch.cuda.synchronize()
    keep, old = -(-new // bs), -(-S // bs)
    assert freed.shape == (B, old - keep) and torch.equal(freed, table_before[:, keep:old])
    assert torch.equal(table[:, :keep], table_before[:, :keep]) and bool((table[:, keep:] == -1).all())
    assert lens_d.tolist() == [new] * B
    rK, rV, rdeg = ckv.paged_gather(K_pool, V_pool, deg_pool, table, new)
    torch.cuda.synchronize()
    assert torch.equal(rK, nK) and torch.equal(rV, nV) and torch.equal(rdeg, ndeg)
    # a gather that runs past the kept blocks meets released (-1) entries: zero rows of degree 1
    gone = ckv.paged_gather(K_pool, V_pool, deg_pool, table, min(S, (keep + 1) * bs))    # reads past the kept blocks
    torch.cuda.synchronize()
    assert not bool(gone[0][:, :, keep * bs:].any()) and bool((gone[2][:, :, keep * bs:] == 1).all())


@pytest.mark.parametrize("seq,chunk,kw", [
    (4096 + 80, 256, dict(retain_ratio=0.25, n_sink=16, n_recent=64)),
    (3001, 512, dict(rounds=[0.8, 0.6], scope="head")),
    (2048, 1024, dict(retain_ratio=0.5)),
])
def test_paged_compress_equals_strided_compress(seq, chunk, kw):
    """In-place compression of a paged cache: the tokens found in the sequences' blocks afterwards
    are bit for bit what ckv_compress gives on the contiguous cache (that path is checked against
    the oracle elsewhere), the released blocks are the tail of each table row, attention over the
    compacted pages matches the oracle."""
    _say(f"paged compress S={seq} c={chunk} {kw}")
    B, H, G, D, bs = 2, 4, 4, 128, 16
    K, V, _ = kv_host(94, B * H, seq, D, "bf16", alpha=0.9, n_outlier=4)
    K, V = K.reshape(B, H, seq, D), V.reshape(B, H, seq, D)
    deg = torch.ones((B, H, seq), dtype=torch.int32)
    lens = torch.full((B,), seq, dtype=torch.int32)
    n_blocks = B * (-(-seq // bs)) + 7
    K_pool, V_pool, deg_pool, table = _pack(K, V, deg, lens, bs, n_blocks, 29)
    table_before = table.clone()
    lens_d = lens.to(DEV)
    cK, cV, cdeg, _ = ckv.compress(K.to(DEV), V.to(DEV), chunk, want_assign=False, **kw)
    new_len, freed = ckv.paged_compress(K_pool, V_pool, deg_pool, table, seq, chunk, lens=lens_d, **kw)
    torch.cuda.synchronize()
    assert new_len == cK.shape[2] and lens_d.tolist() == [new_len] * B
    keep, old = -(-new_len // bs), -(-seq // bs)
    assert torch.equal(freed, table_before[:, keep:old]) and bool((table[:, keep:] == -1).all())
    rK, rV, rdeg = ckv.paged_gather(K_pool, V_pool, deg_pool, table, new_len)
    torch.cuda.synchronize()
    assert torch.equal(rK, cK) and torch.equal(rV, cV) and torch.equal(rdeg, cdeg)
    q = torch.randn((B, H * G, D), generator=torch.Generator().manual_seed(8)).to(torch.bfloat16).to(DEV)
    o = ckv.paged_decode_attn(q, K_pool, V_pool, deg_pool, table, lens_d, max_len=new_len, out_dtype=torch.float32)
    torch.cuda.synchronize()
    for b in range(B):
        ref = oracle.app_attn(f64(q[b]), f64(cK[b]), f64(cV[b]), i64(cdeg[b]))
        assert_rows_close(f64(o[b]), ref, ATTN_TOL, f"attention over compacted pages b{b}")


def test_algorithm1_decode_loop_on_a_paged_cache():
    """The decode loop of Algorithm 1 kept entirely in pages: ckv_paged_append, attention over the
    pages, in-place compression with block release once the cache holds budget + g tokens, blocks
    handed back and out again by a toy free list.  Every step's output must equal, bit for bit,
    the strided OnlineCache on the same tokens (that loop is checked against the oracle in
    test_gpu_online.py); at the end the pages hold exactly the strided cache."""
    from paper_2506_11418_amd.online import OnlineCache
    _say("online loop on pages")
    B, H, G, D, bs = 2, 2, 2, 128, 16
    n, chunk, R, g, n_sink, n_recent, steps = 1024, 128, 0.5, 16, 4, 8, 120
    K, V, _ = kv_host(95, B * H, n + steps, D, "bf16", alpha=0.9, n_outlier=4)
    K, V = K.reshape(B, H, n + steps, D).to(DEV), V.reshape(B, H, n + steps, D).to(DEV)
    qs = torch.randn((steps, B, H * G, D), generator=torch.Generator().manual_seed(5)).to(torch.bfloat16).to(DEV)
    ref = OnlineCache(K[:, :, :n], V[:, :, :n], chunk, R, g, H * G, 0.8, 0.2, 0.2, n_sink, n_recent)
    budget = ref.budget

    # pages: a pool with a free list on the host
    n_blocks, max_blocks = 200, (n + bs - 1) // bs + 2
    free = list(range(n_blocks))[::-1]
    K_pool = torch.zeros((n_blocks, H, bs, D), dtype=torch.bfloat16, device=DEV)
    V_pool = torch.zeros_like(K_pool)
    deg_pool = torch.zeros((n_blocks, H, bs), dtype=torch.int32, device=DEV)
    table_h = torch.full((B, max_blocks), -1, dtype=torch.int32)
    for b in range(B):
        for i in range((n + bs - 1) // bs):
            table_h[b, i] = free.pop()
    table = table_h.to(DEV)
    lens = torch.full((B,), n, dtype=torch.int32, device=DEV)
    ones = torch.ones((B, H, n), dtype=torch.int32, device=DEV)
    ckv.paged_scatter(K[:, :, :n].contiguous(), V[:, :, :n].contiguous(), ones, K_pool, V_pool, deg_pool, table, n)
    # first clustering after prefill (same schedule as the reference helper)
    s, freed = ckv.paged_compress(K_pool, V_pool, deg_pool, table, n, chunk, rounds=ref.rounds_prefill, lens=lens,
                                  n_sink=n_sink, n_recent=n_recent)
    free.extend(freed.flatten().tolist())
    assert s == ref.s
    n_rounds = 0
    for i in range(steps):
        if s % bs == 0:                                   # the next token opens a block: take one from the free list
            for b in range(B):
                table[b, s // bs] = free.pop()
        ckv.paged_append(K[:, :, n + i].contiguous(), V[:, :, n + i].contiguous(), K_pool, V_pool, deg_pool, table, lens)
        s += 1
        # max_len = the current length: the same split of the sequence as the strided call, hence the same bits
        o = ckv.paged_decode_attn(qs[i], K_pool, V_pool, deg_pool, table, lens, max_len=s, out_dtype=torch.float32)
        o_ref = ref.step(qs[i], K[:, :, n + i].contiguous(), V[:, :, n + i].contiguous(), out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert lens.tolist() == [s] * B
        assert torch.equal(o, o_ref), f"step {i}"
        if s >= budget + g:
            s, freed = ckv.paged_compress(K_pool, V_pool, deg_pool, table, s, chunk, rounds=[0.8], lens=lens,
                                          n_sink=n_sink, n_recent=n_recent)
            free.extend(freed.flatten().tolist())
            n_rounds += 1
            assert s == ref.s
    assert n_rounds == ref.n_clusterings and n_rounds >= 1
    gK, gV, gdeg = ckv.paged_gather(K_pool, V_pool, deg_pool, table, s)
    rK, rV, rdeg = ref.view()
    torch.cuda.synchronize()
    assert torch.equal(gK, rK) and torch.equal(gV, rV) and torch.equal(gdeg, rdeg)
    used = set(table[table >= 0].flatten().tolist())
    assert len(used) == B * ((s + bs - 1) // bs) and used.isdisjoint(free) and len(used) + len(free) == n_blocks
