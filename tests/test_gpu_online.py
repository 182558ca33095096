"""GPU parity of the online part of Algorithm 1: ckv_append, attention over the growing cache and
the periodic clustering round (with incoming degrees, sinks and recents), against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from paper_2506_11418_amd.online import OnlineCache
from parity_util import ATTN_TOL, assert_rows_close, check_round_with_edges, f64, i64
from synth import kv_host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def _stream(seed, B, H, n, steps, D, dtype):
    """Prompt cache and decode-time tokens from ONE synthetic sequence of n + steps tokens per
    (batch, head), so the appended keys continue the prompt's local similarity."""
    K, V, _ = kv_host(seed, B * H, n + steps, D, dtype, alpha=0.9, n_outlier=4 if D == 128 else 0)
    K, V = K.reshape(B, H, n + steps, D), V.reshape(B, H, n + steps, D)
    gen = torch.Generator().manual_seed(seed)
    return K, V, gen


@pytest.mark.parametrize("dtype,n,chunk,R,g,n_sink,n_recent,steps", [
    ("bf16", 2128, 256, 0.25, 32, 16, 64, 270),        # 8 prefill rounds (floor 0.2); rounds at steps 68, 261
    ("f32", 600, 64, 0.5, 16, 4, 8, 180),              # rounds at steps 51, 170
    ("bf16", 1024, 128, 0.5, 16, 0, 0, 310),           # rounds at steps 94, 304
])
def test_algorithm1_decode_loop(dtype, n, chunk, R, g, n_sink, n_recent, steps):
    _say(f"online loop {dtype} n={n} c={chunk} R={R} g={g} n1={n_sink} n2={n_recent} steps={steps}")
    B, H, G, D = 2, 2, 2, 128 if dtype == "bf16" else 64
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Kall, Vall, gen = _stream(71, B, H, n, steps, D, dtype)
    qs = torch.randn((steps, B, H * G, D), generator=gen).to(tdt)
    Kd, Vd = Kall.to(DEV), Vall.to(DEV)
    budget = int(R * n + 1e-9)
    rounds = ckv.schedule_annealed(n, chunk, budget, 0.8, 0.2, 0.2, n_sink, n_recent)
    assert rounds == oracle.rounds_to_budget(n, chunk, budget, 0.8, 0.2, 0.2, n_sink, n_recent) and rounds

    # ---- the calls of Algorithm 1 issued one by one, every step checked against the oracle ----
    cap = budget + g
    bufs = [tuple(torch.zeros((B, H, cap, D), dtype=tdt, device=DEV) for _ in range(2)) +
            (torch.zeros((B, H, cap), dtype=torch.int32, device=DEV),) for _ in range(2)]
    cur = 0
    ckv.compress(Kd[:, :, :n], Vd[:, :, :n], chunk, rounds=rounds, want_assign=False,
                 out=(bufs[0][0], bufs[0][1], bufs[0][2], None), n_sink=n_sink, n_recent=n_recent)
    s = oracle.round_lengths(n, chunk, rounds, n_sink, n_recent)[-1]
    assert s <= budget
    start = [t[:, :, :s].clone() for t in bufs[0]]           # the cache the loop starts from
    outs, ran = [], []
    for i in range(steps):
        cK, cV, cdeg = bufs[cur]
        k_new, v_new = Kd[:, :, n + i].contiguous(), Vd[:, :, n + i].contiguous()
        ckv.append(k_new, v_new, cK, cV, cdeg, pos=s)
        s += 1
        K, V, deg = cK[:, :, :s], cV[:, :, :s], cdeg[:, :, :s]
        assert torch.equal(K[:, :, s - 1], k_new) and torch.equal(V[:, :, s - 1], v_new)
        assert bool((deg[:, :, s - 1] == 1).all())
        o = ckv.decode_attn(qs[i].to(DEV), K, V, deg=deg, out_dtype=torch.float32)
        torch.cuda.synchronize()
        outs.append(o)
        if i % 7 == 0 or s >= budget + g:                    # oracle attention on a sample of the steps
            for b in range(B):
                ref = oracle.app_attn(f64(qs[i][b]), f64(K[b]), f64(V[b]), i64(deg[b]))
                assert_rows_close(f64(o[b]), ref, ATTN_TOL, f"step {i} b{b}")
        if s >= budget + g:
            nK, nV, ndeg = bufs[1 - cur]
            ckv.compress(K, V, chunk, rounds=[0.8], deg=deg, out=(nK, nV, ndeg, None), want_assign=False,
                         n_sink=n_sink, n_recent=n_recent)
            gas = ckv.compress(K, V, chunk, rounds=[0.8], deg=deg, n_sink=n_sink, n_recent=n_recent)
            torch.cuda.synchronize()
            s_new = gas[0].shape[2]
            assert torch.equal(gas[0], nK[:, :, :s_new]) and torch.equal(gas[2], ndeg[:, :, :s_new])
            for b in range(B):
                for h in range(H):
                    check_round_with_edges(f64(K[b, h]), f64(V[b, h]), i64(deg[b, h]), chunk, 0.8, dtype, n_sink,
                                           n_recent, f64(gas[0][b, h]), f64(gas[1][b, h]), i64(gas[2][b, h]),
                                           i64(gas[3][b, h]), what=f"decode-time round at step {i} (b{b},h{h})")
            cur, s = 1 - cur, s_new
            ran.append(i)
            assert int(ndeg[:, :, :s].sum()) == B * H * (n + i + 1)
    assert len(ran) >= 2 and ran[0] == budget + g - start[0].shape[2] - 1

    # ---- the same loop through the OnlineCache helper: identical bits ------------------------
    oc = OnlineCache(Kd[:, :, :n], Vd[:, :, :n], chunk, R, g, H * G, 0.8, 0.2, 0.2, n_sink, n_recent)
    assert oc.rounds_prefill == rounds and oc.budget == budget
    for i in range(steps):
        o = oc.step(qs[i].to(DEV), Kd[:, :, n + i].contiguous(), Vd[:, :, n + i].contiguous(), out_dtype=torch.float32)
        assert torch.equal(o, outs[i]), f"helper differs at step {i}"
    assert oc.n_clusterings == len(ran) and oc.s == s
    fK, fV, fdeg = oc.view()
    assert torch.equal(fK, bufs[cur][0][:, :, :s]) and torch.equal(fdeg, bufs[cur][2][:, :, :s])

    # ---- free-running oracle loop from the same starting cache --------------------------------
    for b in range(B):
        ks = [f64(Kall[b, :, n + i]) for i in range(steps)]
        vs = [f64(Vall[b, :, n + i]) for i in range(steps)]
        ref_o, rK, rV, rdeg, rran = oracle.alg1_decode(f64(start[0][b]), f64(start[1][b]), i64(start[2][b]),
                                                       [f64(qs[i][b]) for i in range(steps)], ks, vs, chunk, budget,
                                                       g, [0.8], dtype, n_sink, n_recent)
        assert rran == ran and rK.shape[1] == s
        if np.array_equal(rdeg, i64(bufs[cur][2][b, :, :s])):       # same clustering decisions throughout
            got = np.stack([f64(outs[i][b]) for i in range(steps)])
            assert_rows_close(got, ref_o, ATTN_TOL, f"free-running loop b{b}")
        else:
            _say(f"b{b}: a near-tie was resolved differently; per-round checks above cover it")


def test_append_with_device_lengths():
    """Per-sequence lengths on the device: each sequence's token lands at its own row, lens is
    incremented, a full sequence is left untouched."""
    B, H, D, cap = 4, 2, 128, 40
    gen = torch.Generator(device=DEV).manual_seed(3)
    K = torch.randn((B, H, cap, D), generator=gen, device=DEV).to(torch.bfloat16)
    V = torch.randn((B, H, cap, D), generator=gen, device=DEV).to(torch.bfloat16)
    deg = torch.full((B, H, cap), 7, dtype=torch.int32, device=DEV)
    K0, V0 = K.clone(), V.clone()
    lens = torch.tensor([0, 17, 39, 40], dtype=torch.int32, device=DEV)
    k_new = torch.randn((B, H, D), generator=gen, device=DEV).to(torch.bfloat16)
    v_new = torch.randn((B, H, D), generator=gen, device=DEV).to(torch.bfloat16)
    ckv.append(k_new, v_new, K, V, deg, lens=lens)
    torch.cuda.synchronize()
    assert lens.tolist() == [1, 18, 40, 40]
    expK, expV, expdeg = K0.clone(), V0.clone(), torch.full((B, H, cap), 7, dtype=torch.int32, device=DEV)
    for b, t in enumerate([0, 17, 39]):
        expK[b, :, t], expV[b, :, t], expdeg[b, :, t] = k_new[b], v_new[b], 1
    assert torch.equal(K, expK) and torch.equal(V, expV) and torch.equal(deg, expdeg)
    # attention with those lengths against the oracle (appended tokens have degree 1)
    q = torch.randn((B, H * 4, D), generator=gen, device=DEV).to(torch.bfloat16)
    o = ckv.decode_attn(q, K, V, lens=lens, deg=deg, out_dtype=torch.float32)
    torch.cuda.synchronize()
    for b in range(B):
        ref = oracle.app_attn(f64(q[b]), f64(K[b]), f64(V[b]), i64(deg[b]), int(lens[b]))
        assert_rows_close(f64(o[b]), ref, ATTN_TOL, f"b{b}")
    with pytest.raises(ckv.CkvError):
        ckv.append(k_new, v_new, K, V, deg, pos=cap)
