"""GPU parity: ckv_decode_attn (HIP, through the C ABI) vs the oracle's Eq. 3."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from parity_util import ATTN_TOL, assert_rows_close, f64, i64
from synth import kv_host, query_host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)


def _check(q, K, V, deg, lens, out, tol=ATTN_TOL, what=""):
    B = q.shape[0]
    for b in range(B):
        n = K.shape[2] if lens is None else int(lens[b])
        ref = oracle.app_attn(f64(q[b]), f64(K[b]), f64(V[b]), None if deg is None else i64(deg[b]), n)
        assert_rows_close(f64(out[b]), ref, tol, f"{what} b{b}")


def test_config1_decode_over_compressed_cache_fp32():
    _say("attn config1")
    K, V, rng = kv_host(0, 1, 1024, 64, "f32", alpha=0.9, single_stream=True)
    q = query_host(rng, 1, 1, 64, "f32").to(DEV)
    K, V = K.to(DEV), V.to(DEV)
    cK, cV, cdeg, _ = ckv.compress(K, V, 64, retain_ratio=0.5)
    o = ckv.decode_attn(q, cK, cV, deg=cdeg)
    torch.cuda.synchronize()
    _check(q, cK, cV, cdeg, None, o, tol=1e-4, what="config1")
    # and the approximation is close to attention over the full cache (sanity, loose)
    full = oracle.app_attn(f64(q[0]), f64(K[0]), f64(V[0]))
    assert np.abs(f64(o[0]) - full).max() < 0.5


@pytest.mark.parametrize("B,Hkv,G,L,D,dtype", [
    (1, 8, 4, 8192, 128, "bf16"),      # config 2's compressed cache
    (2, 2, 4, 1000, 128, "bf16"),      # ragged: not a multiple of the slice
    (3, 1, 8, 300, 64, "bf16"),
    (2, 2, 1, 513, 128, "bf16"),
    (1, 2, 2, 77, 32, "f32"),
    (2, 1, 4, 2000, 128, "f32"),
    (1, 1, 1, 1, 64, "f32"),
])
def test_decode_attn_shapes(B, Hkv, G, L, D, dtype):
    _say(f"attn B={B} Hkv={Hkv} G={G} L={L} D={D} {dtype}")
    rng = np.random.default_rng(B * 1000 + L)
    Ks, Vs = [], []
    for b in range(B):
        K, V, _ = kv_host(20 + b, Hkv, L, D, dtype, n_outlier=0)
        Ks.append(K)
        Vs.append(V)
    K, V = torch.cat(Ks).to(DEV), torch.cat(Vs).to(DEV)
    q = query_host(int(rng.integers(1 << 30)), B, Hkv * G, D, dtype).to(DEV)
    deg = torch.from_numpy(rng.integers(1, 6, (B, Hkv, L)).astype(np.int32)).to(DEV)
    lens = torch.from_numpy(rng.integers(1, L + 1, B).astype(np.int32))
    lens[0] = L
    tol = 1e-4 if dtype == "f32" else ATTN_TOL
    o = ckv.decode_attn(q, K, V, lens=lens.to(DEV), deg=deg, out_dtype=torch.float32)
    torch.cuda.synchronize()
    _check(q, K, V, deg, lens, o, tol, "deg+lens")
    o2 = ckv.decode_attn(q, K, V)                                 # vanilla attention, cache dtype out
    torch.cuda.synchronize()
    # a bf16 output carries its own rounding (half an ulp = 2^-9 relative) on top of the bar
    _check(q, K, V, None, None, o2, ATTN_TOL + 2.0 ** -8 if dtype == "bf16" else 1e-4, "vanilla")


def test_outlier_keys_large_logits_bf16():
    """Keys with x10 outlier channels give logits of several tens: the softmax must stay stable."""
    _say("attn outliers")
    K, V, _ = kv_host(31, 2, 4096, 128, "bf16", n_outlier=4)
    q = query_host(32, 1, 8, 128, "bf16")
    K, V, q = K.to(DEV), V.to(DEV), q.to(DEV)
    cK, cV, cdeg, _ = ckv.compress(K, V, 1024, retain_ratio=0.25)
    o = ckv.decode_attn(q, cK, cV, deg=cdeg, out_dtype=torch.float32)
    torch.cuda.synchronize()
    _check(q, cK, cV, cdeg, None, o, ATTN_TOL, "outliers")


def test_zero_length_and_zero_query():
    _say("attn zero length / zero query")
    K, V, _ = kv_host(33, 1, 256, 128, "bf16")
    K, V = K.to(DEV), V.to(DEV)
    cK, cV, cdeg, _ = ckv.compress(K, V, 64, retain_ratio=0.5)
    q = torch.zeros((1, 4, 128), dtype=torch.bfloat16, device=DEV)
    o = ckv.decode_attn(q, cK, cV, deg=cdeg, out_dtype=torch.float32)
    torch.cuda.synchronize()
    # q = 0: degree-weighted mean of centroids = plain mean of the ORIGINAL values (bf16 storage of V')
    assert np.abs(f64(o[0, 0]) - f64(V[0, 0]).mean(0)).max() < 2e-3
    lens = torch.zeros(1, dtype=torch.int32, device=DEV)
    o0 = ckv.decode_attn(torch.ones_like(q), cK, cV, lens=lens, deg=cdeg)
    torch.cuda.synchronize()
    assert float(o0.float().abs().sum()) == 0.0


def test_strided_cache_layout():
    _say("attn strided layout")
    K, V, _ = kv_host(34, 2, 640, 128, "bf16")
    q = query_host(35, 1, 4, 128, "bf16").to(DEV)
    Kb = K.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)     # [B,S,H,D] storage
    Vb = V.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    a = ckv.decode_attn(q, Kb, Vb, out_dtype=torch.float32)
    b = ckv.decode_attn(q, K.to(DEV), V.to(DEV), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_decode_loop_can_be_captured_in_a_hip_graph():
    """The library allocates nothing, synchronises nothing and clears nothing with memset, so the
    per-layer attention calls of a decode step (and an append before them) can be recorded into a
    HIP graph.  Every replay, with eager work and synchronisation between replays, gives the bits of
    the eager calls."""
    _say("attention calls in a HIP graph")
    Ly, Hkv, G, L, D = 6, 4, 4, 3000, 128
    K, V, _ = kv_host(61, Ly * Hkv, L + 1, D, "bf16", n_outlier=0)
    K, V = K.reshape(Ly, Hkv, L + 1, D).to(DEV), V.reshape(Ly, Hkv, L + 1, D).to(DEV)
    rng = np.random.default_rng(3)
    deg = torch.from_numpy(rng.integers(1, 6, (Ly, Hkv, L + 1)).astype(np.int32)).to(DEV)
    q = query_host(9, Ly, Hkv * G, D, "bf16").to(DEV).reshape(Ly, 1, Hkv * G, D)
    k_new, v_new = K[:, :, L].clone(), V[:, :, L].clone()
    ws = torch.zeros(ckv.decode_attn_workspace(ckv.layout_of(K[0:1]), Hkv * G), dtype=torch.uint8, device=DEV)
    o = torch.empty((Ly, 1, Hkv * G, D), dtype=torch.float32, device=DEV)

    def step():
        for l in range(Ly):
            ckv.append(k_new[l:l + 1], v_new[l:l + 1], K[l:l + 1], V[l:l + 1], deg[l:l + 1], pos=L)
            ckv.decode_attn(q[l], K[l:l + 1], V[l:l + 1], deg=deg[l:l + 1], out=o[l], workspace=ws)

    step()
    torch.cuda.synchronize()
    ref = o.clone()
    for l in (0, Ly - 1):
        _check(q[l], K[l:l + 1], V[l:l + 1], deg[l:l + 1], None, ref[l], ATTN_TOL, f"eager layer {l}")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                           # warm-up on the capture stream's side
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in range(4):
        o.zero_()
        K[:, :, L].zero_()                               # the captured append has to write the token again
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, ref), f"replay {i}"
        assert torch.equal(K[:, :, L], k_new)
        step()                                           # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(o, ref)


def test_attn_argument_errors():
    _say("attn argument errors")
    K = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((1, 6, 128), dtype=torch.bfloat16, device=DEV)      # 3 query heads per KV head
    with pytest.raises(ckv.CkvError) as e:
        ckv.decode_attn(q, K, K)
    assert e.value.status == -5
    q = torch.zeros((1, 8, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(ckv.CkvError) as e:
        ckv.decode_attn(q, K, K, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.status == -4
