"""GPU check of ckv_decode_attn_noalloc (the entry point for callers that cannot allocate): through
the C ABI, against ckv_decode_attn on the same inputs, on calls in a row that share the library's
scratch array - the second with a smaller input, the third with more (batch, head) pairs than any
before - and on a recorded call replayed after calls of other shapes."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from parity_util import ATTN_TOL, assert_rows_close, f64, i64
from synth import kv_host, query_host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(seed, B, Hkv, G, L, D):
    rng = np.random.default_rng(seed)
    Ks, Vs = zip(*[kv_host(seed + b, Hkv, L, D, "bf16", n_outlier=0)[:2] for b in range(B)])
    K, V = torch.cat(Ks).to(DEV), torch.cat(Vs).to(DEV)
    q = query_host(seed + 100, B, Hkv * G, D, "bf16").to(DEV)
    deg = torch.from_numpy(rng.integers(1, 6, (B, Hkv, L)).astype(np.int32)).to(DEV)
    lens = torch.from_numpy(rng.integers(L // 2, L + 1, B).astype(np.int32)).to(DEV)
    return q, K, V, deg, lens


def test_noalloc_entry_point_matches_the_workspace_entry_point():
    print("no-alloc attention: three calls in a row on the shared scratch", flush=True)
    cases = [_case(1, 1, 8, 4, 8192, 128),      # a compressed Llama-3-8B layer cache, batch 1
             _case(2, 1, 2, 4, 700, 128),       # smaller input: fewer heads, shorter, ragged
             _case(3, 5, 8, 4, 1500, 128)]      # more (batch, head) pairs than either call before
    outs = []
    for q, K, V, deg, lens in cases:            # back to back on one stream, no synchronisation in between
        o = torch.empty(q.shape, dtype=torch.float32, device=DEV)
        ckv.decode_attn_noalloc(q, K, V, o, lens=lens, deg=deg)
        outs.append(o)
    q, K, V, deg, lens = cases[1]
    again = torch.empty_like(outs[1])
    ckv.decode_attn_noalloc(q, K, V, again, lens=lens, deg=deg)       # and the small one once more after the large one
    torch.cuda.synchronize()
    for i, ((q, K, V, deg, lens), o) in enumerate(zip(cases, outs)):
        ref = ckv.decode_attn(q, K, V, lens=lens, deg=deg, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(o, ref), f"call {i}: differs from ckv_decode_attn"
        for b in range(q.shape[0]):             # and both meet the oracle (Eq. 3) to the attention tolerance
            want = oracle.app_attn(f64(q[b]), f64(K[b]), f64(V[b]), i64(deg[b]), int(lens[b]))
            assert_rows_close(f64(o[b]), want, ATTN_TOL, f"call {i} b{b}")
    assert torch.equal(again, outs[1])


def test_noalloc_call_recorded_in_a_graph_replays_after_calls_of_other_shapes():
    """The entry point launches one kernel and keeps no host state that depends on the calls made
    so far, so a call recorded into a HIP graph gives the eager bits on every replay, whatever
    shapes ran on the shared scratch in between."""
    print("no-alloc attention: recorded call replayed between eager calls of other shapes", flush=True)
    q, K, V, deg, lens = _case(11, 2, 8, 4, 3000, 128)
    others = [_case(12, 6, 8, 4, 900, 128), _case(13, 1, 2, 4, 5000, 128)]
    ref = ckv.decode_attn(q, K, V, lens=lens, deg=deg, out_dtype=torch.float32)
    o = torch.zeros_like(ref)
    ckv.decode_attn_noalloc(q, K, V, o, lens=lens, deg=deg)            # first use outside the capture (address lookup)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            ckv.decode_attn_noalloc(q, K, V, o, lens=lens, deg=deg)
    torch.cuda.synchronize()
    for rep in range(4):
        oq, oK, oV, odeg, olens = others[rep % 2]
        oo = torch.empty(oq.shape, dtype=torch.float32, device=DEV)
        ckv.decode_attn_noalloc(oq, oK, oV, oo, lens=olens, deg=odeg)   # eager, another shape, same scratch
        torch.cuda.synchronize()
        assert torch.equal(oo, ckv.decode_attn(oq, oK, oV, lens=olens, deg=odeg, out_dtype=torch.float32))
        o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, ref), f"replay {rep}"


def test_noalloc_entry_point_rejects_what_its_scratch_cannot_hold():
    L = ckv.lib()
    a = C.c_void_p(4096)
    big = ckv.Layout(256, 8, 4096, 128, 8 * 4096 * 128, 4096 * 128, 128, ckv.BF16, 0)
    need = C.c_size_t(0)
    assert L.ckv_decode_attn_workspace(C.byref(big), 64, C.byref(need)) == 0
    assert need.value > (4 << 20)               # 256 sequences x 64 query heads: more than the array holds
    assert L.ckv_decode_attn_noalloc(a, 64, a, a, C.byref(big), None, None, 0.0, a, 0, None) == -4
    many = ckv.Layout(2500, 8, 64, 32, 8 * 64 * 32, 64 * 32, 32, ckv.F32, 0)
    assert L.ckv_decode_attn_workspace(C.byref(many), 8, C.byref(need)) == 0
    assert need.value < (4 << 20) - (64 << 10)  # the partials would fit, the 20000 arrival counters do not
    assert L.ckv_decode_attn_noalloc(a, 8, a, a, C.byref(many), None, None, 0.0, a, 0, None) == -4
    ok = ckv.Layout(1, 8, 8192, 128, 8 * 8192 * 128, 8192 * 128, 128, ckv.BF16, 0)
    assert L.ckv_decode_attn_noalloc(None, 32, a, a, C.byref(ok), None, None, 0.0, a, 0, None) == -1
    assert L.ckv_decode_attn_noalloc(a, 32, C.c_void_p(4100), a, C.byref(ok), None, None, 0.0, a, 0, None) == -3
    assert L.ckv_decode_attn_noalloc(a, 24, a, a, C.byref(ok), None, None, 0.0, a, 0, None) == -5     # 3 query heads per KV head
