"""GPU parity at the benchmark's full size and launch configuration: the 32-layer x 8-KV-head x
131072-token bf16 cache compressed in ONE ckv_compress call (layers folded into batch), then one
GQA decode step per layer.  Cheap invariants are checked on every (layer, head) on the device;
sampled (layer, head) sequences are checked element by element against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from parity_util import ATTN_TOL, assert_rows_close, check_round, f64, i64
from synth import kv_device

pytestmark = pytest.mark.gpu
DEV = "cuda"
LAYERS, HEADS, QHEADS, SEQ, DIM, CHUNK, RHO = 32, 8, 32, 131072, 128, 1024, 0.25
SAMPLES = [(0, 0), (13, 5), (31, 7)]


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def full_cache():
    _say("generating the 16 GiB cache on the device")
    K = torch.empty((LAYERS, HEADS, SEQ, DIM), dtype=torch.bfloat16, device=DEV)
    V = torch.empty_like(K)
    for l in range(LAYERS):
        kv_device(2024, HEADS, SEQ, DIM, "bf16", 0.9, 4, layer=l, device=DEV, out_k=K[l], out_v=V[l])
    _say("compressing")
    cK, cV, cdeg, assign = ckv.compress(K, V, CHUNK, retain_ratio=RHO)
    torch.cuda.synchronize()
    yield K, V, cK, cV, cdeg, assign
    del K, V, cK, cV, cdeg, assign
    torch.cuda.empty_cache()


def test_invariants_on_every_head(full_cache):
    K, V, cK, cV, cdeg, assign = full_cache
    L2 = SEQ // 4
    assert cK.shape == (LAYERS, HEADS, L2, DIM) and cdeg.shape == (LAYERS, HEADS, L2)
    assert int(cdeg.min()) >= 1
    assert torch.equal(cdeg.sum(dim=-1), torch.full((LAYERS, HEADS), SEQ, dtype=torch.int64, device=DEV))
    assert int(assign.min()) == 0 and int(assign.max()) == L2 - 1
    # every source token is assigned to exactly one centroid, and the centroid's degree counts them
    counts = torch.zeros((LAYERS * HEADS, L2), dtype=torch.int32, device=DEV)
    counts.scatter_add_(1, assign.reshape(LAYERS * HEADS, SEQ).to(torch.int64),
                        torch.ones((LAYERS * HEADS, SEQ), dtype=torch.int32, device=DEV))
    assert torch.equal(counts.reshape(LAYERS, HEADS, L2), cdeg)
    # mass conservation of the values in fp32 (bf16 storage of the centroids costs ~1e-2 per element)
    tot_in = V.float().sum(dim=2)
    tot_out = (cV.float() * cdeg.unsqueeze(-1).float()).sum(dim=2)
    assert float((tot_in - tot_out).abs().max()) < 5.0
    assert bool(torch.isfinite(cK.float()).all()) and bool(torch.isfinite(cV.float()).all())


@pytest.mark.parametrize("layer,head", SAMPLES)
def test_sampled_heads_against_the_oracle(full_cache, layer, head):
    K, V, cK, cV, cdeg, assign = full_cache
    _say(f"oracle check of layer {layer} head {head}")
    Kh = K[layer:layer + 1, head:head + 1].contiguous()
    Vh = V[layer:layer + 1, head:head + 1].contiguous()
    # round by round on the GPU for this one sequence, every round checked against the oracle
    curK, curV, curdeg, maps = Kh, Vh, None, []
    for j, r in enumerate([1.0, 1.0]):
        gK, gV, gdeg, gas = ckv.compress(curK, curV, CHUNK, rounds=[r], deg=curdeg)
        torch.cuda.synchronize()
        d_in = np.ones(curK.shape[2], dtype=np.int64) if curdeg is None else i64(curdeg[0, 0])
        check_round(f64(curK[0, 0]), f64(curV[0, 0]), d_in, CHUNK, r, "bf16", f64(gK[0, 0]), f64(gV[0, 0]),
                    i64(gdeg[0, 0]), i64(gas[0, 0]), what=f"L{layer}H{head} round {j}")
        curK, curV, curdeg = gK, gV, gdeg
        maps.append(gas[0, 0].to(torch.int64))
    # the one big call produced exactly the same bits for this sequence
    assert torch.equal(cK[layer, head], curK[0, 0]) and torch.equal(cV[layer, head], curV[0, 0])
    assert torch.equal(cdeg[layer, head], curdeg[0, 0])
    assert torch.equal(assign[layer, head].to(torch.int64), maps[1][maps[0]])


@pytest.mark.parametrize("layer", [0, 17])
def test_decode_attention_over_the_compressed_layer(full_cache, layer):
    K, V, cK, cV, cdeg, assign = full_cache
    _say(f"decode attention over compressed layer {layer}")
    gen = torch.Generator(device=DEV).manual_seed(77 + layer)
    q = torch.randn((1, QHEADS, DIM), generator=gen, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    o = ckv.decode_attn(q, cK[layer:layer + 1], cV[layer:layer + 1], deg=cdeg[layer:layer + 1],
                        out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = oracle.app_attn(f64(q[0]), f64(cK[layer]), f64(cV[layer]), i64(cdeg[layer]))
    assert_rows_close(f64(o[0]), ref, ATTN_TOL, f"layer {layer}")
