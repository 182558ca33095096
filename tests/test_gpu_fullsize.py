"""GPU parity at the benchmark's full size and launch configuration: the 32-layer x 8-KV-head x
131072-token bf16 cache compressed in ONE ckv_compress call (layers folded into batch), then one
GQA decode step per layer.  Cheap invariants are checked on every (layer, head) on the device;
sampled (layer, head) sequences are checked element by element against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from parity_util import ATTN_TOL, assert_rows_close, check_round, check_round_with_edges, f64, i64
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


# ---- the paper's default-style setting at 128k tokens: sinks 16, recents 64, annealed r, one ranking per head ----
def test_128k_layer_with_sinks_recents_annealed_schedule_and_whole_sequence_selection():
    """One layer (8 KV heads x 131072 tokens), chunk 1024, n1 = 16, n2 = 64, merge fractions 0.8 then
    0.6 (Eq. 4), top-r over all chunks of a head.  Invariants on every head; two heads round by
    round against the oracle, and the one call must equal the rounds issued one by one."""
    _say("128k layer: sinks/recents, annealed schedule, scope=head")
    n1, n2, rounds = 16, 64, [0.8, 0.6]
    K = torch.empty((1, HEADS, SEQ, DIM), dtype=torch.bfloat16, device=DEV)
    V = torch.empty_like(K)
    kv_device(808, HEADS, SEQ, DIM, "bf16", 0.9, 4, layer=0, device=DEV, out_k=K[0], out_v=V[0])
    cK, cV, cdeg, assign = ckv.compress(K, V, CHUNK, rounds=rounds, n_sink=n1, n_recent=n2, scope="head")
    torch.cuda.synchronize()
    out_len = oracle.round_lengths(SEQ, CHUNK, rounds, n1, n2, scope="head")[-1]
    assert cK.shape == (1, HEADS, out_len, DIM)
    assert torch.equal(cdeg.sum(dim=-1), torch.full((1, HEADS), SEQ, dtype=torch.int64, device=DEV))
    assert torch.equal(cK[:, :, :n1], K[:, :, :n1]) and torch.equal(cV[:, :, -n2:], V[:, :, -n2:])
    counts = torch.zeros((HEADS, out_len), dtype=torch.int32, device=DEV)
    counts.scatter_add_(1, assign[0].to(torch.int64), torch.ones((HEADS, SEQ), dtype=torch.int32, device=DEV))
    assert torch.equal(counts, cdeg[0])
    for h in (2, 7):
        _say(f"  oracle check of head {h}")
        curK, curV, curdeg = K[:, h:h + 1].contiguous(), V[:, h:h + 1].contiguous(), None
        for j, r in enumerate(rounds):
            gK, gV, gdeg, gas = ckv.compress(curK, curV, CHUNK, rounds=[r], deg=curdeg, n_sink=n1, n_recent=n2,
                                             scope="head")
            torch.cuda.synchronize()
            d_in = np.ones(curK.shape[2], dtype=np.int64) if curdeg is None else i64(curdeg[0, 0])
            check_round_with_edges(f64(curK[0, 0]), f64(curV[0, 0]), d_in, CHUNK, r, "bf16", n1, n2, f64(gK[0, 0]),
                                   f64(gV[0, 0]), i64(gdeg[0, 0]), i64(gas[0, 0]), what=f"head {h} round {j}",
                                   scope="head")
            curK, curV, curdeg = gK, gV, gdeg
        assert torch.equal(cK[0, h], curK[0, 0]) and torch.equal(cdeg[0, h], curdeg[0, 0])


def test_128k_layer_with_the_papers_own_hyper_parameters():
    """One layer (8 KV heads x 131072 tokens) with the settings of Sec. 6.1: chunk 256, 16 sinks, 64
    recents, merge fractions annealed from 0.8 by 0.2 (Eq. 4; the schedule's floor, which the paper
    leaves open, at 0.2) down to the 25% budget - six rounds, whole chunks through the several-
    chunks-per-workgroup similarity kernel, a ragged tail chunk through the other one.  Invariants
    on every head; one head round by round against the oracle, and the one call must equal the
    rounds issued one by one."""
    _say("128k layer: chunk 256, sinks/recents, six annealed rounds")
    n1, n2, chunk = 16, 64, 256
    rounds = ckv.schedule_annealed(SEQ, chunk, SEQ // 4, 0.8, 0.2, 0.2, n1, n2)
    assert [round(float(r), 3) for r in rounds] == [0.8, 0.6, 0.4, 0.2, 0.2, 0.2]
    K = torch.empty((1, HEADS, SEQ, DIM), dtype=torch.bfloat16, device=DEV)
    V = torch.empty_like(K)
    kv_device(909, HEADS, SEQ, DIM, "bf16", 0.9, 4, layer=0, device=DEV, out_k=K[0], out_v=V[0])
    cK, cV, cdeg, assign = ckv.compress(K, V, chunk, rounds=rounds, n_sink=n1, n_recent=n2)
    torch.cuda.synchronize()
    out_len = oracle.round_lengths(SEQ, chunk, rounds, n1, n2)[-1]
    assert out_len <= SEQ // 4 and cK.shape == (1, HEADS, out_len, DIM)
    assert torch.equal(cdeg.sum(dim=-1), torch.full((1, HEADS), SEQ, dtype=torch.int64, device=DEV))
    assert torch.equal(cK[:, :, :n1], K[:, :, :n1]) and torch.equal(cV[:, :, -n2:], V[:, :, -n2:])
    counts = torch.zeros((HEADS, out_len), dtype=torch.int32, device=DEV)
    counts.scatter_add_(1, assign[0].to(torch.int64), torch.ones((HEADS, SEQ), dtype=torch.int32, device=DEV))
    assert torch.equal(counts, cdeg[0])
    h = 5
    curK, curV, curdeg = K[:, h:h + 1].contiguous(), V[:, h:h + 1].contiguous(), None
    for j, r in enumerate(rounds):
        gK, gV, gdeg, gas = ckv.compress(curK, curV, chunk, rounds=[r], deg=curdeg, n_sink=n1, n_recent=n2)
        torch.cuda.synchronize()
        d_in = np.ones(curK.shape[2], dtype=np.int64) if curdeg is None else i64(curdeg[0, 0])
        check_round_with_edges(f64(curK[0, 0]), f64(curV[0, 0]), d_in, chunk, r, "bf16", n1, n2, f64(gK[0, 0]),
                               f64(gV[0, 0]), i64(gdeg[0, 0]), i64(gas[0, 0]), what=f"head {h} round {j}")
        curK, curV, curdeg = gK, gV, gdeg
    assert torch.equal(cK[0, h], curK[0, 0]) and torch.equal(cV[0, h], curV[0, 0]) and torch.equal(cdeg[0, h], curdeg[0, 0])


# ---- serving decode shape (batch 16, pre-compressed caches, appended tokens) --------------------
def test_serving_decode_batch16_with_appended_tokens():
    """16 sequences of 32768 tokens compressed to 25%, a few decoded tokens appended with degree 1
    (capacity 8192 + 128), per-sequence lengths; compressed (with degrees) and uncompressed
    (degrees = NULL) attention against the oracle on sampled sequences."""
    _say("serving decode: batch 16")
    B, H, S, CAP = 16, HEADS, 32768, 8192 + 128
    K = torch.empty((B, H, S, DIM), dtype=torch.bfloat16, device=DEV)
    V = torch.empty_like(K)
    for b in range(B):
        kv_device(4242, H, S, DIM, "bf16", 0.9, 4, layer=b, device=DEV, out_k=K[b], out_v=V[b])
    cK = torch.zeros((B, H, CAP, DIM), dtype=torch.bfloat16, device=DEV)
    cV = torch.zeros_like(cK)
    cdeg = torch.ones((B, H, CAP), dtype=torch.int32, device=DEV)
    ckv.compress(K, V, CHUNK, retain_ratio=RHO, out=(cK, cV, cdeg, None))       # rows [0, 8192) of the padded cache
    gen = torch.Generator(device=DEV).manual_seed(9)
    n_new = torch.randint(1, 129, (B,), generator=gen, device=DEV)
    cK[:, :, 8192:] = torch.randn((B, H, 128, DIM), generator=gen, device=DEV).to(torch.bfloat16)
    cV[:, :, 8192:] = torch.randn((B, H, 128, DIM), generator=gen, device=DEV).to(torch.bfloat16)
    lens = (8192 + n_new).to(torch.int32)
    q = torch.randn((B, QHEADS, DIM), generator=gen, device=DEV).to(torch.bfloat16)
    o = ckv.decode_attn(q, cK, cV, lens=lens, deg=cdeg, out_dtype=torch.float32)
    o_full = ckv.decode_attn(q, K, V, out_dtype=torch.float32)                  # uncompressed baseline
    torch.cuda.synchronize()
    assert int(cdeg[:, :, :8192].sum()) == B * H * S and bool((cdeg[:, :, 8192:] == 1).all())
    for b in (0, 7, 15):
        ref = oracle.app_attn(f64(q[b]), f64(cK[b]), f64(cV[b]), i64(cdeg[b]), int(lens[b]))
        assert_rows_close(f64(o[b]), ref, ATTN_TOL, f"compressed b{b}")
        ref_full = oracle.app_attn(f64(q[b]), f64(K[b]), f64(V[b]))
        assert_rows_close(f64(o_full[b]), ref_full, ATTN_TOL, f"uncompressed b{b}")


# ---- extreme context: 1M tokens x 32 layers, chunk 2048, layer-streamed ---------------------------
def test_extreme_context_chunk2048_streamed_over_32_layers():
    """The 1 048 576-token workload as bench.py runs it: 32 layers generated and compressed one after
    the other (one ckv_compress call per layer: 8 KV heads, alpha 0.95, chunk 2048, retain 25%), the
    compressed layers kept (32 GiB), then one decode step over all of them.  Invariants on every
    (layer, head); on sampled (layer, head) pairs spread over the run a 65536-token prefix (closed
    under both rounds: 16 round-1 chunks) is checked round by round against the oracle and must equal
    the big call's prefix bit for bit; the decode output of sampled layers is checked against the
    oracle over all 262144 centroids."""
    _say("extreme context: 1M tokens x 32 layers, chunk 2048, layer-streamed")
    Ly, H, S, C = 32, HEADS, 1048576, 2048
    L2, P = S // 4, 65536
    samples = {0: [1], 9: [6], 20: [3], 31: [0, 7]}
    K = torch.empty((1, H, S, DIM), dtype=torch.bfloat16, device=DEV)
    V = torch.empty_like(K)
    cK = torch.empty((Ly, H, L2, DIM), dtype=torch.bfloat16, device=DEV)
    cV = torch.empty_like(cK)
    cdeg = torch.empty((Ly, H, L2), dtype=torch.int32, device=DEV)
    assign = torch.empty((1, H, S), dtype=torch.int32, device=DEV)
    plan = ckv.plan(ckv.layout_of(K), ckv.make_params(C, RHO))
    assert plan.out_seq == L2
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=DEV)
    ones = torch.ones((H, S), dtype=torch.int32, device=DEV)
    for l in range(Ly):
        kv_device(555, H, S, DIM, "bf16", 0.95, 4, layer=l, device=DEV, out_k=K[0], out_v=V[0])
        ckv.compress(K, V, C, retain_ratio=RHO, out=(cK[l:l + 1], cV[l:l + 1], cdeg[l:l + 1], assign), workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(cdeg[l].sum(dim=-1), torch.full((H,), S, dtype=torch.int64, device=DEV)), f"layer {l}"
        counts = torch.zeros((H, L2), dtype=torch.int32, device=DEV)
        counts.scatter_add_(1, assign[0].to(torch.int64), ones)
        assert torch.equal(counts, cdeg[l]), f"layer {l}: degrees do not count the assigned tokens"
        for h in samples.get(l, []):
            _say(f"  oracle check of layer {l} head {h} (prefix of {P} tokens)")
            curK, curV, curdeg = K[:, h:h + 1, :P].contiguous(), V[:, h:h + 1, :P].contiguous(), None
            for j, r in enumerate([1.0, 1.0]):
                gK, gV, gdeg, gas = ckv.compress(curK, curV, C, rounds=[r], deg=curdeg)
                torch.cuda.synchronize()
                d_in = np.ones(curK.shape[2], dtype=np.int64) if curdeg is None else i64(curdeg[0, 0])
                check_round(f64(curK[0, 0]), f64(curV[0, 0]), d_in, C, r, "bf16", f64(gK[0, 0]), f64(gV[0, 0]),
                            i64(gdeg[0, 0]), i64(gas[0, 0]), what=f"1M L{l}H{h} prefix round {j}")
                curK, curV, curdeg = gK, gV, gdeg
            assert torch.equal(cK[l, h, :P // 4], curK[0, 0]) and torch.equal(cV[l, h, :P // 4], curV[0, 0])
            assert torch.equal(cdeg[l, h, :P // 4], curdeg[0, 0])
    del K, V, assign, ws, ones
    assert bool(torch.isfinite(cK.float().sum())) and bool(torch.isfinite(cV.float().sum()))
    # one decode step over the 32 compressed layers, as the benchmark issues it
    gen = torch.Generator(device=DEV).manual_seed(11)
    q = torch.randn((Ly, 1, QHEADS, DIM), generator=gen, device=DEV).to(torch.bfloat16)
    o = torch.empty((Ly, 1, QHEADS, DIM), dtype=torch.float32, device=DEV)
    attn_ws = torch.zeros(ckv.decode_attn_workspace(ckv.layout_of(cK[0:1]), QHEADS), dtype=torch.uint8, device=DEV)
    for l in range(Ly):
        ckv.decode_attn(q[l], cK[l:l + 1], cV[l:l + 1], deg=cdeg[l:l + 1], out=o[l], workspace=attn_ws)
    torch.cuda.synchronize()
    for l in (3, 31):
        _say(f"  oracle attention over compressed layer {l}")
        ref = oracle.app_attn(f64(q[l, 0]), f64(cK[l]), f64(cV[l]), i64(cdeg[l]))
        assert_rows_close(f64(o[l, 0]), ref, ATTN_TOL, f"1M decode layer {l}")
