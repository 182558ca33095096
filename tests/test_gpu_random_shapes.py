"""GPU parity on a fixed list of pseudo-randomly drawn configurations: odd lengths, every chunk
size class, mixed merge fractions, sinks / recents, both selection scopes, incoming degrees.  Each
round is checked against the oracle (teacher-forced); the multi-round call must reproduce the
rounds issued one by one bit for bit (it takes the deferred-value path where it applies)."""

import numpy as np
import pytest
import torch

import oracle
import paper_2506_11418_amd as ckv
from parity_util import check_round_with_edges, f64, i64
from synth import kv_host

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _compress(route, *args, **kw):
    """ckv.compress on a named kernel route (the routes give the same bits)."""
    return ckv.compress(*args, route=route, **kw)


def _cases():
    rng = np.random.default_rng(20250611)
    out = []
    for k in range(28):
        dtype = "bf16" if k % 4 else "f32"
        dim = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([16, 32, 64, 128]))
        chunk = int(rng.choice([2, 4, 8, 16, 64, 256, 512, 1024, 2048]))
        seq = int(rng.integers(1, 4 * chunk + 40)) if chunk >= 256 else int(rng.integers(1, 1500))
        heads = int(rng.integers(1, 4))
        n_rounds = int(rng.integers(1, 4))
        rounds = [float(rng.choice([0.0, 0.25, 0.5, 0.8, 1.0, 1.0, 1.0])) for _ in range(n_rounds)]
        n_sink = int(rng.choice([0, 0, 4, 16]))
        n_recent = int(rng.choice([0, 0, 7, 64]))
        scope = "head" if k % 5 == 3 else "chunk"
        use_deg = bool(k % 3 == 1)
        out.append((k, dtype, heads, seq, dim, chunk, rounds, n_sink, n_recent, scope, use_deg))
    # longer schedules (a second stream, so the cases above stay what they were): deferred pairs
    # after full rounds, in the middle and at the end of a schedule
    rng = np.random.default_rng(20250612)
    for k in range(28, 48):
        dtype = "bf16" if k % 4 else "f32"
        dim = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([16, 32, 64, 128]))
        chunk = int(rng.choice([4, 16, 64, 256, 512, 1024, 2048]))
        seq = int(rng.integers(1, 4 * chunk + 40)) if chunk >= 256 else int(rng.integers(1, 1500))
        rounds = [float(rng.choice([0.5, 0.8, 1.0, 1.0, 1.0])) for _ in range(int(rng.integers(3, 6)))]
        out.append((k, dtype, int(rng.integers(1, 3)), seq, dim, chunk, rounds, int(rng.choice([0, 4])),
                    int(rng.choice([0, 7])), "chunk", bool(k % 3 == 1)))
    # chunk sizes between the kernels' size classes (a third stream): 128 goes to the small-chunk similarity
    # kernel like 64 and 256, 32 / 96 / 384 to the one-chunk-per-workgroup kernel
    rng = np.random.default_rng(20250613)
    for k in range(48, 62):
        dtype = "bf16" if k % 5 else "f32"
        dim = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([32, 64]))
        chunk = int(rng.choice([32, 96, 128, 128, 384]))
        seq = int(rng.integers(chunk, 2600))
        rounds = [float(rng.choice([0.25, 0.5, 0.8, 1.0, 1.0])) for _ in range(int(rng.integers(1, 4)))]
        out.append((k, dtype, int(rng.integers(1, 4)), seq, dim, chunk, rounds, int(rng.choice([0, 16])),
                    int(rng.choice([0, 64])), "head" if k % 7 == 3 else "chunk", bool(k % 3 == 1)))
    return out


@pytest.mark.parametrize("k,dtype,heads,seq,dim,chunk,rounds,n_sink,n_recent,scope,use_deg", _cases())
def test_random_configuration(k, dtype, heads, seq, dim, chunk, rounds, n_sink, n_recent, scope, use_deg):
    print(f"case {k}: {dtype} H={heads} S={seq} D={dim} c={chunk} rounds={rounds} n1={n_sink} n2={n_recent} "
          f"scope={scope} deg={use_deg}", flush=True)
    K, V, _ = kv_host(900 + k, heads, seq, dim, dtype, alpha=0.9, n_outlier=4 if dim == 128 else 0)
    K, V = K.to(DEV), V.to(DEV)
    deg = None
    if use_deg:
        deg = torch.from_numpy(np.random.default_rng(k).integers(1, 9, (1, heads, seq)).astype(np.int32)).to(DEV)
    kw = dict(n_sink=n_sink, n_recent=n_recent, scope=scope)
    curK, curV, curdeg, maps = K, V, deg, []
    for j, r in enumerate(rounds):
        gK, gV, gdeg, gas = ckv.compress(curK, curV, chunk, rounds=[r], deg=curdeg, **kw)
        torch.cuda.synchronize()
        for h in range(heads):
            d_in = np.ones(curK.shape[2], dtype=np.int64) if curdeg is None else i64(curdeg[0, h])
            check_round_with_edges(f64(curK[0, h]), f64(curV[0, h]), d_in, chunk, r, dtype, n_sink, n_recent,
                                   f64(gK[0, h]), f64(gV[0, h]), i64(gdeg[0, h]), i64(gas[0, h]),
                                   what=f"case {k} round {j} h{h}", scope=scope)
        curK, curV, curdeg = gK, gV, gdeg
        maps.append(gas.to(torch.int64))
    gK, gV, gdeg, gas = _compress("defer_always", K, V, chunk, rounds=rounds, deg=deg, **kw)
    torch.cuda.synchronize()
    assert gK.shape[2] == oracle.round_lengths(seq, chunk, rounds, n_sink, n_recent, scope=scope)[-1]
    assert torch.equal(gK, curK) and torch.equal(gV, curV) and torch.equal(gdeg, curdeg)
    comp = maps[0]
    for m in maps[1:]:
        comp = torch.gather(m, 2, comp)
    assert torch.equal(gas.to(torch.int64), comp)
    total = heads * seq if deg is None else int(deg.sum())
    assert int(gdeg.sum()) == total
