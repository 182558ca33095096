"""CPU-only checks of the C-ABI library: it loads, exports what include/ckv.h declares, and its
host-side logic (schedule, lengths, argument validation) agrees with the oracle's integer math.
No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import paper_2506_11418_amd as ckv
from oracle import direct_schedule, round_lengths

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lay(batch=1, heads=2, seq=4096, dim=128, dtype=ckv.BF16):
    return ckv.Layout(batch, heads, seq, dim, heads * seq * dim, seq * dim, dim, dtype)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ckv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(ckv_[a-z_]+)\s*\(", header))
    assert {"ckv_plan", "ckv_match", "ckv_compress", "ckv_decode_attn", "ckv_decode_attn_workspace",
            "ckv_version", "ckv_strerror", "ckv_append", "ckv_schedule_annealed", "ckv_paged_decode_attn",
            "ckv_paged_gather", "ckv_paged_scatter", "ckv_paged_append", "ckv_paged_compress", "ckv_paged_compress_plan"} <= names
    L = ckv.lib()
    for n in names:
        assert hasattr(L, n), n
    assert "gfx950" in ckv.version()
    assert L.ckv_strerror(-4).decode() == "workspace too small"


@pytest.mark.parametrize("rho", [1.0, 0.75, 0.5, 0.375, 0.3, 0.25, 0.125, 0.1])
@pytest.mark.parametrize("seq,chunk", [(32768, 1024), (4096, 256), (1000, 64), (77, 16), (1, 2), (2049, 2048)])
def test_plan_matches_oracle_schedule_and_lengths(rho, seq, chunk):
    pl = ckv.plan(_lay(seq=seq), ckv.make_params(chunk, rho))
    sched = direct_schedule(rho)
    assert len(pl.round_r) == len(sched)
    for a, b in zip(pl.round_r, sched):
        assert abs(a - b) < 1e-6
    assert pl.round_len == round_lengths(seq, chunk, pl.round_r)
    assert pl.out_seq == pl.round_len[-1]


@pytest.mark.parametrize("rounds", [[1.0], [0.5], [0.8, 0.6, 0.4], [1.0, 1.0, 0.3], [0.0]])
def test_plan_explicit_rounds(rounds):
    for seq, chunk in [(5000, 256), (333, 32), (8192, 2048)]:
        pl = ckv.plan(_lay(seq=seq), ckv.make_params(chunk, rounds=rounds))
        assert pl.round_len == round_lengths(seq, chunk, rounds)


@pytest.mark.parametrize("n_sink,n_recent", [(4, 0), (0, 64), (16, 64), (100, 300)])
def test_plan_with_sinks_and_recents(n_sink, n_recent):
    for seq, chunk, rounds in [(5000, 256, [1.0, 0.5]), (333, 32, [0.7]), (300, 64, [1.0, 1.0, 1.0]), (50, 16, [1.0])]:
        pl = ckv.plan(_lay(seq=seq), ckv.make_params(chunk, rounds=rounds, n_sink=n_sink, n_recent=n_recent))
        assert pl.round_len == round_lengths(seq, chunk, rounds, n_sink, n_recent)


@pytest.mark.parametrize("seq,chunk,budget,n_sink,n_recent,r_floor", [
    (10000, 1000, 6000, 0, 0, 0.0), (10000, 1000, 3024, 0, 0, 0.0), (10000, 1000, 2500, 0, 0, 0.2),
    (4096, 256, 1024, 16, 64, 0.2), (32768, 1024, 8192, 16, 64, 0.4), (333, 32, 200, 4, 8, 0.0), (500, 64, 500, 0, 0, 0.0),
])
def test_annealed_schedule_matches_the_oracle_loop(seq, chunk, budget, n_sink, n_recent, r_floor):
    from oracle import rounds_to_budget
    got = ckv.schedule_annealed(seq, chunk, budget, 0.8, 0.2, r_floor, n_sink, n_recent)
    assert got == rounds_to_budget(seq, chunk, budget, 0.8, 0.2, r_floor, n_sink, n_recent)
    if got:
        pl = ckv.plan(_lay(seq=seq), ckv.make_params(chunk, rounds=got, n_sink=n_sink, n_recent=n_recent))
        assert pl.out_seq <= budget < pl.round_len[-2]


def test_annealed_schedule_reports_a_budget_it_cannot_reach():
    with pytest.raises(ckv.CkvError) as e:      # Eq. 4 as printed stalls at 30.24% with the defaults
        ckv.schedule_annealed(10000, 1000, 2500, 0.8, 0.2, 0.0)
    assert e.value.status == -5
    with pytest.raises(ckv.CkvError):           # more than 8 rounds
        ckv.schedule_annealed(1 << 20, 64, 100, 0.8, 0.2, 0.2)
    p = ckv.Params()
    L = ckv.lib()
    assert L.ckv_schedule_annealed(1000, 63, 0, 0, 0, 500, 0.8, 0.2, 0.0, C.byref(p)) == -1
    assert L.ckv_schedule_annealed(1000, 64, 0, 0, 0, 500, 1.5, 0.2, 0.0, C.byref(p)) == -1
    assert L.ckv_schedule_annealed(1000, 64, 0, 0, 7, 500, 0.8, 0.2, 0.0, C.byref(p)) == -1
    assert L.ckv_schedule_annealed(1000, 64, 0, 0, 0, 500, 0.8, 0.2, 0.0, None) == -1


def test_append_rejects_bad_arguments_before_any_launch():
    L = ckv.lib()
    lay, z, a = _lay(seq=128), C.c_void_p(0), C.c_void_p(4096)
    assert L.ckv_append(z, a, a, a, z, C.byref(lay), z, 0, z) == -1
    assert L.ckv_append(a, a, C.c_void_p(4100), a, z, C.byref(lay), z, 0, z) == -3
    assert L.ckv_append(a, a, a, a, z, C.byref(lay), z, 128, z) == -2          # row outside the capacity
    assert L.ckv_append(a, a, a, a, z, C.byref(lay), z, -1, z) == -2
    bad = _lay(seq=128)
    bad.deg_stride = 100                                                       # rows would overlap
    assert L.ckv_append(a, a, a, a, z, C.byref(bad), z, 0, z) == -2


@pytest.mark.parametrize("seq,chunk,rounds,n_sink,n_recent", [
    (5000, 256, [0.3], 0, 0), (5001, 256, [0.7, 0.45], 16, 64), (777, 32, [1.0, 0.5, 0.25], 3, 0), (9, 4, [1.0], 0, 0),
    (131072, 1024, [0.8, 0.6], 16, 64),
])
def test_plan_with_selection_over_the_whole_sequence(seq, chunk, rounds, n_sink, n_recent):
    pl = ckv.plan(_lay(seq=seq), ckv.make_params(chunk, rounds=rounds, n_sink=n_sink, n_recent=n_recent, scope="head"))
    assert pl.round_len == round_lengths(seq, chunk, rounds, n_sink, n_recent, scope="head")
    per_chunk = ckv.plan(_lay(seq=seq), ckv.make_params(chunk, rounds=rounds, n_sink=n_sink, n_recent=n_recent))
    assert pl.workspace_bytes > per_chunk.workspace_bytes or pl.round_len != per_chunk.round_len
    bad = ckv.make_params(chunk, rounds=rounds)
    bad.scope = 3
    assert ckv.lib().ckv_plan(C.byref(_lay(seq=seq)), C.byref(bad), C.byref(ckv.PlanT())) == -1


def test_paged_plan_and_argument_checks():
    L = ckv.lib()
    pl = ckv.PagedLayout(2, 8, 128, ckv.BF16, 16, 300, 1000)
    par = ckv.make_params(256, 0.25, n_sink=16, n_recent=64)
    out_seq, n_freed, nbytes = ckv.paged_compress_plan(pl, 4096 + 80, par)
    assert out_seq == round_lengths(4176, 256, [1.0, 1.0], 16, 64)[-1]
    assert n_freed == -(-4176 // 16) - (-(-out_seq // 16))
    # nothing is gathered: the scratch is ckv_compress's own workspace plus, for this two-round schedule that
    # stays below the size where values are deferred, no staging at all (the last round writes the pages directly)
    inner = ckv.plan(_lay(batch=2, heads=8, seq=4176), par).workspace_bytes
    assert inner <= nbytes < inner + 4096
    # a single round reads the pools while it writes: keys, values and degrees of the result are staged
    one = ckv.make_params(256, rounds=[0.5])
    o1, _, n1 = ckv.paged_compress_plan(pl, 4176, one)
    assert n1 >= ckv.plan(_lay(batch=2, heads=8, seq=4176), one).workspace_bytes + 2 * 8 * o1 * (2 * 128 * 2 + 4)
    # one deferred pair: the last round still reads the original values and degrees, the keys go straight to the pages
    dp = ckv.make_params(256, 0.25, route="defer_always")
    o2, _, n2 = ckv.paged_compress_plan(pl, 4096, dp)
    base = ckv.plan(_lay(batch=2, heads=8, seq=4096), dp).workspace_bytes
    assert base + 2 * 8 * o2 * (128 * 2 + 4) <= n2 < base + 2 * 8 * o2 * (128 * 2 + 4) + 4096
    # per-sequence lengths: lengths after compression per sequence, the most blocks any sequence releases
    outs, nf, _ = ckv.paged_compress_plan(pl, 0, ckv.make_params(256, 0.5), seq_lens=[4096, 1000])
    assert outs == [round_lengths(4096, 256, [1.0])[-1], round_lengths(1000, 256, [1.0])[-1]]
    assert nf == 256 - 128
    z, a = C.c_void_p(0), C.c_void_p(4096)
    bad = ckv.PagedLayout(2, 8, 128, ckv.BF16, 24, 300, 1000)              # block size not a power of two
    assert L.ckv_paged_compress_plan(C.byref(bad), 4096, None, C.byref(ckv.make_params(256, 0.5)), None, None, None) == -2
    assert L.ckv_paged_compress_plan(C.byref(pl), 16 * 300 + 1, None, C.byref(ckv.make_params(256, 0.5)), None, None, None) == -2
    small = ckv.PagedLayout(2, 8, 128, ckv.BF16, 4, 3000, 4000)            # blocks under 8 tokens: no kernel
    assert L.ckv_paged_compress_plan(C.byref(small), 4096, None, C.byref(ckv.make_params(256, 0.5)), None, None, None) == -5
    two = (C.c_int32 * 2)(4096, 0)                                         # an empty sequence
    assert L.ckv_paged_compress_plan(C.byref(pl), 0, two, C.byref(ckv.make_params(256, 0.5)), None, None, None) == -2
    n = C.c_size_t(0)
    assert L.ckv_paged_decode_attn_workspace(C.byref(pl), 32, 4096, C.byref(n)) == 0 and n.value > 0
    assert L.ckv_paged_decode_attn_workspace(C.byref(pl), 30, 4096, C.byref(n)) == -2
    assert L.ckv_paged_decode_attn(a, 32, a, a, z, a, z, C.byref(pl), 4096, 0.0, a, 0, a, n.value, z) == -1   # lens required
    assert L.ckv_paged_decode_attn(a, 32, a, a, z, a, a, C.byref(pl), 4096, 0.0, a, 0, a, 16, z) == -4
    assert L.ckv_paged_append(a, a, a, a, z, a, z, C.byref(pl), z) == -1                                      # lens required
    assert L.ckv_paged_append(a, a, C.c_void_p(4100), a, z, a, a, C.byref(pl), z) == -3
    lay = _lay(batch=2, heads=8, seq=512)
    assert L.ckv_paged_gather(a, a, z, a, C.byref(pl), 1024, a, a, z, C.byref(lay), z) == -2                 # seq > out->seq
    assert L.ckv_paged_scatter(a, a, z, C.byref(lay), a, a, z, a, C.byref(pl), 100, z, z, z) == -2           # old_seq < seq
    assert L.ckv_paged_compress(a, a, z, a, z, C.byref(pl), 4096, None, C.byref(ckv.make_params(256, 0.5)), z, 0, a, 1 << 30, z) == -1
    assert L.ckv_paged_compress(a, a, a, a, z, C.byref(pl), 4096, None, C.byref(ckv.make_params(256, 0.5)), z, 0, a, 1 << 10, z) == -4
    assert L.ckv_paged_compress(a, a, a, a, z, C.byref(pl), 4096, None, C.byref(ckv.make_params(256, 0.5)), a, 10, a, 1 << 30, z) == -2   # freed rows too short


def test_plan_workspace_grows_with_rounds():
    one = ckv.plan(_lay(), ckv.make_params(1024, 0.5)).workspace_bytes
    two = ckv.plan(_lay(), ckv.make_params(1024, 0.25)).workspace_bytes
    assert 0 < one < two
    # two rounds keep one intermediate cache: K, V (bf16) and degrees for 2 heads x 2048 tokens
    assert two - one >= 2 * 2048 * (2 * 128 * 2 + 4)


def test_plan_rejects_bad_arguments():
    L = ckv.lib()
    pt = ckv.PlanT()

    def st(lay, p):
        return L.ckv_plan(C.byref(lay), C.byref(p), C.byref(pt))

    ok = ckv.make_params(256, 0.5)
    assert st(_lay(), ok) == 0
    assert st(_lay(), ckv.make_params(255, 0.5)) == -1          # odd chunk
    assert st(_lay(), ckv.make_params(0, 0.5)) == -1
    assert st(_lay(), ckv.make_params(4096, 0.5)) == -1         # chunk > 2048
    assert st(_lay(), ckv.make_params(256, 0.0)) == -1          # ratio outside (0,1]
    assert st(_lay(), ckv.make_params(256, 1.5)) == -1
    assert st(_lay(), ckv.make_params(256, rounds=[1.2])) == -1
    assert st(_lay(seq=0), ok) == -2
    assert st(_lay(dtype=7), ok) == -1
    bad = _lay()
    bad.stride_s = 100                                          # smaller than dim
    assert st(bad, ok) == -2
    odd = _lay()
    odd.stride_s = 132                                          # 264 bytes: not a multiple of 16
    assert st(odd, ok) == -3
    assert st(_lay(), ckv.make_params(256, 0.5, n_sink=-1)) == -1
    assert st(_lay(), ckv.make_params(256, 0.5, n_recent=-4)) == -1
    assert L.ckv_plan(None, C.byref(ok), C.byref(pt)) == -1


def test_entry_points_reject_null_and_misaligned_pointers_before_any_launch():
    L = ckv.lib()
    lay, p = _lay(), ckv.make_params(256, 0.5)
    z = C.c_void_p(0)
    assert L.ckv_compress(z, z, z, C.byref(lay), C.byref(p), z, z, z, C.byref(lay), z, z, 0, z) == -1
    short = _lay(seq=100)                                       # output shorter than the plan's length
    a = C.c_void_p(4096)
    assert L.ckv_compress(a, a, z, C.byref(lay), C.byref(p), a, a, a, C.byref(short), z, a, 1 << 30, z) == -2
    assert L.ckv_compress(a, a, z, C.byref(lay), C.byref(p), a, a, a, C.byref(lay), z, a, 1 << 30, z) == -1  # overlap
    big = C.c_void_p(1 << 40)
    far = C.c_void_p(1 << 41)
    ws = C.c_void_p(1 << 42)
    assert L.ckv_compress(a, big, z, C.byref(lay), C.byref(p), far, C.c_void_p((1 << 41) + (1 << 30)), ws,
                          C.byref(lay), z, C.c_void_p(1 << 43), 16, z) == -4             # workspace too small
    n = C.c_size_t(0)
    assert L.ckv_decode_attn_workspace(C.byref(lay), 8, C.byref(n)) == 0 and n.value > 0
    assert L.ckv_decode_attn_workspace(C.byref(lay), 3, C.byref(n)) == -2        # 3 % 2 heads
    assert L.ckv_decode_attn(z, 8, z, z, C.byref(lay), z, z, 0.0, z, 1, z, 0, z) == -1
    assert L.ckv_match(z, C.byref(lay), 256, z, z, z) == -1
    assert L.ckv_match(C.c_void_p(8), C.byref(lay), 256, C.c_void_p(16), C.c_void_p(16), z) == -3
    assert L.ckv_match(C.c_void_p(16), C.byref(lay), 251, C.c_void_p(16), C.c_void_p(16), z) == -1   # odd chunk


def test_host_helpers_for_sizes_the_binding_no_longer_computes():
    L = ckv.lib()
    for seq, chunk in [(0, 2), (1, 2), (1000, 64), (131072, 1024), (2049, 2048), (77, 16)]:
        want = sum((min(chunk, seq - g0) + 1) // 2 for g0 in range(0, seq, chunk))      # ceil(L/2) per chunk (Sec. 5.2)
        assert L.ckv_n_sources(seq, chunk) == want
    assert L.ckv_n_sources(100, 3) == -1 and L.ckv_n_sources(-1, 4) == -2
    # Algorithm 1: B = floor(R * n); the paper's 25% budget of its 128k prompts; exact products stay exact
    assert ckv.budget_tokens(0.25, 131072) == 32768
    assert ckv.budget_tokens(0.3, 10) == 3 and ckv.budget_tokens(0.6, 5) == 3 and ckv.budget_tokens(1.0, 7) == 7
    assert ckv.budget_tokens(0.999, 1000) == 999
    assert L.ckv_budget_tokens(0.0, 10) == -1 and L.ckv_budget_tokens(1.5, 10) == -1 and L.ckv_budget_tokens(0.5, -1) == -2
    pl = ckv.PagedLayout(2, 8, 128, ckv.BF16, 16, 300, 1000)
    assert L.ckv_paged_freed_blocks(C.byref(pl), 4176, 1100) == 261 - 69
    assert L.ckv_paged_freed_blocks(C.byref(pl), 16, 16) == 0 and L.ckv_paged_freed_blocks(C.byref(pl), 17, 16) == 1
    assert L.ckv_paged_freed_blocks(C.byref(pl), 10, 11) == -2 and L.ckv_paged_freed_blocks(C.byref(pl), 4801, 1) == -2


def test_route_flags_size_the_workspace_and_reject_nonsense():
    """A deferred pair at the start of the schedule without sinks / recents needs no intermediate
    value cache: the plan for it is smaller by exactly that cache (the route flags change kernels
    and scratch, never lengths)."""
    lay = _lay(batch=32, heads=8, seq=131072)
    full = ckv.plan(lay, ckv.make_params(1024, 0.25, route="full_rounds"))
    auto = ckv.plan(lay, ckv.make_params(1024, 0.25))
    forced = ckv.plan(lay, ckv.make_params(1024, 0.25, route="defer_always"))
    assert full.round_len == auto.round_len == forced.round_len == [131072, 65536, 32768]
    lists = 256 * 128 * 3 * 512 * 2
    assert full.workspace_bytes - auto.workspace_bytes == 256 * 65536 * 128 * 2 - lists
    assert auto.workspace_bytes == forced.workspace_bytes
    small = _lay(seq=8192)          # 16 chunks in the second round: too small to defer unless asked to
    assert ckv.plan(small, ckv.make_params(1024, 0.25)).workspace_bytes == \
        ckv.plan(small, ckv.make_params(1024, 0.25, route="full_rounds")).workspace_bytes
    assert ckv.plan(small, ckv.make_params(1024, 0.25, route="defer_always")).workspace_bytes < \
        ckv.plan(small, ckv.make_params(1024, 0.25)).workspace_bytes
    # sinks / recents keep the staging value cache (their rows are copied in every round)
    with_edges = ckv.plan(lay, ckv.make_params(1024, 0.25, n_sink=16, n_recent=64))
    assert with_edges.workspace_bytes > auto.workspace_bytes + 256 * 60000 * 128 * 2
    p = ckv.make_params(1024, 0.25)
    p.flags = 3
    assert ckv.lib().ckv_plan(C.byref(lay), C.byref(p), C.byref(ckv.PlanT())) == -1
    p.flags = 8
    assert ckv.lib().ckv_plan(C.byref(lay), C.byref(p), C.byref(ckv.PlanT())) == -1
