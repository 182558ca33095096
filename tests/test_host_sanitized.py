"""The host side of the library - the rounds planner (make_plan / carve / route planning), the
annealed schedule, the paged-compression plan and the argument checks that run before any launch -
compiled with AddressSanitizer and UndefinedBehaviorSanitizer (host code only) and driven through the
same cases as test_boundary_host.py.  The sanitized build must report nothing and must return, value
for value, what the regular library returns.  No GPU is needed: every call returns before a launch."""
import ctypes as C
import itertools
import os
import subprocess

import pytest

import paper_2506_11418_amd as ckv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2506_11418_amd", "csrc")
PKG = os.path.join(ROOT, "paper_2506_11418_amd")


def _lay_words(batch, heads, seq, dim, dtype, deg_stride=0, stride_s=None):
    stride_s = dim if stride_s is None else stride_s
    return [batch, heads, seq, dim, heads * seq * stride_s, seq * stride_s, stride_s, dtype, deg_stride]


def _par_words(chunk, rho=1.0, rounds=None, n_sink=0, n_recent=0, scope=0, flags=0):
    r = list(rounds or []) + [0.0] * (8 - len(rounds or []))
    return [chunk, repr(float(rho)), len(rounds or [])] + [repr(float(x)) for x in r] + [n_sink, n_recent, scope, flags]


def _params(chunk, rho=1.0, rounds=None, n_sink=0, n_recent=0, scope=0, flags=0):
    p = ckv.make_params(chunk, rho, rounds, n_sink, n_recent, "head" if scope == 1 else "chunk")
    p.scope, p.flags = scope, flags
    return p


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("hostsan") / "host_sanitize_driver")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, os.path.join(CSRC, "ckv_host.hip"),
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), "-L", PKG, "-l:libckv.so",
           f"-Wl,-rpath,{PKG}", "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    return out


def _cases():
    """(command line for the driver, the regular library's answer in the driver's print format)."""
    L = ckv.lib()
    cases = []

    def plan_case(lay_w, par_w, p):
        lay = ckv.Layout(*lay_w)
        pt = ckv.PlanT()
        st = L.ckv_plan(C.byref(lay), C.byref(p), C.byref(pt))
        want = ["plan", st, pt.out_seq, pt.n_rounds] + list(pt.round_len) + [f"{x:.9g}" for x in pt.round_r] + [pt.workspace_bytes]
        cases.append((["plan"] + lay_w + par_w, want))

    for rho, (seq, chunk) in itertools.product([1.0, 0.75, 0.5, 0.375, 0.3, 0.25, 0.125, 0.1],
                                               [(32768, 1024), (4096, 256), (1000, 64), (77, 16), (1, 2), (2049, 2048)]):
        plan_case(_lay_words(1, 2, seq, 128, ckv.BF16), _par_words(chunk, rho), _params(chunk, rho))
    for rounds, (seq, chunk), (n1, n2), scope, flags in itertools.product(
            [[1.0], [0.5], [0.8, 0.6, 0.4], [1.0, 1.0, 0.3], [0.0], [1.0] * 8],
            [(5000, 256), (333, 32), (8192, 2048), (131072, 1024)], [(0, 0), (16, 64), (100, 300)], [0, 1], [0, 1, 2]):
        plan_case(_lay_words(32, 8, seq, 128, ckv.BF16), _par_words(chunk, 1.0, rounds, n1, n2, scope, flags),
                  _params(chunk, 1.0, rounds, n1, n2, scope, flags))
    # rejected plans: odd chunk, chunk too large, bad ratio, bad scope, both route flags, unknown flag, bad strides
    for par_w, p in [(_par_words(63, 0.5), _params(63, 0.5)), (_par_words(4096, 0.5), _params(4096, 0.5)),
                     (_par_words(64, 0.0), _params(64, 0.0)), (_par_words(64, 0.5, scope=3), _params(64, 0.5, scope=3)),
                     (_par_words(64, 0.5, flags=3), _params(64, 0.5, flags=3)), (_par_words(64, 0.5, flags=8), _params(64, 0.5, flags=8)),
                     (_par_words(64, 1.0, [1.5]), _params(64, 1.0, [1.5])), (_par_words(64, 0.5, n_sink=-1), _params(64, 0.5, n_sink=-1))]:
        plan_case(_lay_words(1, 2, 4096, 128, ckv.BF16), par_w, p)
    plan_case(_lay_words(1, 2, 4096, 128, 7), _par_words(64, 0.5), _params(64, 0.5))                  # bad dtype
    plan_case(_lay_words(1, 2, 4096, 100, ckv.BF16), _par_words(64, 0.5), _params(64, 0.5))            # row not 16-byte
    plan_case(_lay_words(1, 2, 0, 128, ckv.BF16), _par_words(64, 0.5), _params(64, 0.5))               # empty
    plan_case(_lay_words(1, 2, 4096, 128, ckv.BF16, deg_stride=100), _par_words(64, 0.5), _params(64, 0.5))

    for seq, chunk, budget, n1, n2, floor_ in [(10000, 1000, 6000, 0, 0, 0.0), (10000, 1000, 3024, 0, 0, 0.0),
                                               (10000, 1000, 2500, 0, 0, 0.2), (4096, 256, 1024, 16, 64, 0.2),
                                               (32768, 1024, 8192, 16, 64, 0.4), (333, 32, 200, 4, 8, 0.0), (500, 64, 500, 0, 0, 0.0),
                                               (10000, 1000, 2500, 0, 0, 0.0), (1 << 20, 64, 100, 0, 0, 0.2), (1000, 63, 500, 0, 0, 0.0)]:
        for scope in (0, 1):
            p = ckv.Params()
            st = L.ckv_schedule_annealed(seq, chunk, n1, n2, scope, budget, 0.8, 0.2, floor_, C.byref(p))
            cases.append((["anneal", seq, chunk, n1, n2, scope, budget, repr(0.8), repr(0.2), repr(floor_)],
                          ["anneal", st, p.n_rounds] + [f"{x:.9g}" for x in p.r]))

    for (bs, max_blocks, n_blocks), seq, lens, par in [
            ((16, 300, 1000), 4176, [], dict(chunk=256, rho=0.25, n_sink=16, n_recent=64)),
            ((16, 300, 1000), 4176, [], dict(chunk=256, rho=1.0, rounds=[0.5])),
            ((16, 300, 1000), 4096, [], dict(chunk=256, rho=0.25, flags=2)),
            ((16, 300, 1000), 0, [4096, 1000], dict(chunk=256, rho=0.5)),
            ((32, 2048, 70000), 0, [65536, 65536, 3000, 1, 70], dict(chunk=1024, rho=0.25)),
            ((24, 300, 1000), 4096, [], dict(chunk=256, rho=0.5)),
            ((16, 300, 1000), 4801, [], dict(chunk=256, rho=0.5)),
            ((4, 3000, 4000), 4096, [], dict(chunk=256, rho=0.5)),
            ((16, 300, 1000), 0, [4096, 0], dict(chunk=256, rho=0.5))]:
        batch = max(len(lens), 2)
        pl = ckv.PagedLayout(batch, 8, 128, ckv.BF16, bs, max_blocks, n_blocks)
        p = _params(**par)
        hl = (C.c_int32 * len(lens))(*lens) if lens else None
        out = (C.c_int32 * max(len(lens), 1))(*([-1] * max(len(lens), 1)))
        nf, nb = C.c_int32(-1), C.c_size_t(0)
        st = L.ckv_paged_compress_plan(C.byref(pl), seq, hl, C.byref(p), out, C.byref(nf), C.byref(nb))
        cases.append((["pplan", batch, 8, 128, ckv.BF16, bs, max_blocks, n_blocks, seq, len(lens)] + lens + _par_words(**par),
                      ["pplan", st, nf.value, nb.value] + list(out)))

    pl_w = [2, 8, 128, ckv.BF16, 16, 300, 1000]
    pl = ckv.PagedLayout(*pl_w)
    for seq, chunk, ratio, n, old, new in [(1000, 64, 0.25, 131072, 4176, 1100), (0, 2, 0.3, 10, 16, 16), (100, 3, 0.0, 10, 10, 11),
                                           (-1, 4, 1.5, 10, 4801, 1), (2049, 2048, 0.999, 1000, 17, 16)]:
        cases.append((["sizes", seq, chunk, repr(ratio), n] + pl_w + [old, new],
                      ["sizes", L.ckv_n_sources(seq, chunk), L.ckv_budget_tokens(ratio, n),
                       L.ckv_paged_freed_blocks(C.byref(pl), old, new)]))

    for lay_w, qh in [(_lay_words(1, 8, 8192, 128, ckv.BF16), 32), (_lay_words(16, 8, 8320, 128, ckv.BF16), 32),
                      (_lay_words(1, 2, 100, 64, ckv.F32), 3), (_lay_words(256, 8, 4096, 128, ckv.BF16), 64)]:
        n = C.c_size_t(0)
        st = L.ckv_decode_attn_workspace(C.byref(ckv.Layout(*lay_w)), qh, C.byref(n))
        cases.append((["attn_ws"] + lay_w + [qh], ["attn_ws", st, n.value]))

    # argument errors of ckv_compress / ckv_match that the host finds before a launch
    good, pw = _lay_words(1, 2, 4096, 128, ckv.BF16), _par_words(256, 0.5)
    for lay_w, out_w, ws_bytes, k_addr, want in [
            (good, _lay_words(1, 2, 100, 128, ckv.BF16), 1 << 30, 4096, -2),          # output too short
            (good, _lay_words(1, 3, 2048, 128, ckv.BF16), 1 << 30, 4096, -2),         # head count differs
            (good, _lay_words(1, 2, 2048, 128, ckv.BF16), 16, 4096, -4),              # workspace too small
            (good, _lay_words(1, 2, 2048, 128, ckv.BF16), 1 << 30, 4100, -3),         # K misaligned
            (good, _lay_words(1, 2, 2048, 128, ckv.BF16), 1 << 30, 0, -1),            # K null
            (_lay_words(1, 2, 4096, 48, ckv.F32), _lay_words(1, 2, 2048, 48, ckv.F32), 1 << 30, 4096, -5)]:   # no kernel for dim 48
        cases.append((["compress_err"] + lay_w + out_w + pw + [ws_bytes, k_addr], ["compress_err", want]))
    cases.append((["match_err"] + good + [256], ["match_err", -1]))
    cases.append((["match_err"] + good + [255], ["match_err", -1]))
    return cases


def test_sanitized_host_code_agrees_with_the_library_and_reports_nothing(driver):
    cases = _cases()
    assert len(cases) > 500
    text = "\n".join(" ".join(str(w) for w in cmd) for cmd, _ in cases) + "\n"
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["LD_LIBRARY_PATH"] = PKG + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    res = subprocess.run([driver], input=text, capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, f"sanitized driver failed:\n{res.stderr[-4000:]}"
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
    lines = res.stdout.strip().splitlines()
    assert lines[-1].startswith("done ckv") and lines[-1].endswith("workspace too small")
    assert len(lines) == len(cases) + 1
    for (cmd, want), got in zip(cases, lines):
        assert got.split() == [str(w) for w in want], f"{' '.join(str(w) for w in cmd)}\n  sanitized: {got}\n  library:   {want}"
