"""Thin Python binding of libckv (C ABI in include/ckv.h).

Only argument marshalling happens here: torch tensors provide device memory and the current HIP
stream; every step of the path runs in the library's kernels.  There is no CPU fallback: if the
shared library has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckv.so")
MAX_ROUNDS = 8
F32, BF16 = 0, 1
_DT = {torch.float32: F32, torch.bfloat16: BF16}


class CkvError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {lib().ckv_strerror(status).decode()} (status {status})")
        self.status = status


class Layout(C.Structure):
    _fields_ = [("batch", C.c_int32), ("heads", C.c_int32), ("seq", C.c_int32), ("dim", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_s", C.c_int64),
                ("dtype", C.c_int32), ("deg_stride", C.c_int64)]


class Params(C.Structure):
    _fields_ = [("chunk", C.c_int32), ("retain_ratio", C.c_float), ("n_rounds", C.c_int32),
                ("r", C.c_float * MAX_ROUNDS), ("n_sink", C.c_int32), ("n_recent", C.c_int32),
                ("scope", C.c_int32), ("flags", C.c_uint32)]


class PagedLayout(C.Structure):
    _fields_ = [("batch", C.c_int32), ("heads", C.c_int32), ("dim", C.c_int32), ("dtype", C.c_int32),
                ("block_size", C.c_int32), ("max_blocks", C.c_int32), ("n_blocks", C.c_int32)]


class PlanT(C.Structure):
    _fields_ = [("out_seq", C.c_int32), ("n_rounds", C.c_int32),
                ("round_len", C.c_int32 * (MAX_ROUNDS + 1)), ("round_r", C.c_float * MAX_ROUNDS),
                ("workspace_bytes", C.c_size_t)]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("total_ms", C.c_double), ("launches", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    """Load libckv.so (built in-tree by paper_2506_11418_amd.build); fail loudly if missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2506_11418_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int32
        L.ckv_version.restype = C.c_char_p
        L.ckv_strerror.restype = C.c_char_p
        L.ckv_strerror.argtypes = [C.c_int]
        L.ckv_plan.argtypes = [C.POINTER(Layout), C.POINTER(Params), C.POINTER(PlanT)]
        L.ckv_n_sources.argtypes = [i32, i32]
        L.ckv_n_sources.restype = i32
        L.ckv_budget_tokens.argtypes = [C.c_float, i32]
        L.ckv_budget_tokens.restype = i32
        L.ckv_match.argtypes = [vp, C.POINTER(Layout), i32, vp, vp, vp]
        L.ckv_compress.argtypes = [vp, vp, vp, C.POINTER(Layout), C.POINTER(Params), vp, vp, vp,
                                   C.POINTER(Layout), vp, vp, C.c_size_t, vp]
        L.ckv_decode_attn_workspace.argtypes = [C.POINTER(Layout), i32, C.POINTER(C.c_size_t)]
        L.ckv_decode_attn.argtypes = [vp, i32, vp, vp, C.POINTER(Layout), vp, vp, C.c_float, vp, i32,
                                      vp, C.c_size_t, vp]
        L.ckv_decode_attn_noalloc.argtypes = [vp, i32, vp, vp, C.POINTER(Layout), vp, vp, C.c_float, vp, i32, vp]
        L.ckv_schedule_annealed.argtypes = [i32, i32, i32, i32, i32, i32, C.c_float, C.c_float, C.c_float,
                                            C.POINTER(Params)]
        L.ckv_append.argtypes = [vp, vp, vp, vp, vp, C.POINTER(Layout), vp, i32, vp]
        PL = C.POINTER(PagedLayout)
        L.ckv_paged_decode_attn_workspace.argtypes = [PL, i32, i32, C.POINTER(C.c_size_t)]
        L.ckv_paged_decode_attn.argtypes = [vp, i32, vp, vp, vp, vp, vp, PL, i32, C.c_float, vp, i32, vp,
                                            C.c_size_t, vp]
        L.ckv_paged_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, PL, vp]
        L.ckv_paged_gather.argtypes = [vp, vp, vp, vp, PL, i32, vp, vp, vp, C.POINTER(Layout), vp]
        L.ckv_paged_scatter.argtypes = [vp, vp, vp, C.POINTER(Layout), vp, vp, vp, vp, PL, i32, vp, vp, vp]
        L.ckv_paged_freed_blocks.argtypes = [PL, i32, i32]
        L.ckv_paged_freed_blocks.restype = i32
        L.ckv_paged_compress_plan.argtypes = [PL, i32, C.POINTER(i32), C.POINTER(Params), C.POINTER(i32),
                                              C.POINTER(i32), C.POINTER(C.c_size_t)]
        L.ckv_paged_compress.argtypes = [vp, vp, vp, vp, vp, PL, i32, C.POINTER(i32), C.POINTER(Params), vp, i32, vp,
                                         C.c_size_t, vp]
        L.ckv_bench_mfma_ceiling.argtypes = [i32, i32, i32, vp, C.c_size_t, C.POINTER(C.c_double), vp]
        L.ckv_timing_enable.argtypes = [C.c_int]
        L.ckv_timing_select.argtypes = [C.c_char_p]
        L.ckv_timing_read.argtypes = [C.POINTER(KernelTime), C.c_int]
        _lib = L
    return _lib


def version() -> str:
    return lib().ckv_version().decode()


def layout_of(t: torch.Tensor, deg: Optional[torch.Tensor] = None) -> Layout:
    """Layout of a [batch, heads, seq, dim] tensor (any strides, dim contiguous) and of the int32
    degree array [batch, heads, seq] that goes with it (rows evenly spaced, e.g. a slice of a
    [batch, heads, capacity] buffer)."""
    if t.dim() != 4 or t.stride(3) != 1 or t.dtype not in _DT:
        raise ValueError("expected a [batch, heads, seq, dim] float32/bfloat16 tensor with contiguous dim")
    deg_stride = 0
    if deg is not None:
        B, H, S = t.shape[:3]
        if deg.dtype != torch.int32 or tuple(deg.shape) != (B, H, S) or (S > 1 and deg.stride(2) != 1):
            raise ValueError("deg must be int32 [batch, heads, seq] with contiguous seq")
        deg_stride = deg.stride(1) if H > 1 else (deg.stride(0) if B > 1 else S)
        if B > 1 and H > 1 and deg.stride(0) != H * deg.stride(1):
            raise ValueError("deg rows must be evenly spaced over (batch, head)")
    return Layout(t.shape[0], t.shape[1], t.shape[2], t.shape[3], t.stride(0), t.stride(1), t.stride(2),
                  _DT[t.dtype], deg_stride)


SCOPES = {"chunk": 0, "head": 1}
# kernel routes with bit-identical results (ckv_params.flags): None = the library chooses
ROUTES = {None: 0, "full_rounds": 1, "defer_always": 2}


def make_params(chunk: int, retain_ratio: float = 1.0, rounds: Optional[Sequence[float]] = None,
                n_sink: int = 0, n_recent: int = 0, scope: str = "chunk", route: Optional[str] = None) -> Params:
    p = Params()
    p.chunk, p.retain_ratio, p.n_sink, p.n_recent = chunk, retain_ratio, n_sink, n_recent
    p.scope = SCOPES[scope]
    p.flags = ROUTES[route]
    if rounds is not None:
        if not 0 < len(rounds) <= MAX_ROUNDS:
            raise ValueError("rounds must have 1..8 entries")
        p.n_rounds = len(rounds)
        for j, r in enumerate(rounds):
            p.r[j] = r
    return p


@dataclass
class Plan:
    out_seq: int
    round_len: list
    round_r: list
    workspace_bytes: int


def plan(lay: Layout, params: Params) -> Plan:
    pt = PlanT()
    st = lib().ckv_plan(C.byref(lay), C.byref(params), C.byref(pt))
    if st != 0:
        raise CkvError(st, "ckv_plan")
    return Plan(pt.out_seq, list(pt.round_len[: pt.n_rounds + 1]), list(pt.round_r[: pt.n_rounds]),
                pt.workspace_bytes)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def match(K: torch.Tensor, chunk: int):
    """ckv_match: (dst positions int32 [B,H,n_src], scores fp32 [B,H,n_src])."""
    lay = layout_of(K)
    n_src = lib().ckv_n_sources(K.shape[2], chunk)
    if n_src < 0:
        raise CkvError(n_src, "ckv_n_sources")
    dst = torch.empty((K.shape[0], K.shape[1], n_src), dtype=torch.int32, device=K.device)
    score = torch.empty((K.shape[0], K.shape[1], n_src), dtype=torch.float32, device=K.device)
    st = lib().ckv_match(_ptr(K), C.byref(lay), chunk, _ptr(dst), _ptr(score), _stream())
    if st != 0:
        raise CkvError(st, "ckv_match")
    return dst, score


def compress(K: torch.Tensor, V: torch.Tensor, chunk: int, retain_ratio: float = 1.0,
             rounds: Optional[Sequence[float]] = None, deg: Optional[torch.Tensor] = None,
             want_assign: bool = True, out: Optional[tuple] = None,
             workspace: Optional[torch.Tensor] = None, n_sink: int = 0, n_recent: int = 0,
             scope: str = "chunk", route: Optional[str] = None):
    """ckv_compress: returns (K', V', deg', assign or None).  K, V: [B,H,S,D] on the GPU.
    The first n_sink and last n_recent tokens bypass the clustering in every round.
    scope: "chunk" = top-r inside every chunk, "head" = one ranking over all chunks of a sequence.
    route: None, "full_rounds" or "defer_always" (same result bits; see ckv_params.flags).

    `out` may pass preallocated (K_out, V_out, deg_out, assign) and `workspace` a uint8 tensor, so
    that a timed loop allocates nothing."""
    lay = layout_of(K, deg)
    if layout_of(V).dtype != lay.dtype or V.shape != K.shape:
        raise ValueError("K and V must have the same shape and dtype")
    params = make_params(chunk, retain_ratio, rounds, n_sink, n_recent, scope, route)
    pl = plan(lay, params)
    B, H, S, D = K.shape
    if out is None:
        K_out = torch.empty((B, H, pl.out_seq, D), dtype=K.dtype, device=K.device)
        V_out = torch.empty_like(K_out)
        deg_out = torch.empty((B, H, pl.out_seq), dtype=torch.int32, device=K.device)
        assign = torch.empty((B, H, S), dtype=torch.int32, device=K.device) if want_assign else None
    else:
        K_out, V_out, deg_out, assign = out
    if workspace is None:
        workspace = torch.empty(max(pl.workspace_bytes, 256), dtype=torch.uint8, device=K.device)
    olay = layout_of(K_out, deg_out)
    st = lib().ckv_compress(_ptr(K), _ptr(V), _ptr(deg), C.byref(lay), C.byref(params), _ptr(K_out),
                            _ptr(V_out), _ptr(deg_out), C.byref(olay), _ptr(assign), _ptr(workspace),
                            workspace.numel(), _stream())
    if st != 0:
        raise CkvError(st, "ckv_compress")
    return K_out, V_out, deg_out, assign


def decode_attn_workspace(lay: Layout, q_heads: int) -> int:
    n = C.c_size_t(0)
    st = lib().ckv_decode_attn_workspace(C.byref(lay), q_heads, C.byref(n))
    if st != 0:
        raise CkvError(st, "ckv_decode_attn_workspace")
    return n.value


def decode_attn(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, lens: Optional[torch.Tensor] = None,
                deg: Optional[torch.Tensor] = None, scale: float = 0.0, out_dtype=None,
                out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """ckv_decode_attn: q [B,Hq,D], K/V [B,Hkv,L,D], lens [B] int32, deg [B,Hkv,L] int32 -> o [B,Hq,D].
    A `workspace` passed in must have been zero-filled when it was allocated (torch.zeros)."""
    lay = layout_of(K, deg)
    if not q.is_contiguous() or q.dim() != 3 or q.dtype != K.dtype:
        raise ValueError("q must be a contiguous [batch, q_heads, dim] tensor of the cache dtype")
    q_heads = q.shape[1]
    if out is None:
        out = torch.empty(q.shape, dtype=out_dtype or q.dtype, device=q.device)
    if workspace is None:
        workspace = torch.zeros(decode_attn_workspace(lay, q_heads), dtype=torch.uint8, device=q.device)
    st = lib().ckv_decode_attn(_ptr(q), q_heads, _ptr(K), _ptr(V), C.byref(lay), _ptr(lens), _ptr(deg),
                               scale, _ptr(out), _DT[out.dtype], _ptr(workspace), workspace.numel(),
                               _stream())
    if st != 0:
        raise CkvError(st, "ckv_decode_attn")
    return out


def decode_attn_noalloc(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, out: torch.Tensor,
                        lens: Optional[torch.Tensor] = None, deg: Optional[torch.Tensor] = None,
                        scale: float = 0.0) -> torch.Tensor:
    """ckv_decode_attn_noalloc: ckv_decode_attn with the library's own scratch array; the caller
    passes inputs and the output tensor, nothing is allocated."""
    lay = layout_of(K, deg)
    if not q.is_contiguous() or q.dim() != 3 or q.dtype != K.dtype:
        raise ValueError("q must be a contiguous [batch, q_heads, dim] tensor of the cache dtype")
    st = lib().ckv_decode_attn_noalloc(_ptr(q), q.shape[1], _ptr(K), _ptr(V), C.byref(lay), _ptr(lens), _ptr(deg),
                                       scale, _ptr(out), _DT[out.dtype], _stream())
    if st != 0:
        raise CkvError(st, "ckv_decode_attn_noalloc")
    return out


def budget_tokens(cache_ratio: float, n: int) -> int:
    """ckv_budget_tokens: Algorithm 1's cache budget B = floor(R * n)."""
    b = lib().ckv_budget_tokens(cache_ratio, n)
    if b < 0:
        raise CkvError(b, "ckv_budget_tokens")
    return b


def schedule_annealed(seq: int, chunk: int, budget: int, r_init: float = 0.8, delta_r: float = 0.2,
                      r_floor: float = 0.0, n_sink: int = 0, n_recent: int = 0, scope: str = "chunk") -> list:
    """ckv_schedule_annealed: the merge fractions Algorithm 1's loop after prefill uses to bring
    `seq` tokens within `budget` under the annealed schedule."""
    p = Params()
    st = lib().ckv_schedule_annealed(seq, chunk, n_sink, n_recent, SCOPES[scope], budget, r_init, delta_r, r_floor,
                                     C.byref(p))
    if st != 0:
        raise CkvError(st, "ckv_schedule_annealed")
    return list(p.r[: p.n_rounds])


def append(k_new: torch.Tensor, v_new: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
           deg: Optional[torch.Tensor], lens: Optional[torch.Tensor] = None, pos: int = -1) -> None:
    """ckv_append: write one new token per (batch, head) into the cache buffers K, V
    [batch, heads, capacity, dim] (deg [batch, heads, capacity] := 1 there) at row lens[b]
    (device int32, incremented by the call) or at row `pos`."""
    lay = layout_of(K, deg)
    B, H, _, D = K.shape
    for t in (k_new, v_new):
        if tuple(t.shape) != (B, H, D) or not t.is_contiguous() or t.dtype != K.dtype:
            raise ValueError("k_new, v_new must be contiguous [batch, heads, dim] tensors of the cache dtype")
    if layout_of(V).stride_s != lay.stride_s or V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("K and V buffers must share shape and strides")
    st = lib().ckv_append(_ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V), _ptr(deg), C.byref(lay), _ptr(lens),
                          pos, _stream())
    if st != 0:
        raise CkvError(st, "ckv_append")


# ---- block-paged caches ------------------------------------------------------------------------
def paged_layout_of(K_pool: torch.Tensor, block_table: torch.Tensor) -> PagedLayout:
    """K_pool: [n_blocks, heads, block_size, dim] contiguous; block_table: int32 [batch, max_blocks]."""
    if K_pool.dim() != 4 or not K_pool.is_contiguous() or K_pool.dtype not in _DT:
        raise ValueError("pool must be a contiguous [n_blocks, heads, block_size, dim] float32/bfloat16 tensor")
    if block_table.dim() != 2 or block_table.dtype != torch.int32 or not block_table.is_contiguous():
        raise ValueError("block_table must be a contiguous int32 [batch, max_blocks] tensor")
    nb, H, bs, D = K_pool.shape
    return PagedLayout(block_table.shape[0], H, D, _DT[K_pool.dtype], bs, block_table.shape[1], nb)


def paged_decode_attn(q, K_pool, V_pool, deg_pool, block_table, lens, max_len: int, scale: float = 0.0,
                      out_dtype=None, out=None, workspace=None):
    """ckv_paged_decode_attn: Eq. 3 over a block-paged cache read in place."""
    pl = paged_layout_of(K_pool, block_table)
    q_heads = q.shape[1]
    if not q.is_contiguous() or q.dim() != 3 or q.dtype != K_pool.dtype:
        raise ValueError("q must be a contiguous [batch, q_heads, dim] tensor of the cache dtype")
    if out is None:
        out = torch.empty(q.shape, dtype=out_dtype or q.dtype, device=q.device)
    if workspace is None:
        n = C.c_size_t(0)
        st = lib().ckv_paged_decode_attn_workspace(C.byref(pl), q_heads, max_len, C.byref(n))
        if st != 0:
            raise CkvError(st, "ckv_paged_decode_attn_workspace")
        workspace = torch.zeros(n.value, dtype=torch.uint8, device=q.device)
    st = lib().ckv_paged_decode_attn(_ptr(q), q_heads, _ptr(K_pool), _ptr(V_pool), _ptr(deg_pool), _ptr(block_table),
                                     _ptr(lens), C.byref(pl), max_len, scale, _ptr(out), _DT[out.dtype],
                                     _ptr(workspace), workspace.numel(), _stream())
    if st != 0:
        raise CkvError(st, "ckv_paged_decode_attn")
    return out


def paged_append(k_new, v_new, K_pool, V_pool, deg_pool, block_table, lens) -> None:
    """ckv_paged_append: one new token per sequence at position lens[b] (then lens[b] += 1)."""
    pl = paged_layout_of(K_pool, block_table)
    for t in (k_new, v_new):
        if tuple(t.shape) != (pl.batch, pl.heads, pl.dim) or not t.is_contiguous() or t.dtype != K_pool.dtype:
            raise ValueError("k_new, v_new must be contiguous [batch, heads, dim] tensors of the cache dtype")
    st = lib().ckv_paged_append(_ptr(k_new), _ptr(v_new), _ptr(K_pool), _ptr(V_pool), _ptr(deg_pool),
                                _ptr(block_table), _ptr(lens), C.byref(pl), _stream())
    if st != 0:
        raise CkvError(st, "ckv_paged_append")


def paged_gather(K_pool, V_pool, deg_pool, block_table, seq: int):
    """ckv_paged_gather: the first `seq` tokens of every sequence as [batch, heads, seq, dim] tensors."""
    pl = paged_layout_of(K_pool, block_table)
    K = torch.empty((pl.batch, pl.heads, seq, pl.dim), dtype=K_pool.dtype, device=K_pool.device)
    V = torch.empty_like(K)
    deg = torch.empty((pl.batch, pl.heads, seq), dtype=torch.int32, device=K_pool.device)
    lay = layout_of(K, deg)
    st = lib().ckv_paged_gather(_ptr(K_pool), _ptr(V_pool), _ptr(deg_pool), _ptr(block_table), C.byref(pl), seq,
                                _ptr(K), _ptr(V), _ptr(deg), C.byref(lay), _stream())
    if st != 0:
        raise CkvError(st, "ckv_paged_gather")
    return K, V, deg


def paged_scatter(K, V, deg, K_pool, V_pool, deg_pool, block_table, old_seq: int, lens=None):
    """ckv_paged_scatter: write [batch, heads, seq, dim] tensors into the sequences' blocks and
    release the blocks behind them; returns the freed block ids [batch, n_freed]."""
    pl = paged_layout_of(K_pool, block_table)
    lay = layout_of(K, deg)
    n_freed = lib().ckv_paged_freed_blocks(C.byref(pl), old_seq, K.shape[2])
    if n_freed < 0:
        raise CkvError(n_freed, "ckv_paged_freed_blocks")
    freed = torch.empty((pl.batch, n_freed), dtype=torch.int32, device=K.device)
    st = lib().ckv_paged_scatter(_ptr(K), _ptr(V), _ptr(deg), C.byref(lay), _ptr(K_pool), _ptr(V_pool),
                                 _ptr(deg_pool), _ptr(block_table), C.byref(pl), old_seq, _ptr(freed), _ptr(lens),
                                 _stream())
    if st != 0:
        raise CkvError(st, "ckv_paged_scatter")
    return freed


def _host_lens(seq_lens, batch):
    if seq_lens is None:
        return None
    vals = [int(x) for x in seq_lens]
    if len(vals) != batch:
        raise ValueError("seq_lens must have one entry per sequence")
    return (C.c_int32 * batch)(*vals)


def paged_compress_plan(pl: PagedLayout, seq: int, params: Params, seq_lens=None):
    """(length after compression - a list when seq_lens is given -, most blocks a sequence releases,
    workspace bytes).  seq_lens: host sequence of per-sequence lengths, or None (all `seq`)."""
    hl = _host_lens(seq_lens, pl.batch)
    out = (C.c_int32 * (pl.batch if hl is not None else 1))()
    n_freed, nbytes = C.c_int32(0), C.c_size_t(0)
    st = lib().ckv_paged_compress_plan(C.byref(pl), seq, hl, C.byref(params), out, C.byref(n_freed), C.byref(nbytes))
    if st != 0:
        raise CkvError(st, "ckv_paged_compress_plan")
    return (list(out) if hl is not None else out[0]), n_freed.value, nbytes.value


def paged_compress(K_pool, V_pool, deg_pool, block_table, seq: int, chunk: int, retain_ratio: float = 1.0,
                   rounds=None, lens=None, n_sink: int = 0, n_recent: int = 0, scope: str = "chunk",
                   workspace=None, seq_lens=None, route: Optional[str] = None):
    """ckv_paged_compress: compress the sequences in place in the paged cache; returns
    (new length - a list when seq_lens is given -, freed block ids [batch, n_freed], -1 padded)."""
    pl = paged_layout_of(K_pool, block_table)
    params = make_params(chunk, retain_ratio, rounds, n_sink, n_recent, scope, route)
    out_seq, n_freed, nbytes = paged_compress_plan(pl, seq, params, seq_lens)
    freed = torch.empty((pl.batch, n_freed), dtype=torch.int32, device=K_pool.device)
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=K_pool.device)
    st = lib().ckv_paged_compress(_ptr(K_pool), _ptr(V_pool), _ptr(deg_pool), _ptr(block_table), _ptr(lens),
                                  C.byref(pl), seq, _host_lens(seq_lens, pl.batch), C.byref(params), _ptr(freed), n_freed,
                                  _ptr(workspace), workspace.numel(), _stream())
    if st != 0:
        raise CkvError(st, "ckv_paged_compress")
    return out_seq, freed


def mfma_ceiling(mode: int, waves_per_cu: int, iters: int = 20000) -> float:
    """ckv_bench_mfma_ceiling timed through the library's hooks: sustained bf16 MFMA rate in FLOP/s."""
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    flops = C.c_double(0.0)
    for it, n in enumerate((max(iters // 10, 1), iters)):      # a short warm-up launch, then the timed one
        if it == 1:
            timing_select("mfma_ceiling")
            timing_reset()
            timing_enable(True)
        st = lib().ckv_bench_mfma_ceiling(mode, waves_per_cu, n, _ptr(scratch), scratch.numel(), C.byref(flops), _stream())
        if st != 0:
            timing_enable(False)
            timing_select(None)
            raise CkvError(st, "ckv_bench_mfma_ceiling")
        torch.cuda.synchronize()
    timing_enable(False)
    t = timing_read()
    timing_select(None)
    return flops.value / (t["mfma_ceiling"][0] * 1e-3)


def timing_enable(on: bool) -> None:
    lib().ckv_timing_enable(1 if on else 0)


def timing_reset() -> None:
    lib().ckv_timing_reset()


def timing_select(prefix: Optional[str]) -> None:
    """Time only kernels whose timing name starts with `prefix` (None: all)."""
    lib().ckv_timing_select(prefix.encode() if prefix else None)


def timing_read() -> dict:
    buf = (KernelTime * 32)()
    n = lib().ckv_timing_read(buf, 32)
    if n < 0:
        raise CkvError(n, "ckv_timing_read")
    return {buf[i].name.decode(): (buf[i].total_ms, buf[i].launches) for i in range(min(n, 32))}
