"""Thin ctypes binding of the C ABI in include/thrift.h: argument marshalling only.

Every step of the path runs in the HIP kernels of libthrift_hip.so; PyTorch is used for device
memory and for the current stream.  There is no CPU fallback: if the library has not been built
(``python -m paper_2605_23081_amd.build``) importing a function from here raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libthrift_hip.so")

F16, BF16, F32 = 0, 1, 2
_DT = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}

EXPORTS = (
    "thrift_status_string", "thrift_row_budget", "thrift_visible_blocks", "thrift_budget_to_global_k",
    "thrift_select_kmax", "thrift_block_means", "thrift_select_topk", "thrift_select_topk_shared", "thrift_select_ablation", "thrift_quantize_mxfp4",
    "thrift_attn_prefill_workspace", "thrift_attn_prefill", "thrift_attn_prefill_chunk", "thrift_attn_prefill_ordered",
    "thrift_attn_decode_workspace", "thrift_attn_decode", "thrift_attn_decode_shared", "thrift_attn_decode_static",
    "thrift_kv_cache_append",
    "thrift_attention_forward_workspace", "thrift_attention_forward", "thrift_peak_probe",
)

_lib = None


class ThriftError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: status {code} ({status_string(code)})")


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_23081_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        i, d, f, p, sz = C.c_int, C.c_double, C.c_float, C.c_void_p, C.c_size_t
        L.thrift_status_string.restype = C.c_char_p
        L.thrift_status_string.argtypes = [i]
        L.thrift_row_budget.argtypes = [i, d, i]
        L.thrift_visible_blocks.argtypes = [i] * 6
        L.thrift_budget_to_global_k.argtypes = [i, d]
        L.thrift_select_kmax.argtypes = [i, i, i, i, i, d, i, i]
        L.thrift_block_means.argtypes = [p, i, i, i, i, i, i, p, p]
        L.thrift_select_topk.argtypes = [p, p, i, i, i, i, i, i, i, i, i, d, i, i, p, p, i, p]
        L.thrift_select_topk_shared.argtypes = L.thrift_select_topk.argtypes
        L.thrift_select_ablation.argtypes = [i, C.c_uint64, i, i, i, i, i, i, i, d, i, i, p, p, i, p]
        L.thrift_quantize_mxfp4.argtypes = [p, i, i, i, i, i, i, p, p, p]
        L.thrift_attn_prefill_workspace.restype = sz
        L.thrift_attn_prefill_workspace.argtypes = [i] * 8
        L.thrift_attn_prefill.argtypes = [p, p, p, i, p, p, p, p, p, p, p, p, i, i, i, i, i, i, i, i, i, f, p, i, p, p, sz, p]
        L.thrift_attn_prefill_chunk.argtypes = [p, p, p, i, p, p, p, p, p, p, p, p, i, i, i, i, i, i, i, i, i, i, i, f, p, i, p, p, sz, p]
        L.thrift_attn_prefill_ordered.argtypes = [p, p, p, i, p, p, p, p, p, p, p, p, i, i, i, i, i, i, i, i, i, i, i, i, f, p, i, p, p, sz, p]
        L.thrift_attn_decode_workspace.restype = sz
        L.thrift_attn_decode_workspace.argtypes = [i] * 7
        L.thrift_attn_decode.argtypes = [p, i, p, p, p, p, p, p, p, p, i, i, i, i, i, i, d, i, i, f, p, i, p, p, i, p, sz, p]
        L.thrift_attn_decode_shared.argtypes = L.thrift_attn_decode.argtypes
        L.thrift_attn_decode_static.argtypes = [p, i, p, p, p, p, p, p, p, p, i, i, i, i, i, i, d, i, i, f, p, i, p, p, i, p]
        L.thrift_kv_cache_append.argtypes = [p, p, i, i, p, p, p, p, p, p, p, p, p, i, i, i, i, i, p]
        L.thrift_attention_forward_workspace.restype = sz
        L.thrift_attention_forward_workspace.argtypes = [i, i, i, i, i, i, i, i, d, i]
        L.thrift_attention_forward.argtypes = [p, p, p, i, i, i, i, i, i, i, i, i, d, i, i, f, p, i, p, p, sz, p]
        L.thrift_peak_probe.argtypes = [i, i, i, p, sz, C.POINTER(C.c_double), p]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().thrift_status_string(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != 0:
        raise ThriftError(code, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype=None) -> torch.Tensor:
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return t


def _prefill_shapes(q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt, Bq: int) -> None:
    """The C side sees pointers only: check here that every tensor has the dtype and the exact shape the kernel indexes."""
    B, Hq, Nq, D = q.shape
    _, Hkv, Nkv, _ = k.shape
    assert q.dtype == k.dtype == v.dtype and q.dtype in (torch.float16, torch.bfloat16), (q.dtype, k.dtype, v.dtype)
    assert k.shape == v.shape == (B, Hkv, Nkv, D), (k.shape, v.shape)
    Tq, Tv = -(-Nq // Bq), -(-Nkv // 64)
    u8, i32 = torch.uint8, torch.int32
    for name, t, shape, dt in (("q4", q4, (B, Hq, Nq, D // 2), u8), ("qs", qs, (B, Hq, Nq, D // 32), u8),
                               ("k4", k4, (B, Hkv, Nkv, D // 2), u8), ("ks", ks, (B, Hkv, Nkv, D // 32), u8),
                               ("v4", v4, (B, Hkv, Tv, D, 32), u8), ("vs", vs, (B, Hkv, 2 * Tv, D), u8),
                               ("cnt", cnt, (B, Hq, Tq), i32)):
        assert tuple(t.shape) == shape and t.dtype == dt, (name, tuple(t.shape), shape, t.dtype)
    assert idx.dtype == i32 and idx.dim() == 4 and tuple(idx.shape[:3]) == (B, Hq, Tq) and idx.shape[3] >= 1, tuple(idx.shape)


def _cache_shapes(k16, v16, k4, ks, v4, vs, kmean, Bk: int) -> None:
    B, Hkv, Nkv, D = k16.shape
    assert k16.dtype == v16.dtype and k16.dtype in (torch.float16, torch.bfloat16) and v16.shape == k16.shape
    u8 = torch.uint8
    for name, t, shape, dt in (("k4", k4, (B, Hkv, Nkv, D // 2), u8), ("ks", ks, (B, Hkv, Nkv, D // 32), u8),
                               ("v4", v4, (B, Hkv, Nkv // 64, D, 32), u8), ("vs", vs, (B, Hkv, Nkv // 32, D), u8),
                               ("kmean", kmean, (B, Hkv, Nkv // Bk, D), torch.float32)):
        assert tuple(t.shape) == shape and t.dtype == dt, (name, tuple(t.shape), shape, t.dtype)


# ---- host helpers ----

def row_budget(visible: int, budget: float, fixed_k: int = -1) -> int:
    return int(lib().thrift_row_budget(int(visible), float(budget), int(fixed_k)))


def visible_blocks(i: int, Tk: int, Bq: int, Bk: int, causal: bool, q_block_offset: int = 0) -> int:
    return int(lib().thrift_visible_blocks(i, Tk, Bq, Bk, int(causal), q_block_offset))


def budget_to_global_k(n_blocks: int, fraction: float) -> int:
    return int(lib().thrift_budget_to_global_k(int(n_blocks), float(fraction)))


def select_kmax(Tq: int, Tk: int, Bq: int, Bk: int, causal: bool, budget: float, fixed_k: int = -1,
                q_block_offset: int = 0) -> int:
    return int(lib().thrift_select_kmax(Tq, Tk, Bq, Bk, int(causal), float(budget), int(fixed_k), q_block_offset))


# ---- the five compute calls ----

def thrift_block_means(x: torch.Tensor, block: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(x)
    B, H, N, D = x.shape
    if out is None:
        out = torch.empty(B, H, -(-N // max(block, 1)), D, dtype=torch.float32, device=x.device)
    _check(lib().thrift_block_means(_ptr(x), _DT[x.dtype], B, H, N, D, block, _ptr(out), _stream()), "thrift_block_means")
    return out


def thrift_select_topk(qmean: torch.Tensor, kmean: torch.Tensor, Bq: int, Bk: int, causal: bool, budget: float,
                       fixed_k: int = -1, q_block_offset: int = 0, kmax: Optional[int] = None,
                       idx: Optional[torch.Tensor] = None, cnt: Optional[torch.Tensor] = None,
                       group_shared: bool = False) -> Tuple[torch.Tensor, torch.Tensor]:
    _dev(qmean, torch.float32), _dev(kmean, torch.float32)
    B, Hq, Tq, D = qmean.shape
    _, Hkv, Tk, _ = kmean.shape
    if kmax is None:
        kmax = max(1, select_kmax(Tq, Tk, Bq, Bk, causal, budget, fixed_k, q_block_offset))
    if idx is None:
        idx = torch.empty(B, Hq, Tq, kmax, dtype=torch.int32, device=qmean.device)
        cnt = torch.empty(B, Hq, Tq, dtype=torch.int32, device=qmean.device)
    fn = lib().thrift_select_topk_shared if group_shared else lib().thrift_select_topk
    _check(fn(_ptr(qmean), _ptr(kmean), B, Hq, Hkv, Tq, Tk, D, Bq, Bk, int(causal), float(budget),
              int(fixed_k), int(q_block_offset), _ptr(idx), _ptr(cnt), int(kmax), _stream()),
           "thrift_select_topk_shared" if group_shared else "thrift_select_topk")
    return idx, cnt


SELECT_RANDOM, SELECT_DIAGONAL = 1, 2


def thrift_select_ablation(selector: int, seed: int, B: int, Hq: int, Tq: int, Tk: int, Bq: int, Bk: int, causal: bool,
                           budget: float, fixed_k: int = -1, q_block_offset: int = 0, kmax: Optional[int] = None,
                           device=None, idx: Optional[torch.Tensor] = None, cnt: Optional[torch.Tensor] = None
                           ) -> Tuple[torch.Tensor, torch.Tensor]:
    device = torch.device("cuda", torch.cuda.current_device()) if device is None else device
    if kmax is None:
        kmax = max(1, select_kmax(Tq, Tk, Bq, Bk, causal, budget, fixed_k, q_block_offset))
    if idx is None:
        idx = torch.empty(B, Hq, Tq, kmax, dtype=torch.int32, device=device)
        cnt = torch.empty(B, Hq, Tq, dtype=torch.int32, device=device)
    _check(lib().thrift_select_ablation(int(selector), int(seed) & (2 ** 64 - 1), B, Hq, Tq, Tk, Bq, Bk, int(causal), float(budget),
                                        int(fixed_k), int(q_block_offset), _ptr(idx), _ptr(cnt), int(kmax), _stream()),
           "thrift_select_ablation")
    return idx, cnt


def thrift_quantize_mxfp4(x: torch.Tensor, axis: int, codes: Optional[torch.Tensor] = None,
                          scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    _dev(x)
    B, H, N, D = x.shape
    if codes is None:
        if axis == 0:
            codes = torch.empty(B, H, N, D // 2, dtype=torch.uint8, device=x.device)
            scales = torch.empty(B, H, N, D // 32, dtype=torch.uint8, device=x.device)
        else:
            codes = torch.empty(B, H, -(-N // 64), D, 32, dtype=torch.uint8, device=x.device)
            scales = torch.empty(B, H, 2 * -(-N // 64), D, dtype=torch.uint8, device=x.device)
    _check(lib().thrift_quantize_mxfp4(_ptr(x), _DT[x.dtype], B, H, N, D, int(axis), _ptr(codes), _ptr(scales), _stream()),
           "thrift_quantize_mxfp4")
    return codes, scales


def thrift_attn_prefill(q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt, Bq: int, Bk: int, causal: bool,
                        softmax_scale: float = 0.0, out: Optional[torch.Tensor] = None,
                        out_dtype: Optional[torch.dtype] = None, lse: Optional[torch.Tensor] = None) -> torch.Tensor:
    for t in (q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt):
        _dev(t)
    _prefill_shapes(q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt, Bq)
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    if out is None:
        out = torch.empty(B, Hq, N, D, dtype=out_dtype or q.dtype, device=q.device)
    assert tuple(out.shape) == (B, Hq, N, D) and (lse is None or (tuple(lse.shape) == (B, Hq, N) and lse.dtype == torch.float32))
    kmax = idx.shape[-1]
    ws_bytes = lib().thrift_attn_prefill_workspace(B, Hq, Hkv, N, D, Bq, Bk, kmax)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=q.device) if ws_bytes else None
    _check(lib().thrift_attn_prefill(_ptr(q), _ptr(k), _ptr(v), _DT[q.dtype], _ptr(q4), _ptr(qs), _ptr(k4), _ptr(ks),
                                     _ptr(v4), _ptr(vs), _ptr(idx), _ptr(cnt), kmax, B, Hq, Hkv, N, D, Bq, Bk,
                                     int(causal), float(softmax_scale), _ptr(out), _DT[out.dtype], _ptr(lse), _ptr(ws),
                                     ws_bytes, _stream()), "thrift_attn_prefill")
    return out


def thrift_attn_prefill_chunk(q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt, Bq: int, Bk: int, causal: bool, q_block_offset: int,
                              softmax_scale: float = 0.0, out: Optional[torch.Tensor] = None,
                              out_dtype: Optional[torch.dtype] = None, lse: Optional[torch.Tensor] = None,
                              tile_order: int = 0) -> torch.Tensor:
    """q, q4, qs: the chunk's Nq tokens; k, v and their codes: the whole key range.  tile_order 1: Sec. 3.3's order;
    2 / 3: ascending order with the staging schedule fixed (see include/thrift.h)."""
    for t in (q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt):
        _dev(t)
    _prefill_shapes(q, k, v, q4, qs, k4, ks, v4, vs, idx, cnt, Bq)
    B, Hq, Nq, D = q.shape
    Hkv, Nkv = k.shape[1], k.shape[2]
    if out is None:
        out = torch.empty(B, Hq, Nq, D, dtype=out_dtype or q.dtype, device=q.device)
    assert tuple(out.shape) == (B, Hq, Nq, D) and (lse is None or (tuple(lse.shape) == (B, Hq, Nq) and lse.dtype == torch.float32))
    kmax = idx.shape[-1]
    _check(lib().thrift_attn_prefill_ordered(_ptr(q), _ptr(k), _ptr(v), _DT[q.dtype], _ptr(q4), _ptr(qs), _ptr(k4), _ptr(ks),
                                             _ptr(v4), _ptr(vs), _ptr(idx), _ptr(cnt), kmax, B, Hq, Hkv, Nq, int(q_block_offset),
                                             Nkv, D, Bq, Bk, int(causal), int(tile_order), float(softmax_scale), _ptr(out),
                                             _DT[out.dtype], _ptr(lse), None, 0, _stream()), "thrift_attn_prefill_ordered")
    return out


def decode_workspace_bytes(B: int, Hq: int, Hkv: int, Nkv: int, D: int, Bk: int, split_blocks: int) -> int:
    return int(lib().thrift_attn_decode_workspace(B, Hq, Hkv, Nkv, D, Bk, split_blocks))


def thrift_attn_decode(q, k16, v16, k4, ks, v4, vs, kmean, Bk: int, budget: float, fixed_k: int = -1,
                       split_blocks: int = 256, softmax_scale: float = 0.0, seqlens: Optional[torch.Tensor] = None,
                       out: Optional[torch.Tensor] = None, out_dtype: Optional[torch.dtype] = None,
                       workspace: Optional[torch.Tensor] = None, return_selection: bool = False,
                       group_shared: bool = False):
    for t in (q, k16, v16, k4, ks, v4, vs, kmean):
        _dev(t)
    _cache_shapes(k16, v16, k4, ks, v4, vs, kmean, Bk)
    B, Hq, D = q.shape
    _, Hkv, Nkv, _ = k16.shape
    assert q.dtype == k16.dtype and k16.shape[0] == B and k16.shape[3] == D
    if seqlens is not None:
        _dev(seqlens, torch.int32)
        assert tuple(seqlens.shape) == (B,)
    if out is None:
        out = torch.empty(B, Hq, D, dtype=out_dtype or q.dtype, device=q.device)
    assert tuple(out.shape) == (B, Hq, D)
    if workspace is None:
        workspace = torch.empty(max(decode_workspace_bytes(B, Hq, Hkv, Nkv, D, Bk, split_blocks), 16), dtype=torch.uint8,
                                device=q.device)
    idx = cnt = None
    kmax = 0
    if return_selection:
        kmax = max(1, row_budget(Nkv // Bk, budget, fixed_k))
        idx = torch.empty(B, Hq, kmax, dtype=torch.int32, device=q.device)
        cnt = torch.empty(B, Hq, dtype=torch.int32, device=q.device)
    fn = lib().thrift_attn_decode_shared if group_shared else lib().thrift_attn_decode
    _check(fn(_ptr(q), _DT[q.dtype], _ptr(k16), _ptr(v16), _ptr(k4), _ptr(ks), _ptr(v4), _ptr(vs),
              _ptr(kmean), _ptr(seqlens), B, Hq, Hkv, Nkv, D, Bk, float(budget), int(fixed_k),
              int(split_blocks), float(softmax_scale), _ptr(out), _DT[out.dtype], _ptr(idx), _ptr(cnt),
              kmax, _ptr(workspace), workspace.numel(), _stream()),
           "thrift_attn_decode_shared" if group_shared else "thrift_attn_decode")
    return (out, idx, cnt) if return_selection else out


DECODE_STATIC_SCRATCH_BYTES = 32 << 20


def thrift_attn_decode_static(q, k16, v16, k4, ks, v4, vs, kmean, Bk: int, budget: float, out: torch.Tensor,
                              fixed_k: int = -1, split_blocks: int = 256, softmax_scale: float = 0.0,
                              seqlens: Optional[torch.Tensor] = None, idx: Optional[torch.Tensor] = None,
                              cnt: Optional[torch.Tensor] = None) -> torch.Tensor:
    """thrift_attn_decode on the library's static scratch: the caller passes every buffer (out, and idx / cnt if it
    wants the selection back); neither this wrapper nor the C call allocates."""
    for t in (q, k16, v16, k4, ks, v4, vs, kmean, out):
        _dev(t)
    _cache_shapes(k16, v16, k4, ks, v4, vs, kmean, Bk)
    B, Hq, D = q.shape
    _, Hkv, Nkv, _ = k16.shape
    assert q.dtype == k16.dtype and k16.shape[0] == B and k16.shape[3] == D and tuple(out.shape) == (B, Hq, D)
    if seqlens is not None:
        _dev(seqlens, torch.int32)
        assert tuple(seqlens.shape) == (B,)
    if idx is not None:
        assert idx.dtype == torch.int32 and tuple(idx.shape[:2]) == (B, Hq) and cnt is not None and tuple(cnt.shape) == (B, Hq)
    kmax = 0 if idx is None else idx.shape[-1]
    _check(lib().thrift_attn_decode_static(_ptr(q), _DT[q.dtype], _ptr(k16), _ptr(v16), _ptr(k4), _ptr(ks), _ptr(v4), _ptr(vs),
                                           _ptr(kmean), _ptr(seqlens), B, Hq, Hkv, Nkv, D, Bk, float(budget), int(fixed_k),
                                           int(split_blocks), float(softmax_scale), _ptr(out), _DT[out.dtype], _ptr(idx), _ptr(cnt),
                                           kmax, _stream()), "thrift_attn_decode_static")
    return out


class KVCache:
    """Device buffers of the dual cache (Sec. 4.1, Sec. 5): 16-bit K/V, MXFP4 K/V and the key-block means."""

    def __init__(self, B, Hkv, Nkv, D, Bk, dtype, device, fill: Optional[int] = None):
        assert Nkv % Bk == 0
        u8 = torch.uint8

        def mk(*shape, dtype):
            # fill: a byte pattern for every buffer (tests poison the cache to show that nothing unwritten is read)
            if fill is None:
                return torch.empty(shape, dtype=dtype, device=device)
            nbytes = math.prod(shape) * torch.empty((), dtype=dtype).element_size()
            return torch.full((nbytes,), fill, dtype=u8, device=device).view(dtype).view(shape)

        self.B, self.Hkv, self.Nkv, self.D, self.Bk = B, Hkv, Nkv, D, Bk
        self.k16 = mk(B, Hkv, Nkv, D, dtype=dtype)
        self.v16 = mk(B, Hkv, Nkv, D, dtype=dtype)
        self.k4 = mk(B, Hkv, Nkv, D // 2, dtype=u8)
        self.ks = mk(B, Hkv, Nkv, D // 32, dtype=u8)
        self.v4 = mk(B, Hkv, Nkv // 64, D, 32, dtype=u8)
        self.vs = mk(B, Hkv, Nkv // 32, D, dtype=u8)
        self.kmean = mk(B, Hkv, Nkv // Bk, D, dtype=torch.float32)
        self.seqlens = torch.zeros(B, dtype=torch.int32, device=device)

    def append(self, k_new, v_new, new_lens: Optional[torch.Tensor] = None):
        """Append k_new, v_new [B,Hkv,n,D] (all n tokens, or new_lens[b] of them) and advance seqlens."""
        thrift_kv_cache_append(k_new, v_new, self.seqlens, self.k16, self.v16, self.k4, self.ks, self.v4, self.vs,
                               self.kmean, self.Bk, new_lens)
        n = k_new.shape[2]
        step = torch.full_like(self.seqlens, n) if new_lens is None else new_lens.clamp(0, n).to(torch.int32)
        self.seqlens = torch.minimum(self.seqlens + step, torch.full_like(self.seqlens, self.Nkv))


def thrift_kv_cache_append(k_new, v_new, seqlens, k16, v16, k4, ks, v4, vs, kmean, Bk: int,
                           new_lens: Optional[torch.Tensor] = None) -> None:
    for t in (k_new, v_new, k16, v16, k4, ks, v4, vs, kmean):
        _dev(t)
    _dev(seqlens, torch.int32)
    if new_lens is not None:
        _dev(new_lens, torch.int32)
    assert k_new.shape == v_new.shape and k_new.dtype == v_new.dtype == k16.dtype == v16.dtype
    _cache_shapes(k16, v16, k4, ks, v4, vs, kmean, Bk)
    B, Hkv, n_new, D = k_new.shape
    _, _, Nkv, _ = k16.shape
    assert tuple(k16.shape[:2]) == (B, Hkv) and k16.shape[3] == D and tuple(seqlens.shape) == (B,)
    assert new_lens is None or tuple(new_lens.shape) == (B,)
    _check(lib().thrift_kv_cache_append(_ptr(k_new), _ptr(v_new), _DT[k_new.dtype], n_new, _ptr(seqlens), _ptr(new_lens),
                                        _ptr(k16), _ptr(v16), _ptr(k4), _ptr(ks), _ptr(v4), _ptr(vs), _ptr(kmean),
                                        B, Hkv, Nkv, D, Bk, _stream()), "thrift_kv_cache_append")


PEAK_MFMA_MXFP4, PEAK_MFMA_16, PEAK_HBM_READ, PEAK_VALU_SOFTMAX, PEAK_TILE_MIX = range(5)


def thrift_peak_probe(kind: int, buffer: torch.Tensor, iters: int = 2000, dtype: torch.dtype = torch.bfloat16) -> float:
    """Enqueue one measurement microbenchmark (see include/thrift.h) on the current stream; returns the work of the
    launch (flops, bytes or wave-tiles).  The caller times it."""
    _dev(buffer, torch.uint8)
    work = C.c_double(0.0)
    _check(lib().thrift_peak_probe(int(kind), _DT[dtype], int(iters), _ptr(buffer), buffer.numel(), C.byref(work), _stream()),
           "thrift_peak_probe")
    return float(work.value)


# ---- Alg. 1 end to end: the user-level form of the paper's signature ----

class PrefillPlan:
    """Buffers of one prefill problem, allocated once so that repeated steps do not allocate."""

    def __init__(self, B, Hq, Hkv, N, D, Bq, Bk, causal, budget, dtype, device, fixed_k=-1, out_dtype=None,
                 selector: int = 0, seed: int = 0, tile_order: int = 0):
        self.args = (B, Hq, Hkv, N, D, Bq, Bk, causal, budget, fixed_k)
        self.tile_order = tile_order                        # 0: Alg. 1's ascending order; 1: the order of the kernel in Sec. 3.3
        self.selector, self.seed = selector, seed           # 0: the paper's heuristic; else an App. A ablation selector
        dev = device
        u8, f32, i32 = torch.uint8, torch.float32, torch.int32
        Tq, Tk = -(-N // Bq), -(-N // Bk)                   # N need not be a multiple of the blocks
        self.Tq, self.Tk = Tq, Tk
        self.qmean = torch.empty(B, Hq, Tq, D, dtype=f32, device=dev)
        self.kmean = torch.empty(B, Hkv, Tk, D, dtype=f32, device=dev)
        self.kmax = max(1, select_kmax(Tq, Tk, Bq, Bk, causal, budget, fixed_k))
        self.idx = torch.empty(B, Hq, Tq, self.kmax, dtype=i32, device=dev)
        self.cnt = torch.empty(B, Hq, Tq, dtype=i32, device=dev)
        self.q4 = torch.empty(B, Hq, N, D // 2, dtype=u8, device=dev)
        self.qs = torch.empty(B, Hq, N, D // 32, dtype=u8, device=dev)
        self.k4 = torch.empty(B, Hkv, N, D // 2, dtype=u8, device=dev)
        self.ks = torch.empty(B, Hkv, N, D // 32, dtype=u8, device=dev)
        self.v4 = torch.empty(B, Hkv, -(-N // 64), D, 32, dtype=u8, device=dev)
        self.vs = torch.empty(B, Hkv, 2 * -(-N // 64), D, dtype=u8, device=dev)
        self.out = torch.empty(B, Hq, N, D, dtype=out_dtype or dtype, device=dev)

    def run(self, q, k, v, softmax_scale: float = 0.0, prepass: bool = True, attention: bool = True) -> torch.Tensor:
        B, Hq, Hkv, N, D, Bq, Bk, causal, budget, fixed_k = self.args
        if prepass:
            thrift_block_means(q, Bq, out=self.qmean)
            thrift_block_means(k, Bk, out=self.kmean)
            if self.selector == 0:
                thrift_select_topk(self.qmean, self.kmean, Bq, Bk, causal, budget, fixed_k, kmax=self.kmax, idx=self.idx, cnt=self.cnt)
            else:
                thrift_select_ablation(self.selector, self.seed, B, Hq, self.Tq, self.Tk, Bq, Bk, causal, budget, fixed_k,
                                       kmax=self.kmax, idx=self.idx, cnt=self.cnt)
            thrift_quantize_mxfp4(q, 0, self.q4, self.qs)
            thrift_quantize_mxfp4(k, 0, self.k4, self.ks)
            thrift_quantize_mxfp4(v, 1, self.v4, self.vs)
        if attention:
            thrift_attn_prefill_chunk(q, k, v, self.q4, self.qs, self.k4, self.ks, self.v4, self.vs, self.idx, self.cnt, Bq, Bk,
                                      causal, 0, softmax_scale, out=self.out, tile_order=self.tile_order)
        return self.out


def thrift_attention(q, k, v, causal: bool = True, Bq: int = 128, Bk: int = 64, budget: float = 0.05,
                     fixed_k: int = -1, softmax_scale: float = 0.0, out_dtype=None,
                     workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                     lse: Optional[torch.Tensor] = None, tile_order: int = 0) -> torch.Tensor:
    """Alg. 1: Q, K, V, block sizes and FP16 budget in, attention output out (thrift_attention_forward: one C call)."""
    for t in (q, k, v):
        _dev(t)
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    assert q.dtype == k.dtype == v.dtype and k.shape == v.shape == (B, Hkv, N, D), (q.dtype, k.dtype, v.dtype, k.shape, v.shape)
    need = int(lib().thrift_attention_forward_workspace(B, Hq, Hkv, N, D, Bq, Bk, int(causal), float(budget), int(fixed_k)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty(B, Hq, N, D, dtype=out_dtype or q.dtype, device=q.device)
    _check(lib().thrift_attention_forward(_ptr(q), _ptr(k), _ptr(v), _DT[q.dtype], B, Hq, Hkv, N, D, Bq, Bk, int(causal),
                                          float(budget), int(fixed_k), int(tile_order), float(softmax_scale), _ptr(out), _DT[out.dtype],
                                          _ptr(lse), _ptr(workspace), workspace.numel(), _stream()), "thrift_attention_forward")
    return out
