"""ctypes front end of the CPU oracle (oracle/thrift_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the HIP package, and the HIP
package never imports it.  Inputs are numpy arrays; 16-bit float tensors travel
as their raw uint16 bit patterns so that both sides see identical bits.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "thrift_oracle.c")
_LIB = os.path.join(_HERE, "libthrift_oracle.so")

F16, BF16 = 0, 1


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (strict IEEE arithmetic, OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        L.oracle_round_to_dtype.restype = C.c_double
        L.oracle_round_to_dtype.argtypes = [C.c_double, C.c_int]
        L.oracle_e2m1_decode.restype = C.c_double
        L.oracle_e2m1_decode.argtypes = [C.c_int]
        L.oracle_mx_quantize_group.restype = C.c_uint8
        L.oracle_error_bound_rhs.restype = C.c_double
        L.oracle_row_k.argtypes = [C.c_int, C.c_double, C.c_int]
        L.oracle_paper_global_k.argtypes = [C.c_int, C.c_double]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def bits_of(t) -> Tuple[np.ndarray, int]:
    """torch fp16/bf16 CPU tensor -> (uint16 numpy view, dtype code)."""
    import torch

    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float16:
        return t.view(torch.int16).numpy().view(np.uint16), F16
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16), BF16
    raise TypeError(t.dtype)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def round_to_dtype(x: float, dtype: int) -> float:
    return float(lib().oracle_round_to_dtype(float(x), dtype))


def block_means(x: np.ndarray, dtype: int, block: int) -> np.ndarray:
    x = _u16(x)
    B, H, N, D = x.shape
    out = np.empty((B, H, -(-N // block), D), np.float32)      # a short last block is the mean of its own tokens
    lib().oracle_block_means(_p(x), dtype, B, H, N, D, block, _p(out))
    return out


def row_k(visible: int, budget: float, fixed_k: int = -1) -> int:
    return int(lib().oracle_row_k(int(visible), float(budget), int(fixed_k)))


def paper_global_k(n: int, f: float) -> int:
    return int(lib().oracle_paper_global_k(int(n), float(f)))


def visible_blocks(i: int, Tk: int, Bq: int, Bk: int, causal: bool, q_block_offset: int = 0) -> int:
    return int(lib().oracle_visible_blocks(i, Tk, Bq, Bk, int(causal), q_block_offset))


def block_scores(qmean: np.ndarray, kmean: np.ndarray) -> np.ndarray:
    qmean = np.ascontiguousarray(qmean, np.float32)
    kmean = np.ascontiguousarray(kmean, np.float32)
    B, Hq, Tq, D = qmean.shape
    _, Hkv, Tk, _ = kmean.shape
    out = np.empty((B, Hq, Tq, Tk), np.float64)
    lib().oracle_block_scores(_p(qmean), _p(kmean), B, Hq, Hkv, Tq, Tk, D, _p(out))
    return out


def select_topk(qmean: np.ndarray, kmean: np.ndarray, Bq: int, Bk: int, causal: bool, budget: float,
                fixed_k: int = -1, q_block_offset: int = 0, kmax: Optional[int] = None, group_shared: bool = False):
    """group_shared: one set per (batch, KV head, query block) from the scores summed over the group's query heads."""
    qmean = np.ascontiguousarray(qmean, np.float32)
    kmean = np.ascontiguousarray(kmean, np.float32)
    B, Hq, Tq, D = qmean.shape
    _, Hkv, Tk, _ = kmean.shape
    if kmax is None:
        kmax = max(1, max(row_k(visible_blocks(i, Tk, Bq, Bk, causal, q_block_offset), budget, fixed_k) for i in range(Tq)))
    idx = np.empty((B, Hq, Tq, kmax), np.int32)
    cnt = np.empty((B, Hq, Tq), np.int32)
    fn = lib().oracle_select_topk_shared if group_shared else lib().oracle_select_topk
    rc = fn(_p(qmean), _p(kmean), B, Hq, Hkv, Tq, Tk, D, Bq, Bk, int(causal),
            C.c_double(budget), int(fixed_k), int(q_block_offset), _p(idx), _p(cnt), kmax)
    if rc != 0:
        raise ValueError("kmax too small")
    return idx, cnt


SELECT_RANDOM, SELECT_DIAGONAL = 1, 2


def splitmix64_output(seed: int, n_plus_1: int) -> int:
    f = lib().oracle_splitmix64_output
    f.restype = C.c_uint64
    return int(f(C.c_uint64(seed & (2 ** 64 - 1)), C.c_uint64(n_plus_1 & (2 ** 64 - 1))))


def select_ablation(selector: int, seed: int, B: int, Hq: int, Tq: int, Tk: int, Bq: int, Bk: int, causal: bool,
                    budget: float, fixed_k: int = -1, q_block_offset: int = 0, kmax: Optional[int] = None):
    """App. A selectors (random / diagonal) at the heuristic's per-row budget; output as select_topk."""
    if kmax is None:
        kmax = max(1, max(row_k(visible_blocks(i, Tk, Bq, Bk, causal, q_block_offset), budget, fixed_k) for i in range(Tq)))
    idx = np.empty((B, Hq, Tq, kmax), np.int32)
    cnt = np.empty((B, Hq, Tq), np.int32)
    rc = lib().oracle_select_ablation(int(selector), C.c_uint64(seed & (2 ** 64 - 1)), B, Hq, Tq, Tk, Bq, Bk, int(causal),
                                      C.c_double(budget), int(fixed_k), int(q_block_offset), _p(idx), _p(cnt), kmax)
    if rc == -2:
        raise ValueError("unknown selector")
    if rc != 0:
        raise ValueError("kmax too small")
    return idx, cnt


def e4m3_round(x: float) -> float:
    f = lib().oracle_e4m3_round
    f.restype = C.c_double
    return float(f(C.c_double(x)))


def nvfp4_qdq(x: np.ndarray) -> np.ndarray:
    """NVFP4 quantise-dequantise of consecutive groups of 16 (the paper's format; study aid)."""
    x = np.ascontiguousarray(x, np.float64)
    out = np.empty_like(x)
    lib().oracle_nvfp4_qdq(_p(x), C.c_long(x.size), _p(out))
    return out


def mx_nosat_qdq(x: np.ndarray) -> np.ndarray:
    """MXFP4 quantise-dequantise of consecutive groups of 32 with the scale rule that never saturates (study aid)."""
    x = np.ascontiguousarray(x, np.float64)
    out = np.empty_like(x)
    lib().oracle_mx_nosat_qdq(_p(x), C.c_long(x.size), _p(out))
    return out


def mx_quantize_group(x: Sequence[float]) -> Tuple[np.ndarray, int]:
    x = np.ascontiguousarray(x, np.float64)
    codes = np.empty(x.shape[0], np.uint8)
    s = lib().oracle_mx_quantize_group(_p(x), x.shape[0], _p(codes))
    return codes, int(s)


def quantize_mxfp4(x: np.ndarray, dtype: int, axis: int):
    """-> (codes [B,H,N,D] one code per byte, scales [B,H,N,D/32] or [B,H,ceil(N/32),D])."""
    x = _u16(x)
    B, H, N, D = x.shape
    codes = np.empty((B, H, N, D), np.uint8)
    scales = np.empty((B, H, N, D // 32) if axis == 0 else (B, H, -(-N // 32), D), np.uint8)
    lib().oracle_quantize_mxfp4(_p(x), dtype, B, H, N, D, axis, _p(codes), _p(scales))
    return codes, scales


def dequantize_mxfp4(codes: np.ndarray, scales: np.ndarray, axis: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.uint8)
    B, H, N, D = codes.shape
    out = np.empty((B, H, N, D), np.float64)
    lib().oracle_dequantize_mxfp4(_p(codes), _p(scales), B, H, N, D, axis, _p(out))
    return out


def attn_exact(q, k, v, dtype: int, causal: bool, scale: float, rows: np.ndarray, q_pos0: int = 0,
               want_lse: bool = False):
    """rows: [n,3] int32 (b, h, t).  -> out [n, D] (and lse [n])."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, Hq, Nq, D = q.shape
    _, Hkv, Nk, _ = k.shape
    rows = np.ascontiguousarray(rows, np.int32).reshape(-1, 3)
    out = np.empty((rows.shape[0], D), np.float64)
    lse = np.empty(rows.shape[0], np.float64) if want_lse else None
    lib().oracle_attn_exact(_p(q), _p(k), _p(v), dtype, B, Hq, Hkv, Nq, Nk, D, int(causal), int(q_pos0),
                            C.c_double(scale), _p(rows), rows.shape[0], _p(out), _p(lse))
    return (out, lse) if want_lse else out


def attn_thrift_prefill(q, k, v, dtype: int, idx, cnt, Bq: int, Bk: int, causal: bool, scale: float,
                        units: np.ndarray, tile_order: int = 0, quantize_p: bool = True, force_path: int = -1,
                        want_lse: bool = False, q_block_offset: int = 0, fmt: int = 0):
    """units: [n,3] int32 (b, h, i).  -> out [n, Bq, D] fp64 (and lse [n, Bq]).

    q may hold fewer tokens than k, v (chunked prefill): query block i then stands at block position
    i + q_block_offset of the sequence.  fmt 1: the paper's NVFP4 numerics instead of MXFP4; fmt 2: MXFP4 with the
    scale rule that never saturates (study aids; fmt 2 needs N % 32 == 0)."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, Hq, Nq, D = q.shape
    Hkv, N = k.shape[1], k.shape[2]
    units = np.ascontiguousarray(units, np.int32).reshape(-1, 3)
    kmax = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, np.int32)
        cnt = np.ascontiguousarray(cnt, np.int32)
        kmax = idx.shape[-1]
    out = np.empty((units.shape[0], Bq, D), np.float64)
    lse = np.empty((units.shape[0], Bq), np.float64) if want_lse else None
    rc = lib().oracle_attn_thrift_prefill_chunk(_p(q), _p(k), _p(v), dtype, _p(idx), _p(cnt), kmax, B, Hq, Hkv, Nq,
                                                int(q_block_offset), N, D, Bq, Bk,
                                                int(causal), C.c_double(scale), int(tile_order), int(quantize_p),
                                                int(force_path), int(fmt), _p(units), units.shape[0], _p(out), _p(lse))
    if rc != 0:
        raise ValueError("unsupported shape")
    return (out, lse) if want_lse else out


def attn_thrift_decode(q, k, v, dtype: int, idx, cnt, Bk: int, scale: float, split_blocks: int,
                       seqlens: Optional[np.ndarray] = None, quantize_p: bool = True, force_path: int = -1):
    """q [B,Hq,D]; k,v [B,Hkv,Nkv,D]; idx [B,Hq,kmax]; cnt [B,Hq] -> out [B,Hq,D] fp64."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, Hq, D = q.shape
    _, Hkv, Nkv, _ = k.shape
    kmax = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, np.int32)
        cnt = np.ascontiguousarray(cnt, np.int32)
        kmax = idx.shape[-1]
    if seqlens is not None:
        seqlens = np.ascontiguousarray(seqlens, np.int32)
    out = np.empty((B, Hq, D), np.float64)
    rc = lib().oracle_attn_thrift_decode(_p(q), _p(k), _p(v), dtype, _p(idx), _p(cnt), kmax, _p(seqlens), B, Hq, Hkv,
                                         Nkv, D, Bk, C.c_double(scale), int(split_blocks), int(quantize_p),
                                         int(force_path), _p(out))
    if rc != 0:
        raise ValueError("unsupported shape")
    return out


def error_bound_rhs(q_row, k_head, v_head, dtype: int, Bk: int, n_visible: int, scale: float):
    """Eq. (4) right-hand side for one query row; returns (total, per-key-block split)."""
    q_row, k_head, v_head = _u16(q_row), _u16(k_head), _u16(v_head)
    Nk, D = k_head.shape
    per = np.empty(Nk // Bk, np.float64)
    tot = lib().oracle_error_bound_rhs(_p(q_row), _p(k_head), _p(v_head), dtype, Nk, D, Bk, int(n_visible),
                                       C.c_double(scale), _p(per))
    return float(tot), per
