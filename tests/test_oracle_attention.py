"""Pins for the oracle's attention routines (CPU only).

The exact routine is pinned to a numpy brute force and to torch's fp64
scaled_dot_product_attention.  The mixed-precision routine is pinned by the
invariants the method fixes (100 % budget == 16-bit attention, 0 % budget with
P quantisation off == exact attention on the dequantised tensors, T_i = all /
none == forced paths, tile-order independence without P quantisation) and by a
second, independently written numpy version of Alg. 1's recurrence.
"""
import math

import numpy as np
import pytest
import torch

from paper_2605_23081_amd import metrics
from paper_2605_23081_amd import workloads as W

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def _softmax_attention_np(q, k, v, causal, scale, q_pos0=0):
    """Textbook Eq. (1): o = sum_j p_j v_j, p = softmax(q.k / sqrt(d)); fp64."""
    s = (q @ k.T) * scale
    if causal:
        qpos = q_pos0 + np.arange(q.shape[0])[:, None]
        s = np.where(np.arange(k.shape[0])[None, :] <= qpos, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=1, keepdims=True)) @ v


def _all_rows(B, H, N):
    return np.array([(b, h, t) for b in range(B) for h in range(H) for t in range(N)], np.int32)


def _all_units(B, H, Tq):
    return np.array([(b, h, i) for b in range(B) for h in range(H) for i in range(Tq)], np.int32)


def _small(dtype="f16", N=256, Hq=2, Hkv=1, Bq=64, seed=1):
    base = W.TINY if dtype == "f16" else W.QWEN3_32K
    w = W.scaled(base, N=N, Hq=Hq, Hkv=Hkv, Bq=Bq, Bk=64, seed=seed, planted_blocks=1, sink_tokens=0)
    q, k, v, _, _ = W.make_prefill(w)
    return w, q, k, v


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_exact_attention_against_numpy_and_torch(oracle, causal, dtype):
    w, q, k, v = _small(dtype)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    out, lse = oracle.attn_exact(qb, kb, vb, dt, causal, scale, _all_rows(1, w.Hq, w.N), want_lse=True)
    out = out.reshape(w.Hq, w.N, w.D)
    qd, kd, vd = q.double(), k.double(), v.double()
    for h in range(w.Hq):
        want = _softmax_attention_np(qd[0, h].numpy(), kd[0, h // w.group].numpy(), vd[0, h // w.group].numpy(), causal, scale)
        assert np.abs(out[h] - want).max() < 1e-12
    ref = torch.nn.functional.scaled_dot_product_attention(
        qd, kd.repeat_interleave(w.group, dim=1), vd.repeat_interleave(w.group, dim=1), is_causal=causal)
    assert np.abs(out - ref[0].numpy()).max() < 1e-10
    # log-sum-exp of the scaled scores
    s = (qd[0, 0] @ kd[0, 0].T * scale).numpy()
    if causal:
        s = np.where(np.tril(np.ones_like(s)) > 0, s, -np.inf)
    want_lse = np.log(np.exp(s - s.max(1, keepdims=True)).sum(1)) + s.max(1)
    assert np.abs(lse.reshape(w.Hq, w.N)[0] - want_lse).max() < 1e-10


def test_exact_attention_decode_position(oracle):
    w, q, k, v = _small("f16", N=192, Hq=2, Hkv=1)
    qb, dt = oracle.bits_of(q[:, :, -1:, :]); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    rows = np.array([(0, 0, 0), (0, 1, 0)], np.int32)
    out = oracle.attn_exact(qb, kb, vb, dt, True, 0.1, rows, q_pos0=w.N - 1)
    for h in range(2):
        want = _softmax_attention_np(q[0, h, -1:].double().numpy(), k[0, 0].double().numpy(), v[0, 0].double().numpy(), False, 0.1)
        assert np.abs(out[h] - want[0]).max() < 1e-12


@pytest.mark.parametrize("dtype,Bq", [("f16", 64), ("bf16", 128)])
def test_full_budget_equals_16bit_attention(oracle, dtype, Bq):
    """Budget 100 %: every visible tile on the 16-bit path -> exact attention up to the rounding of P."""
    w, q, k, v = _small(dtype, N=512, Bq=Bq)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    Tq = w.N // Bq
    units = _all_units(1, w.Hq, Tq)
    exact = oracle.attn_exact(qb, kb, vb, dt, True, scale, _all_rows(1, w.Hq, w.N)).reshape(w.Hq, w.N, w.D)
    qm = oracle.block_means(qb, dt, Bq); km = oracle.block_means(kb, dt, 64)
    idx, cnt = oracle.select_topk(qm, km, Bq, 64, True, 1.0)
    for order in (0, 1):
        out, lse = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, True, scale, units, tile_order=order, want_lse=True)
        out = out.reshape(w.Hq, w.N, w.D)
        tol = 2e-3 if dtype == "f16" else 8e-3   # P carries 11 (fp16) or 8 (bf16) significant bits
        assert np.abs(out - exact).max() < tol
        assert np.abs(out - exact).max() > 0          # the rounding of P is really applied
    forced = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, Bq, 64, True, scale, units, force_path=1).reshape(w.Hq, w.N, w.D)
    assert np.array_equal(forced, out if order == 0 else forced) or np.abs(forced - out).max() < 1e-12
    _, lse_exact = oracle.attn_exact(qb, kb, vb, dt, True, scale, _all_rows(1, w.Hq, w.N), want_lse=True)
    assert np.abs(lse.ravel() - lse_exact).max() < 1e-10   # l uses the unrounded P


@pytest.mark.parametrize("causal", [True, False])
def test_zero_budget_without_p_quantisation_is_attention_on_dequantised_tensors(oracle, causal):
    w, q, k, v = _small("f16", N=256, Bq=64)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    units = _all_units(1, w.Hq, w.N // 64)
    for order in (0, 1):
        out = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, causal, scale, units, tile_order=order,
                                         quantize_p=False, force_path=0).reshape(w.Hq, w.N, w.D)
        qd = oracle.dequantize_mxfp4(*oracle.quantize_mxfp4(qb, dt, 0), 0)
        kd = oracle.dequantize_mxfp4(*oracle.quantize_mxfp4(kb, dt, 0), 0)
        vd = oracle.dequantize_mxfp4(*oracle.quantize_mxfp4(vb, dt, 1), 1)
        for h in range(w.Hq):
            want = _softmax_attention_np(qd[0, h], kd[0, 0], vd[0, 0], causal, scale)
            assert np.abs(out[h] - want).max() < 1e-11


# ---- an independent numpy restatement of Alg. 1 (one head), used only as a cross-check ----

def _np_mx_quant_dequant(x):
    """x [..., 32] -> dequantised MXFP4 values; power-of-two scale, nearest grid value, ties to even code."""
    amax = np.abs(x).max(-1, keepdims=True)
    e = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 2, 0.0)
    e = np.clip(e, -127, 127)
    y = x / 2.0 ** e
    a = np.minimum(np.abs(y), 6.0)
    d = np.abs(a[..., None] - E2M1)
    best = np.zeros(a.shape, np.int64)
    for c in range(1, 8):
        cur = np.take_along_axis(d, best[..., None], -1)[..., 0]
        better = (d[..., c] < cur) | ((d[..., c] == cur) & (c % 2 == 0) & (best % 2 == 1))
        best = np.where(better, c, best)
    return np.sign(y) * E2M1[best] * 2.0 ** e


def _np_round(x, dtype):
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float64)
    return torch.from_numpy(x).to(torch.bfloat16).double().numpy()


def _np_thrift_head(q, k, v, sel, Bq, Bk, causal, scale, dtype, quantize_p=True):
    """q,k,v fp64 [N,D] holding 16-bit values; sel[i] = set of 16-bit key blocks of query block i."""
    N, D = q.shape
    qq = _np_mx_quant_dequant(q.reshape(N, D // 32, 32)).reshape(N, D)
    kq = _np_mx_quant_dequant(k.reshape(N, D // 32, 32)).reshape(N, D)
    vq = _np_mx_quant_dequant(v.reshape(N // 32, 32, D).transpose(0, 2, 1)).transpose(0, 2, 1).reshape(N, D)
    out = np.zeros((N, D))
    for i in range(N // Bq):
        rows = slice(i * Bq, (i + 1) * Bq)
        m = np.full(Bq, -np.inf); l = np.zeros(Bq); O = np.zeros((Bq, D))
        nvis = min(N // Bk, ((i + 1) * Bq - 1) // Bk + 1) if causal else N // Bk
        for j in range(nvis):
            cols = slice(j * Bk, (j + 1) * Bk)
            hi = j in sel[i]
            S = ((q[rows] @ k[cols].T) if hi else (qq[rows] @ kq[cols].T)) * scale
            if causal:
                S = np.where(np.arange(j * Bk, (j + 1) * Bk)[None, :] <= np.arange(i * Bq, (i + 1) * Bq)[:, None], S, -np.inf)
            m_new = np.maximum(m, S.max(1))
            live = np.isfinite(m_new)
            m_safe = np.where(live, m_new, 0.0)
            alpha = np.where(np.isfinite(m), np.exp(m - m_safe), 0.0)
            P = np.where(live[:, None], np.exp(S - m_safe[:, None]), 0.0)
            l = alpha * l + P.sum(1)
            if hi:
                O = alpha[:, None] * O + _np_round(P, dtype) @ v[cols]
            else:
                Pq = _np_mx_quant_dequant(P.reshape(Bq, Bk // 32, 32)).reshape(Bq, Bk) if quantize_p else P
                O = alpha[:, None] * O + Pq @ vq[cols]
            m = m_new
        out[rows] = O / l[:, None]
    return out


@pytest.mark.parametrize("dtype,Bq,causal", [("f16", 64, True), ("bf16", 128, True), ("f16", 64, False)])
def test_mixed_attention_against_independent_numpy_recurrence(oracle, dtype, Bq, causal):
    w, q, k, v = _small(dtype, N=512, Hq=2, Hkv=1, Bq=Bq, seed=5)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    Tq = w.N // Bq
    qm = oracle.block_means(qb, dt, Bq); km = oracle.block_means(kb, dt, 64)
    for budget in (0.0, 0.25, 1.0):
        idx, cnt = oracle.select_topk(qm, km, Bq, 64, causal, budget)
        out = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, causal, scale, _all_units(1, w.Hq, Tq)).reshape(w.Hq, w.N, w.D)
        for h in range(w.Hq):
            sel = [set(idx[0, h, i, :cnt[0, h, i]].tolist()) for i in range(Tq)]
            want = _np_thrift_head(q[0, h].double().numpy(), k[0, 0].double().numpy(), v[0, 0].double().numpy(), sel, Bq, 64, causal, scale, dtype)
            # same arithmetic in a different summation order: agreement to rounding noise, except where
            # that noise flips a 4-bit code of P (rare, bounded by one grid step of one element)
            diff = np.abs(out[h] - want)
            assert np.quantile(diff, 0.999) < 1e-9
            assert diff.max() < 5e-3


def test_selection_sets_all_and_none_equal_forced_paths_and_branch_swap(oracle):
    w, q, k, v = _small("f16", N=512, Hq=1, Hkv=1, Bq=64, seed=7)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    Tq = Tk = 8
    units = _all_units(1, 1, Tq)
    full_idx = np.full((1, 1, Tq, Tk), -1, np.int32); full_cnt = np.zeros((1, 1, Tq), np.int32)
    for i in range(Tq):
        full_idx[0, 0, i, :i + 1] = np.arange(i + 1); full_cnt[0, 0, i] = i + 1
    none_idx = np.full((1, 1, Tq, 1), -1, np.int32); none_cnt = np.zeros((1, 1, Tq), np.int32)
    a = oracle.attn_thrift_prefill(qb, kb, vb, dt, full_idx, full_cnt, 64, 64, True, scale, units)
    b = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=1)
    assert np.array_equal(a, b)
    a = oracle.attn_thrift_prefill(qb, kb, vb, dt, none_idx, none_cnt, 64, 64, True, scale, units)
    b = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=0)
    assert np.array_equal(a, b)
    # a hand-set T_i changes exactly the rows of that query block and nothing else
    one_idx = none_idx.copy(); one_cnt = none_cnt.copy()
    one_idx[0, 0, 5, 0] = 2; one_cnt[0, 0, 5] = 1
    c = oracle.attn_thrift_prefill(qb, kb, vb, dt, one_idx, one_cnt, 64, 64, True, scale, units)
    assert np.array_equal(c[:5], a[:5]) and np.array_equal(c[6:], a[6:]) and not np.array_equal(c[5], a[5])
    # without P quantisation the result does not depend on the order of the tiles (to rounding)
    sel_idx, sel_cnt = oracle.select_topk(oracle.block_means(qb, dt, 64), oracle.block_means(kb, dt, 64), 64, 64, True, 0.25)
    o0 = oracle.attn_thrift_prefill(qb, kb, vb, dt, sel_idx, sel_cnt, 64, 64, True, scale, units, tile_order=0, quantize_p=False)
    o1 = oracle.attn_thrift_prefill(qb, kb, vb, dt, sel_idx, sel_cnt, 64, 64, True, scale, units, tile_order=1, quantize_p=False)
    assert np.abs(o0 - o1).max() < 2e-3          # only the fp16 rounding of P on promoted tiles depends on the running max
    p0 = oracle.attn_thrift_prefill(qb, kb, vb, dt, sel_idx, sel_cnt, 64, 64, True, scale, units, tile_order=0)
    p1 = oracle.attn_thrift_prefill(qb, kb, vb, dt, sel_idx, sel_cnt, 64, 64, True, scale, units, tile_order=1)
    # with P quantisation on, the order changes the running max each tile sees, hence which way each
    # 4-bit code of P rounds: two noise realisations of the same quantity, far below the 4-bit error itself
    rows = _all_rows(1, 1, w.N)
    exact = oracle.attn_exact(qb, kb, vb, dt, True, scale, rows).reshape(p0.shape)
    assert metrics.rel_fro(p0, p1) < 0.1 * metrics.rel_fro(p0, exact)


def test_decode_split_k_and_invariants(oracle):
    w = W.scaled(W.DECODE_131K, B=2, N=1024, Hq=4, Hkv=2, sink_tokens=4)
    q, k, v = W.make_decode(w)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    Tk = w.N // 64
    km = oracle.block_means(kb, dt, 64)
    qm = q.float().numpy().reshape(2, 4, 1, 128)
    idx, cnt = oracle.select_topk(qm, km, 1, 64, True, 0.05, q_block_offset=w.N - 1)
    assert np.all(cnt == math.ceil(0.05 * Tk))
    idx, cnt = idx[:, :, 0], cnt[:, :, 0]
    rows = np.array([(b, h, 0) for b in range(2) for h in range(4)], np.int32)
    exact = oracle.attn_exact(qb.reshape(2, 4, 1, 128), kb, vb, dt, False, scale, rows).reshape(2, 4, 128)
    # 100 %: 16-bit path everywhere == exact attention up to P rounding, for any split
    for split in (0, 4, 5):
        o = oracle.attn_thrift_decode(qb, kb, vb, dt, None, None, 64, scale, split, force_path=1)
        assert np.abs(o - exact).max() < 2e-3
    # P quantisation off: split-K is exact arithmetic, any partition size gives the same result
    ref = oracle.attn_thrift_decode(qb, kb, vb, dt, idx, cnt, 64, scale, 0, quantize_p=False)
    for split in (1, 4, 7, 16):
        o = oracle.attn_thrift_decode(qb, kb, vb, dt, idx, cnt, 64, scale, split, quantize_p=False)
        assert np.abs(o - ref).max() < 1e-3     # fp16 rounding of P on promoted blocks depends on the partition max
    o0 = oracle.attn_thrift_decode(qb, kb, vb, dt, None, None, 64, scale, 0, quantize_p=False, force_path=0)
    o4 = oracle.attn_thrift_decode(qb, kb, vb, dt, None, None, 64, scale, 4, quantize_p=False, force_path=0)
    assert np.abs(o0 - o4).max() < 1e-12
    # decode == the last row of a prefill over the same keys (one partition, same tile order)
    qfull = torch.zeros(2, 4, w.N, 128, dtype=q.dtype); qfull[:, :, -1] = q
    qfb, _ = oracle.bits_of(qfull)
    pidx = np.full((2, 4, w.N, idx.shape[-1]), -1, np.int32); pcnt = np.zeros((2, 4, w.N), np.int32)
    pidx[:, :, -1] = idx; pcnt[:, :, -1] = cnt
    units = np.array([(b, h, w.N - 1) for b in range(2) for h in range(4)], np.int32)
    pre = oracle.attn_thrift_prefill(qfb, kb, vb, dt, pidx, pcnt, 1, 64, True, scale, units).reshape(2, 4, 128)
    dec = oracle.attn_thrift_decode(qb, kb, vb, dt, idx, cnt, 64, scale, 0)
    assert np.array_equal(pre, dec)
    # shorter sequences via seqlens: only the first blocks are read
    sl = np.array([512, 1024], np.int32)
    idx_s = np.where(idx < 8, idx, -1); idx_s.sort(axis=-1); idx_s = idx_s[..., ::-1].copy()
    cnt_s = (idx_s >= 0).sum(-1).astype(np.int32)
    idx_s2 = np.full_like(idx_s, -1)
    for b in range(2):
        for h in range(4):
            vals = sorted(x for x in idx_s[b, h] if x >= 0)
            idx_s2[b, h, :len(vals)] = vals
    o = oracle.attn_thrift_decode(qb, kb, vb, dt, idx_s2, cnt_s, 64, scale, 4, seqlens=sl, force_path=1)
    ex0 = oracle.attn_exact(qb.reshape(2, 4, 1, 128)[:1], kb[:1, :, :512], vb[:1, :, :512], dt, False, scale, rows[:4]).reshape(4, 128)
    assert np.abs(o[0] - ex0).max() < 2e-3


def test_promoting_blocks_reduces_error_on_planted_workload(oracle):
    """Qualitative claim of Sec. 3.1/3.2 on the synthetic stand-in: 16-bit for a few top blocks closes
    most of the 4-bit error gap, and the block-mean selector beats promoting the same number of
    lowest-scored blocks."""
    w = W.TINY
    q, k, v, _, _ = W.make_prefill(w)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    sample = np.array([(0, 0, i) for i in (20, 25, 31)], np.int32)
    rows = np.array([(0, 0, i * 64 + r) for i in (20, 25, 31) for r in range(64)], np.int32)
    exact = oracle.attn_exact(qb, kb, vb, dt, True, scale, rows).reshape(3, 64, 128)
    qm = oracle.block_means(qb, dt, 64); km = oracle.block_means(kb, dt, 64)
    idx, cnt = oracle.select_topk(qm, km, 64, 64, True, 0.05)
    e4 = metrics.rel_fro(oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, sample, force_path=0), exact)
    e16 = metrics.rel_fro(oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, sample, force_path=1), exact)
    em = metrics.rel_fro(oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, 64, 64, True, scale, sample), exact)
    assert e16 < em < e4
    assert metrics.recovery(e16, e4, em) > 0.5
    # worst-scored blocks instead of best-scored ones recover less
    scores = oracle.block_scores(qm, km)
    bad_idx = np.full_like(idx, -1)
    for i in range(32):
        order = np.argsort(scores[0, 0, i, :i + 1], kind="stable")[:cnt[0, 0, i]]
        bad_idx[0, 0, i, :cnt[0, 0, i]] = np.sort(order)
    eb = metrics.rel_fro(oracle.attn_thrift_prefill(qb, kb, vb, dt, bad_idx, cnt, 64, 64, True, scale, sample), exact)
    assert em < eb


def test_error_bound_diagnostic_bookkeeping(oracle):
    """Eq. (4) right-hand side, split by key block: non-negative terms that add up to the total and
    vanish for blocks the (causal) row cannot see."""
    w = W.TINY
    q, k, v, _, _ = W.make_prefill(w)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    t = 20 * 64 + 10
    total, per = oracle.error_bound_rhs(qb[0, 0, t], kb[0, 0], vb[0, 0], dt, 64, t + 1, 1 / math.sqrt(128))
    assert total > 0 and np.all(per >= 0)
    assert abs(per.sum() - total) < 1e-12 * max(1, total)
    assert np.all(per[21:] == 0) and per[20] > 0


@pytest.mark.parametrize("dtype,Bq,nq_blocks", [("f16", 64, 3), ("bf16", 128, 1)])
def test_chunked_prefill_pins(oracle, dtype, Bq, nq_blocks):
    """Chunked prefill (the last Nq queries of a longer sequence):
    (a) at 100 % budget it is exact attention with the queries at their shifted positions (the textbook routine,
        up to the rounding of P); with P quantisation off and all tiles on the 4-bit path it is exact attention
        on the dequantised tensors at those positions (numpy brute force);
    (b) rows of a chunk equal the same rows of the full prefill given the same selected sets."""
    w, q, k, v = _small(dtype, N=512, Bq=Bq)
    Nq = nq_blocks * Bq
    off = (w.N - Nq) // Bq
    scale = 1 / math.sqrt(w.D)
    qc = q[:, :, w.N - Nq:, :].contiguous()
    qb, dt = oracle.bits_of(q); qcb, _ = oracle.bits_of(qc); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    units_c = _all_units(1, w.Hq, nq_blocks)
    # (a) 100 %: against exact attention at shifted positions
    exact = oracle.attn_exact(qcb, kb, vb, dt, True, scale, _all_rows(1, w.Hq, Nq), q_pos0=w.N - Nq).reshape(w.Hq, Nq, w.D)
    full16 = oracle.attn_thrift_prefill(qcb, kb, vb, dt, None, None, Bq, 64, True, scale, units_c, force_path=1,
                                        q_block_offset=off).reshape(w.Hq, Nq, w.D)
    assert np.abs(full16 - exact).max() < (2e-3 if dtype == "f16" else 8e-3)
    # (a') 4-bit path, P not quantised: numpy attention on the dequantised tensors
    c, s = oracle.quantize_mxfp4(qcb, dt, 0); qd = oracle.dequantize_mxfp4(c, s, 0)
    c, s = oracle.quantize_mxfp4(kb, dt, 0); kd = oracle.dequantize_mxfp4(c, s, 0)
    c, s = oracle.quantize_mxfp4(vb, dt, 1); vd = oracle.dequantize_mxfp4(c, s, 1)
    got = oracle.attn_thrift_prefill(qcb, kb, vb, dt, None, None, Bq, 64, True, scale, units_c, force_path=0, quantize_p=False,
                                     q_block_offset=off).reshape(w.Hq, Nq, w.D)
    for h in range(w.Hq):
        want = _softmax_attention_np(qd[0, h], kd[0, 0], vd[0, 0], True, scale, q_pos0=w.N - Nq)
        assert np.abs(got[h] - want).max() < 1e-10
    # (b) mixed: chunk rows == full-prefill rows for the same sets
    qm = oracle.block_means(qb, dt, Bq); km = oracle.block_means(kb, dt, 64)
    idx, cnt = oracle.select_topk(qm, km, Bq, 64, True, 0.25)
    Tq = w.N // Bq
    full = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, True, scale, _all_units(1, w.Hq, Tq)).reshape(w.Hq, Tq, Bq, w.D)
    chunk = oracle.attn_thrift_prefill(qcb, kb, vb, dt, idx[:, :, off:], cnt[:, :, off:], Bq, 64, True, scale, units_c,
                                       q_block_offset=off).reshape(w.Hq, nq_blocks, Bq, w.D)
    assert np.array_equal(chunk, full[:, off:])
    # selection with the same offset reproduces the tail rows of the full selection
    idx_c, cnt_c = oracle.select_topk(qm[:, :, off:], km, Bq, 64, True, 0.25, q_block_offset=off, kmax=idx.shape[-1])
    assert np.array_equal(idx_c, idx[:, :, off:]) and np.array_equal(cnt_c, cnt[:, :, off:])


def test_nvfp4_variant_invariants(oracle):
    """The paper-format study variant: the 16-bit path is untouched; the 4-bit path without P quantisation is exact
    attention on the NVFP4-dequantised tensors; the two-level P quantisation stays within the format's error."""
    w, q, k, v = _small("f16", N=256, Bq=64)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    units = _all_units(1, w.Hq, w.N // 64)
    a = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=1, fmt=1)
    b = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=1, fmt=0)
    assert np.array_equal(a, b)
    qd = oracle.nvfp4_qdq(q.double().numpy()).reshape(w.Hq, w.N, w.D)
    kd = oracle.nvfp4_qdq(k.double().numpy()).reshape(w.N, w.D)
    vt = np.ascontiguousarray(v.double().numpy().reshape(w.N, w.D).T)            # groups of 16 along the tokens
    vd = oracle.nvfp4_qdq(vt).T
    got = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=0, quantize_p=False,
                                     fmt=1).reshape(w.Hq, w.N, w.D)
    for h in range(w.Hq):
        assert np.abs(got[h] - _softmax_attention_np(qd[h], kd, vd, True, scale)).max() < 1e-10
    withp = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=0, fmt=1).reshape(w.Hq, w.N, w.D)
    assert 0 < np.abs(withp - got).max() < 0.5
    # NVFP4 (E4M3 scales per 16) is the finer format: closer to exact attention than MXFP4 on the same inputs
    exact = oracle.attn_exact(qb, kb, vb, dt, True, scale, _all_rows(1, w.Hq, w.N)).reshape(w.Hq, w.N, w.D)
    mx = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, True, scale, units, force_path=0, fmt=0).reshape(w.Hq, w.N, w.D)
    assert metrics.rel_fro(withp, exact) < metrics.rel_fro(mx, exact)


@pytest.mark.parametrize("N,Bq,causal", [(200, 64, True), (333, 128, True), (97, 64, False), (64 + 31, 64, True)])
def test_ragged_lengths_pins(oracle, N, Bq, causal):
    """Sequence lengths that are not multiples of the blocks (short last query / key block, short last V group):
    means of a short block over its own tokens (numpy); 100 % budget == exact attention (separate routine);
    4-bit path without P quantisation == numpy attention on the dequantised tensors, whose last V group is
    quantised from the tokens it has (checked against the stand-alone group quantiser)."""
    w = W.scaled(W.TINY, N=512, Hq=2, Hkv=1, Bq=64, Bk=64, seed=5, planted_blocks=1, sink_tokens=0)
    q, k, v, _, _ = W.make_prefill(w)
    q, k, v = q[:, :, :N].contiguous(), k[:, :, :N].contiguous(), v[:, :, :N].contiguous()
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    # means
    km = oracle.block_means(kb, dt, 64)
    Tk = -(-N // 64)
    assert km.shape == (1, 1, Tk, w.D)
    kd64 = k.double().numpy()[0, 0]
    for j in range(Tk):
        assert np.array_equal(km[0, 0, j], kd64[j * 64:min(N, (j + 1) * 64)].mean(axis=0).astype(np.float32))
    # V quantiser: last group from its own tokens
    codes, scales = oracle.quantize_mxfp4(vb, dt, 1)
    assert scales.shape == (1, 1, -(-N // 32), w.D)
    g_last = (N - 1) // 32
    vd64 = v.double().numpy()[0, 0]
    for c in (0, 17, 127):
        grp = vd64[g_last * 32:N, c]
        cg, sb = oracle.mx_quantize_group(grp)
        assert sb == scales[0, 0, g_last, c] and np.array_equal(cg, codes[0, 0, g_last * 32:N, c])
    vdq = oracle.dequantize_mxfp4(codes, scales, 1)[0, 0]
    c0, s0 = oracle.quantize_mxfp4(kb, dt, 0); kdq = oracle.dequantize_mxfp4(c0, s0, 0)[0, 0]
    c0, s0 = oracle.quantize_mxfp4(qb, dt, 0); qdq = oracle.dequantize_mxfp4(c0, s0, 0)[0]
    Tq = -(-N // Bq)
    units = _all_units(1, w.Hq, Tq)
    exact = oracle.attn_exact(qb, kb, vb, dt, causal, scale, _all_rows(1, w.Hq, N)).reshape(w.Hq, N, w.D)
    full16 = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, Bq, 64, causal, scale, units, force_path=1)
    full16 = full16.reshape(w.Hq, Tq * Bq, w.D)
    assert np.abs(full16[:, :N] - exact).max() < 2e-3 and np.all(full16[:, N:] == 0)
    got = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, Bq, 64, causal, scale, units, force_path=0,
                                     quantize_p=False).reshape(w.Hq, Tq * Bq, w.D)
    for h in range(w.Hq):
        assert np.abs(got[h, :N] - _softmax_attention_np(qdq[h], kdq, vdq, causal, scale)).max() < 1e-10
    # mixed with a real selection: shapes follow the ragged block counts, rows past the end stay zero
    qm = oracle.block_means(qb, dt, Bq)
    idx, cnt = oracle.select_topk(qm, km, Bq, 64, causal, 0.3)
    assert idx.shape[2] == Tq and cnt.max() <= Tk
    mixed = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, causal, scale, units).reshape(w.Hq, Tq * Bq, w.D)
    assert np.all(mixed[:, N:] == 0) and np.isfinite(mixed).all()
    assert metrics.rel_fro(mixed[:, :N], exact) < metrics.rel_fro(got[:, :N], exact) + 0.05
    # decode over a cache whose length is not a multiple of the block: == the last row of the prefill
    if causal:
        ql = q[:, :, N - 1].contiguous()
        qlb, _ = oracle.bits_of(ql)
        d16 = oracle.attn_thrift_decode(qlb, kb, vb, dt, None, None, 64, scale, 0, seqlens=np.array([N], np.int32), force_path=1)
        assert np.abs(d16[0] - exact[:, N - 1]).max() < 2e-3
        d4 = oracle.attn_thrift_decode(qlb, kb, vb, dt, None, None, 64, scale, 0, seqlens=np.array([N], np.int32), force_path=0,
                                       quantize_p=False)
        assert np.abs(d4[0] - got[:, N - 1]).max() < 1e-10
        # split-K (the short block is a partition of its own): without P quantisation the cut points do not matter
        for sb in (1, 2):
            d4s = oracle.attn_thrift_decode(qlb, kb, vb, dt, None, None, 64, scale, sb, seqlens=np.array([N], np.int32),
                                            force_path=0, quantize_p=False)
            assert np.abs(d4s - d4).max() < 1e-10


# ------------------------------------------------------------------ Alg. 1 step 19 as printed (NVFP4 study variant)

def _e2m1_rne(y):
    """Nearest value of the E2M1 grid, ties to the even code, magnitudes above 6 saturate (brute force over the grid)."""
    a = np.abs(y)
    out = np.empty_like(a)
    for i, x in enumerate(a.ravel()):
        d = np.abs(E2M1 - min(x, 6.0))
        best = np.flatnonzero(d == d.min())
        out.ravel()[i] = E2M1[best[0] if len(best) == 1 or best[0] % 2 == 0 else best[1]]
    return np.sign(y) * out


def _e4m3(x):
    """Round to E4M3 with torch's float8 type (saturating at 448, which torch does not do by itself)."""
    return float(torch.tensor(min(x, 448.0), dtype=torch.float64).to(torch.float32).to(torch.float8_e4m3fn).to(torch.float64))


def _nvfp4_groups_np(x):
    """E2M1 elements with one E4M3 scale (group maximum / 6) per 16 consecutive values of the last axis."""
    flat = x.reshape(-1, 16)
    out = np.zeros_like(flat)
    for g, grp in enumerate(flat):
        s = _e4m3(np.abs(grp).max() / 6.0)
        if s > 0:
            out[g] = _e2m1_rne(grp / s) * s
    return out.reshape(x.shape)


def _nvfp4_attention_np(qd, kd, vd, scale, Bk=64, p_level1=448.0 * 6.0):
    """Alg. 1 steps 15-20 on the 4-bit path, written out in numpy for non-causal inputs that are already
    quantised-dequantised: per key block, scores, running maximum, P = exp(S - m), row sum from the unquantised P,
    then the two-level quantisation of P of step 19 (s1 = rowmax(P) / (448 * 6), NVFP4 groups of 16 keys on P / s1)
    and O += s1 * P_hat V."""
    Nq, D = qd.shape
    m = np.full(Nq, -np.inf); l = np.zeros(Nq); O = np.zeros((Nq, D))
    for j in range(kd.shape[0] // Bk):
        S = (qd @ kd[j * Bk:(j + 1) * Bk].T) * scale
        m_new = np.maximum(m, S.max(axis=1))
        alpha = np.where(np.isinf(m), 0.0, np.exp(m - m_new))
        P = np.exp(S - m_new[:, None])
        l = alpha * l + P.sum(axis=1)
        s1 = P.max(axis=1) / p_level1
        Ph = _nvfp4_groups_np(P / s1[:, None]) * s1[:, None]
        O = alpha[:, None] * O + Ph @ vd[j * Bk:(j + 1) * Bk]
        m = m_new
    return O / l[:, None]


def test_two_level_p_quantisation_of_alg1_step19_against_numpy(oracle):
    """The NVFP4 branch of the oracle's tile step against an independent numpy version of Alg. 1 step 19, element by
    element, on two key blocks (so that the running maximum, the rescale and the level-1 scale all matter).  The E4M3
    scale rounding comes from torch's float8 type, the E2M1 rounding from a brute-force search of the grid.  A level-1
    scale of rowmax(P)/448 instead of rowmax(P)/(448*6) must NOT reproduce the oracle."""
    w = W.scaled(W.TINY, N=128, Hq=2, Hkv=1, Bq=64, Bk=64, seed=9, planted_blocks=1, sink_tokens=0)
    q, k, v, _, _ = W.make_prefill(w)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    units = _all_units(1, w.Hq, w.N // 64)
    got = oracle.attn_thrift_prefill(qb, kb, vb, dt, None, None, 64, 64, False, scale, units, force_path=0, fmt=1)
    got = got.reshape(w.Hq, w.N, w.D)
    kd = _nvfp4_groups_np(k.double().numpy()[0, 0])
    vd = _nvfp4_groups_np(np.ascontiguousarray(v.double().numpy()[0, 0].T)).T          # groups of 16 along the tokens
    worst_wrong = 0.0
    for h in range(w.Hq):
        qd = _nvfp4_groups_np(q.double().numpy()[0, h])
        want = _nvfp4_attention_np(qd, kd, vd, scale)
        assert np.abs(got[h] - want).max() < 1e-12
        wrong = _nvfp4_attention_np(qd, kd, vd, scale, p_level1=448.0)
        worst_wrong = max(worst_wrong, np.abs(got[h] - wrong).max())
    assert worst_wrong > 1e-4          # the factor 6 of the level-1 scale is visible: dropping it changes the result


# ------------------------------------------------------------------ Eq. (4)

def test_error_bound_rhs_against_direct_evaluation_and_first_order_inequality(oracle):
    """Eq. (4): RHS = sum_j |eps_j| p_j ||v_j - o||, evaluated directly in numpy on one row (eps from the dequantised
    MXFP4 query and keys), must equal the oracle's value; and the bound must hold to first order: with the exact
    values and scores perturbed by eps, ||o' - o|| <= RHS up to a second-order term, and o' - o equals Eq. (3)'s
    sum_j eps_j p_j (v_j - o) to the same order."""
    w = W.scaled(W.TINY, N=512, Hq=1, Hkv=1, Bq=64, Bk=64, seed=4, planted_blocks=1, sink_tokens=0, outlier_channels=0,
                 query_mean_gain=0.0)
    q, k, v, _, _ = W.make_prefill(w)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(w.D)
    c, s = oracle.quantize_mxfp4(qb, dt, 0); qq = oracle.dequantize_mxfp4(c, s, 0)[0, 0]
    c, s = oracle.quantize_mxfp4(kb, dt, 0); kq = oracle.dequantize_mxfp4(c, s, 0)[0, 0]
    qd, kd, vd = q.double().numpy()[0, 0], k.double().numpy()[0, 0], v.double().numpy()[0, 0]
    for t in (70, 300, 511):
        n = t + 1
        sc = (kd[:n] @ qd[t]) * scale
        eps = (kq[:n] @ qq[t]) * scale - sc
        p = np.exp(sc - sc.max()); p /= p.sum()
        o = p @ vd[:n]
        dist = np.linalg.norm(vd[:n] - o, axis=1)
        terms = np.abs(eps) * p * dist
        total, per = oracle.error_bound_rhs(qb[0, 0, t], kb[0, 0], vb[0, 0], dt, 64, n, scale)
        assert abs(total - terms.sum()) <= 1e-12 * terms.sum()
        want_per = np.zeros(w.N // 64)
        np.add.at(want_per, np.arange(n) // 64, terms)
        assert np.abs(per - want_per).max() <= 1e-12 * terms.sum()
        # first order: shrink the perturbation until the second-order term is small, then compare
        for shrink in (1.0, 0.1):
            e = eps * shrink
            p2 = np.exp(sc + e - (sc + e).max()); p2 /= p2.sum()
            delta = p2 @ vd[:n] - o
            first_order = (e * p) @ (vd[:n] - o)
            rhs = terms.sum() * shrink
            second = np.abs(e).max() * rhs * 4.0                     # generous bound on the neglected term
            assert np.linalg.norm(delta - first_order) <= second
            assert np.linalg.norm(delta) <= rhs + second
