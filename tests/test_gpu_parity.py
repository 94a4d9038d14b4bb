"""GPU parity: every C-ABI entry point against the CPU oracle on identical seeded inputs.

Bars (from the build's target): selected block ids exact wherever neighbouring scores differ by more
than 1e-6 relative; MXFP4 codes and scales bit-exact; block means bit-exact; outputs of all-16-bit
runs within 2e-3 max abs; mixed outputs within 3e-2 max abs.
"""
import math

import numpy as np
import pytest
import torch

from paper_2605_23081_amd import workloads as W
from tests.gpu_util import check_selection, to_np, unpack_axis0, unpack_axis1

pytestmark = pytest.mark.gpu

TOL16 = 2e-3
TOLMIX = 3e-2


@pytest.fixture(scope="module")
def T():
    from paper_2605_23081_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return binding


def _say(msg):
    print(msg, flush=True)


def _small_bf16(N=1024, Hq=4, Hkv=2, Bq=128, seed=3, **kw):
    return W.scaled(W.QWEN3_32K, N=N, Hq=Hq, Hkv=Hkv, Bq=Bq, seed=seed, **kw)


def _units(B, H, Tq):
    return np.array([(b, h, i) for b in range(B) for h in range(H) for i in range(Tq)], np.int32)


# ------------------------------------------------------------------ block means

@pytest.mark.parametrize("wl,block", [(W.TINY, 64), (_small_bf16(), 128), (_small_bf16(), 64), (_small_bf16(N=384, Bq=64), 96)])
def test_block_means_bit_exact(T, oracle, wl, block):
    _say(f"block_means {wl.name} N={wl.N} block={block}")
    q, k, v, _, _ = W.make_prefill(wl)
    for t in (q, k):
        bits, dt = oracle.bits_of(t)
        want = oracle.block_means(bits, dt, block)
        got = to_np(T.thrift_block_means(t.cuda(), block))
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


# ------------------------------------------------------------------ quantiser

def _edge_tensor(dtype):
    """[1,1,64,128] with groups that exercise zeros, signed zeros, saturation, ties, tiny and huge magnitudes."""
    g = torch.Generator().manual_seed(11)
    x = torch.randn(1, 1, 64, 128, generator=g)
    x[0, 0, 0, :32] = 0.0
    x[0, 0, 1, :32] = -0.0
    x[0, 0, 2, :32] = torch.tensor([7.0] + [0.25 * i for i in range(31)])           # ties at every half step, max in (6,8)
    x[0, 0, 3, :32] = torch.tensor([4.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0] * 4) * torch.tensor([1, -1] * 16)
    x[0, 0, 4, :32] = 60000.0 if dtype == torch.float16 else 3.0e38
    x[0, 0, 5, :32] = 6.0e-8 if dtype == torch.float16 else 1.0e-30
    x[0, 0, 6, :32] = torch.linspace(-1e-3, 1e-3, 32)
    x[0, 0, 7, 32:64] = torch.tensor([1e4] + [1e-4] * 31)                             # everything but the max underflows to 0
    if dtype == torch.bfloat16:
        x[0, 0, 8, :32] = 1.0e-38                                                    # scale byte would be < 1
        x[0, 0, 9, :32] = torch.tensor([2.0 ** -126 * (i + 1) / 8 for i in range(32)])
    x[0, 0, 32:, 64:] *= 100.0
    return x.to(dtype)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_quantize_bit_exact_edges_and_random(T, oracle, dtype):
    _say(f"quantize edges {dtype}")
    wl = W.TINY if dtype == torch.float16 else _small_bf16()
    q, k, v, _, _ = W.make_prefill(W.scaled(wl, N=512))
    for name, x in (("edges", _edge_tensor(dtype)), ("q", q), ("k", k), ("v", v)):
        bits, dt = oracle.bits_of(x)
        for axis in (0, 1):
            want_c, want_s = oracle.quantize_mxfp4(bits, dt, axis)
            codes, scales = T.thrift_quantize_mxfp4(x.cuda(), axis)
            got_c = unpack_axis0(to_np(codes)) if axis == 0 else unpack_axis1(to_np(codes))
            assert np.array_equal(to_np(scales), want_s), (name, axis)
            bad = np.argwhere(got_c != want_c)
            assert bad.size == 0, (name, axis, bad[:5], got_c[tuple(bad[0])], want_c[tuple(bad[0])])


# ------------------------------------------------------------------ selection

def _select_case(T, oracle, wl, budget, causal=True, fixed_k=-1):
    q, k, v, _, _ = W.make_prefill(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k)
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx_r, cnt_r = oracle.select_topk(qm, km, wl.Bq, wl.Bk, causal, budget, fixed_k)
    qm_g = T.thrift_block_means(q.cuda(), wl.Bq); km_g = T.thrift_block_means(k.cuda(), wl.Bk)
    idx_g, cnt_g = T.thrift_select_topk(qm_g, km_g, wl.Bq, wl.Bk, causal, budget, fixed_k)
    assert idx_g.shape[-1] == max(1, idx_r.shape[-1]) or idx_g.shape[-1] >= idx_r.shape[-1]
    ig = to_np(idx_g)[..., :idx_r.shape[-1]] if idx_r.shape[-1] <= idx_g.shape[-1] else to_np(idx_g)
    assert np.all(to_np(idx_g)[..., idx_r.shape[-1]:] == -1)
    return check_selection(ig, to_np(cnt_g), idx_r, cnt_r, oracle.block_scores(qm, km))


@pytest.mark.parametrize("budget", [0.0, 0.05, 0.25, 1.0])
def test_select_topk_sets(T, oracle, budget):
    _say(f"select tiny budget={budget}")
    assert _select_case(T, oracle, W.TINY, budget) == 0
    _say(f"select bf16 GQA budget={budget}")
    assert _select_case(T, oracle, _small_bf16(N=4096, Hq=4, Hkv=2), budget) == 0


def test_select_topk_variants(T, oracle):
    _say("select non-causal / fixed_k / 80 blocks (two chunks, ragged) / odd group size")
    assert _select_case(T, oracle, _small_bf16(N=2048), 0.1, causal=False) == 0
    assert _select_case(T, oracle, _small_bf16(N=2048), 0.0, fixed_k=5) == 0
    assert _select_case(T, oracle, _small_bf16(N=5120, Hq=3, Hkv=1, Bq=64), 0.05) == 0
    assert _select_case(T, oracle, _small_bf16(N=5120, Hq=6, Hkv=2, Bq=128), 0.3) == 0


def test_select_topk_ties(T, oracle):
    _say("select with exact ties")
    g = torch.Generator().manual_seed(5)
    qm = torch.randint(-2, 3, (1, 2, 8, 128), generator=g).float()
    km = torch.randint(-2, 3, (1, 1, 96, 128), generator=g).float()
    km[0, 0, 70] = km[0, 0, 3]; km[0, 0, 71] = km[0, 0, 3]
    for fixed_k in (1, 4, 17, 96):
        idx_r, cnt_r = oracle.select_topk(qm.numpy(), km.numpy(), 64, 64, False, 0.0, fixed_k)
        idx_g, cnt_g = T.thrift_select_topk(qm.cuda(), km.cuda(), 64, 64, False, 0.0, fixed_k)
        assert np.array_equal(to_np(idx_g), idx_r) and np.array_equal(to_np(cnt_g), cnt_r)


# ------------------------------------------------------------------ prefill

def _prefill_both(T, oracle, wl, budget, causal=True, force_sel=None, out_dtype=torch.float32):
    """Runs GPU and oracle with the ORACLE's selection fed to both; returns (gpu out, oracle out)."""
    q, k, v, _, _ = W.make_prefill(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(wl.D)
    Tq = wl.N // wl.Bq
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx, cnt = oracle.select_topk(qm, km, wl.Bq, wl.Bk, causal, budget) if force_sel is None else force_sel
    want, want_lse = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, causal, scale,
                                                _units(wl.B, wl.Hq, Tq), want_lse=True)
    want = want.reshape(wl.B, wl.Hq, wl.N, wl.D)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    lse = torch.empty(wl.B, wl.Hq, wl.N, dtype=torch.float32, device="cuda")
    got = T.thrift_attn_prefill(qg, kg, vg, q4, qs, k4, ks, v4, vs, torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(),
                                wl.Bq, wl.Bk, causal, 0.0, out_dtype=out_dtype, lse=lse)
    torch.cuda.synchronize()
    return to_np(got.float()), want, to_np(lse), want_lse.reshape(wl.B, wl.Hq, wl.N)


@pytest.mark.parametrize("wl", [W.TINY, _small_bf16(N=1024), _small_bf16(N=640, Hq=2, Hkv=1, Bq=64)])
def test_prefill_all_16bit_tiles(T, oracle, wl):
    _say(f"prefill 100% {wl.name} N={wl.N} Bq={wl.Bq}")
    got, want, lse, want_lse = _prefill_both(T, oracle, wl, 1.0)
    err = np.abs(got - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= TOL16
    assert np.abs(lse - want_lse).max() <= 1e-3


@pytest.mark.parametrize("wl", [W.TINY, _small_bf16(N=1024)])
def test_prefill_all_4bit_tiles(T, oracle, wl):
    _say(f"prefill 0% {wl.name} N={wl.N} Bq={wl.Bq}")
    got, want, _, _ = _prefill_both(T, oracle, wl, 0.0)
    err = np.abs(got - want)
    _say(f"  max abs err {err.max():.3e}  p99.9 {np.quantile(err, 0.999):.3e}")
    assert err.max() <= TOLMIX


@pytest.mark.parametrize("budget", [0.05, 0.10, 0.25])
@pytest.mark.parametrize("wl", [W.TINY, _small_bf16(N=2048)])
def test_prefill_mixed(T, oracle, wl, budget):
    _say(f"prefill mixed {wl.name} N={wl.N} Bq={wl.Bq} budget={budget}")
    got, want, lse, want_lse = _prefill_both(T, oracle, wl, budget)
    err = np.abs(got - want)
    _say(f"  max abs err {err.max():.3e}  p99.9 {np.quantile(err, 0.999):.3e}")
    assert err.max() <= TOLMIX


def test_prefill_non_causal_and_output_dtypes(T, oracle):
    wl = _small_bf16(N=512, Hq=2, Hkv=1)
    _say("prefill non-causal, bf16/f32 outputs")
    got, want, _, _ = _prefill_both(T, oracle, wl, 0.25, causal=False)
    assert np.abs(got - want).max() <= TOLMIX
    got16, want, _, _ = _prefill_both(T, oracle, wl, 0.25, causal=False, out_dtype=torch.bfloat16)
    # bf16 output: one rounding of the fp32 result
    assert np.abs(got16 - torch.from_numpy(got).to(torch.bfloat16).float().numpy()).max() == 0
    wl = W.scaled(W.TINY, N=512)
    got, want, _, _ = _prefill_both(T, oracle, wl, 0.25, out_dtype=torch.float16)
    assert np.abs(got - want).max() <= TOLMIX


def test_prefill_end_to_end_alg1(T, oracle):
    """Q, K, V in, output out, every stage on the GPU (means, TopK, quantisation, attention)."""
    wl = _small_bf16(N=2048)
    _say("prefill end-to-end Alg. 1")
    q, k, v, _, _ = W.make_prefill(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx, cnt = oracle.select_topk(qm, km, wl.Bq, wl.Bk, True, 0.05)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, True, 1 / math.sqrt(wl.D),
                                      _units(1, wl.Hq, wl.N // wl.Bq)).reshape(1, wl.Hq, wl.N, wl.D)
    got = T.thrift_attention(q.cuda(), k.cuda(), v.cuda(), True, wl.Bq, wl.Bk, 0.05, out_dtype=torch.float32)
    assert np.abs(to_np(got) - want).max() <= TOLMIX
    # determinism: a second run gives the same bits
    got2 = T.thrift_attention(q.cuda(), k.cuda(), v.cuda(), True, wl.Bq, wl.Bk, 0.05, out_dtype=torch.float32)
    assert torch.equal(got, got2)


# ------------------------------------------------------------------ decode

def _decode_case(T, oracle, wl, budget, split_blocks, seqlens=None, fixed_k=-1):
    q, k, v = W.make_decode(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(wl.D)
    B, Hq, Tk = wl.B, wl.Hq, wl.N // wl.Bk
    km = oracle.block_means(kb, dt, wl.Bk)
    qm = q.float().numpy().reshape(B, Hq, 1, wl.D)
    sl = None if seqlens is None else np.asarray(seqlens, np.int32)
    kmax = max(1, oracle.row_k(Tk, budget, fixed_k))
    idx_r = np.full((B, Hq, kmax), -1, np.int32); cnt_r = np.zeros((B, Hq), np.int32)
    for b in range(B):
        tkb = Tk if sl is None else sl[b] // wl.Bk
        i_b, c_b = oracle.select_topk(qm[b:b + 1], km[b:b + 1, :, :tkb], 1, wl.Bk, False, budget, fixed_k)
        idx_r[b, :, :i_b.shape[-1]] = i_b[0, :, 0]; cnt_r[b] = c_b[0, :, 0]
    # one recurrence of Alg. 1 per partition of split_blocks key blocks, on both sides
    want = oracle.attn_thrift_decode(qb, kb, vb, dt, idx_r, cnt_r, wl.Bk, scale, split_blocks, seqlens=sl)
    kg, vg = k.cuda(), v.cuda()
    k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    kmean = T.thrift_block_means(kg, wl.Bk)
    got, idx_g, cnt_g = T.thrift_attn_decode(q.cuda(), kg, vg, k4, ks, v4, vs, kmean, wl.Bk, budget, fixed_k, split_blocks,
                                             seqlens=None if sl is None else torch.from_numpy(sl).cuda(),
                                             out_dtype=torch.float32, return_selection=True)
    torch.cuda.synchronize()
    scores = np.zeros((B, Hq, Tk))
    for b in range(B):
        scores[b] = oracle.block_scores(qm[b:b + 1], km[b:b + 1])[0, :, 0]
    swaps = check_selection(to_np(idx_g), to_np(cnt_g), idx_r, cnt_r, scores)
    return to_np(got), want, swaps


@pytest.mark.parametrize("budget", [0.0, 0.05, 0.25, 1.0])
def test_decode_parity(T, oracle, budget):
    wl = W.scaled(W.DECODE_131K, B=2, N=4096, Hq=8, Hkv=2)
    _say(f"decode B=2 N=4096 budget={budget}")
    got, want, swaps = _decode_case(T, oracle, wl, budget, 16)
    err = np.abs(got - want).max()
    _say(f"  max abs err {err:.3e} swaps {swaps}")
    assert swaps == 0
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)


def test_decode_partition_sizes(T, oracle):
    """split_blocks names the key blocks per partition: one recurrence of Alg. 1 per partition, partitions merged by
    log-sum-exp.  Sizes that are not multiples of four, a size larger than the cache (one partition), and the size of
    the benchmark configuration."""
    wl = W.scaled(W.DECODE_131K, B=2, N=8192, Hq=8, Hkv=2)
    q, k, v = W.make_decode(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(wl.D)
    km = oracle.block_means(kb, dt, wl.Bk)
    qm = q.float().numpy().reshape(wl.B, wl.Hq, 1, wl.D)
    kg, vg = k.cuda(), v.cuda()
    k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    kmean = T.thrift_block_means(kg, wl.Bk)
    idx_r, cnt_r = oracle.select_topk(qm, km, 1, wl.Bk, False, 0.05)
    idx_r, cnt_r = idx_r[:, :, 0], cnt_r[:, :, 0]
    for split in (1, 3, 7, 32, 128, 256):
        got = to_np(T.thrift_attn_decode(q.cuda(), kg, vg, k4, ks, v4, vs, kmean, wl.Bk, 0.05, split_blocks=split, out_dtype=torch.float32))
        want = oracle.attn_thrift_decode(qb, kb, vb, dt, idx_r, cnt_r, wl.Bk, scale, split)
        err = np.abs(got - want).max()
        _say(f"decode split_blocks={split}: max abs err {err:.3e}")
        assert err <= TOLMIX


def test_decode_variants(T, oracle):
    _say("decode bf16, group of 1, ragged partition, seqlens, fixed_k")
    wl = W.scaled(W.DECODE_131K, B=2, N=2560, Hq=4, Hkv=4, dtype="bf16")
    got, want, swaps = _decode_case(T, oracle, wl, 0.1, 16)          # 40 blocks: partitions of 16,16,8
    assert swaps == 0 and np.abs(got - want).max() <= TOLMIX
    wl = W.scaled(W.DECODE_131K, B=3, N=2048, Hq=8, Hkv=2)
    got, want, swaps = _decode_case(T, oracle, wl, 0.05, 8, seqlens=[2048, 640, 64])
    assert swaps == 0 and np.abs(got - want).max() <= TOLMIX
    got, want, swaps = _decode_case(T, oracle, wl, 0.0, 32, fixed_k=3)
    assert swaps == 0 and np.abs(got - want).max() <= TOLMIX


# ------------------------------------------------------------------ edge cases

@pytest.mark.parametrize("wl,budget", [
    (W.scaled(W.TINY, N=64), 1.0),                                  # one query block, one key block
    (W.scaled(W.TINY, N=64), 0.0),
    (_small_bf16(N=128, Hq=1, Hkv=1), 0.5),                         # Bq=128 over two key blocks, diagonal only
    (_small_bf16(N=512, Hq=16, Hkv=8, B=2), 0.1),                   # batch 2, 16 (b, kv head) units: XCD-spread mapping
    (W.scaled(W.TINY, N=1024, Hq=8, Hkv=8, B=1), 0.25),             # 8 units, group of 1, Bq=64
    (_small_bf16(N=768, Hq=6, Hkv=2), 0.05),                        # group of 3, 6 query blocks
])
def test_prefill_edge_shapes(T, oracle, wl, budget):
    _say(f"prefill edge {wl.name} B={wl.B} N={wl.N} Hq={wl.Hq} Hkv={wl.Hkv} Bq={wl.Bq} budget={budget}")
    got, want, lse, want_lse = _prefill_both(T, oracle, wl, budget)
    err = np.abs(got - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)
    assert np.abs(lse - want_lse).max() <= 1e-3


def test_prefill_padded_selection_scale_and_guards(T, oracle):
    """idx wider than needed (padding -1), explicit softmax scale, and canaries around the output."""
    wl = _small_bf16(N=1024, Hq=4, Hkv=2)
    _say("prefill with padded idx, explicit scale, guarded output")
    q, k, v, _, _ = W.make_prefill(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 0.07
    Tq = wl.N // wl.Bq
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx, cnt = oracle.select_topk(qm, km, wl.Bq, wl.Bk, True, 0.1, kmax=7)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, True, scale, _units(1, wl.Hq, Tq)).reshape(1, wl.Hq, wl.N, wl.D)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    n = wl.Hq * wl.N * wl.D
    guard = 4096
    buf = torch.full((n + 2 * guard,), 12345.0, dtype=torch.float32, device="cuda")
    out = buf[guard:guard + n].view(1, wl.Hq, wl.N, wl.D)
    T.thrift_attn_prefill(qg, kg, vg, q4, qs, k4, ks, v4, vs, torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(),
                          wl.Bq, wl.Bk, True, scale, out=out)
    torch.cuda.synchronize()
    assert torch.all(buf[:guard] == 12345.0) and torch.all(buf[guard + n:] == 12345.0)
    assert np.abs(to_np(out) - want).max() <= TOLMIX
    # the GPU selection with a wider idx gives the same lists, padded with -1
    idx_g, cnt_g = T.thrift_select_topk(T.thrift_block_means(qg, wl.Bq), T.thrift_block_means(kg, wl.Bk), wl.Bq, wl.Bk, True, 0.1, kmax=7)
    assert np.array_equal(to_np(idx_g), idx) and np.array_equal(to_np(cnt_g), cnt)


def test_select_single_row_and_offset(T, oracle):
    _say("select: one query block, decode-style offset")
    g = torch.Generator().manual_seed(9)
    qm = torch.randn(2, 4, 1, 128, generator=g)
    km = torch.randn(2, 2, 200, 128, generator=g)
    for causal, off, budget in ((False, 0, 0.05), (True, 12799, 0.05), (True, 6399, 0.3)):
        idx_r, cnt_r = oracle.select_topk(qm.numpy(), km.numpy(), 1, 64, causal, budget, q_block_offset=off)
        idx_g, cnt_g = T.thrift_select_topk(qm.cuda(), km.cuda(), 1, 64, causal, budget, q_block_offset=off)
        assert np.array_equal(to_np(idx_g)[..., :idx_r.shape[-1]], idx_r) and np.array_equal(to_np(cnt_g), cnt_r)


@pytest.mark.parametrize("Hq,Hkv,Tq,Tk,causal,off", [
    (4, 2, 9, 300, False, 0),          # 18 rows per KV head: a full workgroup of 16 rows and a ragged one; 5 chunks (a part group of 4)
    (2, 1, 20, 2048, True, 2008 * 64), # 40 rows, 32 chunks, a causal frontier that differs from row to row
    (1, 1, 5, 2100, False, 0),         # more than 2048 key blocks: the 4-row kernel with 64 key registers
    (8, 2, 3, 70, False, 0),           # fewer than 16 rows per KV head: the 4-row kernel, ragged
    (2, 2, 33, 257, True, 225 * 64)])  # one key past a staged group of 256
def test_select_topk_kernel_shapes(T, oracle, Hq, Hkv, Tq, Tk, causal, off):
    """Every instantiation of the selection kernel (rows per workgroup, key registers per lane) against the oracle,
    bit for bit, per-head and group-shared."""
    _say(f"select shapes Hq={Hq} Hkv={Hkv} Tq={Tq} Tk={Tk} causal={causal} off={off}")
    g = torch.Generator().manual_seed(1000 * Tq + Tk)
    qm = torch.randn(1, Hq, Tq, 128, generator=g)
    km = torch.randn(1, Hkv, Tk, 128, generator=g)
    for shared in (False, True):
        idx_r, cnt_r = oracle.select_topk(qm.numpy(), km.numpy(), 64, 64, causal, 0.07, q_block_offset=off, group_shared=shared)
        idx_g, cnt_g = T.thrift_select_topk(qm.cuda(), km.cuda(), 64, 64, causal, 0.07, q_block_offset=off, group_shared=shared)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(cnt_g), cnt_r)
        assert np.array_equal(to_np(idx_g)[..., :idx_r.shape[-1]], idx_r) and np.all(to_np(idx_g)[..., idx_r.shape[-1]:] == -1)


# head groups of every kernel shape: one head per wavefront (G <= 4, some wavefronts without a head at G = 3), two (G <= 8,
# some with one at G = 5, 6, 7), more (the transposed tiles: G = 12, 32)
@pytest.mark.parametrize("Hq,Hkv,B,N,split", [(32, 1, 1, 1024, 16), (4, 4, 1, 640, 64), (16, 2, 2, 1536, 4), (12, 2, 2, 1024, 8),
                                              (5, 1, 1, 1024, 16), (3, 1, 2, 1024, 3), (24, 2, 1, 1024, 8), (7, 1, 2, 1536, 5),
                                              # partitions longer than the kernel's window of cached selection words (8 x 64 blocks)
                                              (8, 2, 1, 69632, 1088), (16, 1, 1, 40960, 640), (24, 1, 1, 36864, 576),
                                              # launch order: 2048 items (two per thread of the ordering workgroup); 16384 items
                                              # (more than it sorts: natural order)
                                              (8, 2, 2, 65536, 2), (8, 8, 4, 32768, 1)])
def test_decode_edge_shapes(T, oracle, Hq, Hkv, B, N, split):
    wl = W.scaled(W.DECODE_131K, B=B, N=N, Hq=Hq, Hkv=Hkv)
    _say(f"decode edge B={B} N={N} Hq={Hq} Hkv={Hkv} split={split}")
    got, want, swaps = _decode_case(T, oracle, wl, 0.1, split)
    err = np.abs(got - want).max()
    _say(f"  max abs err {err:.3e}")
    assert swaps == 0 and err <= TOLMIX


def test_decode_is_deterministic_and_keeps_guards(T, oracle):
    wl = W.scaled(W.DECODE_131K, B=2, N=2048, Hq=8, Hkv=2)
    q, k, v = W.make_decode(wl)
    kg, vg = k.cuda(), v.cuda()
    k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    kmean = T.thrift_block_means(kg, 64)
    n = wl.B * wl.Hq * wl.D
    buf = torch.full((n + 512,), 777.0, dtype=torch.float32, device="cuda")
    out = buf[256:256 + n].view(wl.B, wl.Hq, wl.D)
    a = T.thrift_attn_decode(q.cuda(), kg, vg, k4, ks, v4, vs, kmean, 64, 0.05, split_blocks=8, out=out).clone()
    b = T.thrift_attn_decode(q.cuda(), kg, vg, k4, ks, v4, vs, kmean, 64, 0.05, split_blocks=8, out=out).clone()
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert torch.all(buf[:256] == 777.0) and torch.all(buf[256 + n:] == 777.0)


def test_decode_launch_order_is_a_permutation_heaviest_first(T, oracle):
    """The split-K workgroups take their (sequence, KV head, partition) from a list the call writes into the last array
    of its workspace: every item exactly once, by descending bytes to stage (1 per key block + 4 per block that some head
    of the group has promoted).  A list that missed an item would leave that item's partial unwritten."""
    wl = W.scaled(W.DECODE_131K, B=3, N=4096, Hq=8, Hkv=2)
    split, Tk, G = 16, wl.N // wl.Bk, wl.Hq // wl.Hkv
    q, k, v = W.make_decode(wl)
    kg, vg = k.cuda(), v.cuda()
    k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    kmean = T.thrift_block_means(kg, wl.Bk)
    sl = np.array([4096, 1500, 0], np.int32)
    nbytes = T.decode_workspace_bytes(wl.B, wl.Hq, wl.Hkv, wl.N, wl.D, wl.Bk, split)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    _, idx, cnt = T.thrift_attn_decode(q.cuda(), kg, vg, k4, ks, v4, vs, kmean, wl.Bk, 0.1, split_blocks=split,
                                       seqlens=torch.from_numpy(sl).cuda(), workspace=ws, return_selection=True)
    torch.cuda.synchronize()
    nsplit = (Tk + split - 1) // split
    items = wl.B * wl.Hkv * nsplit
    region = (4 * items + 255) // 256 * 256
    order = ws[nbytes - region:nbytes - region + 4 * items].cpu().numpy().view(np.int32)
    assert np.array_equal(np.sort(order), np.arange(items))
    idx, cnt = to_np(idx), to_np(cnt)
    weight = np.zeros(items, np.int64)
    for b in range(wl.B):
        full = min(int(sl[b]), wl.N) // wl.Bk
        for kvh in range(wl.Hkv):
            promoted = np.zeros(Tk, bool)
            for h in range(kvh * G, (kvh + 1) * G):
                promoted[idx[b, h, :cnt[b, h]]] = True
            for part in range(nsplit):
                lo, hi = min(full, part * split), min(full, (part + 1) * split)
                weight[(b * wl.Hkv + kvh) * nsplit + part] = (hi - lo) + 4 * int(promoted[lo:hi].sum())
    assert 5 * split < 1023            # every weight has a bin of its own at this partition size: the order is exact
    assert np.all(np.diff(weight[order]) <= 0)
    assert weight.max() > weight.min()


# ------------------------------------------------------------------ App. A ablation selectors
@pytest.mark.parametrize("selector", [1, 2])
def test_select_ablation_bit_exact(T, oracle, selector):
    cases = [  # B, Hq, Tq, Tk, Bq, Bk, causal, budget, fixed_k, offset
        (1, 1, 32, 32, 64, 64, True, 0.05, -1, 0),
        (2, 3, 16, 32, 128, 64, True, 0.25, -1, 0),
        (1, 2, 9, 80, 64, 64, False, 0.1, -1, 0),          # two 64-block chunks, ragged
        (1, 2, 5, 40, 64, 64, True, 0.0, 7, 3),            # fixed k, shifted causal frontier
        (1, 1, 4, 12, 64, 64, True, 0.0, -1, 0),           # empty budget
        (1, 1, 1, 2048, 1, 64, True, 0.05, -1, 131071),    # decode-shaped row over 2048 blocks
    ]
    for (B, Hq, Tq, Tk, Bq, Bk, causal, budget, fixed_k, off) in cases:
        _say(f"ablation selector {selector}: B={B} Hq={Hq} Tq={Tq} Tk={Tk} Bq={Bq} causal={causal} f={budget} k={fixed_k} off={off}")
        for seed in (0, 0x9e3779b97f4a7c15, 2 ** 64 - 1):
            idx_r, cnt_r = oracle.select_ablation(selector, seed, B, Hq, Tq, Tk, Bq, Bk, causal, budget, fixed_k, off)
            idx_g, cnt_g = T.thrift_select_ablation(selector, seed, B, Hq, Tq, Tk, Bq, Bk, causal, budget, fixed_k, off)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(cnt_g), cnt_r)
            assert np.array_equal(to_np(idx_g)[..., :idx_r.shape[-1]], idx_r) and np.all(to_np(idx_g)[..., idx_r.shape[-1]:] == -1)
            if selector == 2:
                break                                       # the seed plays no part


def test_select_ablation_guards_and_prefill(T, oracle):
    _say("ablation selector guards; random selection through the fused kernel")
    with pytest.raises(T.ThriftError) as e:
        T.thrift_select_ablation(3, 0, 1, 1, 4, 4, 64, 64, True, 0.5)
    assert e.value.code == 2
    with pytest.raises(T.ThriftError) as e:
        T.thrift_select_ablation(1, 0, 1, 1, 4, 4, 64, 64, True, 1.5)
    assert e.value.code == 4
    wl = _small_bf16(N=1024)
    Tq, Tk = wl.N // wl.Bq, wl.N // wl.Bk
    sel = oracle.select_ablation(1, 11, wl.B, wl.Hq, Tq, Tk, wl.Bq, wl.Bk, True, 0.25)
    got, want, _, _ = _prefill_both(T, oracle, wl, 0.25, force_sel=sel)
    err = np.abs(got - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= TOLMIX
    # the plan object with the selector switched on reproduces the same selection on the GPU
    q, k, v, _, _ = W.make_prefill(wl)
    plan = T.PrefillPlan(wl.B, wl.Hq, wl.Hkv, wl.N, wl.D, wl.Bq, wl.Bk, True, 0.25, q.dtype, torch.device("cuda"),
                         out_dtype=torch.float32, selector=1, seed=11)
    out = plan.run(q.cuda(), k.cuda(), v.cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(plan.idx)[..., :sel[0].shape[-1]], sel[0]) and np.array_equal(to_np(plan.cnt), sel[1])
    assert np.abs(to_np(out) - want).max() <= TOLMIX


# ------------------------------------------------------------------ chunked prefill
@pytest.mark.parametrize("wl,nq_blocks,budget,causal", [
    (_small_bf16(N=2048), 3, 0.1, True),                       # three 128-row blocks at the end of 2048 keys
    (_small_bf16(N=1024, Hq=2, Hkv=1, Bq=64), 5, 0.25, True),  # Bq = 64
    (_small_bf16(N=1024), 1, 1.0, True),                       # one block, every tile on the 16-bit path
    (_small_bf16(N=1024), 2, 0.0, True),                       # every tile on the 4-bit path
    (W.TINY, 4, 0.05, False),                                  # non-causal: the offset plays no part
])
def test_prefill_chunk(T, oracle, wl, nq_blocks, budget, causal):
    _say(f"chunked prefill {wl.name} N={wl.N} Bq={wl.Bq} chunk={nq_blocks} blocks f={budget} causal={causal}")
    q, k, v, _, _ = W.make_prefill(wl)
    Nq = nq_blocks * wl.Bq
    off = (wl.N - Nq) // wl.Bq
    qc = q[:, :, wl.N - Nq:, :].contiguous()
    qcb, dt = oracle.bits_of(qc); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(wl.D)
    qm = oracle.block_means(qcb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx, cnt = oracle.select_topk(qm, km, wl.Bq, wl.Bk, causal, budget, q_block_offset=off)
    want = oracle.attn_thrift_prefill(qcb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, causal, scale, _units(wl.B, wl.Hq, nq_blocks),
                                      q_block_offset=off).reshape(wl.B, wl.Hq, Nq, wl.D)
    qg, kg, vg = qc.cuda(), k.cuda(), v.cuda()
    # the whole pre-pass on the GPU with the same offset
    qm_g = T.thrift_block_means(qg, wl.Bq); km_g = T.thrift_block_means(kg, wl.Bk)
    idx_g, cnt_g = T.thrift_select_topk(qm_g, km_g, wl.Bq, wl.Bk, causal, budget, q_block_offset=off)
    assert np.array_equal(to_np(cnt_g), cnt) and np.array_equal(to_np(idx_g)[..., :idx.shape[-1]], idx)
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    got = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, idx_g, cnt_g, wl.Bq, wl.Bk, causal, off,
                                      out_dtype=torch.float32)
    torch.cuda.synchronize()
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)
    if causal:
        # the chunk's rows are the same rows of the full prefill, bit for bit, given the same sets
        qf = q.cuda()
        q4f, qsf = T.thrift_quantize_mxfp4(qf, 0)
        Tq = wl.N // wl.Bq
        idx_f = torch.full((wl.B, wl.Hq, Tq, idx_g.shape[-1]), -1, dtype=torch.int32, device="cuda")
        cnt_f = torch.zeros((wl.B, wl.Hq, Tq), dtype=torch.int32, device="cuda")
        idx_f[:, :, off:] = idx_g; cnt_f[:, :, off:] = cnt_g
        full = T.thrift_attn_prefill(qf, kg, vg, q4f, qsf, k4, ks, v4, vs, idx_f, cnt_f, wl.Bq, wl.Bk, True, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(full[:, :, wl.N - Nq:], got)


def test_prefill_chunk_guards(T):
    _say("chunked prefill guards")
    wl = _small_bf16(N=1024)
    q, k, v, _, _ = W.make_prefill(wl)
    qg, kg, vg = q[:, :, :256].contiguous().cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    idx = torch.full((wl.B, wl.Hq, 2, 1), -1, dtype=torch.int32, device="cuda"); cnt = torch.zeros((wl.B, wl.Hq, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(T.ThriftError) as e:     # the chunk would end after the last key
        T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, idx, cnt, 128, 64, True, 7)
    assert e.value.code == 2
    with pytest.raises(T.ThriftError) as e:
        T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, idx, cnt, 128, 64, True, -1)
    assert e.value.code == 2
    out = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, idx, cnt, 128, 64, True, 6)   # the last two blocks: fine
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()


# ------------------------------------------------------------------ group-shared selection (GQA extension)
def test_select_topk_shared_bit_exact(T, oracle):
    for wl, budget, causal, fixed_k in [(_small_bf16(N=4096, Hq=8, Hkv=2), 0.05, True, -1),
                                        (_small_bf16(N=2048, Hq=6, Hkv=2, Bq=64), 0.25, False, -1),
                                        (_small_bf16(N=5120, Hq=3, Hkv=1, Bq=64), 0.0, True, 9),     # two chunks of key blocks
                                        (_small_bf16(N=1024, Hq=4, Hkv=4), 0.1, True, -1)]:         # groups of one head
        _say(f"shared selection N={wl.N} Hq={wl.Hq} Hkv={wl.Hkv} Bq={wl.Bq} f={budget} causal={causal} k={fixed_k}")
        q, k, v, _, _ = W.make_prefill(wl)
        qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k)
        qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
        idx_r, cnt_r = oracle.select_topk(qm, km, wl.Bq, wl.Bk, causal, budget, fixed_k, group_shared=True)
        qm_g = T.thrift_block_means(q.cuda(), wl.Bq); km_g = T.thrift_block_means(k.cuda(), wl.Bk)
        idx_g, cnt_g = T.thrift_select_topk(qm_g, km_g, wl.Bq, wl.Bk, causal, budget, fixed_k, group_shared=True)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(cnt_g), cnt_r)
        assert np.array_equal(to_np(idx_g)[..., :idx_r.shape[-1]], idx_r) and np.all(to_np(idx_g)[..., idx_r.shape[-1]:] == -1)
        G = wl.Hq // wl.Hkv
        ig = to_np(idx_g).reshape(wl.B, wl.Hkv, G, *idx_g.shape[2:])
        assert all(np.array_equal(ig[:, :, 0], ig[:, :, g]) for g in range(G))        # one set per group


@pytest.mark.parametrize("budget", [0.05, 0.25])
def test_decode_shared_selection(T, oracle, budget):
    wl = W.scaled(W.DECODE_131K, B=2, N=4096, Hq=8, Hkv=2)
    _say(f"decode with group-shared selection B=2 N=4096 budget={budget}")
    q, k, v = W.make_decode(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    B, Hq, Tk = wl.B, wl.Hq, wl.N // wl.Bk
    km = oracle.block_means(kb, dt, wl.Bk)
    qm = q.float().numpy().reshape(B, Hq, 1, wl.D)
    idx_r, cnt_r = oracle.select_topk(qm, km, 1, wl.Bk, False, budget, group_shared=True)
    idx_r, cnt_r = idx_r[:, :, 0], cnt_r[:, :, 0]
    want = oracle.attn_thrift_decode(qb, kb, vb, dt, idx_r, cnt_r, wl.Bk, 1 / math.sqrt(wl.D), 16)
    kg, vg = k.cuda(), v.cuda()
    k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    kmean = T.thrift_block_means(kg, wl.Bk)
    got, idx_g, cnt_g = T.thrift_attn_decode(q.cuda(), kg, vg, k4, ks, v4, vs, kmean, wl.Bk, budget, -1, 16,
                                             out_dtype=torch.float32, return_selection=True, group_shared=True)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(cnt_g), cnt_r) and np.array_equal(to_np(idx_g)[..., :idx_r.shape[-1]], idx_r)
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= TOLMIX


# ------------------------------------------------------------------ tile order of Sec. 3.3 (4-bit blocks first)
@pytest.mark.parametrize("wl,budget,causal", [
    (W.TINY, 0.05, True),
    (_small_bf16(N=2048), 0.25, True),
    (_small_bf16(N=1024, Hq=2, Hkv=1, Bq=64), 0.5, True),
    (_small_bf16(N=1024), 1.0, True),                       # no 4-bit block at all
    (_small_bf16(N=1024), 0.0, True),                       # no promoted block at all
    (_small_bf16(N=1024), 0.1, False),
])
def test_prefill_two_phase_order(T, oracle, wl, budget, causal):
    _say(f"two-phase tile order {wl.name} N={wl.N} Bq={wl.Bq} f={budget} causal={causal}")
    q, k, v, _, _ = W.make_prefill(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(wl.D)
    Tq = wl.N // wl.Bq
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx, cnt = oracle.select_topk(qm, km, wl.Bq, wl.Bk, causal, budget)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, causal, scale, _units(wl.B, wl.Hq, Tq),
                                      tile_order=1).reshape(wl.B, wl.Hq, wl.N, wl.D)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    ig, cg = torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda()
    got = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, ig, cg, wl.Bq, wl.Bk, causal, 0,
                                      out_dtype=torch.float32, tile_order=1)
    torch.cuda.synchronize()
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)
    if budget in (0.0, 1.0):                                # a single phase: the same arithmetic as the ascending walk
        asc = T.thrift_attn_prefill(qg, kg, vg, q4, qs, k4, ks, v4, vs, ig, cg, wl.Bq, wl.Bk, causal, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(asc, got)
    # the same order from the persistent launch (items taken from a device counter): the same bits, twice in a row
    for _ in range(2):
        pers = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, ig, cg, wl.Bq, wl.Bk, causal, 0,
                                           out_dtype=torch.float32, tile_order=4)
        torch.cuda.synchronize()
        assert torch.equal(pers, got)
    with pytest.raises(T.ThriftError) as e:
        T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, ig, cg, wl.Bq, wl.Bk, causal, 0, tile_order=5)
    assert e.value.code == 2


# ------------------------------------------------------------------ the two schedules of the ascending walk
@pytest.mark.parametrize("wl,N,budget,causal", [
    (_small_bf16(N=2048), 2048, 0.25, True),
    (_small_bf16(N=1024), 1024, 1.0, True),                  # promoted blocks only: both slots carry 16-bit tiles
    (_small_bf16(N=1024), 1024, 0.0, True),
    (_small_bf16(N=1024, Hq=6, Hkv=2), 1000, 0.3, True),    # short last blocks
    (_small_bf16(N=1024), 1024, 0.5, False),
    (W.scaled(W.TINY, N=1024, Hq=2, Hkv=1, Bq=128), 1024, 0.4, True),   # fp16
    (_small_bf16(N=128, Hq=1, Hkv=1), 128, 0.5, True),       # one query block over two key blocks
    (_small_bf16(N=128, Hq=1, Hkv=1), 65, 1.0, True),
])
def test_prefill_schedules_agree_bit_for_bit(T, oracle, wl, N, budget, causal):
    """tile_order 2 (three workgroups per CU, promoted tiles half a step ahead) and 3 (two workgroups per CU, every
    block a whole step ahead) run the same arithmetic in the same order: equal bits, and parity with the oracle."""
    _say(f"schedules {wl.name} N={N} f={budget} causal={causal}")
    q, k, v, _, _ = W.make_prefill(wl)
    q, k, v = q[:, :, :N].contiguous(), k[:, :, :N].contiguous(), v[:, :, :N].contiguous()
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    Tq = -(-N // wl.Bq)
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx, cnt = oracle.select_topk(qm, km, wl.Bq, wl.Bk, causal, budget)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, causal, 1 / math.sqrt(wl.D),
                                      _units(wl.B, wl.Hq, Tq)).reshape(wl.B, wl.Hq, Tq * wl.Bq, wl.D)[:, :, :N]
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    if idx.shape[-1] == 0:
        idx = np.full(idx.shape[:-1] + (1,), -1, np.int32)
    ig, cg = torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda()
    outs = [T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, ig, cg, wl.Bq, wl.Bk, causal, 0,
                                        out_dtype=torch.float32, tile_order=order) for order in (0, 2, 3)]
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[1], outs[2])
    err = np.abs(to_np(outs[2]) - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)


# ------------------------------------------------------------------ lengths that are not multiples of the blocks
@pytest.mark.parametrize("N", [200, 333, 95, 33, 1])
def test_ragged_means_and_quantiser(T, oracle, N):
    _say(f"ragged pre-pass N={N}")
    wl = _small_bf16(N=512, Hq=2, Hkv=2)
    q, k, v, _, _ = W.make_prefill(wl)
    for t in (q[:, :, :N].contiguous(), v[:, :, :N].contiguous()):
        bits, dt = oracle.bits_of(t)
        for block in (64, 128, 96):
            got = to_np(T.thrift_block_means(t.cuda(), block))
            want = oracle.block_means(bits, dt, block)
            assert got.shape == want.shape and np.array_equal(got.view(np.uint32), want.view(np.uint32))
        want_c, want_s = oracle.quantize_mxfp4(bits, dt, 0)
        codes, scales = T.thrift_quantize_mxfp4(t.cuda(), 0)
        assert np.array_equal(unpack_axis0(to_np(codes)), want_c) and np.array_equal(to_np(scales), want_s)
        want_c, want_s = oracle.quantize_mxfp4(bits, dt, 1)
        codes, scales = T.thrift_quantize_mxfp4(t.cuda(), 1)
        got_c = unpack_axis1(to_np(codes))                       # [B,H,64*ceil(N/64),D]
        assert np.array_equal(got_c[:, :, :N], want_c) and np.all(got_c[:, :, N:] == 0)
        ng = want_s.shape[2]
        assert np.array_equal(to_np(scales)[:, :, :ng], want_s) and np.all(to_np(scales)[:, :, ng:] == 127)


@pytest.mark.parametrize("N,Bq,budget,causal,order", [
    (200, 64, 0.25, True, 0), (333, 128, 0.1, True, 0), (1000, 128, 0.05, True, 0), (97, 64, 0.5, False, 0),
    (777, 128, 1.0, True, 0), (450, 128, 0.0, True, 0), (333, 128, 0.3, True, 1), (65, 128, 0.05, True, 0),
])
def test_prefill_ragged_lengths(T, oracle, N, Bq, budget, causal, order):
    _say(f"prefill with N={N} (not a multiple of the blocks) Bq={Bq} f={budget} causal={causal} order={order}")
    wl = _small_bf16(N=1024, Hq=4, Hkv=2, Bq=Bq)
    q, k, v, _, _ = W.make_prefill(wl)
    q, k, v = q[:, :, :N].contiguous(), k[:, :, :N].contiguous(), v[:, :, :N].contiguous()
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    scale = 1 / math.sqrt(wl.D)
    Tq = -(-N // Bq)
    qm = oracle.block_means(qb, dt, Bq); km = oracle.block_means(kb, dt, 64)
    idx, cnt = oracle.select_topk(qm, km, Bq, 64, causal, budget)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, causal, scale, _units(wl.B, wl.Hq, Tq),
                                      tile_order=order).reshape(wl.B, wl.Hq, Tq * Bq, wl.D)[:, :, :N]
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    idx_g, cnt_g = T.thrift_select_topk(T.thrift_block_means(qg, Bq), T.thrift_block_means(kg, 64), Bq, 64, causal, budget)
    assert np.array_equal(to_np(cnt_g), cnt) and np.array_equal(to_np(idx_g)[..., :idx.shape[-1]], idx)
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    lse = torch.full((wl.B, wl.Hq, N), 7.0, dtype=torch.float32, device="cuda")
    res = torch.empty(wl.B, wl.Hq, N, wl.D, dtype=torch.float32, device="cuda")
    T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, idx_g, cnt_g, Bq, 64, causal, 0, out=res, lse=lse,
                                tile_order=order)
    torch.cuda.synchronize()
    err = np.abs(to_np(res) - want).max()
    _say(f"  max abs err {err:.3e}")
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)
    assert torch.isfinite(lse).all() and not (lse == 7.0).any()
    # the one-call form allocates by the same rules
    got2 = T.thrift_attention(qg, kg, vg, causal, Bq, 64, budget, out_dtype=torch.float32)
    torch.cuda.synchronize()
    if order == 0:
        assert torch.equal(got2, res)


# ------------------------------------------------------------------ dual cache: append and decode at any length

def _check_cache(T, oracle, cache, k_all, v_all, lens):
    """The cache must equal the pre-pass applied to each sequence's prefix; nothing else may have been written."""
    k16, v16 = to_np(cache.k16.view(torch.int16)), to_np(cache.v16.view(torch.int16))
    k4, ks, v4, vs, km = (to_np(x) for x in (cache.k4, cache.ks, cache.v4, cache.vs, cache.kmean))
    for b, n in enumerate(lens):
        nb = -(-n // 64)
        if n == 0:
            continue
        kb, dt = oracle.bits_of(k_all[b:b + 1, :, :n].contiguous()); vb, _ = oracle.bits_of(v_all[b:b + 1, :, :n].contiguous())
        assert np.array_equal(k16[b, :, :n].view(np.uint16), kb[0]) and np.array_equal(v16[b, :, :n].view(np.uint16), vb[0])
        want_c, want_s = oracle.quantize_mxfp4(kb, dt, 0)
        assert np.array_equal(unpack_axis0(k4[b:b + 1, :, :n]), want_c) and np.array_equal(ks[b:b + 1, :, :n], want_s)
        want_c, want_s = oracle.quantize_mxfp4(vb, dt, 1)
        got_c = unpack_axis1(v4[b:b + 1, :, :nb])
        assert np.array_equal(got_c[:, :, :n], want_c) and np.all(got_c[:, :, n:] == 0)
        ng = want_s.shape[2]
        assert np.array_equal(vs[b:b + 1, :, :ng], want_s) and np.all(vs[b:b + 1, :, ng:2 * nb] == 127)
        want_m = oracle.block_means(kb, dt, 64)
        assert np.array_equal(km[b:b + 1, :, :nb].view(np.uint32), want_m.view(np.uint32))
    return k16, v16, k4, ks, v4, vs, km


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_cache_append_equals_prepass_of_prefix(T, oracle, dtype):
    _say(f"cache append {dtype}")
    B, Hkv, Nkv = 3, 2, 512
    wl = W.scaled(W.DECODE_131K, B=B, N=Nkv, Hq=4, Hkv=Hkv, dtype=dtype)
    _, k, v = W.make_decode(wl)
    POISON = 0xFF
    cache = T.KVCache(B, Hkv, Nkv, wl.D, 64, k.dtype, "cuda", fill=POISON)
    lens = [0] * B
    # chunks and single tokens; steps that stay inside a group, cross a group, cross blocks, fill to the capacity
    steps = [(70, [70, 33, 0]), (1, None), (1, [1, 0, 1]), (96, [64, 31, 95]), (130, [130, 130, 7]), (1, None), (300, [300, 2, 1])]
    for n_max, per in steps:
        take = [n_max] * B if per is None else per
        new_k = torch.zeros(B, Hkv, n_max, wl.D, dtype=k.dtype); new_v = torch.zeros_like(new_k)
        for b in range(B):
            t = min(take[b], Nkv - lens[b])
            new_k[b, :, :t] = k[b, :, lens[b]:lens[b] + t]; new_v[b, :, :t] = v[b, :, lens[b]:lens[b] + t]
        nl = None if per is None else torch.tensor(per, dtype=torch.int32).cuda()
        cache.append(new_k.cuda(), new_v.cuda(), nl)
        lens = [min(Nkv, lens[b] + take[b]) for b in range(B)]
        assert to_np(cache.seqlens).tolist() == lens
        arrays = _check_cache(T, oracle, cache, k, v, lens)
    # what lies past each sequence's last touched block still holds the fill pattern
    k16, v16, k4, ks, v4, vs, km = arrays
    for b, n in enumerate(lens):
        nb = -(-n // 64)
        assert np.all(k16[b, :, n:].view(np.uint8) == POISON) and np.all(v16[b, :, n:].view(np.uint8) == POISON)
        assert np.all(k4[b, :, n:] == POISON) and np.all(ks[b, :, n:] == POISON)
        assert np.all(v4[b, :, nb:] == POISON) and np.all(vs[b, :, 2 * nb:] == POISON)
        assert np.all(km[b, :, nb:].view(np.uint8) == POISON)
    assert lens[0] == Nkv                                     # one sequence reached the capacity and dropped the rest


@pytest.mark.parametrize("budget,shared", [(0.05, False), (0.25, False), (1.0, False), (0.0, False), (0.1, True)])
def test_decode_at_any_length(T, oracle, budget, shared):
    """Decode over caches built by appends, lengths that leave the last key block partly filled; everything the
    appends did not write holds an all-ones byte pattern (NaN as a float of any width)."""
    lens = [2047, 641, 65, 1, 1984]
    B, Hq, Hkv, Nkv, split = len(lens), 8, 2, 2048, 16
    _say(f"decode at lengths {lens} budget={budget} shared={shared}")
    wl = W.scaled(W.DECODE_131K, B=B, N=Nkv, Hq=Hq, Hkv=Hkv)
    q, k, v = W.make_decode(wl)
    cache = T.KVCache(B, Hkv, Nkv, wl.D, 64, k.dtype, "cuda", fill=0xFF)
    nl = torch.tensor(lens, dtype=torch.int32).cuda()
    cache.append(k.cuda(), v.cuda(), nl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    qm = q.float().numpy().reshape(B, Hq, 1, wl.D)
    Tk = Nkv // 64
    kmax = max(1, oracle.row_k(Tk, budget, -1))
    idx_r = np.full((B, Hq, kmax), -1, np.int32); cnt_r = np.zeros((B, Hq), np.int32)
    scores = np.zeros((B, Hq, Tk))
    for b, n in enumerate(lens):
        km_b = oracle.block_means(np.ascontiguousarray(kb[b:b + 1, :, :n]), dt, 64)
        i_b, c_b = oracle.select_topk(qm[b:b + 1], km_b, 1, 64, False, budget, -1, group_shared=shared)
        idx_r[b, :, :i_b.shape[-1]] = i_b[0, :, 0]; cnt_r[b] = c_b[0, :, 0]
        sc = oracle.block_scores(qm[b:b + 1], km_b)[0, :, 0]
        if shared:
            sc = np.repeat(sc.reshape(Hkv, Hq // Hkv, -1).sum(1), Hq // Hkv, axis=0)
        scores[b, :, :sc.shape[-1]] = sc
    sl = np.asarray(lens, np.int32)
    want = oracle.attn_thrift_decode(qb, kb, vb, dt, idx_r, cnt_r, 64, 1 / math.sqrt(wl.D), split, seqlens=sl)
    got, idx_g, cnt_g = T.thrift_attn_decode(q.cuda(), cache.k16, cache.v16, cache.k4, cache.ks, cache.v4, cache.vs, cache.kmean,
                                             64, budget, -1, split, seqlens=cache.seqlens, out_dtype=torch.float32,
                                             return_selection=True, group_shared=shared)
    torch.cuda.synchronize()
    swaps = check_selection(to_np(idx_g), to_np(cnt_g), idx_r, cnt_r, scores)
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e} swaps {swaps}")
    assert np.isfinite(to_np(got)).all() and swaps == 0
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)
    # one more token: the appended token changes the last block's mean, its V group and the selection
    cache.append(k[:, :, :1].contiguous().cuda(), v[:, :, :1].contiguous().cuda())
    assert to_np(cache.seqlens).tolist() == [n + 1 for n in lens]


def test_decode_empty_sequence_gives_zeros(T, oracle):
    wl = W.scaled(W.DECODE_131K, B=2, N=256, Hq=4, Hkv=2)
    q, k, v = W.make_decode(wl)
    cache = T.KVCache(2, 2, 256, wl.D, 64, k.dtype, "cuda", fill=0xFF)
    cache.append(k.cuda(), v.cuda(), torch.tensor([0, 100], dtype=torch.int32).cuda())
    got = T.thrift_attn_decode(q.cuda(), cache.k16, cache.v16, cache.k4, cache.ks, cache.v4, cache.vs, cache.kmean, 64, 0.25, -1, 4,
                               seqlens=cache.seqlens, out_dtype=torch.float32)
    g = to_np(got)
    assert np.all(g[0] == 0) and np.isfinite(g[1]).all() and np.abs(g[1]).max() > 0


def test_one_call_forward_equals_the_staged_calls(T, oracle):
    """thrift_attention_forward chains the same seven launches as the staged entry points: equal bits, also for a
    length that is not a multiple of the blocks, with LSE, a reused workspace and a non-causal problem."""
    for wl, N, causal, budget in ((_small_bf16(N=1024, Hq=4, Hkv=2), 1024, True, 0.1), (_small_bf16(N=512, Hq=2, Hkv=1), 333, True, 0.25),
                                  (W.scaled(W.TINY, N=512), 512, False, 0.2)):
        _say(f"one-call forward {wl.name} N={N} causal={causal}")
        q, k, v, _, _ = W.make_prefill(wl)
        qg, kg, vg = (t[:, :, :N].contiguous().cuda() for t in (q, k, v))
        plan = T.PrefillPlan(wl.B, wl.Hq, wl.Hkv, N, wl.D, wl.Bq, wl.Bk, causal, budget, qg.dtype, "cuda", out_dtype=torch.float32)
        want = plan.run(qg, kg, vg).clone()
        lse = torch.empty(wl.B, wl.Hq, N, dtype=torch.float32, device="cuda")
        ws = torch.full((T.lib().thrift_attention_forward_workspace(wl.B, wl.Hq, wl.Hkv, N, wl.D, wl.Bq, wl.Bk, int(causal), budget, -1),),
                        0xFF, dtype=torch.uint8, device="cuda")
        for _ in range(2):                                  # the second call reuses the workspace of the first
            got = T.thrift_attention(qg, kg, vg, causal, wl.Bq, wl.Bk, budget, out_dtype=torch.float32, workspace=ws, lse=lse)
            torch.cuda.synchronize()
            assert torch.equal(got, want)
        lse_staged = torch.empty_like(lse)
        T.thrift_attn_prefill(qg, kg, vg, plan.q4, plan.qs, plan.k4, plan.ks, plan.v4, plan.vs, plan.idx, plan.cnt, wl.Bq, wl.Bk, causal,
                              out_dtype=torch.float32, lse=lse_staged)
        torch.cuda.synchronize()
        assert torch.equal(lse, lse_staged) and torch.isfinite(lse).all()
        with pytest.raises(T.ThriftError) as e:
            T.thrift_attention(qg, kg, vg, causal, wl.Bq, wl.Bk, budget, workspace=ws[: ws.numel() // 2])
        assert e.value.code == 5


# ------------------------------------------------------------------ seeded random shapes
def _random_prefill_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for t in range(n):
        Bq = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 2, 4]))
        Hkv = int(rng.choice([1, 2]))
        N = int(rng.integers(1, 1101))
        causal = bool(rng.random() < 0.75)
        budget = float(rng.choice([0.0, 0.03, 0.1, 0.3, 0.6, 1.0]))
        fixed_k = int(rng.integers(0, 5)) if rng.random() < 0.2 else -1
        order = int(rng.choice([0, 1, 2, 3]))
        dtype = "bf16" if rng.random() < 0.6 else "f16"
        cases.append((t, N, Bq, G * Hkv, Hkv, causal, budget, fixed_k, order, dtype))
    return cases


@pytest.mark.parametrize("case", _random_prefill_cases(28, 20260523), ids=lambda c: f"r{c[0]}-N{c[1]}-Bq{c[2]}-o{c[8]}")
def test_prefill_random_shapes(T, oracle, case):
    t, N, Bq, Hq, Hkv, causal, budget, fixed_k, order, dtype = case
    _say(f"random prefill {case}")
    wl = W.scaled(W.QWEN3_32K, N=1152, Hq=Hq, Hkv=Hkv, Bq=Bq, seed=100 + t, dtype=dtype)
    q, k, v, _, _ = W.make_prefill(wl)
    q, k, v = q[:, :, :N].contiguous(), k[:, :, :N].contiguous(), v[:, :, :N].contiguous()
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    Tq = -(-N // Bq)
    qm = oracle.block_means(qb, dt, Bq); km = oracle.block_means(kb, dt, 64)
    idx, cnt = oracle.select_topk(qm, km, Bq, 64, causal, budget, fixed_k)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, causal, 1 / math.sqrt(wl.D), _units(1, Hq, Tq),
                                      tile_order=1 if order == 1 else 0).reshape(1, Hq, Tq * Bq, wl.D)[:, :, :N]
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    qm_g = T.thrift_block_means(qg, Bq); km_g = T.thrift_block_means(kg, 64)
    idx_g, cnt_g = T.thrift_select_topk(qm_g, km_g, Bq, 64, causal, budget, fixed_k)
    swaps = check_selection(to_np(idx_g)[..., :idx.shape[-1]], to_np(cnt_g), idx, cnt, oracle.block_scores(qm, km))
    got = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, idx_g, cnt_g, Bq, 64, causal, 0,
                                      out_dtype=torch.float32, tile_order=order)
    torch.cuda.synchronize()
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e} swaps {swaps}")
    all16 = budget == 1.0 and fixed_k < 0
    assert swaps == 0 and np.isfinite(to_np(got)).all()
    assert err <= (TOL16 if all16 else TOLMIX)


def _random_decode_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for t in range(n):
        G = int(rng.choice([1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2]))
        B = int(rng.integers(1, 4))
        Nkv = int(rng.choice([512, 1024, 2048]))
        lens = [int(rng.integers(1, Nkv + 1)) for _ in range(B)]
        budget = float(rng.choice([0.0, 0.05, 0.2, 1.0]))
        split = int(rng.choice([4, 8, 16]))
        shared = bool(rng.random() < 0.3)
        dtype = "bf16" if rng.random() < 0.5 else "f16"
        cases.append((t, B, G * Hkv, Hkv, Nkv, tuple(lens), budget, split, shared, dtype))
    return cases


@pytest.mark.parametrize("case", _random_decode_cases(16, 8205), ids=lambda c: f"d{c[0]}-B{c[1]}-Hq{c[2]}-N{c[4]}")
def test_decode_random_shapes(T, oracle, case):
    t, B, Hq, Hkv, Nkv, lens, budget, split, shared, dtype = case
    _say(f"random decode {case}")
    wl = W.scaled(W.DECODE_131K, B=B, N=Nkv, Hq=Hq, Hkv=Hkv, seed=300 + t, dtype=dtype)
    q, k, v = W.make_decode(wl)
    cache = T.KVCache(B, Hkv, Nkv, wl.D, 64, k.dtype, "cuda", fill=0xFF)
    # two appends: a prefix, then the rest
    first = [n // 2 for n in lens]
    kg, vg = k.cuda(), v.cuda()
    cache.append(kg, vg, torch.tensor(first, dtype=torch.int32).cuda())
    rest = max(n - f for n, f in zip(lens, first))
    k2 = torch.zeros(B, Hkv, rest, wl.D, dtype=k.dtype); v2 = torch.zeros_like(k2)
    for b in range(B):
        m = lens[b] - first[b]
        k2[b, :, :m] = k[b, :, first[b]:lens[b]]; v2[b, :, :m] = v[b, :, first[b]:lens[b]]
    cache.append(k2.cuda(), v2.cuda(), torch.tensor([n - f for n, f in zip(lens, first)], dtype=torch.int32).cuda())
    assert to_np(cache.seqlens).tolist() == list(lens)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    qm = q.float().numpy().reshape(B, Hq, 1, wl.D)
    Tk = Nkv // 64
    kmax = max(1, oracle.row_k(Tk, budget, -1))
    idx_r = np.full((B, Hq, kmax), -1, np.int32); cnt_r = np.zeros((B, Hq), np.int32)
    scores = np.zeros((B, Hq, Tk))
    for b, n in enumerate(lens):
        km_b = oracle.block_means(np.ascontiguousarray(kb[b:b + 1, :, :n]), dt, 64)
        i_b, c_b = oracle.select_topk(qm[b:b + 1], km_b, 1, 64, False, budget, -1, group_shared=shared)
        idx_r[b, :, :i_b.shape[-1]] = i_b[0, :, 0]; cnt_r[b] = c_b[0, :, 0]
        sc = oracle.block_scores(qm[b:b + 1], km_b)[0, :, 0]
        if shared:
            sc = np.repeat(sc.reshape(Hkv, Hq // Hkv, -1).sum(1), Hq // Hkv, axis=0)
        scores[b, :, :sc.shape[-1]] = sc
    want = oracle.attn_thrift_decode(qb, kb, vb, dt, idx_r, cnt_r, 64, 1 / math.sqrt(wl.D), split, seqlens=np.asarray(lens, np.int32))
    got, idx_g, cnt_g = T.thrift_attn_decode(q.cuda(), cache.k16, cache.v16, cache.k4, cache.ks, cache.v4, cache.vs, cache.kmean,
                                             64, budget, -1, split, seqlens=cache.seqlens, out_dtype=torch.float32,
                                             return_selection=True, group_shared=shared)
    torch.cuda.synchronize()
    swaps = check_selection(to_np(idx_g), to_np(cnt_g), idx_r, cnt_r, scores)
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e} swaps {swaps}")
    assert swaps == 0 and np.isfinite(to_np(got)).all()
    assert err <= (TOL16 if budget == 1.0 else TOLMIX)


@pytest.mark.parametrize("order", [0, 1, 2, 3])
def test_prefill_hand_set_lists_with_ids_out_of_view(T, oracle, order):
    """Hand-set promoted lists (ascending) that also name blocks a causal row cannot see, an empty list and a list
    that promotes everything: blocks out of view are ignored in every tile order, as in the oracle."""
    wl = _small_bf16(N=1024, Hq=2, Hkv=1)
    _say(f"hand-set lists, order {order}")
    q, k, v, _, _ = W.make_prefill(wl)
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    Tq, Tk, kmax = wl.N // wl.Bq, wl.N // wl.Bk, 16
    idx = np.full((1, wl.Hq, Tq, kmax), -1, np.int32); cnt = np.zeros((1, wl.Hq, Tq), np.int32)
    for h in range(wl.Hq):
        for i in range(Tq):
            vis = min(Tk, 2 * (i + 1))
            if i % 4 == 0:
                ids = []                                                    # nothing promoted
            elif i % 4 == 1:
                ids = list(range(min(vis, kmax)))                          # the first blocks, consecutive
            elif i % 4 == 2:
                ids = sorted({0, vis - 1, vis, vis + 1, Tk - 1})           # two of them (three for the last rows) out of view
            else:
                ids = sorted({1, 2, vis - 2, vis - 1, Tk - 1} | ({5 + h} if vis > 6 else set()))
            ids = [j for j in ids if 0 <= j < Tk][:kmax]
            idx[0, h, i, :len(ids)] = ids; cnt[0, h, i] = len(ids)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, True, 1 / math.sqrt(wl.D), _units(1, wl.Hq, Tq),
                                      tile_order=1 if order == 1 else 0).reshape(1, wl.Hq, wl.N, wl.D)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    got = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(),
                                      wl.Bq, wl.Bk, True, 0, out_dtype=torch.float32, tile_order=order)
    torch.cuda.synchronize()
    err = np.abs(to_np(got) - want).max()
    _say(f"  max abs err {err:.3e}")
    assert np.isfinite(to_np(got)).all() and err <= TOLMIX


@pytest.mark.parametrize("order", [0, 1, 2, 3])
def test_prefill_malformed_list_entries_are_never_followed(T, oracle, order):
    """A list that breaks the contract (negative ids inside the count, ids past the last block, entries out of order,
    a count beyond the list length) yields unspecified numbers but must never turn into an address outside the
    tensors: the call completes, and a correct call right after it gives the right answer."""
    wl = _small_bf16(N=512, Hq=2, Hkv=1)
    q, k, v, _, _ = W.make_prefill(wl)
    Tq, kmax = wl.N // wl.Bq, 4
    idx = np.tile(np.array([-1, -5, 10_000, 2], np.int32), (1, wl.Hq, Tq, 1))
    cnt = np.full((1, wl.Hq, Tq), 9, np.int32)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    q4, qs = T.thrift_quantize_mxfp4(qg, 0); k4, ks = T.thrift_quantize_mxfp4(kg, 0); v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    _say(f"malformed lists, order {order}")
    T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(),
                                wl.Bq, wl.Bk, True, 0, out_dtype=torch.float32, tile_order=order)
    torch.cuda.synchronize()
    qb, dt = oracle.bits_of(q); kb, _ = oracle.bits_of(k); vb, _ = oracle.bits_of(v)
    qm = oracle.block_means(qb, dt, wl.Bq); km = oracle.block_means(kb, dt, wl.Bk)
    idx_r, cnt_r = oracle.select_topk(qm, km, wl.Bq, wl.Bk, True, 0.25)
    want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx_r, cnt_r, wl.Bq, wl.Bk, True, 1 / math.sqrt(wl.D), _units(1, wl.Hq, Tq),
                                      tile_order=1 if order == 1 else 0).reshape(1, wl.Hq, wl.N, wl.D)
    got = T.thrift_attn_prefill_chunk(qg, kg, vg, q4, qs, k4, ks, v4, vs, torch.from_numpy(idx_r).cuda(), torch.from_numpy(cnt_r).cuda(),
                                      wl.Bq, wl.Bk, True, 0, out_dtype=torch.float32, tile_order=order)
    torch.cuda.synchronize()
    assert np.abs(to_np(got) - want).max() <= TOLMIX


@pytest.mark.parametrize("order", [0, 1])
def test_prefill_degenerate_inputs(T, oracle, order):
    """All-zero inputs (uniform attention over zeros), and zero Q, K with constant V: every probability is exactly 1,
    its 4-bit code is exact, so the output is the constant on both paths: exactly in the oracle, up to the rounding of
    the final multiplication by 1/l on the GPU."""
    B, Hq, Hkv, N, D, Bq = 1, 2, 1, 512, 128, 128
    z = torch.zeros(B, Hq, N, D, dtype=torch.bfloat16)
    zk = torch.zeros(B, Hkv, N, D, dtype=torch.bfloat16)
    for const in (0.0, 1.0, -3.0):
        v = torch.full((B, Hkv, N, D), const, dtype=torch.bfloat16)
        got = T.thrift_attention(z.cuda(), zk.cuda(), v.cuda(), True, Bq, 64, 0.25, out_dtype=torch.float32, tile_order=order)
        torch.cuda.synchronize()
        assert torch.all((got - const).abs() <= 2e-7 * abs(const)), (const, (got - const).abs().max())
        qb, dt = oracle.bits_of(z); kb, _ = oracle.bits_of(zk); vb, _ = oracle.bits_of(v)
        qm = oracle.block_means(qb, dt, Bq); km = oracle.block_means(kb, dt, 64)
        idx, cnt = oracle.select_topk(qm, km, Bq, 64, True, 0.25)
        want = oracle.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, Bq, 64, True, 1 / math.sqrt(D), _units(B, Hq, N // Bq), tile_order=order)
        assert np.all(want == const)
        # ties everywhere: the selection takes the smallest ids, on both sides
        idx_g, cnt_g = T.thrift_select_topk(T.thrift_block_means(z.cuda(), Bq), T.thrift_block_means(zk.cuda(), 64), Bq, 64, True, 0.25)
        assert np.array_equal(to_np(idx_g)[..., :idx.shape[-1]], idx) and np.array_equal(to_np(cnt_g), cnt)


# ------------------------------------------------------------------ measurement microbenchmarks
def test_peak_probes_run_and_report_their_work(T):
    """Every thrift_peak_probe kind launches, leaves the device healthy and reports the work its launch did (the figure
    bench.py divides by the measured time)."""
    _say("peak probes")
    buf = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    grid, iters = 256 * 3 * 16, 20
    want = {T.PEAK_MFMA_MXFP4: grid * 4 * iters * 16 * 2.0 * 32 * 32 * 64, T.PEAK_MFMA_16: grid * 4 * iters * 16 * 2.0 * 32 * 32 * 16,
            T.PEAK_HBM_READ: float(((64 << 20) - 65536) // 16384 * 16384), T.PEAK_VALU_SOFTMAX: float(grid * 4 * iters),
            T.PEAK_TILE_MIX: float(grid * 4 * iters)}
    for kind, work in want.items():
        for dtype in ((torch.bfloat16, torch.float16) if kind == T.PEAK_MFMA_16 else (torch.bfloat16,)):
            got = T.thrift_peak_probe(kind, buf, iters, dtype)
            torch.cuda.synchronize()
            assert got == work, (kind, got, work)
    assert torch.all(buf[-65536 - (1 << 20):-65536] == 1)      # the HBM probe only reads; the others write at the front
