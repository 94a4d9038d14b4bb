"""Pins for the oracle's block means, block-pair scores, budget rules and TopK (CPU only)."""
import os

import numpy as np
import pytest
import torch

from paper_2605_23081_amd import metrics
from paper_2605_23081_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_block_means_against_numpy_mean(oracle):
    q, k, v, _, _ = W.make_prefill(W.scaled(W.TINY, N=512))
    for t, blk in ((q, 64), (k, 64), (k, 128)):
        bits, dt = oracle.bits_of(t)
        got = oracle.block_means(bits, dt, blk)
        want = t.double().numpy().reshape(1, 1, 512 // blk, blk, 128).mean(axis=3).astype(np.float32)
        assert np.array_equal(got, want)
    # bf16 path and several heads
    w = W.scaled(W.QWEN3_32K, N=256, Hq=4, Hkv=2)
    q, k, v, _, _ = W.make_prefill(w)
    bits, dt = oracle.bits_of(q)
    got = oracle.block_means(bits, dt, 128)
    want = q.double().numpy().reshape(1, 4, 2, 128, 128).mean(axis=3).astype(np.float32)
    assert np.array_equal(got, want)


def test_block_scores_against_einsum(oracle):
    rng = np.random.default_rng(0)
    qm = rng.standard_normal((2, 4, 5, 128)).astype(np.float32)
    km = rng.standard_normal((2, 2, 7, 128)).astype(np.float32)
    got = oracle.block_scores(qm, km)
    kme = np.repeat(km, 2, axis=1)  # query head h uses kv head h // 2
    want = np.einsum("bhid,bhjd->bhij", qm.astype(np.float64), kme.astype(np.float64))
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    # no 1/sqrt(d) and not symmetric in the operands' head mapping
    assert not np.allclose(got, want / np.sqrt(128))


def test_row_budget_rule_golden_and_edges(oracle):
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLDEN, "budget_rows_tiny.txt")) if l[0] != "#"]
    assert len(rows) == 32
    assert [oracle.row_k(v, 0.05) for v, _ in rows] == [k for _, k in rows]
    assert sum(oracle.row_k(v, 0.05) for v, _ in rows) == 44
    assert metrics.causal_tiles(2048, 64, 64) == 528
    for v in (1, 3, 20, 1000):
        assert oracle.row_k(v, 0.0) == 0           # 0 % == pure 4-bit attention
        assert oracle.row_k(v, 1.0) == v           # 100 % == all tiles 16-bit
        assert oracle.row_k(v, 1e-9) in (0, 1)
        assert oracle.row_k(v, 0.25) == max(1, -(-v // 4))
        assert oracle.row_k(v, 0.10) == max(1, -(-v // 10))  # exact ceiling, no float drift at multiples of 10
        assert oracle.row_k(v, 0.5, fixed_k=7) == min(7, v)


def test_paper_global_k_rule(oracle):
    # identity printed in App. B: sum_i min(i, k) = k n - k(k-1)/2
    for n in (1, 5, 32, 257):
        for k in range(1, n + 1):
            assert sum(min(i, k) for i in range(1, n + 1)) == k * n - k * (k - 1) // 2
    for n, f in ((32, 0.05), (512, 0.05), (2048, 0.10), (2048, 0.25), (100, 1.0)):
        k = oracle.paper_global_k(n, f)
        fr = lambda kk: (kk * n - kk * (kk - 1) / 2) / (n * (n + 1) / 2)
        assert 1 <= k <= n
        assert all(abs(fr(k) - f) <= abs(fr(kk) - f) + 1e-15 for kk in range(1, n + 1))


def test_visible_blocks_against_position_brute_force(oracle):
    for Bq, Bk, N in ((64, 64, 512), (128, 64, 1024), (64, 128, 1024), (1, 64, 256)):
        Tq, Tk = N // Bq, N // Bk
        for i in range(Tq):
            want = sum(1 for j in range(Tk) if j * Bk <= (i + 1) * Bq - 1)
            assert oracle.visible_blocks(i, Tk, Bq, Bk, True) == want
            assert oracle.visible_blocks(i, Tk, Bq, Bk, False) == Tk
    # decode: a one-token query block at the last position sees the whole cache
    assert oracle.visible_blocks(0, 2048, 1, 64, True, q_block_offset=131071) == 2048


def _topk_by_full_sort(scores_row, k):
    order = np.lexsort((np.arange(scores_row.size), -scores_row))  # score descending, then index ascending
    return np.sort(order[:k])


@pytest.mark.parametrize("causal", [True, False])
def test_topk_against_exhaustive_sort(oracle, causal):
    rng = np.random.default_rng(3)
    B, Hq, Hkv, Tq, Tk, D, Bq, Bk = 1, 4, 2, 16, 32, 128, 128, 64
    qm = rng.standard_normal((B, Hq, Tq, D)).astype(np.float32)
    km = rng.standard_normal((B, Hkv, Tk, D)).astype(np.float32)
    km[0, 0, 5] = km[0, 0, 9]   # exact duplicates -> ties resolved towards the smaller index
    km[0, 1, 2] = km[0, 1, 30]
    km[0, 1, 3] = km[0, 1, 30]
    scores = oracle.block_scores(qm, km)
    for budget in (0.0, 0.05, 0.25, 0.6, 1.0):
        idx, cnt = oracle.select_topk(qm, km, Bq, Bk, causal, budget)
        for h in range(Hq):
            for i in range(Tq):
                vis = oracle.visible_blocks(i, Tk, Bq, Bk, causal)
                k = oracle.row_k(vis, budget)
                assert cnt[0, h, i] == k
                want = _topk_by_full_sort(scores[0, h, i, :vis], k)
                assert np.array_equal(idx[0, h, i, :k], want)
                assert np.all(idx[0, h, i, k:] == -1)
                assert np.all(idx[0, h, i, :k] < vis)
    # a tie at the cut: with k = 1 and two equal best blocks the smaller index wins
    qm1 = np.zeros((1, 1, 1, D), np.float32); qm1[..., 0] = 1
    km1 = np.zeros((1, 1, 8, D), np.float32); km1[0, 0, 6, 0] = 2; km1[0, 0, 3, 0] = 2
    idx, cnt = oracle.select_topk(qm1, km1, 64, 64, False, 0.0, fixed_k=1)
    assert cnt[0, 0, 0] == 1 and idx[0, 0, 0, 0] == 3


def test_topk_rank_counting_brute_force(oracle):
    rng = np.random.default_rng(4)
    qm = rng.integers(-2, 3, (1, 1, 6, 128)).astype(np.float32)   # small integers: many exact ties
    km = rng.integers(-2, 3, (1, 1, 12, 128)).astype(np.float32)
    s = oracle.block_scores(qm, km)[0, 0]
    idx, cnt = oracle.select_topk(qm, km, 64, 64, False, 0.0, fixed_k=5)
    for i in range(6):
        rank = [sum(1 for jj in range(12) if s[i, jj] > s[i, j] or (s[i, jj] == s[i, j] and jj < j)) for j in range(12)]
        want = [j for j in range(12) if rank[j] < 5]
        assert list(idx[0, 0, i, :5]) == want


def test_planted_blocks_are_selected(oracle):
    """The heuristic's purpose (Sec. 3.2): blocks whose keys align with the mean query rank first."""
    w = W.TINY
    q, k, v, _, _ = W.make_prefill(w)
    qb, dt = oracle.bits_of(q)
    kb, _ = oracle.bits_of(k)
    qm = oracle.block_means(qb, dt, w.Bq)
    km = oracle.block_means(kb, dt, w.Bk)
    idx, cnt = oracle.select_topk(qm, km, w.Bq, w.Bk, True, 0.05)
    planted = W.planted_block_ids(w, 0, 0)
    assert cnt.sum() == 44
    for i in range(w.N // w.Bq):
        chosen = idx[0, 0, i, :cnt[0, 0, i]].tolist()
        vis_planted = [p for p in planted if p <= i]
        assert set(vis_planted[:cnt[0, 0, i]]) <= set(chosen)


def test_recovery_definition_matches_paper_table():
    fp16, fp4, thrift, pct = [float(x) for x in [l for l in open(os.path.join(GOLDEN, "paper_recovery.txt")) if l[0] != "#"][0].split()]
    assert round(100 * metrics.recovery(fp16, fp4, thrift), 1) == pct
    # error-like scores (lower is better) use the same ratio
    assert abs(metrics.recovery(0.01, 0.11, 0.02) - 0.9) < 1e-12
    # blended peak: 5 % at 2.5 PF and 95 % at 10 PF -> 8.70 PF; equal to the matched-compute 28.75 %
    assert abs(metrics.blended_peak(0.05, 2.5, 10.0) - 10.0 / (4 * 0.2875)) < 1e-12


# ---------------------------------------------------------------- App. A ablation selectors

def test_splitmix64_published_vector(oracle):
    want = [int(l) for l in open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")) if l[0] != "#"]
    assert [oracle.splitmix64_output(1234567, n + 1) for n in range(5)] == want


def test_diagonal_selector_is_the_most_recent_blocks(oracle):
    Tq, Tk, Bq, Bk = 16, 32, 128, 64
    idx, cnt = oracle.select_ablation(oracle.SELECT_DIAGONAL, 0, 1, 2, Tq, Tk, Bq, Bk, True, 0.25)
    for i in range(Tq):
        vis = 2 * (i + 1)                                  # hand count: blocks 0 .. 2i+1 are visible
        k = max(1, -(-vis // 4))
        assert cnt[0, 1, i] == k
        assert idx[0, 1, i, :k].tolist() == list(range(vis - k, vis))
        assert (idx[0, 1, i, k:] == -1).all()
    # non-causal: the tail of the whole key range; fixed k
    idx, cnt = oracle.select_ablation(oracle.SELECT_DIAGONAL, 0, 1, 1, 4, 10, 64, 64, False, 0.0, fixed_k=3)
    assert (cnt == 3).all() and (idx[0, 0, :, :3] == np.array([7, 8, 9])).all()


def test_random_selector_properties(oracle):
    B, Hq, Tq, Tk, Bq, Bk = 2, 3, 24, 24, 64, 64
    idx, cnt = oracle.select_ablation(oracle.SELECT_RANDOM, 7, B, Hq, Tq, Tk, Bq, Bk, True, 0.25)
    idx2, cnt2 = oracle.select_ablation(oracle.SELECT_RANDOM, 7, B, Hq, Tq, Tk, Bq, Bk, True, 0.25)
    idx3, _ = oracle.select_ablation(oracle.SELECT_RANDOM, 8, B, Hq, Tq, Tk, Bq, Bk, True, 0.25)
    assert np.array_equal(idx, idx2) and np.array_equal(cnt, cnt2)         # deterministic in the seed
    assert not np.array_equal(idx, idx3)                                   # and depends on it
    rows = set()
    for b in range(B):
        for h in range(Hq):
            for i in range(Tq):
                vis = i + 1
                k = oracle.row_k(vis, 0.25)
                assert cnt[b, h, i] == k
                ids = idx[b, h, i, :k].tolist()
                assert ids == sorted(set(ids)) and 0 <= ids[0] and ids[-1] < vis    # distinct, ascending, visible
                # brute force: rank the visible blocks by their published-generator keys
                rowid = (b * Hq + h) * Tq + i
                keys = [oracle.splitmix64_output(7, ((rowid << 32) | j) + 1) for j in range(vis)]
                want = sorted(sorted(range(vis), key=lambda j: (-keys[j], j))[:k])
                assert ids == want
                rows.add(tuple(ids))
    assert len(rows) > B * Hq * Tq // 2                                    # rows differ from each other


def test_random_selector_is_uniform(oracle):
    """Every visible block is promoted with probability k/vis: chi-square over many rows (non-causal, one k)."""
    B, Hq, Tq, Tk = 1, 8, 512, 16
    idx, cnt = oracle.select_ablation(oracle.SELECT_RANDOM, 123, B, Hq, Tq, Tk, 64, 64, False, 0.0, fixed_k=4)
    counts = np.bincount(idx[..., :4].ravel(), minlength=Tk).astype(np.float64)
    n = B * Hq * Tq
    expect = n * 4 / Tk
    # a single cell of a uniform 4-of-16 draw has variance n*p*(1-p); 15 degrees of freedom after the sum constraint
    chi2 = ((counts - expect) ** 2 / (expect * (1 - 4 / Tk))).sum()
    assert counts.sum() == 4 * n and chi2 < 45.0, chi2                     # P(chi2_15 > 45) < 1e-4


# ---------------------------------------------------------------- group-shared selection (GQA extension)

def test_group_shared_selection(oracle):
    rng = np.random.default_rng(11)
    B, Hq, Hkv, Tq, Tk, D = 2, 6, 2, 10, 20, 128
    qm = rng.standard_normal((B, Hq, Tq, D)).astype(np.float32)
    km = rng.standard_normal((B, Hkv, Tk, D)).astype(np.float32)
    qm[0, 0, 3] = 0; qm[0, 1, 3] = 0; qm[0, 2, 3] = 0            # a row of all-equal (zero) group scores: ties by id
    G = Hq // Hkv
    idx, cnt = oracle.select_topk(qm, km, 128, 64, True, 0.3, group_shared=True)
    per_head = oracle.block_scores(qm, km)                        # [B,Hq,Tq,Tk] fp64, pinned to numpy elsewhere
    for b in range(B):
        for g in range(Hkv):
            total = per_head[b, g * G:(g + 1) * G].sum(axis=0)    # exact here: few terms, fp64
            for i in range(Tq):
                vis = min(Tk, 2 * (i + 1))
                k = oracle.row_k(vis, 0.3)
                order = np.lexsort((np.arange(vis), -total[i, :vis]))     # descending score, ascending id
                want = sorted(order[:k].tolist())
                for h in range(g * G, (g + 1) * G):
                    assert cnt[b, h, i] == k and idx[b, h, i, :k].tolist() == want and (idx[b, h, i, k:] == -1).all()
    assert idx[0, 0, 3, :cnt[0, 0, 3]].tolist() == list(range(cnt[0, 0, 3]))       # the tie row takes the smallest ids
    # one head per group: identical to the per-head rule
    a = oracle.select_topk(qm[:, :2], km, 128, 64, True, 0.3, group_shared=True)
    b_ = oracle.select_topk(qm[:, :2], km, 128, 64, True, 0.3)
    assert np.array_equal(a[0], b_[0]) and np.array_equal(a[1], b_[1])
    # a summed score is the score of the summed query (linearity): same sets when the means are small integers (exact sums)
    qi = rng.integers(-3, 4, (1, 4, 5, D)).astype(np.float32); ki = rng.integers(-3, 4, (1, 1, 12, D)).astype(np.float32)
    s1 = oracle.select_topk(qi, ki, 64, 64, False, 0.0, fixed_k=4, group_shared=True)
    s2 = oracle.select_topk(qi.sum(axis=1, keepdims=True), ki, 64, 64, False, 0.0, fixed_k=4)
    assert all(np.array_equal(s1[0][0, h], s2[0][0, 0]) for h in range(4))
