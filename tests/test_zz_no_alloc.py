"""thrift_attn_decode_static (the entry point that allocates nothing) against thrift_attn_decode.

Two calls in a row on the library's static scratch, the second on a smaller problem, each compared with the
workspace-taking entry point on the same inputs: outputs and selections must be identical bit for bit (both
run the same kernels in the same order).  A problem whose workspace exceeds the static array is refused.
"""
import pytest
import torch

from paper_2605_23081_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    from paper_2605_23081_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return binding


def _cache(T, wl):
    q, k, v = W.make_decode(wl)
    kg, vg = k.cuda(), v.cuda()
    k4, ks = T.thrift_quantize_mxfp4(kg, 0)
    v4, vs = T.thrift_quantize_mxfp4(vg, 1)
    return q.cuda(), kg, vg, k4, ks, v4, vs, T.thrift_block_means(kg, wl.Bk)


def _both(T, wl, budget, split, seqlens=None):
    args = _cache(T, wl)
    sl = None if seqlens is None else torch.tensor(seqlens, dtype=torch.int32).cuda()
    want, idx_w, cnt_w = T.thrift_attn_decode(*args, wl.Bk, budget, -1, split, seqlens=sl, out_dtype=torch.float32,
                                              return_selection=True)
    out = torch.full_like(want, float("nan"))
    idx = torch.full_like(idx_w, -7)
    cnt = torch.full_like(cnt_w, -7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    T.thrift_attn_decode_static(*args, wl.Bk, budget, out, split_blocks=split, seqlens=sl, idx=idx, cnt=cnt)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return out, want, idx, idx_w, cnt, cnt_w


def test_static_scratch_decode_matches_workspace_decode_twice(T):
    # first call: 2 sequences x 4096 tokens; second call, right after, on the same scratch: 1 sequence x 1024 tokens
    # with a length that leaves the last block partly filled
    cases = [(W.scaled(W.DECODE_131K, B=2, N=4096, Hq=8, Hkv=2), 0.05, 16, None),
             (W.scaled(W.DECODE_131K, B=1, N=1024, Hq=8, Hkv=2, seed=5), 0.25, 8, [1000])]
    for wl, budget, split, seqlens in cases:
        print(f"decode_static B={wl.B} N={wl.N} budget={budget} split={split} seqlens={seqlens}", flush=True)
        out, want, idx, idx_w, cnt, cnt_w = _both(T, wl, budget, split, seqlens)
        assert torch.equal(cnt, cnt_w)
        assert torch.equal(idx, idx_w)
        assert torch.equal(out, want)
        assert bool(torch.isfinite(out).all())


def test_static_scratch_decode_rejects_oversized_problem(T):
    # 64 sequences x 131072 tokens would need about 85 MB of workspace: refused before anything is launched
    B, Hq, Hkv, Nkv, D, Bk = 64, 32, 8, 131072, 128, 64
    assert T.decode_workspace_bytes(B, Hq, Hkv, Nkv, D, Bk, 256) > T.DECODE_STATIC_SCRATCH_BYTES
    u8 = torch.zeros(16, dtype=torch.uint8, device="cuda")
    code = T.lib().thrift_attn_decode_static(u8.data_ptr(), T.BF16, u8.data_ptr(), u8.data_ptr(), u8.data_ptr(), u8.data_ptr(),
                                             u8.data_ptr(), u8.data_ptr(), u8.data_ptr(), None, B, Hq, Hkv, Nkv, D, Bk,
                                             0.05, -1, 256, 0.0, u8.data_ptr(), T.F32, None, None, 0, None)
    assert code == 5    # THRIFT_ERR_WORKSPACE
