"""Helpers of the GPU parity tests: byte-layout decoding written from include/thrift.h, oracle plumbing."""
import numpy as np
import torch


def unpack_axis0(codes: np.ndarray) -> np.ndarray:
    """[B,H,N,D/2] packed -> [B,H,N,D] one code per byte (element 2t in the low nibble of byte t)."""
    lo, hi = codes & 0xF, codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(*codes.shape[:-1], codes.shape[-1] * 2)


def unpack_axis1(codes: np.ndarray) -> np.ndarray:
    """[B,H,N/64,D,32] packed -> [B,H,N,D]: byte t of (block, channel) holds tokens 2t (low) and 2t+1."""
    B, H, T, D, _ = codes.shape
    lo, hi = codes & 0xF, codes >> 4
    tok = np.stack([lo, hi], axis=-1).reshape(B, H, T, D, 64)      # [.., channel, token]
    return tok.transpose(0, 1, 2, 4, 3).reshape(B, H, T * 64, D)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def check_selection(idx_gpu, cnt_gpu, idx_ref, cnt_ref, scores, rel=1e-6):
    """Selected sets must be equal; a swap a (oracle only) <-> b (GPU only) is tolerated only when
    the oracle's fp64 scores of a and b differ by at most rel * max(|s_a|, |s_b|).  Returns the
    number of tolerated swaps."""
    assert np.array_equal(cnt_gpu, cnt_ref)
    swaps = 0
    flat_i = idx_gpu.reshape(-1, idx_gpu.shape[-1])
    flat_r = idx_ref.reshape(-1, idx_ref.shape[-1])
    flat_c = cnt_ref.reshape(-1)
    flat_s = scores.reshape(-1, scores.shape[-1])
    for row in range(flat_i.shape[0]):
        k = flat_c[row]
        g, r = flat_i[row, :k], flat_r[row, :k]
        assert np.all(flat_i[row, k:] == -1)
        assert np.all(np.diff(g) > 0), "ids must be strictly ascending"
        if np.array_equal(g, r):
            continue
        only_r = sorted(set(r.tolist()) - set(g.tolist()))
        only_g = sorted(set(g.tolist()) - set(r.tolist()))
        assert len(only_r) == len(only_g)
        sr = sorted(flat_s[row, only_r]); sg = sorted(flat_s[row, only_g])
        for a, b in zip(sr, sg):
            assert abs(a - b) <= rel * max(abs(a), abs(b)), (row, only_r, only_g)
            swaps += 1
    return swaps
