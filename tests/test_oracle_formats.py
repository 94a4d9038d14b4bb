"""Pins for the oracle's number formats and MXFP4 quantiser (CPU only).

Each check compares the oracle with something that is not the oracle: numpy's /
torch's own fp16 / bf16 conversions, the E2M1 value table of the OCP MX
specification (tests/golden/e2m1_values.txt), a brute-force nearest-grid search,
or properties the format fixes (idempotence, error bound, saturation).
"""
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _e2m1_table():
    tab = {}
    for line in open(os.path.join(GOLDEN, "e2m1_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        c, v = line.split()
        tab[int(c)] = float(v)
    return tab


def _all_f16_bits():
    u = np.arange(65536, dtype=np.uint16)
    f = u.view(np.float16)
    ok = np.isfinite(f)
    return u[ok]


def _all_bf16_bits():
    u = np.arange(65536, dtype=np.uint16)
    ex = (u >> 7) & 0xFF
    return u[ex != 255]


def _bf16_to_f64(u):
    return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_fp16_and_bf16_decoding_matches_numpy_and_torch(oracle):
    # block mean over a block of one token is the value itself: pins the bit decoding.
    u = _all_f16_bits()
    n = (u.size // 64) * 64
    x = u[:n].reshape(1, 1, n // 64, 64)
    got = oracle.block_means(x, oracle.F16, 1)
    want = x.view(np.float16).astype(np.float32)
    assert np.array_equal(got, want)  # (-0 sums to +0; every other pattern must decode exactly)
    ub = _all_bf16_bits()
    n = (ub.size // 64) * 64
    xb = ub[:n].reshape(1, 1, n // 64, 64)
    got = oracle.block_means(xb, oracle.BF16, 1)
    want = torch.from_numpy(xb.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert np.array_equal(got, want)


def test_round_to_dtype_matches_library_rounding(oracle):
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.standard_normal(2000), rng.standard_normal(2000) * 1e-6, rng.uniform(0, 1, 2000),
                         [0.0, 1.0, 0.5, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 65504.0, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11,
                          1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 2.0 ** -133]])
    for x in xs:
        assert oracle.round_to_dtype(x, oracle.F16) == float(np.float64(x).astype(np.float16)), x
        want = float(torch.tensor(x, dtype=torch.float64).to(torch.bfloat16).double())
        assert oracle.round_to_dtype(x, oracle.BF16) == want, x


def test_e2m1_decode_table(oracle):
    tab = _e2m1_table()
    for c, v in tab.items():
        d = oracle.lib().oracle_e2m1_decode(c)
        assert d == v and np.signbit(d) == np.signbit(v)


def _nearest_code(y, tab):
    """Brute force: closest grid value, ties to the even code, |y|>6 -> 6, sign kept."""
    mags = [tab[c] for c in range(8)]
    a = abs(y)
    best, bd = 0, None
    for c in range(8):
        d = abs(a - mags[c])
        if bd is None or d < bd or (d == bd and c % 2 == 0 and best % 2 == 1):
            best, bd = c, d
    return best | (8 if np.signbit(y) else 0)


def test_e2m1_rounding_against_brute_force_and_tie_table(oracle):
    tab = _e2m1_table()
    # scale byte 127 (max in [4,8)) so that the other elements are encoded unscaled
    pts = np.concatenate([np.linspace(-6.5, 6.5, 1041), [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -2.5, -5.0, 0.0, -0.0]])
    for chunk in np.array_split(pts, 40):
        grp = np.zeros(32)
        grp[0] = 4.0
        grp[1:1 + len(chunk)] = chunk[:31]
        codes, sb = oracle.mx_quantize_group(grp)
        assert sb == 127
        for y, c in zip(grp, codes):
            assert c == _nearest_code(y, tab), (y, c)
    # the ties of round-to-nearest-even on this grid
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    grp = np.zeros(32)
    grp[0] = 4.0
    for t, (y, want) in enumerate(ties.items()):
        grp[1 + t] = y
        grp[10 + t] = -y
    codes, _ = oracle.mx_quantize_group(grp)
    for t, (y, want) in enumerate(ties.items()):
        assert tab[int(codes[1 + t])] == want
        assert tab[int(codes[10 + t])] == -want and codes[10 + t] & 8


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_quantiser_exhaustive_lone_nonzero(oracle, fmt):
    """Every finite 16-bit pattern as the only non-zero of a group: scale = exponent - 2 (clamped),
    element = the value scaled into [4,8) -> code 4.0 or 6.0 (saturating above 6)."""
    tab = _e2m1_table()
    if fmt == "f16":
        bits = _all_f16_bits()
        vals = bits.view(np.float16).astype(np.float64)
        dt = oracle.F16
    else:
        bits = _all_bf16_bits()
        vals = _bf16_to_f64(bits)
        dt = oracle.BF16
    n = bits.size
    x = np.zeros((1, 1, n, 32), np.uint16)
    x[0, 0, :, 5] = bits
    codes, scales = oracle.quantize_mxfp4(x, dt, 0)
    assert scales.shape == (1, 1, n, 1)
    for i in range(0, n, 7):  # stride keeps the Python loop short; every exponent and mantissa class is hit
        v = vals[i]
        if v == 0:
            assert scales[0, 0, i, 0] == 127
            assert codes[0, 0, i, 5] == (8 if np.signbit(v) else 0)
            continue
        e = int(np.floor(np.log2(abs(v)))) - 2
        e = max(-127, min(127, e))
        assert scales[0, 0, i, 0] == e + 127, (v, scales[0, 0, i, 0])
        y = v / 2.0 ** e
        assert codes[0, 0, i, 5] == _nearest_code(y, tab), (v, y)
        assert np.all(codes[0, 0, i, :5] == 0) and np.all(codes[0, 0, i, 6:] == 0)


def test_quantiser_properties_random_groups(oracle):
    tab = _e2m1_table()
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((1, 2, 64, 128)) * rng.choice([1e-3, 1.0, 30.0], size=(1, 2, 64, 1))).astype(np.float16)
    for axis in (0, 1):
        codes, scales = oracle.quantize_mxfp4(x.view(np.uint16), oracle.F16, axis)
        deq = oracle.dequantize_mxfp4(codes, scales, axis)
        xf = x.astype(np.float64)
        if axis == 0:
            e = scales.astype(np.int64).repeat(32, axis=3) - 127
            amax = np.abs(xf).reshape(1, 2, 64, 4, 32).max(-1).repeat(32, axis=3)
        else:
            e = scales.astype(np.int64).repeat(32, axis=2) - 127
            amax = np.abs(xf).reshape(1, 2, 2, 32, 128).max(3).repeat(32, axis=2)
        # the group maximum lands in [4,8) after scaling (the power-of-two rule)
        ymax = amax / 2.0 ** e
        assert np.all((ymax >= 4) & (ymax < 8))
        y = xf / 2.0 ** e
        err = np.abs(deq - xf) / 2.0 ** e
        mag = np.abs(y)
        half_gap = np.where(mag <= 2, 0.25, np.where(mag <= 4, 0.5, 1.0))
        sat = mag > 6
        assert np.all(err[~sat] <= half_gap[~sat] + 1e-12)
        assert np.all(np.abs(deq[sat]) == 6 * 2.0 ** e[sat])
        assert np.all(np.sign(deq) * np.sign(xf) >= 0)
        # brute force on every element
        flat_y, flat_c = y.ravel(), codes.ravel()
        for t in range(0, flat_y.size, 13):
            assert flat_c[t] == _nearest_code(flat_y[t], tab)
        # idempotence: values already on the grid re-quantise to the same codes and scales
        deq16 = deq.astype(np.float16)
        assert np.array_equal(deq16.astype(np.float64), deq)
        codes2, scales2 = oracle.quantize_mxfp4(deq16.view(np.uint16), oracle.F16, axis)
        deq2 = oracle.dequantize_mxfp4(codes2, scales2, axis)
        assert np.array_equal(deq2, deq)


def test_axis1_groups_run_along_tokens(oracle):
    # a single large token must only change the scale of its own 32-token group, for every channel
    x = np.full((1, 1, 64, 32), 1.0, np.float16)
    x[0, 0, 40, :] = 100.0
    codes, scales = oracle.quantize_mxfp4(x.view(np.uint16), oracle.F16, 1)
    assert scales.shape == (1, 1, 2, 32)
    assert np.all(scales[0, 0, 0] == 125) and np.all(scales[0, 0, 1] == 127 + 4)
    codes0, scales0 = oracle.quantize_mxfp4(x.view(np.uint16), oracle.F16, 0)
    assert scales0.shape == (1, 1, 64, 1)
    assert scales0[0, 0, 40, 0] == 131 and scales0[0, 0, 0, 0] == 125


def test_cache_footprint_closed_form():
    # 4-bit elements + one 8-bit scale per 32 elements on top of a 16-bit cache: +26.6 %
    # (the paper's +28 % is the same count for an 8-bit scale per 16 elements: (4+8/16)/16 = 28.1 %).
    assert abs((4 + 8 / 32) / 16 - 0.265625) < 1e-12
    assert abs((4 + 8 / 16) / 16 - 0.28125) < 1e-12
    # matched-compute identity of Sec. 4.4: 5 % of tiles at full cost + 95 % at a quarter = 28.75 %
    assert abs(0.05 + 0.95 / 4 - 0.2875) < 1e-12


# ---------------------------------------------------------------- NVFP4 study variant (the paper's printed format)

def test_e4m3_rounding_against_torch(oracle):
    import torch
    rng = np.random.default_rng(21)
    xs = np.concatenate([rng.uniform(0, 460, 4000), np.exp(rng.uniform(np.log(2.0 ** -12), np.log(448.0), 4000)),
                         [0.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 448.0, 447.9, 464.0, 1.0, 1.0625, 1.1875]])
    got = np.array([oracle.e4m3_round(float(x)) for x in xs])
    ref = torch.tensor(np.minimum(xs, 448.0)).to(torch.float8_e4m3fn).to(torch.float64).numpy()   # torch does not saturate: clamp first
    assert np.array_equal(got, ref)
    assert oracle.e4m3_round(1e6) == 448.0 and oracle.e4m3_round(-3.0) == -3.0


def test_nvfp4_group_against_brute_force(oracle):
    import torch
    rng = np.random.default_rng(22)
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    for trial in range(300):
        x = rng.standard_normal(16) * np.exp(rng.uniform(-6, 6))
        if trial % 7 == 0:
            x[rng.integers(0, 16)] *= 30.0
        got = oracle.nvfp4_qdq(x)
        scale = float(torch.tensor(min(np.abs(x).max() / 6.0, 448.0)).to(torch.float8_e4m3fn).to(torch.float64))
        y = np.abs(x) / scale
        want = np.array([grid[np.argmin(np.abs(grid - min(v, 6.0)))] for v in y]) * scale * np.sign(x)
        ties = np.isin(np.minimum(y, 6.0), [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
        assert np.array_equal(got[~ties], want[~ties])
        if 2.0 ** -6 <= scale < 448.0:                        # normal E4M3 range: the scale is within 1/16 of max/6
            assert np.abs(x).max() <= 6.0 * scale * (1 + 1 / 16)
    assert np.array_equal(oracle.nvfp4_qdq(np.zeros(32)), np.zeros(32))
    # two groups are independent
    a, b = rng.standard_normal(16), 100 * rng.standard_normal(16)
    assert np.array_equal(oracle.nvfp4_qdq(np.concatenate([a, b])), np.concatenate([oracle.nvfp4_qdq(a), oracle.nvfp4_qdq(b)]))


def test_mx_nosat_group_against_brute_force(oracle):
    """The scale rule without saturation: the power-of-two scale is the smallest that keeps max|x|/scale <= 6
    (found here by scanning exponents), elements go to the nearest grid value; it coincides with the floor rule
    unless the group's maximum falls in (6,8) scale units, and then nothing saturates."""
    rng = np.random.default_rng(23)
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    differed = 0
    for trial in range(400):
        x = rng.standard_normal(32) * np.exp(rng.uniform(-6, 6))
        if trial % 5 == 0:
            x[rng.integers(0, 32)] = 7.0 * 2.0 ** rng.integers(-5, 5)       # a maximum the floor rule saturates
        got = oracle.mx_nosat_qdq(x)
        amax = np.abs(x).max()
        e = next(e for e in range(-140, 140) if amax / 2.0 ** e <= 6.0)
        y = np.abs(x) / 2.0 ** e
        assert y.max() <= 6.0 and (y.max() > 3.0)                           # smallest such exponent
        want = np.array([grid[np.argmin(np.abs(grid - v))] for v in y]) * 2.0 ** e * np.sign(x)
        ties = np.isin(y, [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
        assert np.array_equal(got[~ties], want[~ties])
        codes, sb = oracle.mx_quantize_group(x)
        floor_dq = np.array([oracle.lib().oracle_e2m1_decode(int(c)) for c in codes]) * 2.0 ** (sb - 127)
        if amax / 2.0 ** (sb - 127) <= 6.0:
            assert np.array_equal(got, floor_dq)
        else:
            differed += 1
            assert sb - 127 == e - 1 and np.abs(floor_dq).max() == 6.0 * 2.0 ** (e - 1) < amax
            assert abs(np.abs(got).max() - amax) <= 0.5 * 2.0 ** e
    assert differed >= 40
    assert np.array_equal(oracle.mx_nosat_qdq(np.zeros(32)), np.zeros(32))
