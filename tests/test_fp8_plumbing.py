"""The FP8 E4M3 helpers of the workload module against the format's definition (CPU only): they feed the GPU
path its bytes and the oracle the decoded values, so a wrong table would hide behind agreeing sides."""
import numpy as np

import workloads as wl


def e4m3_value(code: int) -> float:
    """OCP FP8 E4M3 ("FN": no infinities, one NaN pattern per sign): 1 sign, 4 exponent (bias 7), 3 mantissa bits."""
    s, e, m = code >> 7, (code >> 3) & 15, code & 7
    if e == 15 and m == 7:
        return float("nan")
    v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
    return -v if s else v


def test_decode_matches_the_format_definition():
    codes = np.array([c for c in range(256) if not (c & 0x7F) == 0x7F], np.uint8)
    got = wl.widen(wl.fp8_e4m3_to_bf16_bits(codes))
    want = np.array([e4m3_value(int(c)) for c in codes])
    assert np.array_equal(got, want)
    assert want.max() == 448.0 and np.abs(want[want != 0]).min() == 2.0 ** -9


def test_encode_rounds_to_nearest_and_roundtrips():
    codes = np.array([c for c in range(256) if not (c & 0x7F) == 0x7F], np.uint8)
    vals = wl.widen(wl.fp8_e4m3_to_bf16_bits(codes)).astype(np.float32)
    back = wl.fp8_e4m3_encode(vals)
    assert np.array_equal(wl.widen(wl.fp8_e4m3_to_bf16_bits(back)), vals.astype(np.float64))
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(20000) * 100).astype(np.float32)
    x = x[np.abs(x) < 440]
    q = wl.widen(wl.fp8_e4m3_to_bf16_bits(wl.fp8_e4m3_encode(x)))
    grid = np.unique(np.abs(np.array([e4m3_value(int(c)) for c in codes])))
    nearest = grid[np.abs(grid[None, :] - np.abs(x[:, None].astype(np.float64))).argmin(axis=1)] * np.sign(x)
    tie = np.isclose(np.abs(np.abs(q) - np.abs(x)), np.abs(np.abs(nearest) - np.abs(x)))   # either neighbour at an exact tie
    assert tie.all()


def test_fp8_workload_uses_the_range():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="f", V=512, d_t=256, d_d=64)
    w8, scale = wl.w_lm_fp8(w, 3)
    assert w8.dtype == np.uint8 and w8.shape == (w.V, w.d_t)
    dec = wl.widen(wl.fp8_e4m3_to_bf16_bits(w8))
    assert 400 < np.abs(dec).max() <= 448
    ref = wl.widen(wl.w_lm(w, 3)) / scale
    assert np.abs(dec - ref).max() <= 0.0625 * np.abs(ref).max()      # 3 mantissa bits: half an ulp is 1/16 relative
