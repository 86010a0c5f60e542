"""Pins for the CPU oracle: every check here compares it with something that is
not the oracle itself -- a closed form, a library routine on a special case, an
independent formulation, or brute force on tiny inputs.  None needs a GPU."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1907_02129_amd.workloads import CONFIGS, ConvShape, make_tensors, random_small_shape, \
    f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape: ConvShape, rng, integer=False):
    if integer:
        x = rng.integers(-4, 5, size=(shape.N, shape.Hin, shape.Win, shape.C)).astype(np.float64)
        w = rng.integers(-4, 5, size=(shape.K, shape.R, shape.S, shape.C)).astype(np.float64)
    else:
        x = rng.standard_normal((shape.N, shape.Hin, shape.Win, shape.C))
        w = rng.standard_normal((shape.K, shape.R, shape.S, shape.C))
    return x, w


def _extent(i, lo, hi, d, k, s):
    return (i + lo + hi - d * (k - 1) - 1) // s + 1


# ---------------------------------------------------------------- geometry
def test_output_extents_match_hand_worked_table():
    for line in open(os.path.join(GOLDEN, "output_extents.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, h, w = line.split()
        assert oracle.out_extent(CONFIGS[name]) == (int(h), int(w)), name


def test_output_extent_matches_torch_conv_shape():
    rng = np.random.default_rng(11)
    for _ in range(50):
        s = random_small_shape(rng)
        xt = torch.zeros(1, 1, s.Hin + s.PT + s.PB, s.Win + s.PL + s.PR)
        yt = torch.nn.functional.conv2d(xt, torch.zeros(1, 1, s.R, s.S), stride=(s.SY, s.SX),
                                        dilation=(s.DY, s.DX))
        assert oracle.out_extent(s) == tuple(yt.shape[2:])


# ---------------------------------------------------------------- direct convolution
def test_hand_computed_window_sums():
    want = np.loadtxt(os.path.join(GOLDEN, "hand_window_sum.txt"))
    s = ConvShape("hand", 1, 3, 3, 1, 1, 2, 2)
    x = np.arange(1, 10, dtype=np.float64).reshape(1, 3, 3, 1)
    w = np.ones((1, 2, 2, 1))
    assert np.array_equal(oracle.conv2d(s, x, w)[0, :, :, 0], want)


def test_pointwise_conv_is_a_matmul():
    # 1x1 kernel, unit stride, no padding: out[M][K] = in[M][C] . filt[K][C]^T (abstract; section 3.2)
    rng = np.random.default_rng(1)
    s = ConvShape("pw", 2, 5, 7, 6, 4, 1, 1)
    x, w = _rand(s, rng)
    got = oracle.conv2d(s, x, w).reshape(-1, s.K)
    want = x.reshape(-1, s.C) @ w.reshape(s.K, s.C).T
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("seed", range(6))
def test_delta_filter_reproduces_shifted_strided_input(seed):
    # filt[oc0][ky0][kx0][ic0] = 1, rest 0  =>  out[..][oc0] = in[n][oy*SY+ky0*DY-PT][ox*SX+kx0*DX-PL][ic0]
    rng = np.random.default_rng(100 + seed)
    s = ConvShape("delta", 2, 9, 7, 3, 2, 3, 4, SY=1 + seed % 2, SX=1 + (seed // 2) % 3, DY=1 + (seed + 1) % 2,
                  DX=1 + seed % 3, PT=3, PL=1, PB=seed % 3, PR=2)
    Hout, Wout = oracle.out_extent(s)
    x = rng.standard_normal((s.N, s.Hin, s.Win, s.C))
    for ky0, kx0, ic0, oc0 in [(0, 0, 0, 0), (2, 3, 2, 1), (1, 2, 1, 0), (2, 0, 0, 1)]:
        w = np.zeros((s.K, s.R, s.S, s.C))
        w[oc0, ky0, kx0, ic0] = 1.0
        got = oracle.conv2d(s, x, w)
        want = np.zeros_like(got)
        for oy in range(Hout):
            for ox in range(Wout):
                iy, ix = oy * s.SY + ky0 * s.DY - s.PT, ox * s.SX + kx0 * s.DX - s.PL
                if 0 <= iy < s.Hin and 0 <= ix < s.Win:
                    want[:, oy, ox, oc0] = x[:, iy, ix, ic0]
        assert np.array_equal(got, want)


def test_padding_names_top_is_y_left_is_x():
    # Listing 1 names the pads the other way round; a 1-pixel image with PT != PL tells the readings apart.
    s = ConvShape("pad", 1, 1, 1, 1, 1, 1, 1, PT=2, PL=0, PB=0, PR=1)
    x = np.full((1, 1, 1, 1), 7.0)
    got = oracle.conv2d(s, x, np.ones((1, 1, 1, 1)))[0, :, :, 0]
    assert got.shape == (3, 2)
    assert np.array_equal(got, np.array([[0, 0], [0, 0], [7, 0]], dtype=np.float64))


@pytest.mark.parametrize("seed", range(4))
def test_all_ones_filter_gives_window_sums(seed):
    # summed-area table over the zero-padded image, one table per dilation phase
    rng = np.random.default_rng(200 + seed)
    s = ConvShape("ones", 1, 11, 13, 2, 3, 3, 2, SY=1 + seed % 2, SX=2, DY=1 + seed % 3, DX=1 + (seed + 1) % 2,
                  PT=2, PL=1, PB=1, PR=3)
    Hout, Wout = oracle.out_extent(s)
    x = rng.integers(-9, 10, size=(s.N, s.Hin, s.Win, s.C)).astype(np.float64)
    got = oracle.conv2d(s, x, np.ones((s.K, s.R, s.S, s.C)))
    chan = x.sum(axis=3)[0]
    padded = np.zeros((s.Hin + s.PT + s.PB, s.Win + s.PL + s.PR))
    padded[s.PT:s.PT + s.Hin, s.PL:s.PL + s.Win] = chan
    for oy in range(Hout):
        for ox in range(Wout):
            y0, x0 = oy * s.SY, ox * s.SX
            sub = padded[y0::s.DY, x0::s.DX]          # dilation-subsampled image anchored at the window
            sat = np.zeros((sub.shape[0] + 1, sub.shape[1] + 1))
            sat[1:, 1:] = sub.cumsum(0).cumsum(1)
            want = sat[s.R, s.S] - sat[0, s.S] - sat[s.R, 0] + sat[0, 0]
            assert np.all(got[0, oy, ox, :] == want)


def _scatter_form(s, x, w):
    """Independent formulation: loop over input pixels and push contributions to outputs."""
    Hout, Wout = _extent(s.Hin, s.PT, s.PB, s.DY, s.R, s.SY), _extent(s.Win, s.PL, s.PR, s.DX, s.S, s.SX)
    out = np.zeros((s.N, Hout, Wout, s.K))
    for iy in range(s.Hin):
        for ix in range(s.Win):
            for ky in range(s.R):
                for kx in range(s.S):
                    ny, nx = iy + s.PT - ky * s.DY, ix + s.PL - kx * s.DX
                    if ny % s.SY or nx % s.SX:
                        continue
                    oy, ox = ny // s.SY, nx // s.SX
                    if 0 <= oy < Hout and 0 <= ox < Wout:
                        out[:, oy, ox, :] += x[:, iy, ix, :] @ w[:, ky, kx, :].T
    return out


def _torch_conv(s, x, w):
    """Library routine: zero-pad explicitly, then torch's NCHW convolution in float64."""
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)
    xt = torch.nn.functional.pad(xt, (s.PL, s.PR, s.PT, s.PB))
    wt = torch.from_numpy(w).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(xt, wt, stride=(s.SY, s.SX), dilation=(s.DY, s.DX))
    return y.permute(0, 2, 3, 1).numpy()


def test_random_tiny_shapes_against_scatter_form_and_torch():
    rng = np.random.default_rng(7)
    for _ in range(200):
        s = random_small_shape(rng)
        x, w = _rand(s, rng, integer=True)       # small integers: every formulation is exact in double
        got = oracle.conv2d(s, x, w)
        assert np.array_equal(got, _scatter_form(s, x, w)), s
        assert np.array_equal(got, _torch_conv(s, x, w)), s


def test_benchmark_like_shape_against_torch():
    # a mid-sized strided / dilated / asymmetric case with real-valued data
    rng = np.random.default_rng(8)
    s = ConvShape("mid", 2, 17, 19, 16, 12, 3, 5, SY=2, SX=1, DY=1, DX=2, PT=2, PL=1, PB=0, PR=3)
    x, w = _rand(s, rng)
    np.testing.assert_allclose(oracle.conv2d(s, x, w), _torch_conv(s, x, w), rtol=1e-12, atol=1e-12)


def test_linearity_and_rank_one_filter():
    rng = np.random.default_rng(9)
    s = ConvShape("lin", 1, 8, 9, 3, 2, 3, 3, PT=1, PL=1, PB=1, PR=1)
    x, w1 = _rand(s, rng, integer=True)
    _, w2 = _rand(s, rng, integer=True)
    assert np.array_equal(oracle.conv2d(s, x, 2 * w1 - 3 * w2),
                          2 * oracle.conv2d(s, x, w1) - 3 * oracle.conv2d(s, x, w2))
    # filter = u (R) x v (S) on one channel pair: a vertical then a horizontal 1-D pass
    s1 = ConvShape("sep", 1, 8, 9, 1, 1, 3, 3)
    x = rng.integers(-5, 6, size=(1, 8, 9, 1)).astype(np.float64)
    u, v = np.array([1.0, -2.0, 3.0]), np.array([2.0, 0.0, -1.0])
    got = oracle.conv2d(s1, x, np.outer(u, v).reshape(1, 3, 3, 1))
    sv = ConvShape("v", 1, 8, 9, 1, 1, 3, 1)
    sh = ConvShape("h", 1, 6, 9, 1, 1, 1, 3)
    mid = oracle.conv2d(sv, x, u.reshape(1, 3, 1, 1))
    assert np.array_equal(got, oracle.conv2d(sh, mid, v.reshape(1, 1, 3, 1)))


def test_abs_sum_and_pixel_stride():
    rng = np.random.default_rng(10)
    s = ConvShape("abs", 1, 6, 6, 3, 2, 3, 3, PT=1, PL=1, PB=1, PR=1)
    x, w = _rand(s, rng)
    out, mag = oracle.conv2d_abs(s, x, w)
    np.testing.assert_allclose(mag, oracle.conv2d(s, np.abs(x), np.abs(w)), rtol=1e-13)
    assert np.array_equal(out, oracle.conv2d(s, x, w))
    # a 4th, unused channel in the pixel row (stride 4, C = 3) must not change anything
    x4 = np.concatenate([x, rng.standard_normal((1, 6, 6, 1))], axis=3)
    assert np.array_equal(oracle.conv2d(s, x4, w), out)


def test_bf16_widening_is_exact():
    v = np.array([1.0, -2.5, 3.140625, 1e-3, 65280.0], dtype=np.float32)
    bits = f32_to_bf16_bits(v)
    back = oracle.to_f64(bits)
    tb = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(back, tb)


# ---------------------------------------------------------------- quantised path
def test_u8i8_against_integer_matmul_and_centring_identity():
    rng = np.random.default_rng(12)
    for _ in range(40):
        s = random_small_shape(rng, dtype="u8i8")
        x, w = make_tensors(s)
        cen = oracle.conv2d_u8i8(s, x, w, 128, centred=True)
        raw = oracle.conv2d_u8i8(s, x, w, 128, centred=False)
        # independent: centred values through the float64 pin-checked routine above (exact for these sizes)
        want = _torch_conv(s, x.astype(np.float64) - 128.0, w.astype(np.float64))
        assert np.array_equal(cen.astype(np.float64), want), s
        # raw - 128 * sum of all filter weights of the channel == centred
        wsum = w.astype(np.int64).reshape(s.K, -1).sum(axis=1)
        assert np.array_equal(raw.astype(np.int64) - 128 * wsum, cen.astype(np.int64)), s


# ---------------------------------------------------------------- indirection buffer
def _valid_count(out_n, stride, ksz, dil, pad, in_n):
    return sum(1 for o in range(out_n) for k in range(ksz) if 0 <= o * stride + k * dil - pad < in_n)


@pytest.mark.parametrize("name", list(CONFIGS))
def test_indirection_counts_closed_form(name):
    s = CONFIGS[name]
    Hout, Wout = oracle.out_extent(s)
    ent = oracle.indirection(s)
    assert ent.shape == (s.N * Hout * Wout, s.R * s.S)          # size does not depend on C (section 1.1)
    vy = _valid_count(Hout, s.SY, s.R, s.DY, s.PT, s.Hin)
    vx = _valid_count(Wout, s.SX, s.S, s.DX, s.PL, s.Win)
    assert int((ent < 0).sum()) == s.N * (Hout * s.R * Wout * s.S - vy * vx)   # separable count of padding taps
    ok = ent[ent >= 0]
    assert ok.min() >= 0 and ok.max() < s.N * s.Hin * s.Win
    assert np.all(ent[ent < 0] == -1)


def test_indirection_padding_fractions_of_benchmark_shapes():
    # fractions worked out by hand from the separable count, e.g. 3x3 pad 1 on 56x56:
    # 1 - (166/168)^2 = 2.367 %
    want = {"cfg1_tiny_f32": 15.97, "cfg2_3x3_c64": 2.37, "cfg3a_3x3_s2": 2.37, "cfg3b_3x3_d2": 4.12,
            "cfg3c_5x5_asym": 1.44, "cfg4_int8_3x3": 4.71, "cfg5a_1x1": 0.0, "cfg5b_7x7_s2": 1.52}
    for name, pct in want.items():
        ent = oracle.indirection(CONFIGS[name])
        assert abs(100.0 * (ent < 0).mean() - pct) < 0.01, name


def test_indirection_pointwise_cases():
    s = ConvShape("id", 2, 5, 6, 3, 2, 1, 1)
    assert np.array_equal(oracle.indirection(s)[:, 0], np.arange(2 * 5 * 6))       # identity map
    s2 = ConvShape("sub", 2, 6, 8, 3, 2, 1, 1, SY=2, SX=3)
    grid = np.arange(2 * 6 * 8).reshape(2, 6, 8)[:, ::2, ::3].reshape(-1)          # subsampled grid
    assert np.array_equal(oracle.indirection(s2)[:, 0], grid)


def test_indirection_entries_by_brute_force():
    rng = np.random.default_rng(13)
    for _ in range(60):
        s = random_small_shape(rng)
        Hout, Wout = _extent(s.Hin, s.PT, s.PB, s.DY, s.R, s.SY), _extent(s.Win, s.PL, s.PR, s.DX, s.S, s.SX)
        ent = oracle.indirection(s).reshape(s.N, Hout, Wout, s.R, s.S)
        pix = np.arange(s.N * s.Hin * s.Win).reshape(s.N, s.Hin, s.Win)
        padded = np.full((s.N, s.Hin + s.PT + s.PB + s.DY * s.R, s.Win + s.PL + s.PR + s.DX * s.S), -1)
        padded[:, s.PT:s.PT + s.Hin, s.PL:s.PL + s.Win] = pix
        for ky in range(s.R):
            for kx in range(s.S):
                want = padded[:, ky * s.DY::s.SY, kx * s.DX::s.SX][:, :Hout, :Wout]
                assert np.array_equal(ent[:, :, :, ky, kx], want), s


def test_indirect_gemm_through_entries_equals_direct_convolution():
    # "fused im2col + GEMM" (section 2.2): walking the entries gives the convolution itself
    rng = np.random.default_rng(14)
    for _ in range(40):
        s = random_small_shape(rng)
        x, w = _rand(s, rng, integer=True)
        assert np.array_equal(oracle.indirect_gemm(s, oracle.indirection(s), x, w), oracle.conv2d(s, x, w)), s


def test_padded_channel_layout_equals_three_channel_problem():
    s4 = CONFIGS["cfg5b_7x7_s2"].with_(N=1, Hin=20, Win=22)
    x4, w4 = make_tensors(s4)
    assert not x4[..., 3].any() and not w4[..., 3].any()
    s3 = s4.with_(C=3)
    got3 = oracle.conv2d(s3, x4, np.ascontiguousarray(w4[..., :3]))    # pixel stride 4, C = 3
    assert np.array_equal(got3, oracle.conv2d(s4, x4, w4))


# ---------------------------------------------------------------- output stage (bias, ReLU, requantisation)
def test_epilogue_bias_and_relu_against_their_definitions():
    """Integer-valued data: the convolution is exact in double, so bias and ReLU can be checked exactly against
    plain numpy broadcasting on the unfused result."""
    rng = np.random.default_rng(11)
    s = ConvShape("ep", 2, 7, 6, 5, 4, 3, 2, SY=2, SX=1, PT=1, PL=0, PB=1, PR=1, dtype="f32")
    x = rng.integers(-4, 5, size=(s.N, s.Hin, s.Win, s.C)).astype(np.float32)
    w = rng.integers(-3, 4, size=(s.K, s.R, s.S, s.C)).astype(np.float32)
    bias = rng.integers(-20, 21, size=s.K).astype(np.float64)
    y = oracle.conv2d(s, x, w)
    assert np.array_equal(oracle.epilogue(y, bias, False), y + bias[None, None, None, :])
    assert np.array_equal(oracle.epilogue(y, None, True), np.maximum(y, 0.0))
    assert np.array_equal(oracle.epilogue(y, bias, True), np.maximum(y + bias, 0.0))
    assert np.array_equal(oracle.epilogue(y), y)                                   # nothing asked: nothing changes
    # a bias on one channel only moves that channel, by exactly the bias
    one = np.zeros(s.K); one[2] = 7.0
    d = oracle.epilogue(y, one) - y
    assert np.all(d[..., 2] == 7.0) and not d[..., [0, 1, 3]].any()
    # int32 accumulators
    yi = rng.integers(-1000, 1000, size=(3, 4, 5, 6)).astype(np.int32)
    bi = rng.integers(-500, 500, size=6).astype(np.int32)
    assert np.array_equal(oracle.epilogue(yi, bi, True), np.maximum(yi + bi, 0))
    assert oracle.epilogue(yi, bi, True).dtype == np.int32


def test_requantisation_rounds_to_nearest_even_in_single_precision_and_saturates():
    # hand cases: scale 0.5 makes every odd accumulator a tie
    y = np.array([0, 1, 2, 3, 4, 5, -1, -2, -3, 600, -600, 2**31 - 1, -2**31], dtype=np.int32)
    q = oracle.requantise_u8(y, 0.5, 10)
    #            0   0.5->0  1  1.5->2  2  2.5->2  -0.5->-0  -1  -1.5->-2  300->sat  -300->sat  huge  -huge
    assert q.tolist() == [10, 10, 11, 12, 12, 12, 10, 9, 8, 255, 0, 255, 0]
    # against the same formula written with numpy's float32 arithmetic (rint is ties-to-even)
    rng = np.random.default_rng(12)
    y = rng.integers(-40_000_000, 40_000_000, size=20000).astype(np.int32)         # beyond 2^24: the conversion rounds
    for scale, zp in ((1.7e-5, 128), (3.0517578125e-05, 0), (0.00390625, 255), (1.0, 3)):
        r = np.rint(y.astype(np.float32) * np.float32(scale))
        want = np.clip(np.clip(r, -1e9, 1e9).astype(np.int64) + zp, 0, 255).astype(np.uint8)
        assert np.array_equal(oracle.requantise_u8(y, scale, zp), want)
    # monotone in the accumulator, and the zero point is the code of accumulator 0
    ys = np.sort(y)
    qs = oracle.requantise_u8(ys, 1.7e-5, 128).astype(np.int32)
    assert np.all(np.diff(qs) >= 0) and oracle.requantise_u8(np.zeros(1, np.int32), 1.7e-5, 128)[0] == 128
