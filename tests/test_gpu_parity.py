"""GPU parity: the HIP path against the CPU oracle on the same seeded inputs, through the C ABI.

Tolerances (stated by the task's correctness bar):
  u8i8 : bit-exact int32
  bf16 : max |y - r| / max |r| <= 1e-2 against the double-precision oracle
  f32  : same measure <= 1e-4
and, stricter, a rounding bound that holds for any summation order of an fp32 accumulator:
  |y - r| <= 2 * n * 2^-24 * sum |x*w|   (n = R*S*C terms; bf16 products are exact in fp32).
"""
import numpy as np
import pytest
import torch

import icv_layout as layout
import plan_hooks as hooks
import oracle
from paper_1907_02129_amd import binding as icv
from paper_1907_02129_amd.workloads import CONFIGS, ConvShape, make_tensors

pytestmark = pytest.mark.gpu
TOL = {"bf16": 1e-2, "f32": 1e-4}


@pytest.fixture(scope="module", autouse=True)
def _lib():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    icv.load_library()


def _say(*a):
    print(*a, flush=True)


def check_against_oracle(s: ConvShape, got: np.ndarray, x: np.ndarray, w: np.ndarray):
    if s.dtype == "u8i8":
        want = oracle.conv2d_u8i8(s, x, w, s.zero_point, centred=True)
        assert got.dtype == np.int32
        assert np.array_equal(got, want), f"{s.name}: {(got != want).sum()} of {want.size} differ"
        return
    want, mag = oracle.conv2d_abs(s, x, w)
    err = np.abs(got.astype(np.float64) - want)
    rel = err.max() / np.abs(want).max()
    assert rel <= TOL[s.dtype], f"{s.name}: max rel err {rel:.3e}"
    n_terms = s.R * s.S * s.C
    bound = 2.0 * n_terms * 2.0 ** -24 * mag + 1e-30
    worst = (err / bound).max()
    assert worst <= 1.0, f"{s.name}: error is {worst:.2f}x the fp32 accumulation bound"


_ORACLE_CACHE = {}


def oracle_accumulators(s: ConvShape, x, w):
    """(accumulators, sum |x*w| or None) of a named benchmark shape, computed once per test session."""
    if s.name not in _ORACLE_CACHE:
        if s.dtype == "u8i8":
            _ORACLE_CACHE[s.name] = (oracle.conv2d_u8i8(s, x, w, s.zero_point, centred=True), None)
        else:
            _ORACLE_CACHE[s.name] = oracle.conv2d_abs(s, x, w)
    return _ORACLE_CACHE[s.name]


def check_against_accumulators(s: ConvShape, got: np.ndarray, want, mag):
    if s.dtype == "u8i8":
        assert got.dtype == np.int32
        assert np.array_equal(got, want), f"{s.name}: {(got != want).sum()} of {want.size} differ"
        return
    err = np.abs(got.astype(np.float64) - want)
    rel = err.max() / np.abs(want).max()
    assert rel <= TOL[s.dtype], f"{s.name}: max rel err {rel:.3e}"
    bound = 2.0 * (s.R * s.S * s.C) * 2.0 ** -24 * mag + 1e-30
    worst = (err / bound).max()
    assert worst <= 1.0, f"{s.name}: error is {worst:.2f}x the fp32 accumulation bound"


def run_indirect(s: ConvShape, x, w, plan=0, out_pixel_stride=0):
    xd, wd = icv.to_device(x), icv.to_device(w)
    buf = icv.prepare(s, wd, plan=plan, out_pixel_stride=out_pixel_stride)
    buf.output.fill_(-7)
    icv.run(buf, xd)
    torch.cuda.synchronize()
    return buf, xd


def run_im2col(s: ConvShape, buf, xd):
    ws = torch.empty(icv.im2col_bytes(buf.p), dtype=torch.uint8, device="cuda:0")
    out = torch.full_like(buf.output, -7)
    icv.conv2d_nhwc_im2col(buf.p, xd, buf.packed, ws, out)
    torch.cuda.synchronize()
    return out, ws


# ---------------------------------------------------------------- indirection buffer
@pytest.mark.parametrize("name", list(CONFIGS))
def test_indirection_matches_oracle_entry_by_entry(name):
    s = CONFIGS[name]
    _say("indirection", name)
    p = icv.make_params(s)
    Hout, Wout = icv.output_size(p)
    ind = torch.full((icv.indirection_bytes(p) // 4,), 12345, dtype=torch.int32, device="cuda:0")
    icv.setup_indirection(p, ind)
    torch.cuda.synchronize()
    got, tail = layout.logical_indirection(p, ind, s.N * Hout * Wout)
    assert np.array_equal(got, oracle.indirection(s))
    assert np.all(tail == -1)                                   # rows past M read the zero row


SMALL_IND = [
    ConvShape("i1", 2, 9, 7, 3, 2, 3, 4, SY=2, SX=1, DY=1, DX=2, PT=3, PL=1, PB=0, PR=2, dtype="f32"),
    ConvShape("i2", 3, 13, 11, 64, 8, 5, 2, SY=1, SX=3, DY=2, DX=1, PT=0, PL=2, PB=4, PR=0),
    ConvShape("i3", 1, 1, 1, 64, 8, 1, 1),
    ConvShape("i4", 5, 6, 40, 64, 8, 1, 1, SY=2, SX=3),
    ConvShape("i5", 1, 30, 30, 64, 8, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, dtype="u8i8", zero_point=128),
]


@pytest.mark.parametrize("s", SMALL_IND, ids=lambda s: s.name)
def test_indirection_small_shapes(s):
    _say("indirection", s)
    p = icv.make_params(s)
    Hout, Wout = icv.output_size(p)
    ind = torch.full((icv.indirection_bytes(p) // 4,), 12345, dtype=torch.int32, device="cuda:0")
    icv.setup_indirection(p, ind)
    torch.cuda.synchronize()
    got, tail = layout.logical_indirection(p, ind, s.N * Hout * Wout)
    assert np.array_equal(got, oracle.indirection(s))
    assert np.all(tail == -1)


# ---------------------------------------------------------------- full-size benchmark shapes, every element
@pytest.mark.parametrize("name", list(CONFIGS))
def test_benchmark_shape_matches_oracle(name):
    s = CONFIGS[name]
    _say("conv", name, icv.plan_name(icv.make_params(s)))
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    check_against_accumulators(s, buf.output.cpu().numpy(), *oracle_accumulators(s, x, w))


def _other_kernel_families():
    """(shape, plan) pairs: each benchmark shape with every kernel family that covers it besides the library's choice
    -- the families bench.py's comparison columns time at full size."""
    out = []
    try:
        icv.load_library()
    except (RuntimeError, OSError):
        return out                  # no library at collection time: the fixture below reports it
    for name, s in CONFIGS.items():
        chosen = icv.plan_name(icv.make_params(s))
        for plan, tag in ((icv.PLAN_GATHER, "gather"), (icv.PLAN_WINDOW, "window"), (icv.PLAN_FILTER_REGS, "filter_regs"),
                          (icv.PLAN_PER_IMAGE, "per_image")):
            other = icv.plan_name(icv.make_params(s, plan=plan))
            if other and (other != chosen or plan in (icv.PLAN_PER_IMAGE, icv.PLAN_GATHER)) and not other.startswith("generic") and s.N > 1:
                out.append(pytest.param(name, plan, id=f"{name}-{tag}"))
    return out


@pytest.mark.parametrize("name,plan", _other_kernel_families())
def test_benchmark_shape_with_the_other_kernel_families(name, plan):
    s = CONFIGS[name]
    _say("conv", name, icv.plan_name(icv.make_params(s, plan=plan)))
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w, plan=plan)
    check_against_accumulators(s, buf.output.cpu().numpy(), *oracle_accumulators(s, x, w))


@pytest.mark.parametrize("name", ["cfg2_3x3_c64", "cfg3a_3x3_s2", "cfg3b_3x3_d2", "cfg4_int8_3x3"])
def test_batch_256_launches_on_sampled_images(name):
    """The steady-state launches bench.py times (the benchmark shapes at batch 256, the library's own choice of kernel,
    which differs from the one at the benchmark's batch): every output element of the first, the last and two inner
    images against the oracle run on those images alone -- an image's output depends on no other image."""
    s = CONFIGS[name].with_(N=256, name=name + "_n256")
    _say("conv", s.name, icv.plan_name(icv.make_params(s)))
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    one = s.with_(N=1, name=s.name + "_one_image")
    for n in (0, 97, 200, 255):
        check_against_oracle(one, buf.output[n:n + 1].cpu().numpy(), x[n:n + 1], w)


# ---------------------------------------------------------------- small shapes: several tiles, ragged tails
def _small_shapes():
    out = []
    # bf16: ragged M (not a multiple of any tile), ragged K, C giving one / several stages per tap
    out.append(ConvShape("s_bf16_c64_k96", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=21))
    out.append(ConvShape("s_bf16_c32_k40", 1, 37, 11, 32, 40, 5, 5, PT=2, PL=2, PB=1, PR=1, seed=22))
    out.append(ConvShape("s_bf16_c96_k130", 3, 15, 17, 96, 130, 3, 2, SY=2, SX=1, DY=1, DX=2, PT=1, PL=0, PB=2, PR=3, seed=23))
    out.append(ConvShape("s_bf16_c256_k64_1x1", 2, 21, 13, 256, 64, 1, 1, seed=24))
    out.append(ConvShape("s_bf16_c128_s2", 2, 22, 26, 128, 72, 3, 3, SY=2, SX=2, PT=1, PL=1, PB=1, PR=1, seed=25))
    out.append(ConvShape("s_bf16_one_pixel", 1, 1, 1, 64, 8, 1, 1, seed=26))
    out.append(ConvShape("s_bf16_all_padding_rows", 1, 2, 2, 32, 16, 3, 3, DY=2, DX=2, PT=4, PL=4, PB=4, PR=4, seed=27))
    # int8
    out.append(ConvShape("s_i8_c64_k96", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=128, seed=31))
    out.append(ConvShape("s_i8_c192_k200", 1, 17, 9, 192, 200, 3, 3, DY=2, DX=2, PT=2, PL=2, PB=2, PR=2, dtype="u8i8", zero_point=9, seed=32))
    out.append(ConvShape("s_i8_c128_s2", 3, 14, 14, 128, 64, 5, 3, SY=2, SX=2, PT=2, PL=1, PB=2, PR=1, dtype="u8i8", zero_point=128, seed=33))
    # short pixel rows (8, 16, 32 bytes): the flattened-reduction tensor-core kernel
    out.append(ConvShape("s_bf16_c4_7x7", 2, 30, 26, 4, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=34))
    out.append(ConvShape("s_bf16_c8_3x3", 3, 13, 17, 8, 40, 3, 3, DY=2, DX=1, PT=2, PL=1, PB=2, PR=1, seed=35))
    out.append(ConvShape("s_bf16_c16_5x5", 1, 21, 9, 16, 64, 5, 5, SY=1, SX=2, PT=2, PL=2, PB=2, PR=2, seed=36))
    out.append(ConvShape("s_i8_c8_5x5", 2, 11, 23, 8, 33, 5, 5, PT=2, PL=2, PB=1, PR=1, dtype="u8i8", zero_point=131, seed=37))
    out.append(ConvShape("s_i8_c32_3x3", 1, 16, 16, 32, 64, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=128, seed=38))
    # ... with more filters than one workgroup keeps in LDS (several column groups, the last one narrower), and a
    # filter count that leaves a whole 32-column block of the 64-padded packed filter unused
    out.append(ConvShape("s_bf16_c4_7x7_k200", 2, 20, 18, 4, 200, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=39))
    out.append(ConvShape("s_i8_c8_5x5_k300", 1, 11, 23, 8, 300, 5, 5, PT=2, PL=2, PB=1, PR=1, dtype="u8i8", zero_point=128, seed=40))
    out.append(ConvShape("s_bf16_c16_3x3_k96", 2, 13, 9, 16, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=45))
    out.append(ConvShape("s_bf16_c16_1x1_k33", 2, 13, 9, 16, 33, 1, 1, seed=46))
    # vector-ALU fallback: odd channel counts; and a zero point other than 128 (tensor cores: the filter-sum term)
    out.append(ConvShape("s_f32_odd", 2, 9, 10, 5, 7, 3, 3, SY=2, SX=1, PT=1, PL=2, PB=0, PR=1, dtype="f32", dist="uniform", seed=41))
    out.append(ConvShape("s_bf16_c3", 1, 12, 12, 3, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=42))
    out.append(ConvShape("s_i8_zp7", 1, 9, 9, 64, 16, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=7, seed=43))
    out.append(ConvShape("s_i8_c5", 1, 9, 9, 5, 16, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=128, seed=44))
    return out


@pytest.mark.parametrize("s", _small_shapes(), ids=lambda s: s.name)
def test_small_shapes_match_oracle(s):
    _say("conv", s.name, icv.plan_name(icv.make_params(s)))
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    if "lowc" in icv.plan_name(buf.p):
        # the short-row kernel reads compact 16-bit entries by default; the gather plan keeps it on the int32 offsets
        assert layout.tile_records(buf.p, buf.indirection) is not None
        buf32, _ = run_indirect(s, x, w, plan=icv.PLAN_GATHER)
        assert layout.tile_records(buf32.p, buf32.indirection) is None and icv.plan_name(buf32.p) == icv.plan_name(buf.p)
        assert torch.equal(buf32.output, buf.output)


def _random_tensor_core_shapes(n=36):
    """Random shapes the tensor-core plans accept: channel counts that are multiples of 32 (bf16) / 64 (uint8),
    any kernel size, stride, dilation and (asymmetric) padding, batches whose images end inside row tiles."""
    rng = np.random.default_rng(2024)
    out = []
    while len(out) < n:
        dtype = "u8i8" if len(out) % 3 == 2 else "bf16"
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        DY, DX = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        SY, SX = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        PT, PL, PB, PR = (int(v) for v in rng.integers(0, 5, size=4))
        Hin, Win = int(rng.integers(1, 34)), int(rng.integers(1, 40))
        if Hin + PT + PB < DY * (R - 1) + 1 or Win + PL + PR < DX * (S - 1) + 1:
            continue
        C = int(rng.integers(1, 5)) * (64 if dtype == "u8i8" else 32)
        K = int(rng.integers(1, 160))
        out.append(ConvShape(f"r{len(out)}_{dtype}_{R}x{S}", int(rng.integers(1, 4)), Hin, Win, C, K, R, S, SY=SY, SX=SX,
                             DY=DY, DX=DX, PT=PT, PL=PL, PB=PB, PR=PR, dtype=dtype,
                             zero_point=128 if dtype == "u8i8" else 0, seed=1000 + len(out)))
    return out


@pytest.mark.parametrize("s", _random_tensor_core_shapes(), ids=lambda s: s.name)
def test_random_tensor_core_shapes_match_oracle(s):
    name = icv.plan_name(icv.make_params(s))
    _say("conv", s.name, name, s)
    assert name.startswith(("mfma_", "gemm_"))
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)


def _tile_cases():
    cases = [pytest.param(None, 0, id="vector_alu")]          # (row staging is a property of the tensor-core kernels)
    for i, name in enumerate(hooks.TILES):
        for algo, tag in ((0, "auto"), (icv.PLAN_GATHER, "gather"), (icv.PLAN_WINDOW, "window")):
            cases.append(pytest.param(i, algo, id=f"{name}-{tag}"))
    return cases


@pytest.mark.parametrize("tile,algo", _tile_cases())
@pytest.mark.parametrize("dtype", ["bf16", "u8i8"])
def test_every_tile(tile, dtype, algo):
    """Every tile of the tensor-core kernels (and the vector-ALU kernel) on shapes with row, column and channel tails."""
    plan = icv.PLAN_VECTOR_ALU if tile is None else algo | hooks.tile(tile)
    zp = (128, 0, 201) if dtype == "u8i8" else (0, 0, 0)      # uint8: the tensor cores take any zero point
    for s in (ConvShape("v_a", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype=dtype, zero_point=zp[0], seed=51),
              ConvShape("v_b", 1, 20, 33, 128, 200, 2, 3, SY=1, SX=2, PT=0, PL=1, PB=1, PR=1, dtype=dtype, zero_point=zp[1], seed=52),
              ConvShape("v_c", 3, 11, 9, 32 if dtype == "bf16" else 64, 33, 3, 3, DY=2, DX=1, PT=2, PL=1, PB=2, PR=1,
                        dtype=dtype, zero_point=zp[2], seed=53)):
        _say("tile", plan, icv.plan_name(icv.make_params(s, plan=plan)), s.name)
        x, w = make_tensors(s)
        try:
            buf, xd = run_indirect(s, x, w, plan=plan)
        except icv.IcvError as e:
            # the pixel-range kernel declines a tile whose range does not fit LDS -- loudly, not wrongly
            assert e.status == icv.ICV_ERR_UNSUPPORTED and algo == icv.PLAN_WINDOW, (plan, s.name, e)
            continue
        name = icv.plan_name(buf.p)
        if algo == icv.PLAN_WINDOW:
            assert "patch" in name
        if tile is not None and "generic" not in name and ("patch" in name or tile in hooks.GATHER_TILES):
            assert hooks.TILES[tile] in name, name
        check_against_oracle(s, buf.output.cpu().numpy(), x, w)


# ---------------------------------------------------------------- pixel range kept in LDS
def _patch_shapes():
    mk = ConvShape
    return [
        # several channel chunks per row (256-byte rows), tiles crossing image boundaries, K tail
        mk("p_chunks", 3, 13, 17, 128, 72, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=71),
        # stride 2 both ways, 5x5, asymmetric padding
        mk("p_s2", 2, 31, 29, 64, 64, 5, 5, SY=2, SX=2, PT=2, PL=2, PB=1, PR=1, seed=72),
        # dilation 2 x 3, different strides
        mk("p_dil", 2, 24, 40, 64, 130, 3, 3, SY=1, SX=2, DY=2, DX=3, PT=2, PL=3, PB=2, PR=3, seed=73),
        # no padding at all: the image-to-image step of the pixel range is larger than a row step
        mk("p_valid", 4, 12, 12, 32, 64, 3, 3, seed=74),
        # padding larger than the kernel reach: whole tiles of zero-row entries at the borders
        mk("p_bigpad", 1, 9, 70, 64, 32, 2, 2, PT=3, PL=3, PB=3, PR=3, seed=75),
        # one short tile only
        mk("p_tiny", 1, 5, 6, 64, 16, 2, 2, PT=1, PL=1, seed=76),
        # padded pixel stride (power of two) with fewer channels used
        mk("p_stride", 2, 14, 14, 32, 48, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=77),
        # int8, 256-byte rows
        mk("p_i8", 2, 15, 15, 256, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=128, seed=78),
        mk("p_i8_s2", 2, 21, 18, 64, 64, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=254, seed=79),
    ]


@pytest.mark.parametrize("s", _patch_shapes(), ids=lambda s: s.name)
@pytest.mark.parametrize("knobs", [0, hooks.ring(2), hooks.ring(3), hooks.ring(5), hooks.KCB64, hooks.ring(2) | hooks.KCB64,
                                   hooks.group(1), hooks.group(3) | hooks.KCB64, hooks.group(5) | hooks.ring(2), hooks.group(2),
                                   hooks.per_cu(2), hooks.per_cu(2) | hooks.KCB64 | hooks.ring(2), hooks.per_cu(2) | hooks.group(2)],
                         ids=["auto", "ring2", "ring3", "ring5", "kcb64", "ring2_kcb64", "group1", "group3_kcb64",
                              "group5_ring2", "group2", "two_per_cu", "two_per_cu_kcb64_ring2", "two_per_cu_group2"])
@pytest.mark.parametrize("tile", [0, hooks.tile(0), hooks.tile(3), hooks.tile(6)], ids=["tile_auto", "128x64", "256x64", "128x128"])
def test_pixel_range_kernel_matches_oracle(s, knobs, tile):
    # small shapes get the smallest tile when the library chooses; the larger ones are forced
    plan = icv.PLAN_WINDOW | knobs | tile
    stride = 64 if s.name == "p_stride" else 0
    x, w = make_tensors(s)
    if stride:
        xp = np.zeros(x.shape[:-1] + (stride,), dtype=x.dtype)
        xp[..., :s.C] = x
        xp[..., s.C:] = 0x7fc0                                     # NaN bit patterns in the unused channels
    else:
        xp = x
    p = icv.make_params(s, plan, in_pixel_stride=stride)
    name = icv.plan_name(p)
    if tile and not name:
        # this tile's pixel range (or its row numbers) does not fit LDS for the shape: refused as a whole, loudly
        assert icv.indirection_bytes(p) == 0 and icv.packed_filter_bytes(p) == 0
        with pytest.raises(icv.IcvError) as e:
            icv.prepare(s, icv.to_device(w), plan=plan, in_pixel_stride=stride)
        assert e.value.status == icv.ICV_ERR_UNSUPPORTED
        return
    assert "patch" in name, name
    _say("pixel-range", s.name, name, "knobs", knobs)
    buf = icv.prepare(s, icv.to_device(w), plan=plan, in_pixel_stride=stride)
    xd = icv.to_device(xp)
    icv.run(buf, xd)
    torch.cuda.synchronize()
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)


@pytest.mark.parametrize("s", _patch_shapes()[:6] + [CONFIGS["cfg3c_5x5_asym"].with_(N=2),
                                                     # the short-row kernel reads the same compact form
                                                     ConvShape("p_lowc", 2, 30, 26, 4, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=80),
                                                     ConvShape("p_lowc16", 3, 9, 11, 16, 40, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=81)],
                         ids=lambda s: s.name)
def test_range_records_match_oracle_entries(s):
    """Per row tile: smallest valid entry and pixel count up to the largest, from the oracle's entries."""
    x, w = make_tensors(s)
    buf = icv.prepare(s, icv.to_device(w), plan=icv.PLAN_WINDOW)
    torch.cuda.synchronize()
    got = layout.tile_records(buf.p, buf.indirection)
    assert got is not None
    rec, rows = got
    mr = icv.indirection_index(buf.p, 0, 1)
    want = oracle.indirection(s)
    M, T = want.shape
    esz = 1 if s.dtype == "u8i8" else 2
    cap = icv.tile_span_bound(buf.p, mr)
    for t in range(rec.shape[0]):
        blk = want[t * mr:(t + 1) * mr]                    # (rows of the tile, T) pixel index or -1
        v = blk[blk >= 0]
        first = int(v.min()) if v.size else 0
        if v.size:
            assert rec[t, 0] == first * s.C * esz and rec[t, 1] == int(v.max()) - first + 1, t
        else:
            assert tuple(rec[t, :2]) == (0, 1), t
        assert rec[t, 1] <= cap and rec[t, 2] == 0 and rec[t, 3] == 0
        # the entries as row numbers of the tile's range; the zero row (and rows past M) is one number beyond it
        got_rows = rows[t, :, :blk.shape[0]].T.astype(np.int64)
        zero = got_rows[blk < 0]
        assert np.array_equal(got_rows[blk >= 0], blk[blk >= 0] - first)
        if zero.size:
            assert zero.min() == zero.max() >= cap
        if blk.shape[0] < mr:
            assert np.all(rows[t, :, blk.shape[0]:] >= cap)


# ---------------------------------------------------------------- filter in registers, input window in an LDS ring
FREG = icv.PLAN_FILTER_REGS


def _freg_shapes():
    mk = ConvShape
    q = dict(dtype="u8i8", zero_point=128)
    return [
        # 3x3 on 128- and 256-byte rows; K of one, two, four column blocks with tails; several passes per workgroup
        mk("r_c64_k40", 2, 37, 41, 64, 40, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=301),
        mk("r_c64_k64", 3, 29, 31, 64, 64, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=302),
        mk("r_c128_k130", 2, 23, 19, 128, 130, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=303),
        mk("r_c128_k300", 1, 17, 21, 128, 300, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=304),
        mk("r_c64_k20", 2, 33, 18, 64, 20, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=305),
        # stride 2, dilation, asymmetric and oversized padding, no padding, rows that wrap images
        mk("r_s2", 2, 31, 29, 128, 72, 3, 3, SY=2, SX=2, PT=1, PL=1, PB=1, PR=1, seed=306),
        mk("r_dil", 2, 24, 40, 64, 96, 3, 3, SY=1, SX=2, DY=2, DX=3, PT=2, PL=3, PB=2, PR=3, seed=307),
        mk("r_valid", 5, 12, 12, 64, 64, 3, 3, seed=308),
        mk("r_bigpad", 2, 9, 30, 64, 32, 3, 3, PT=5, PL=4, PB=6, PR=7, seed=309),
        mk("r_bigpad_s3", 3, 7, 11, 64, 48, 3, 3, SY=3, SX=2, PT=4, PL=5, PB=5, PR=6, seed=310),
        mk("r_tiny_images", 40, 3, 3, 64, 32, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=311),
        mk("r_one_block", 1, 4, 5, 64, 16, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=312),
        mk("r_stride_pad", 2, 14, 30, 64, 48, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=313),      # run with a pixel stride of 96
        # 5x5 on 64-byte rows
        mk("r_5x5", 2, 33, 35, 32, 64, 5, 5, PT=2, PL=2, PB=1, PR=1, seed=314),
        mk("r_5x5_s2", 2, 40, 26, 32, 100, 5, 5, SY=2, SX=2, PT=2, PL=2, PB=2, PR=2, seed=315),
        # uint8 x int8
        mk("r_i8_c128", 2, 25, 27, 128, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=316, dtype="u8i8", zero_point=0),
        mk("r_i8_c256", 2, 15, 22, 256, 264, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=317, dtype="u8i8", zero_point=255),
        mk("r_i8_c128_s2", 3, 21, 18, 128, 64, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, seed=318, dtype="u8i8", zero_point=77),
        mk("r_i8_5x5", 1, 30, 30, 64, 40, 5, 5, PT=2, PL=2, PB=2, PR=2, seed=319, **q),
        # 3x3 on 64-byte rows (appended: the fused-output test below picks shapes of this list by position)
        mk("r_c32_k128", 2, 31, 27, 32, 128, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=320),
        mk("r_c32_k40_s2", 3, 26, 19, 32, 40, 3, 3, SY=2, SX=2, PT=1, PL=1, PB=1, PR=1, seed=321),
        mk("r_i8_c64", 2, 22, 33, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=322, **q),
        # fp32 tensors: 16, 32, 64 channels are 64-, 128-, 256-byte rows
        mk("r_f32_c64", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="f32", seed=323),
        mk("r_f32_c32_s2", 3, 26, 19, 32, 40, 3, 3, SY=2, SX=2, PT=1, PL=1, PB=1, PR=1, dtype="f32", seed=324),
        mk("r_f32_c16_dil", 2, 24, 40, 16, 130, 3, 3, SY=1, SX=2, DY=2, DX=3, PT=2, PL=3, PB=2, PR=3, dtype="f32", seed=325),
        mk("r_f32_5x5", 2, 33, 35, 16, 64, 5, 5, PT=2, PL=2, PB=1, PR=1, dtype="f32", seed=326),
    ]


@pytest.mark.parametrize("s", _freg_shapes(), ids=lambda s: s.name)
def test_filter_in_registers_kernel_matches_oracle(s):
    stride = 96 if s.name == "r_stride_pad" else 0
    x, w = make_tensors(s)
    xp = x
    if stride:
        xp = np.zeros(x.shape[:-1] + (stride,), dtype=x.dtype)
        xp[..., :s.C] = x
        xp[..., s.C:] = 0x7fc0                                     # NaN bit patterns in the unused channels
    p = icv.make_params(s, FREG, in_pixel_stride=stride)
    name = icv.plan_name(p)
    assert "freg" in name, name
    _say("filter-in-registers", s.name, name)
    buf = icv.prepare(s, icv.to_device(w), plan=FREG, in_pixel_stride=stride)
    buf.output.fill_(-7)
    icv.run(buf, icv.to_device(xp))
    torch.cuda.synchronize()
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    # the buffer this plan builds: entry by entry the oracle's, and every block's base record is the closed-form
    # lower end of the block's pixel range
    got, tail = layout.logical_indirection(buf.p, buf.indirection, buf.M)
    assert np.array_equal(got, oracle.indirection(s)) and np.all(tail == -1)
    rec, _ = layout.tile_records(buf.p, buf.indirection)
    esz = {"u8i8": 1, "bf16": 2, "f32": 4}[s.dtype]
    for b in range(rec.shape[0]):
        first, _last = icv.row_pixel_range(buf.p, 32 * b, min(32 * b + 31, buf.M - 1))
        assert rec[b, 2] == first and rec[b, 0] == first * (stride or s.C) * esz


def _random_freg_shapes(n=60):
    """Random problems of the kinds the filter-in-registers kernel is built for (3x3 on 64-, 128- and 256-byte rows, 5x5
    on 64-byte rows): any stride, dilation and padding, images from one pixel up, batches that end inside blocks."""
    rng = np.random.default_rng(77)
    out = []
    while len(out) < n:
        kind = len(out) % 5
        dtype = "u8i8" if kind == 3 else ("f32" if kind == 4 else "bf16")
        per_elem = {"u8i8": 2, "bf16": 1, "f32": 0.5}[dtype]       # channels per 2 bytes
        if kind == 0:
            R, C = 5, 32
        else:
            R, C = 3, int(int(rng.choice([32, 64, 128])) * per_elem)
        DY, DX = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        SY, SX = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        PT, PL, PB, PR = (int(v) for v in rng.integers(0, 6, size=4))
        Hin, Win = int(rng.integers(1, 30)), int(rng.integers(1, 45))
        if Hin + PT + PB < DY * (R - 1) + 1 or Win + PL + PR < DX * (R - 1) + 1:
            continue
        out.append(ConvShape(f"rr{len(out)}_{dtype}_{R}x{R}_c{C}", int(rng.integers(1, 7)), Hin, Win, C, int(rng.integers(1, 150)),
                             R, R, SY=SY, SX=SX, DY=DY, DX=DX, PT=PT, PL=PL, PB=PB, PR=PR, dtype=dtype,
                             zero_point=int(rng.integers(0, 256)) if dtype == "u8i8" else 0, seed=2000 + len(out)))
    return out


@pytest.mark.parametrize("s", _random_freg_shapes(), ids=lambda s: s.name)
def test_filter_in_registers_kernel_on_random_shapes(s):
    p = icv.make_params(s, FREG)
    name = icv.plan_name(p)
    if not name:
        # (a window of two passes that does not fit LDS: refused as a whole)
        assert icv.indirection_bytes(p) == 0
        return
    assert "freg" in name, name
    _say("filter-in-registers", s.name, name, s)
    x, w = make_tensors(s)
    buf = icv.prepare(s, icv.to_device(w), plan=FREG)
    buf.output.fill_(-7)
    icv.run(buf, icv.to_device(x))
    torch.cuda.synchronize()
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    got, tail = layout.logical_indirection(buf.p, buf.indirection, buf.M)
    assert np.array_equal(got, oracle.indirection(s)) and np.all(tail == -1)


@pytest.mark.parametrize("s", [_freg_shapes()[i] for i in (1, 2, 5, 13, 16, 19, 22)], ids=lambda s: s.name)
@pytest.mark.parametrize("relu,narrow", [(True, True), (False, False), (True, False)], ids=["relu_narrow", "linear_acc", "relu_acc"])
def test_filter_in_registers_kernel_with_fused_output(s, relu, narrow):
    x, w = make_tensors(s)
    if s.dtype == "u8i8":
        acc, mag = oracle.conv2d_u8i8(s, x, w, s.zero_point, centred=True), None
    else:
        acc, mag = oracle.conv2d_abs(s, x, w)
    run_fused_case(s, x, w, acc, mag, relu, narrow, plan=FREG, out_pixel_stride=s.K + 8 if narrow else 0)
    if relu and narrow:
        # the same with the batch-independent buffer (images that end inside a block store through the guarded path)
        run_fused_case(s, x, w, acc, mag, relu, narrow, plan=FREG | icv.PLAN_PER_IMAGE, out_pixel_stride=s.K + 8)


# ---------------------------------------------------------------- fp32 tensors on the matrix cores
def _f32_mfma_shapes():
    mk = lambda *a, **k: ConvShape(*a, dtype="f32", **k)
    return [
        mk("f_c64", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=401),
        mk("f_c16", 3, 17, 15, 16, 40, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=402),             # 64-byte rows, K tail
        mk("f_5x5_s2", 2, 31, 29, 32, 64, 5, 5, SY=2, SX=2, PT=2, PL=2, PB=1, PR=1, seed=403),
        mk("f_dil", 2, 24, 40, 16, 130, 3, 3, SY=1, SX=2, DY=2, DX=3, PT=2, PL=3, PB=2, PR=3, seed=404),
        mk("f_valid", 4, 12, 12, 32, 64, 3, 3, seed=405),
        mk("f_stride", 2, 14, 14, 16, 48, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=406),          # run with a pixel stride of 32
        mk("f_tiny", 1, 5, 6, 16, 16, 2, 2, PT=1, PL=1, seed=407),
    ]


@pytest.mark.parametrize("s", _f32_mfma_shapes(), ids=lambda s: s.name)
@pytest.mark.parametrize("tile", [0, icv.PLAN_WINDOW, hooks.tile(0), hooks.tile(2), hooks.tile(6)],
                         ids=["auto", "window_auto", "128x64", "256x64", "128x128"])
def test_fp32_tensors_on_the_matrix_cores(s, tile):
    """fp32 input and filter (section 3.1's precision) through 32x32x2 fp32 products: the library's choice (the
    filter-in-registers kernel where it applies), the pixel-range kernel with its own choice of tile and with each tile."""
    stride = 32 if s.name == "f_stride" else 0
    x, w = make_tensors(s)
    xp = x
    if stride:
        xp = np.full(x.shape[:-1] + (stride,), np.nan, dtype=x.dtype)     # NaN in the unused channels
        xp[..., :s.C] = x
    p = icv.make_params(s, tile, in_pixel_stride=stride)
    name = icv.plan_name(p)
    if tile == 0 or (tile != icv.PLAN_WINDOW and "patch" not in name):
        # (a forced tile whose pixel range does not fit LDS for the shape: rows are gathered per kernel element instead)
        assert name.startswith("mfma_f32"), name
    else:
        assert name.startswith("mfma_f32") and "patch" in name, name
    _say("fp32 mfma", s.name, name)
    buf = icv.prepare(s, icv.to_device(w), plan=tile, in_pixel_stride=stride)
    buf.output.fill_(-7)
    icv.run(buf, icv.to_device(xp))
    torch.cuda.synchronize()
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    if tile == 0:
        # the same problem with rows gathered per kernel element (section 2.2 as printed), in fp32 on the matrix cores too
        g = icv.prepare(s, icv.to_device(w), plan=icv.PLAN_GATHER, in_pixel_stride=stride)
        assert icv.plan_name(g.p).startswith("mfma_f32") and "patch" not in icv.plan_name(g.p)
        g.output.fill_(-7)
        icv.run(g, icv.to_device(xp))
        torch.cuda.synchronize()
        check_against_oracle(s, g.output.cpu().numpy(), x, w)


def test_fp32_pointwise_convolution_and_ablation_on_the_matrix_cores():
    """1x1 stride-1 in fp32 runs as the plain GEMM on the input; the im2col + GEMM comparison path runs in fp32 too."""
    s = ConvShape("f_1x1", 3, 7, 11, 64, 72, 1, 1, dtype="f32", seed=411)
    x, w = make_tensors(s)
    assert icv.plan_name(icv.make_params(s)).startswith("gemm_f32")
    buf, xd = run_indirect(s, x, w)
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    s = _f32_mfma_shapes()[0]
    x, w = make_tensors(s)
    buf = icv.prepare(s, icv.to_device(w), plan=icv.PLAN_GATHER)
    ws = torch.empty(icv.im2col_bytes(buf.p), dtype=torch.uint8, device="cuda:0")
    assert ws.numel() > 0
    out = torch.full_like(buf.output, -7)
    icv.conv2d_nhwc_im2col(buf.p, icv.to_device(x), buf.packed, ws, out)
    torch.cuda.synchronize()
    check_against_oracle(s, out.cpu().numpy(), x, w)


@pytest.mark.parametrize("s", _f32_mfma_shapes()[:3], ids=lambda s: s.name)
@pytest.mark.parametrize("relu,narrow", [(True, True), (False, False)], ids=["relu_narrow", "linear_acc"])
def test_fp32_tensors_on_the_matrix_cores_with_fused_output(s, relu, narrow):
    x, w = make_tensors(s)
    acc, mag = oracle.conv2d_abs(s, x, w)
    assert icv.plan_name(icv.make_params(s)).startswith("mfma_f32")
    run_fused_case(s, x, w, acc, mag, relu, narrow, out_pixel_stride=s.K + 8 if narrow else 0)


# ---------------------------------------------------------------- 1x1 stride-1: plain GEMM on the input tensor
@pytest.mark.parametrize("s", [
    ConvShape("g_exact", 2, 16, 16, 64, 64, 1, 1, seed=81),                        # M a multiple of every tile
    ConvShape("g_ragged", 3, 7, 11, 128, 72, 1, 1, seed=82),                       # M = 231: last tile mostly past M
    ConvShape("g_one_row", 1, 1, 1, 64, 200, 1, 1, seed=83),
    ConvShape("g_i8", 2, 9, 13, 256, 96, 1, 1, dtype="u8i8", zero_point=5, seed=84),
], ids=lambda s: s.name)
@pytest.mark.parametrize("pixel_stride", [0, 320])
def test_pointwise_convolution_runs_as_gemm_on_the_input(s, pixel_stride):
    x, w = make_tensors(s)
    xp = x
    if pixel_stride:
        # the tensor ends right after the last pixel's channels: reading a row past M would leave the allocation
        flat = np.full(x.shape[0] * x.shape[1] * x.shape[2] * pixel_stride, 0x7f if s.dtype == "u8i8" else 0x7fc0, dtype=x.dtype)
        v = flat.reshape(-1, pixel_stride)
        v[:, :s.C] = x.reshape(-1, s.C)
        xp = flat
    for plan in (0, icv.PLAN_GATHER):                           # dispatch to the GEMM, and the gathered path for comparison
        p = icv.make_params(s, plan, in_pixel_stride=pixel_stride)
        assert icv.plan_name(p).startswith("gemm_" if plan == 0 else "mfma_"), icv.plan_name(p)
        _say("pointwise", s.name, icv.plan_name(p), "pixel stride", pixel_stride)
        buf = icv.prepare(s, icv.to_device(w), plan=plan, in_pixel_stride=pixel_stride)
        buf.output.fill_(-7)
        icv.run(buf, icv.to_device(xp))
        torch.cuda.synchronize()
        check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    # anything that needs an indirection buffer keeps using it
    assert icv.plan_name(icv.make_params(s.with_(SY=2, SX=2))).startswith("mfma_")
    assert icv.plan_name(icv.make_params(s.with_(PT=1, PB=1))).startswith("mfma_")


# ---------------------------------------------------------------- batch-independent indirection buffer
PER_IMAGE = icv.PLAN_PER_IMAGE

PER_IMAGE_SHAPES = [
    CONFIGS["cfg1_tiny_f32"].with_(N=3),                                                            # vector ALU
    ConvShape("b_patch", 3, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=101),                # 437 pixels per image
    ConvShape("b_patch_chunks", 2, 13, 17, 128, 72, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=102),
    ConvShape("b_gather", 4, 13, 17, 96, 40, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, seed=103),   # rows per element
    ConvShape("b_gather_1x1_s2", 3, 15, 15, 64, 64, 1, 1, SY=2, SX=2, seed=104),
    ConvShape("b_lowc", 3, 30, 26, 4, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=105),
    ConvShape("b_i8", 3, 15, 15, 256, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=19, seed=106),
    ConvShape("b_tiny_images", 9, 3, 3, 64, 32, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=107),            # 9 pixels per image
    CONFIGS["cfg3c_5x5_asym"].with_(N=2),                                                           # 12321 = 48 * 256 + 33
    # the filter-in-registers kernel on the one-image buffer: images of a whole number of 32-pixel blocks
    ConvShape("b_regs", 5, 16, 24, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=108),                 # 12 blocks per image
    ConvShape("b_regs_s2", 3, 32, 32, 128, 130, 3, 3, SY=2, SX=2, PT=1, PL=1, PB=1, PR=1, seed=109),
    ConvShape("b_regs_5x5", 3, 8, 12, 32, 64, 5, 5, PT=2, PL=2, PB=2, PR=2, seed=110),              # 3 blocks per image
    ConvShape("b_regs_i8", 3, 16, 16, 256, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=200, seed=112),
    ConvShape("b_regs_one_block_images", 9, 4, 8, 64, 32, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=113),  # a pass spans 4 images
    ConvShape("b_regs_dil", 4, 16, 16, 64, 200, 3, 3, DY=2, DX=2, PT=2, PL=2, PB=2, PR=2, seed=114),
    CONFIGS["cfg3b_3x3_d2"].with_(N=3),
    ConvShape("b_regs_f32", 3, 19, 23, 32, 72, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="f32", seed=116),   # 437 pixels per image
    ConvShape("b_window_c256", 3, 19, 23, 256, 72, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=117),            # pixel-range kernel
]


@pytest.mark.parametrize("s", PER_IMAGE_SHAPES, ids=lambda s: s.name)
def test_batch_independent_buffer_matches_oracle(s):
    x, w = make_tensors(s)
    name = icv.plan_name(icv.make_params(s, plan=PER_IMAGE))
    _say("per-image", s.name, name)
    buf, xd = run_indirect(s, x, w, plan=PER_IMAGE)
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    # the buffer is that of one image: entry by entry the oracle's entries of batch element 0
    one = s.with_(N=1)
    built = icv.prepare(one, icv.to_device(w), plan=PER_IMAGE)
    got, pad = layout.logical_indirection(built.p, built.indirection, built.M)
    assert np.array_equal(got, oracle.indirection(one)) and np.all(pad == -1)
    assert icv.indirection_bytes(buf.p) == icv.indirection_bytes(icv.make_params(one, plan=PER_IMAGE))


def test_batch_independent_buffer_serves_any_batch_size():
    """Built once, used for batches of 1, 2 and 5 images without touching it (section 2.3: a batch-size increase
    only needs the entries of the new images; here there are none to add)."""
    for base in (ConvShape("b_grow", 1, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=111),
                 ConvShape("b_grow_regs", 1, 16, 24, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=115)):   # filter in registers
        big = base.with_(N=5)
        x, w = make_tensors(big)
        built = icv.prepare(base, icv.to_device(w), plan=PER_IMAGE)
        for n in (1, 2, 5):
            s = base.with_(N=n)
            xs = np.ascontiguousarray(x[:n])
            other = icv.prepare(s, icv.to_device(w), plan=PER_IMAGE)       # output, packed filter for this batch size
            icv.conv2d_nhwc(other.p, icv.to_device(xs), other.packed, built.indirection, other.zero_row, other.output)
            torch.cuda.synchronize()
            check_against_oracle(s, other.output.cpu().numpy(), xs, w)


# ---------------------------------------------------------------- the paper's model layers
from paper_1907_02129_amd.workloads import resnet18_layers, squeezenet10_layers

MODEL_LAYERS = resnet18_layers(2) + squeezenet10_layers(2)


@pytest.mark.parametrize("s", MODEL_LAYERS, ids=lambda s: s.name)
def test_model_layers_match_oracle(s):
    """Every distinct convolution of ResNet-18 and SqueezeNet 1.0 (section 3.1, Table 2) at batch 2, with the plan
    the library picks and with the batch-independent buffer.  Channel counts the tensor-core kernels cannot address
    (3; 48) run twice: stored padded with zeros, as the benchmark's sweep keeps them, and as they are (which takes
    the vector-ALU kernel)."""
    stored = icv.stored_for_tensor_cores(s)
    for sh in ([stored, s] if stored is not s else [s]):
        x, w = make_tensors(sh)
        for plan in (0, PER_IMAGE):
            name = icv.plan_name(icv.make_params(sh, plan=plan))
            _say("layer", sh.name, "C", sh.C, name)
            assert ("generic" in name) == (sh is not stored)
            buf, xd = run_indirect(sh, x, w, plan=plan)
            check_against_oracle(sh, buf.output.cpu().numpy(), x, w)


# ---------------------------------------------------------------- grids with workgroups that find no tile
@pytest.mark.parametrize("plan", [0, icv.PLAN_GATHER, hooks.tile(0), hooks.tile(2), hooks.tile(4), icv.PLAN_GATHER | hooks.tile(4)],
                         ids=["auto", "gathered", "128x64", "256x64_c4x1", "64x64", "64x64_gathered"])
@pytest.mark.parametrize("tiles64", [9, 13, 23])
def test_tile_counts_that_are_not_a_multiple_of_eight(plan, tiles64):
    """The XCD-aware tile order launches a multiple of 8 workgroups; with 9, 13 or 23 tiles of 64 rows (fewer of the
    larger tiles) some workgroups own no tile and must leave without touching anything."""
    rows = 64 * tiles64 - 17                                   # ragged last tile
    for s in (ConvShape("z_3x3", 1, 1, rows, 64, 64, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=131),
              ConvShape("z_1x1", 1, 1, rows, 64, 96, 1, 1, seed=132),
              ConvShape("z_1x1_s2", 1, 2, 2 * rows, 64, 32, 1, 1, SY=2, SX=2, seed=133)):
        name = icv.plan_name(icv.make_params(s, plan=plan))
        if not name:
            continue
        _say("tiles", s.name, name)
        x, w = make_tensors(s)
        buf, xd = run_indirect(s, x, w, plan=plan)
        check_against_oracle(s, buf.output.cpu().numpy(), x, w)


def test_batch_independent_buffer_with_fused_output_and_pixel_strides():
    s = ConvShape("bf_combo", 3, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=134)
    x, w = make_tensors(s)
    xs = np.zeros(x.shape[:-1] + (128,), dtype=x.dtype)
    xs[..., :s.C] = x
    xs[..., s.C:] = 0x7fc0                                      # NaN bit patterns in the unused channels
    acc, mag = oracle.conv2d_abs(s, x, w)
    run_fused_case(s, x, w, acc, mag, True, True, plan=PER_IMAGE, in_pixel_stride=128, out_pixel_stride=100, x_stored=xs)


# ---------------------------------------------------------------- one zero row for several operators
def test_one_zero_row_shared_by_operators_of_different_width():
    """Section 2.3: the explicit zero vector need not be contiguous with the input and can be shared between
    convolution operators.  One zero row, sized for the widest operator, serves three of them (the kernels that
    gather rows per kernel element and the vector-ALU kernel fetch it for every padding entry)."""
    shapes = [ConvShape("zr_c128", 2, 11, 13, 128, 48, 3, 3, PT=2, PL=2, PB=2, PR=2, seed=141),
              ConvShape("zr_c64", 1, 9, 17, 64, 72, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, seed=142),
              ConvShape("zr_c32", 3, 7, 7, 32, 40, 5, 5, PT=2, PL=2, PB=2, PR=2, seed=143)]
    widest = max(shapes, key=lambda s: s.C)
    zero_row = torch.empty(icv.zero_row_bytes(icv.make_params(widest)), dtype=torch.uint8, device="cuda:0")
    icv.init_zero_row(icv.make_params(widest), zero_row)
    for plan in (icv.PLAN_GATHER, icv.PLAN_VECTOR_ALU):        # gathered tensor-core kernel, vector-ALU kernel
        for s in shapes:
            x, w = make_tensors(s)
            buf = icv.prepare(s, icv.to_device(w), plan=plan)
            _say("shared zero row", s.name, icv.plan_name(buf.p))
            buf.zero_row.fill_(0x7f)                           # the operator's own zero row is not the one used
            icv.conv2d_nhwc(buf.p, icv.to_device(x), buf.packed, buf.indirection, zero_row, buf.output)
            torch.cuda.synchronize()
            check_against_oracle(s, buf.output.cpu().numpy(), x, w)


# ---------------------------------------------------------------- launches captured into a HIP graph
@pytest.mark.parametrize("s", [
    ConvShape("h_regs", 3, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=121),
    ConvShape("h_patch", 3, 19, 23, 256, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=126),
    ConvShape("h_gather", 2, 13, 17, 96, 40, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, seed=122),
    ConvShape("h_lowc", 2, 30, 26, 4, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=123),
    ConvShape("h_gemm", 2, 21, 13, 256, 64, 1, 1, seed=124),
    ConvShape("h_i8", 2, 15, 15, 256, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=64, seed=125),
], ids=lambda s: s.name)
def test_graph_replays_match_eager(s):
    """The conv call is kernel launches only (no allocation, no memset, no synchronisation), so it can be captured;
    every replay, with eager work and synchronisations in between, must give the eager result bit for bit."""
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)                 # eager result (also does the one-time function set-up)
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    eager = buf.output.clone()
    _say("graph", s.name, icv.plan_name(buf.p))
    assert ("freg" in icv.plan_name(buf.p)) == (s.name in ("h_regs", "h_i8")) and ("patch" in icv.plan_name(buf.p)) == (s.name == "h_patch")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        icv.run(buf, xd)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        icv.run(buf, xd)
    for rep in range(3):
        buf.output.fill_(-7)                        # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(buf.output, eager), (s.name, rep)


# ---------------------------------------------------------------- fused output stage
def _bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


FUSED_SHAPES = [
    CONFIGS["cfg1_tiny_f32"],                                                                     # vector-ALU kernel
    ConvShape("f_patch", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=91),               # filter in registers, then the pixel-range kernel
    ConvShape("f_gather", 2, 13, 17, 96, 40, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, seed=92),  # per-element gather
    ConvShape("f_gemm", 3, 7, 11, 128, 72, 1, 1, seed=93),                                        # GEMM on the input
    ConvShape("f_lowc", 2, 30, 26, 4, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=94),     # short rows
    ConvShape("f_i8_patch", 2, 15, 15, 256, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=3, seed=95),
    ConvShape("f_i8_lowc", 2, 11, 23, 8, 33, 5, 5, PT=2, PL=2, PB=1, PR=1, dtype="u8i8", zero_point=250, seed=96),
    ConvShape("f_i8_alu", 1, 9, 9, 5, 16, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=7, seed=97),
    ConvShape("f_i8_zp0", 2, 13, 14, 64, 40, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=0, seed=99),   # after a ReLU
    ConvShape("f_i8_gemm_zp", 2, 9, 13, 256, 96, 1, 1, dtype="u8i8", zero_point=17, seed=100),
]


def run_fused_case(s, x, w, acc, mag, relu, narrow, plan=0, in_pixel_stride=0, out_pixel_stride=0, x_stored=None):
    """One icv_conv2d_nhwc_fused call checked element by element: integer work bit-exact; float work within the
    accumulation bound (any order), the bias add, and for a bfloat16 output one rounding to 8 significant bits."""
    rng = np.random.default_rng(s.seed + 500)
    quant = s.dtype == "u8i8"
    buf = icv.prepare(s, icv.to_device(w), plan=plan, in_pixel_stride=in_pixel_stride, out_pixel_stride=out_pixel_stride)
    _say("fused", s.name, icv.plan_name(buf.p), "relu" if relu else "", "narrow" if narrow else "")
    xd = icv.to_device(x if x_stored is None else x_stored)
    oshape = acc.shape[:-1] + (out_pixel_stride or s.K,)
    if quant:
        bias = rng.integers(-5000, 5000, size=s.K).astype(np.int32)
        want = oracle.epilogue(acc, bias, relu)
        # (a scale at which both ends of the accumulators' range clamp, whichever way an input zero point skews them)
        reach = float(min(want.max(), -want.min())) if want.min() < 0 < want.max() else float(np.abs(want).max())
        scale, zp = float(np.float32(200.0 / reach)), 77
        bias_dev = icv.to_device(bias)
        ep = icv.make_epilogue(bias_dev, relu, icv.ICV_OUT_U8 if narrow else icv.ICV_OUT_ACC, scale, zp)
        out = torch.full(oshape, 201 if narrow else -7, dtype=torch.uint8 if narrow else torch.int32, device="cuda:0")
        icv.conv2d_nhwc_fused(buf.p, xd, buf.packed, buf.indirection, buf.zero_row, ep, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.all(got[..., s.K:] == (201 if narrow else -7))            # a pixel stride's padding is not written
        got = got[..., :s.K]
        want = oracle.requantise_u8(want, scale, zp) if narrow else want
        assert np.array_equal(got, want), f"{(got != want).sum()} of {want.size} differ"      # integer work: bit-exact
        if narrow:
            assert got.min() == (zp if relu else 0) and got.max() == 255                         # the codes use the range, both clamps
        return
    bias = (rng.standard_normal(s.K) * np.abs(acc).max() * 0.3).astype(np.float32)
    want = oracle.epilogue(acc, bias.astype(np.float64), relu)
    # bf16 output is offered for the float paths, the fp32 kernel included
    out_type = icv.ICV_OUT_BF16 if narrow else icv.ICV_OUT_ACC
    bias_dev = icv.to_device(bias)
    ep = icv.make_epilogue(bias_dev, relu, out_type)
    out = torch.full(oshape, 9.0, dtype=torch.bfloat16 if out_type == icv.ICV_OUT_BF16 else torch.float32, device="cuda:0")
    icv.conv2d_nhwc_fused(buf.p, xd, buf.packed, buf.indirection, buf.zero_row, ep, out)
    torch.cuda.synchronize()
    if out_type == icv.ICV_OUT_BF16:
        got = _bf16_bits_to_f64(out.view(torch.int16).cpu().numpy().view(np.uint16))
    else:
        got = out.cpu().numpy().astype(np.float64)
    assert np.all(got[..., s.K:] == 9.0)
    got = got[..., :s.K]
    err = np.abs(got - want)
    # a bfloat16 output carries 8 significant bits whatever the inputs were: the bf16 bar applies to it
    assert err.max() / np.abs(want).max() <= (TOL["bf16"] if out_type == icv.ICV_OUT_BF16 else TOL[s.dtype])
    n_terms = s.R * s.S * s.C + 1
    bound = 2.0 * n_terms * 2.0 ** -24 * (mag + np.abs(bias)[None, None, None, :]) + 1e-30
    if out_type == icv.ICV_OUT_BF16:
        bound = bound + 2.0 ** -8 * np.abs(want)
    assert (err / bound).max() <= 1.0
    if relu:
        assert got.min() == 0.0 and (got == 0).mean() > 0.05


@pytest.mark.parametrize("s", FUSED_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("relu", [False, True], ids=["linear", "relu"])
@pytest.mark.parametrize("narrow", [False, True], ids=["acc_type", "narrow_out"])
def test_fused_output_stage_matches_oracle(s, relu, narrow):
    x, w = make_tensors(s)
    if s.dtype == "u8i8":
        acc, mag = oracle.conv2d_u8i8(s, x, w, s.zero_point, centred=True), None
    else:
        acc, mag = oracle.conv2d_abs(s, x, w)
    run_fused_case(s, x, w, acc, mag, relu, narrow)
    # where the library's choice is the filter-in-registers kernel, the pixel-range kernel's fused stage as well
    window = icv.plan_name(icv.make_params(s, plan=icv.PLAN_WINDOW))
    if window and window != icv.plan_name(icv.make_params(s)):
        run_fused_case(s, x, w, acc, mag, relu, narrow, plan=icv.PLAN_WINDOW)


@pytest.mark.parametrize("name", [n for n in CONFIGS if n != "cfg1_tiny_f32"])
@pytest.mark.parametrize("relu,narrow", [(True, True), (False, False)], ids=["relu_narrow_out", "linear_acc_type"])
def test_fused_output_stage_on_benchmark_shapes(name, relu, narrow):
    """The fused instantiations of the very kernels the benchmark times, on the full-size shapes, every element."""
    s = CONFIGS[name]
    x, w = make_tensors(s)
    acc, mag = oracle_accumulators(s, x, w)
    run_fused_case(s, x, w, acc, mag, relu, narrow)


def test_fused_with_nothing_to_fuse_equals_the_plain_call_and_rejects_bad_stages():
    s = ConvShape("f_same", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=98)
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    plain = buf.output.clone()
    buf.output.fill_(-7)
    icv.conv2d_nhwc_fused(buf.p, xd, buf.packed, buf.indirection, buf.zero_row, icv.make_epilogue(), buf.output)
    torch.cuda.synchronize()
    assert torch.equal(plain, buf.output)
    for bad in (icv.make_epilogue(out_type=icv.ICV_OUT_U8, out_scale=0.1),          # uint8 codes of a float path
                icv.make_epilogue(out_type=7), icv.make_epilogue(relu=2)):
        with pytest.raises(icv.IcvError) as e:
            icv.conv2d_nhwc_fused(buf.p, xd, buf.packed, buf.indirection, buf.zero_row, bad, buf.output)
        assert e.value.status == icv.ICV_ERR_INVALID_ARG
    q = CONFIGS["cfg4_int8_3x3"].with_(N=1)
    xq, wq = make_tensors(q)
    bq, xqd = run_indirect(q, xq, wq)
    for bad in (icv.make_epilogue(out_type=icv.ICV_OUT_BF16), icv.make_epilogue(out_type=icv.ICV_OUT_U8, out_scale=0.0),
                icv.make_epilogue(out_type=icv.ICV_OUT_U8, out_scale=float("nan")),
                icv.make_epilogue(out_type=icv.ICV_OUT_U8, out_scale=0.1, out_zero_point=256)):
        with pytest.raises(icv.IcvError) as e:
            icv.conv2d_nhwc_fused(bq.p, xqd, bq.packed, bq.indirection, bq.zero_row, bad, bq.output)
        assert e.value.status == icv.ICV_ERR_INVALID_ARG


# ---------------------------------------------------------------- properties of the path
def test_output_pixel_stride_and_untouched_gaps():
    s = ConvShape("ostride", 2, 10, 12, 64, 40, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=61)
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w, out_pixel_stride=48)
    out = buf.output.cpu().numpy()
    assert out.shape[-1] == 48 and np.all(out[..., 40:] == -7)        # only the first K of each pixel written
    check_against_oracle(s, np.ascontiguousarray(out[..., :40]), x, w)


def test_padded_channel_layout():
    # 3 real channels stored with a pixel stride of 4 (fourth input / filter channel zero)
    s4 = CONFIGS["cfg5b_7x7_s2"].with_(N=2, Hin=40, Win=36)
    x, w = make_tensors(s4)
    buf, xd = run_indirect(s4, x, w)
    # the oracle on the three real channels (it reads the input with its pixel stride of 4)
    check_against_oracle(s4.with_(C=3), buf.output.cpu().numpy(), x, np.ascontiguousarray(w[..., :3]))


@pytest.mark.parametrize("name", ["cfg2_3x3_c64", "cfg3a_3x3_s2", "cfg4_int8_3x3", "cfg3c_5x5_asym", "cfg5b_7x7_s2"])
def test_im2col_gemm_ablation_agrees_with_indirect_path(name):
    # "fused im2col + GEMM" (section 2.2): both paths compute the same thing
    s = CONFIGS[name].with_(N=2)
    _say("ablation", name)
    x, w = make_tensors(s)
    direct, xd = run_indirect(s, x, w)
    buf = icv.prepare(s, icv.to_device(w), plan=icv.PLAN_GATHER)          # the filter packed for the plain GEMM kernels
    out2, ws = run_im2col(s, buf, xd)
    got1, got2 = direct.output.cpu().numpy(), out2.cpu().numpy()
    # each path is held to the per-element bound against the oracle (which also bounds their difference)
    check_against_oracle(s, got1, x, w)
    check_against_oracle(s, got2, x, w)
    if s.dtype == "u8i8":
        assert np.array_equal(got1, got2)
    # the patch matrix itself: row m, tap t holds the pixel row the indirection entry names
    M, T = buf.M, s.R * s.S
    esz = 1 if s.dtype == "u8i8" else 2
    mr = icv.indirection_index(buf.p, 0, 1)                         # row tile (T > 1 in all these shapes)
    kp = icv.im2col_bytes(buf.p) // (-(-M // mr) * mr)               # bytes per patch row (padded for short rows)
    rows = ws.cpu().numpy()[:M * kp].reshape(M, kp)
    assert not rows[:, T * s.C * esz:].any()
    rows = rows[:, :T * s.C * esz].reshape(M, T, s.C * esz)
    ent = oracle.indirection(s)
    xb = x.reshape(-1, s.C).view(np.uint8).reshape(-1, s.C * esz)
    fill = np.full(s.C * esz, s.zero_point if s.dtype == "u8i8" else 0, dtype=np.uint8)
    src = np.concatenate([xb, fill[None]], axis=0)
    assert np.array_equal(rows, src[ent])          # entry -1 indexes the appended fill row


@pytest.mark.parametrize("s", [ConvShape("abl_img", 2, 19, 23, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=151),
                               ConvShape("abl_img_i8", 3, 15, 15, 256, 80, 3, 3, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=41, seed=152),
                               ConvShape("abl_img_lowc", 2, 30, 26, 4, 70, 7, 7, SY=2, SX=2, PT=3, PL=3, PB=3, PR=3, seed=153)],
                         ids=lambda s: s.name)
def test_im2col_gemm_ablation_with_the_batch_independent_plan(s):
    """The ablation reads the filter as icv_pack_filter laid it out for the problem's plan, whatever tile that plan
    chose: with the batch-independent buffer the tile is picked for a full chip, not for this small batch."""
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w, plan=icv.PLAN_GATHER | PER_IMAGE)
    check_against_oracle(s, buf.output.cpu().numpy(), x, w)
    out2, _ = run_im2col(s, buf, xd)
    check_against_oracle(s, out2.cpu().numpy(), x, w)


def test_small_generic_im2col_path():
    s = ConvShape("g_im2col", 2, 9, 10, 5, 7, 3, 3, SY=2, SX=1, PT=1, PL=2, PB=0, PR=1, dtype="f32", dist="uniform", seed=71)
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    out2, _ = run_im2col(s, buf, xd)
    check_against_oracle(s, out2.cpu().numpy(), x, w)


def test_determinism_and_buffer_reuse_with_new_input_pointer():
    s = CONFIGS["cfg2_3x3_c64"].with_(N=4)
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    first = buf.output.clone()
    icv.run(buf, xd)
    torch.cuda.synchronize()
    assert torch.equal(first, buf.output)
    # entries are indices, so the same buffer serves an input tensor at another address
    pad = torch.empty(4096, dtype=torch.uint8, device="cuda:0")   # shifts the next allocation
    xd2 = xd.clone()
    assert xd2.data_ptr() != xd.data_ptr()
    icv.run(buf, xd2)
    torch.cuda.synchronize()
    assert torch.equal(first, buf.output)
    del pad


def test_runs_on_a_side_stream():
    s = CONFIGS["cfg2_3x3_c64"].with_(N=2)
    x, w = make_tensors(s)
    buf, xd = run_indirect(s, x, w)
    want = buf.output.clone()
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    buf.output.zero_()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        icv.run(buf, xd)
    st.synchronize()
    assert torch.equal(want, buf.output)


@pytest.mark.gpu
def test_mfma_peak_measurement_is_plausible():
    """The measured tensor-core ceilings: positive, below the data-sheet peak (a loop cannot beat the hardware), above a
    tenth of it (every SIMD is multiplying), int8 about twice bf16, and toggling operands never faster than constant
    ones beyond the run-to-run noise."""
    for dtype, sheet in (("bf16", 2.5e15), ("u8i8", 5.0e15)):
        const = icv.measure_mfma_peak(dtype, 2, False)
        varied = icv.measure_mfma_peak(dtype, 2, True)
        for r in (const, varied):
            assert 0.1 * sheet < r < 1.02 * sheet, (dtype, r)
        assert varied < 1.05 * const, (dtype, const, varied)
    assert 1.5 < icv.measure_mfma_peak("u8i8", 2) / icv.measure_mfma_peak("bf16", 2) < 2.5

