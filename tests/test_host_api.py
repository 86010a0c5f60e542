"""Host-side checks that need no GPU: the library loads, exports what the header declares, and its
geometry / validation logic agrees with the oracle's statement of the problem."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import plan_hooks as hooks
from paper_1907_02129_amd import binding as icv
from paper_1907_02129_amd.workloads import CONFIGS, ConvShape, random_small_shape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return icv.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "icv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(icv_[a-z0-9_]+)\s*\(", header))
    assert declared == set(icv.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_params_struct_matches_header():
    header = open(os.path.join(ROOT, "include", "icv.h")).read()
    body = re.search(r"typedef struct icv_conv_params \{(.*?)\} icv_conv_params;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = [n.strip() for decl in re.findall(r"int32_t([^;]*);", body) for n in decl.split(",")]
    assert names == [f[0] for f in icv.icv_conv_params._fields_]


@pytest.mark.parametrize("name", list(CONFIGS))
def test_output_size_and_buffer_sizes(lib, name):
    s = CONFIGS[name]
    p = icv.make_params(s)
    Hout, Wout = icv.output_size(p)
    assert (Hout, Wout) == oracle.out_extent(s)
    M, T = s.N * Hout * Wout, s.R * s.S
    nbytes = icv.indirection_bytes(p)
    # the layout the library reports accounts for every byte of the buffer: entries in the width the kernel reads,
    # tile records, and the int32 form where it is kept beside a 2-byte form; padding is less than one row tile
    L = icv.get_indirection_layout(p)
    assert L.tile_rows in (32, 64, 128, 256) and L.tiles == -(-M // L.tile_rows)
    n = L.tiles * L.tile_rows * T
    parts = [(L.entries_at, n * L.entry_bytes)]
    if L.record_bytes:
        parts.append((L.records_at, L.tiles * L.record_bytes))
    if L.int32_entries_at >= 0 and L.entry_bytes != 4:
        parts.append((L.int32_entries_at, n * 4))
    parts.sort()
    assert parts[0][0] == 0 and all(a + b == c for (a, b), (c, _) in zip(parts, parts[1:]))
    assert parts[-1][0] + parts[-1][1] == nbytes
    assert (L.entry_bytes == 2) == (L.record_bytes == 16) and (L.records_at >= 0) == (L.record_bytes > 0)
    # the entries do not depend on the number of input channels (section 1.1); with the row staging fixed,
    # neither does the tile the library picks
    per_tap = icv.PLAN_GATHER
    assert (icv.indirection_bytes(icv.make_params(s.with_(C=s.C * 2), plan=per_tap)) ==
            icv.indirection_bytes(icv.make_params(s, plan=per_tap))) or s.dtype == "f32"
    esz = {"f32": 4, "bf16": 2, "u8i8": 1}[s.dtype]
    assert icv.packed_filter_bytes(p) >= s.K * T * s.C * esz
    assert icv.zero_row_bytes(p) >= s.C * esz and icv.zero_row_bytes(p) % 16 == 0
    # the ablation runs with a plan whose packed filter the plain GEMM kernels read
    abl = icv.make_params(s, plan=per_tap)
    assert icv.im2col_bytes(abl) >= M * T * s.C * esz
    if "freg" in icv.plan_name(p):
        assert icv.im2col_bytes(p) == 0
    assert icv.plan_name(p) != ""


def test_output_size_random_shapes(lib):
    rng = np.random.default_rng(3)
    for _ in range(200):
        s = random_small_shape(rng)
        assert icv.output_size(icv.make_params(s)) == oracle.out_extent(s)


def test_indirection_index_is_tile_tap_row_order(lib):
    s = CONFIGS["cfg2_3x3_c64"]
    p = icv.make_params(s)
    T = 9
    mr = icv.indirection_index(p, 0, 1)            # tap stride = rows per tile
    assert mr >= 32 and mr % 32 == 0
    assert icv.indirection_index(p, 0, 0) == 0 and icv.indirection_index(p, 1, 0) == 1
    assert icv.indirection_index(p, mr, 0) == mr * T
    seen = {icv.indirection_index(p, m, t) for m in range(2 * mr) for t in range(T)}
    assert seen == set(range(2 * mr * T))          # a bijection onto the first two tiles
    assert icv.indirection_index(p, -1, 0) == -1 and icv.indirection_index(p, 0, T) == -1


def _status(lib, s, **over):
    p = icv.make_params(s)
    for k, v in over.items():
        setattr(p, k, v)
    return lib.icv_output_size(ctypes.byref(p), None, None)


def test_invalid_arguments_are_rejected(lib):
    s = CONFIGS["cfg2_3x3_c64"]
    assert _status(lib, s) == icv.ICV_OK
    for field in ("N", "Hin", "Win", "C", "K", "R", "S", "SY", "SX", "DY", "DX"):
        assert _status(lib, s, **{field: 0}) == icv.ICV_ERR_INVALID_ARG, field      # empty problems
        assert _status(lib, s, **{field: -3}) == icv.ICV_ERR_INVALID_ARG, field
    for field in ("PT", "PL", "PB", "PR"):
        assert _status(lib, s, **{field: -1}) == icv.ICV_ERR_INVALID_ARG, field
    assert _status(lib, s, dtype=7) == icv.ICV_ERR_INVALID_ARG
    assert _status(lib, s, in_pixel_stride=32) == icv.ICV_ERR_INVALID_ARG           # stride < C
    assert _status(lib, s, out_pixel_stride=8) == icv.ICV_ERR_INVALID_ARG           # stride < K
    assert _status(lib, s, R=80, PT=0, PB=0) == icv.ICV_ERR_INVALID_ARG             # kernel larger than input
    assert _status(lib, s, N=1 << 20) == icv.ICV_ERR_INVALID_ARG                    # input of 2 GiB or more
    assert _status(lib, s, plan=5) == icv.ICV_ERR_INVALID_ARG                       # no such algorithm
    assert _status(lib, s, plan=1 << 4) == icv.ICV_ERR_INVALID_ARG                  # bits that must be 0
    assert _status(lib, s, plan=1 << 23) == icv.ICV_ERR_INVALID_ARG
    assert _status(lib, s, plan=-1) == icv.ICV_ERR_INVALID_ARG
    assert _status(lib, s, plan=icv.PLAN_FILTER_REGS) == icv.ICV_OK                 # filter in registers, forced
    assert _status(lib, s, plan=icv.PLAN_FILTER_REGS | icv.PLAN_PER_IMAGE) == icv.ICV_OK
    assert _status(lib, s, plan=icv.PLAN_FILTER_REGS | icv.PLAN_PER_IMAGE, Hin=55) == icv.ICV_OK     # images of 96.25 blocks
    assert _status(lib, s, plan=icv.PLAN_FILTER_REGS, R=7, S=7, PT=3, PL=3, PB=3, PR=3) == icv.ICV_ERR_UNSUPPORTED   # ... not for 7x7
    assert _status(lib, s, plan=hooks.tile(0) | hooks.ring(13)) == icv.ICV_ERR_INVALID_ARG     # ring deeper than 12
    assert _status(lib, s, plan=hooks.tile(0) | hooks.ring(1)) == icv.ICV_ERR_INVALID_ARG      # a ring needs two slots
    assert _status(lib, s, plan=hooks.tile(7)) == icv.ICV_ERR_INVALID_ARG                      # seven tiles
    assert _status(lib, s, plan=icv.PLAN_VECTOR_ALU | hooks.tile(0)) == icv.ICV_ERR_INVALID_ARG
    assert _status(lib, CONFIGS["cfg4_int8_3x3"], input_zero_point=300) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_output_size(None, None, None) == icv.ICV_ERR_INVALID_ARG
    assert icv.indirection_bytes(icv.make_params(s.with_(N=0))) == 0


def test_null_and_misaligned_pointers_are_rejected_before_any_launch(lib):
    p = icv.make_params(CONFIGS["cfg2_3x3_c64"])
    vp = ctypes.c_void_p
    assert lib.icv_setup_indirection(ctypes.byref(p), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_setup_indirection(ctypes.byref(p), vp(0x1004), vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_conv2d_nhwc(ctypes.byref(p), vp(0), vp(0), vp(0), vp(0), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_pack_filter(ctypes.byref(p), vp(0), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_init_zero_row(ctypes.byref(p), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    for name in ("cfg2_3x3_c64", "cfg3b_3x3_d2"):     # plans without ablation: a tile the GEMM lacks, filter in registers
        q = icv.make_params(CONFIGS[name])
        assert lib.icv_im2col(ctypes.byref(q), vp(0), vp(0), vp(0)) == icv.ICV_ERR_UNSUPPORTED and icv.im2col_bytes(q) == 0
    p = icv.make_params(CONFIGS["cfg2_3x3_c64"], plan=icv.PLAN_GATHER)
    assert lib.icv_im2col(ctypes.byref(p), vp(0), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_gemm_nhwc(ctypes.byref(p), vp(0), vp(0), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    ep = icv.make_epilogue()
    a = vp(0x1000)
    assert lib.icv_conv2d_nhwc_fused(ctypes.byref(p), a, a, a, a, None, a, vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_conv2d_nhwc_fused(ctypes.byref(p), a, a, a, a, ctypes.byref(ep), vp(0), vp(0)) == icv.ICV_ERR_INVALID_ARG
    for bad in (icv.make_epilogue(out_type=icv.ICV_OUT_U8, out_scale=1.0), icv.make_epilogue(out_type=3),
                icv.make_epilogue(relu=-1)):
        # rejected by the host checks, before anything is launched on the (made-up) pointers
        assert lib.icv_conv2d_nhwc_fused(ctypes.byref(p), a, a, a, a, ctypes.byref(bad), a, vp(0)) == icv.ICV_ERR_INVALID_ARG


def test_mfma_peak_measurement_rejects_bad_arguments_before_any_launch(lib):
    v = ctypes.c_double(-1.0)
    vp = ctypes.c_void_p
    F32, BF16 = icv.DTYPES["f32"], icv.DTYPES["bf16"]
    for dtype, waves, varied in ((F32, 2, 0), (BF16, 0, 0), (BF16, 5, 0), (BF16, 2, 2), (BF16, 2, -1), (7, 1, 0)):
        assert lib.icv_measure_mfma_peak(dtype, waves, varied, ctypes.byref(v), vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert lib.icv_measure_mfma_peak(BF16, 2, 0, None, vp(0)) == icv.ICV_ERR_INVALID_ARG
    assert v.value == -1.0


def test_status_strings(lib):
    assert icv.status_string(0) == "ok"
    assert "invalid" in icv.status_string(icv.ICV_ERR_INVALID_ARG)
    assert icv.status_string(-99) == "unknown status"


def test_plans(lib):
    assert icv.plan_name(icv.make_params(CONFIGS["cfg1_tiny_f32"])).startswith("generic")
    assert icv.plan_name(icv.make_params(CONFIGS["cfg2_3x3_c64"])).startswith("mfma_bf16")
    assert icv.plan_name(icv.make_params(CONFIGS["cfg4_int8_3x3"])).startswith("mfma_i8")
    # any uint8 zero point runs on the tensor cores; the packed filter then carries K int32 filter sums behind it
    for zp in (0, 3, 255):
        q = icv.make_params(CONFIGS["cfg4_int8_3x3"].with_(zero_point=zp))
        assert icv.plan_name(q) == icv.plan_name(icv.make_params(CONFIGS["cfg4_int8_3x3"]))
        assert icv.packed_filter_bytes(q) == 256 * 9 * 256 + 256 * 4
    assert icv.packed_filter_bytes(icv.make_params(CONFIGS["cfg2_3x3_c64"])) == 64 * 9 * 64 * 2
    # 1x1 stride 1 without padding is a plain GEMM on the input tensor (section 3.2's advice to switch primitives)
    assert icv.plan_name(icv.make_params(CONFIGS["cfg5a_1x1"])).startswith("gemm_bf16")
    assert icv.plan_name(icv.make_params(CONFIGS["cfg5a_1x1"].with_(SX=2, SY=2))).startswith("mfma_bf16")
    # odd channel counts fall back to the vector-ALU kernel instead of failing
    odd = ConvShape("odd", 1, 8, 8, 5, 3, 3, 3)
    assert icv.plan_name(icv.make_params(odd)).startswith("generic")


def _exact_span(shape, rows):
    """Largest (max - min + 1) over the valid oracle entries of any window of `rows` consecutive output pixels
    that starts at a multiple of `rows` (the library's row tiles)."""
    from oracle import direct_conv as oracle
    ind = oracle.indirection(shape)                     # [M][T] pixel index or -1
    M = ind.shape[0]
    worst = 0
    for m0 in range(0, M, rows):
        blk = ind[m0:m0 + rows]
        v = blk[blk >= 0]
        if v.size:
            worst = max(worst, int(v.max() - v.min() + 1))
    return worst


def test_output_pixel_decomposition_is_exact_up_to_the_largest_tensors(lib):
    """The kernels split an output pixel number into (n, oy, ox) with a multiply and a shift instead of two divisions.
    For a 1x1 unpadded stride-1 convolution output pixel m names input pixel m and nothing else, so the closed-form
    window ends must both be m: checked at the ends, around every row and image boundary sampled, and at random m,
    on extents up to the 2 GiB limit of the input (one uint8 channel) and on strided ones, where the decomposition
    is visible through iy = oy*SY, ix = ox*SX."""
    import numpy as np
    rng = np.random.default_rng(5)
    extents = [(1, 46340, 46340), (1, 3, 715827882), (1, 715827882, 3), (2047, 1024, 1024), (1, 1, 2147483647),
               (7, 65537, 4681), (3, 1, 7), (5, 17, 1), (1 << 20, 1, 2047), (11, 9973, 19541)]
    for N, H, W in extents:
        s = ConvShape("big", N, H, W, 1, 1, 1, 1, dtype="u8i8", zero_point=128)
        p = icv.make_params(s)
        assert icv.output_size(p) == (H, W)
        M = N * H * W
        ms = {0, M - 1, M // 2}
        for _ in range(40):
            r = int(rng.integers(0, N * H))
            ms.update(m for m in (r * W - 1, r * W, r * W + 1, r * W + W - 1) if 0 <= m < M)
        ms.update(int(v) for v in rng.integers(0, M, size=200))
        for m in ms:
            assert icv.row_pixel_range(p, m, m) == (m, m), (N, H, W, m)
    for N, Hin, Win, SY, SX in [(3, 20001, 30011, 2, 3), (1, 2, 1000000007, 1, 2), (5000, 301, 707, 3, 2)]:
        s = ConvShape("big_s", N, Hin, Win, 1, 1, 1, 1, SY=SY, SX=SX, dtype="u8i8", zero_point=128)
        p = icv.make_params(s)
        Hout, Wout = icv.output_size(p)
        M = N * Hout * Wout
        for m in [0, M - 1] + [int(v) for v in rng.integers(0, M, size=300)]:
            n, rem = divmod(m, Hout * Wout)
            oy, ox = divmod(rem, Wout)
            want = (n * Hin + oy * SY) * Win + ox * SX
            assert icv.row_pixel_range(p, m, m) == (want, want), (N, Hin, Win, m)


def test_row_pixel_range_brackets_every_window_of_output_pixels(lib):
    """The sliding input window of the filter-in-registers kernel rests on two closed forms: a lower end that depends
    on a window's first output pixel alone and an upper end that depends on its last one alone.  Brute force on the
    oracle's entries: every valid entry of every window lies between them, both ends never move backwards, and the
    window is never longer than icv_tile_span_bound says (which is what sizes the LDS ring)."""
    import numpy as np
    from oracle import direct_conv as oracle
    from paper_1907_02129_amd.workloads import random_small_shape
    rng = np.random.default_rng(11)
    shapes = [random_small_shape(rng) for _ in range(200)]
    # paddings beyond the kernel's reach, where the clamped ends differ from the unclipped positions
    shapes += [random_small_shape(rng).with_(PT=int(rng.integers(0, 7)), PL=int(rng.integers(0, 7)),
                                             PB=int(rng.integers(0, 7)), PR=int(rng.integers(0, 7))) for _ in range(150)]
    shapes += [CONFIGS[n].with_(N=2) for n in ("cfg2_3x3_c64", "cfg3a_3x3_s2", "cfg3b_3x3_d2", "cfg3c_5x5_asym")]
    attained_lo = attained_hi = 0
    for shape in shapes:
        p = icv.make_params(shape)
        if not icv.plan_name(p):
            continue                                    # the redrawn padding left no output pixel
        ind = oracle.indirection(shape)
        M = ind.shape[0]
        valid = ind >= 0
        lo_row = np.where(valid, ind, np.iinfo(np.int32).max).min(axis=1)       # per output pixel
        hi_row = np.where(valid, ind, -1).max(axis=1)
        # suffix minimum / prefix maximum: what "this pixel or any later (earlier) one" names
        lo_from = np.minimum.accumulate(lo_row[::-1])[::-1]
        hi_upto = np.maximum.accumulate(hi_row)
        firsts = np.array([icv.row_pixel_range(p, m, m)[0] for m in range(M)])
        lasts = np.array([icv.row_pixel_range(p, m, m)[1] for m in range(M)])
        assert np.all(firsts <= lo_from), shape
        assert np.all(lasts >= hi_upto), shape
        assert np.all(np.diff(firsts) >= 0) and np.all(np.diff(lasts) >= 0), shape
        assert firsts.min() >= 0 and lasts.max() <= shape.N * shape.Hin * shape.Win - 1
        attained_lo += int(np.any(firsts == lo_from))
        attained_hi += int(np.any(lasts == hi_upto))
        for rows in (1, 3, 32, 64, 200):
            if rows > M:
                continue
            span = lasts[rows - 1:] - firsts[:M - rows + 1] + 1
            assert span.max() <= icv.tile_span_bound(p, rows), (shape, rows, int(span.max()))
            f, l = icv.row_pixel_range(p, 0, rows - 1)
            assert (f, l) == (firsts[0], lasts[rows - 1])
    assert attained_lo > 250 and attained_hi > 250          # the ends are tight, not merely safe
    p = icv.make_params(CONFIGS["cfg2_3x3_c64"])
    assert lib.icv_row_pixel_range(ctypes.byref(p), 5, 4, None, None) == icv.ICV_ERR_INVALID_ARG


def test_tile_span_bound_covers_every_tile(lib):
    """The LDS patch is sized by a closed-form bound; it must cover the pixel span of every row tile.  Checked by
    brute force on the oracle's indirection entries for random shapes and the benchmark shapes."""
    import numpy as np
    from paper_1907_02129_amd.workloads import random_small_shape
    rng = np.random.default_rng(5)
    tight = 0
    for i in range(300):
        shape = random_small_shape(rng)
        p = icv.make_params(shape)
        for rows in (1, 2, 7, 32, 128):
            bound = icv.tile_span_bound(p, rows)
            exact = _exact_span(shape, rows)
            assert bound >= exact, (shape, rows, bound, exact)
            tight += bound == exact
    assert tight > 0                                    # the bound is attained, not merely huge
    for name in ("cfg2_3x3_c64", "cfg3a_3x3_s2", "cfg3b_3x3_d2", "cfg3c_5x5_asym", "cfg4_int8_3x3"):
        shape = CONFIGS[name].with_(N=2)
        p = icv.make_params(shape)
        for rows in (128, 256):
            bound, exact = icv.tile_span_bound(p, rows), _exact_span(shape, rows)
            assert exact <= bound <= exact + 2 * shape.Win + shape.Hin * shape.Win // 8, (name, rows, bound, exact)
    assert icv.tile_span_bound(icv.make_params(CONFIGS["cfg2_3x3_c64"]), 0) == -1
    # the worked numbers: 3x3 stride 1 on 56 x 56 -> 255 steps + 2 rows + 2 pixels + 1
    assert icv.tile_span_bound(icv.make_params(CONFIGS["cfg2_3x3_c64"]), 256) == 255 + 2 * 56 + 2 + 1


def test_range_records_are_counted_in_the_buffer_size(lib):
    s = CONFIGS["cfg2_3x3_c64"]
    streamed = icv.make_params(s, plan=icv.PLAN_GATHER)
    patch = icv.make_params(s, plan=icv.PLAN_WINDOW)
    assert "patch" in icv.plan_name(patch) and "patch" not in icv.plan_name(streamed)
    mr = icv.indirection_index(patch, 0, 1)
    tiles = -(-(s.N * 56 * 56) // mr)
    assert icv.indirection_bytes(patch) == tiles * 16 + tiles * mr * 9 * 2      # records, 16-bit entries; no int32 form
    mr_s = icv.indirection_index(streamed, 0, 1)
    tiles_s = -(-(s.N * 56 * 56) // mr_s)
    assert icv.indirection_bytes(streamed) == tiles_s * mr_s * 9 * 4
    # a single kernel element has nothing to re-use: rows are gathered per element
    assert "patch" not in icv.plan_name(icv.make_params(CONFIGS["cfg5a_1x1"]))
    # forcing the pixel-range kernel where it cannot run is an error, not a silent fallback
    assert _status(lib, CONFIGS["cfg5a_1x1"], plan=icv.PLAN_WINDOW) == icv.ICV_ERR_UNSUPPORTED


def test_batch_independent_indirection_buffer_sizes(lib):
    """ICV_PLAN_PER_IMAGE: the buffer describes one image, so its size does not depend on N (section 2.3 re-initialises
    the buffer when the batch grows; with one image per buffer there is nothing to re-initialise)."""
    PER_IMAGE = icv.PLAN_PER_IMAGE
    for name in ("cfg2_3x3_c64", "cfg3c_5x5_asym", "cfg5b_7x7_s2", "cfg1_tiny_f32"):
        s = CONFIGS[name]
        one = icv.indirection_bytes(icv.make_params(s.with_(N=1), plan=PER_IMAGE))
        assert one > 0
        for n in (2, 7, s.N):
            assert icv.indirection_bytes(icv.make_params(s.with_(N=n), plan=PER_IMAGE)) == one
        # the kernel and tile do not depend on N either (the buffer's layout follows the tile)
        assert len({icv.plan_name(icv.make_params(s.with_(N=n), plan=PER_IMAGE)) for n in (1, 2, 7, s.N)}) == 1
        assert icv.indirection_bytes(icv.make_params(s)) > one or s.N == 1
        # the index function addresses pixels of one image only
        p = icv.make_params(s, plan=PER_IMAGE)
        Hout, Wout = icv.output_size(p)
        assert icv.indirection_index(p, Hout * Wout - 1, 0) >= 0
        assert icv.indirection_index(p, s.N * Hout * Wout - 1, 0) == -1 or s.N == 1
    # a 1x1 stride-1 convolution reads no entries at all; the option changes nothing for it
    g = CONFIGS["cfg5a_1x1"]
    assert icv.plan_name(icv.make_params(g, plan=PER_IMAGE)).startswith("gemm_")


def test_model_layer_lists_match_the_papers_table_2():
    """The layer sweep's shapes are written from the published architectures; their distinct operators, counted by
    type, must be what the paper's Table 2 prints (fixture), which a missing, duplicated or mistyped layer breaks."""
    import os
    from collections import Counter
    from paper_1907_02129_amd.workloads import resnet18_layers, squeezenet10_layers, layer_type
    want = {"resnet18": Counter(), "squeezenet": Counter()}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table2_layer_types.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            kind, a, b = line.strip().split(",")
            if int(a):
                want["resnet18"][kind] = int(a)
            if int(b):
                want["squeezenet"][kind] = int(b)
    for model, fn in (("resnet18", resnet18_layers), ("squeezenet", squeezenet10_layers)):
        layers = fn(2)
        assert Counter(layer_type(s) for s in layers) == want[model]
        # distinct parameter sets, distinct names, every shape valid for the library
        keys = {(s.Hin, s.c_logical or s.C, s.K, s.R, s.SY, s.PT) for s in layers}
        assert len(keys) == len(layers) == len({s.name for s in layers})
        for s in layers:
            p = icv.make_params(s)
            assert icv.output_size(p)[0] > 0 and icv.indirection_bytes(p) > 0
            assert s.R == s.S and s.SY == s.SX and (s.c_logical or s.C) <= s.C
    # the 3x3 convolutions keep the image size (padding 1); the stems halve it
    first = resnet18_layers(1)[0]
    assert icv.output_size(icv.make_params(first)) == (112, 112)
    assert icv.output_size(icv.make_params(squeezenet10_layers(1)[0])) == (109, 109)


def test_random_plans_and_shapes_never_confuse_the_host_logic(lib):
    """Every (shape, plan) pair is either refused as a whole or gets a kernel name and consistent buffer sizes;
    the tile the sizes are computed for is the one the index function reports."""
    import numpy as np
    from paper_1907_02129_amd.workloads import random_small_shape
    rng = np.random.default_rng(99)
    seen = set()
    for i in range(400):
        dtype = ("f32", "bf16", "u8i8")[i % 3]
        s = random_small_shape(rng, dtype, c_mult=(1, 32, 64)[i % 3] if i % 2 else 4, max_hw=40, max_ck=4)
        s = s.with_(N=int(rng.integers(1, 40)))
        plan = int(rng.integers(0, 16)) | (int(rng.integers(0, 1 << 15)) << 8 if i % 4 else 0)
        p = icv.make_params(s, plan=plan)
        name = icv.plan_name(p)
        sizes = (icv.indirection_bytes(p), icv.packed_filter_bytes(p), icv.zero_row_bytes(p))
        if not name:
            assert sizes == (0, 0, 0), (s, plan, sizes)
            continue
        seen.add(name.split("_")[0])
        Hout, Wout = icv.output_size(p)
        T = s.R * s.S
        rows = Hout * Wout * (1 if plan & icv.PLAN_PER_IMAGE and not name.startswith("gemm_") else s.N)
        assert all(v > 0 for v in sizes)
        L = icv.get_indirection_layout(p)
        assert sizes[0] >= L.entry_bytes * rows * T and sizes[0] % 4 == 0
        assert icv.indirection_index(p, 0, 0) == 0
        assert icv.indirection_index(p, rows - 1, T - 1) >= 0
        if T > 1:
            mr = icv.indirection_index(p, 0, 1)
            assert mr == L.tile_rows and mr in (32, 64, 128, 256)
            assert sizes[0] >= L.entry_bytes * (-(-rows // mr) * mr) * T
    assert {"generic", "mfma"} <= seen
