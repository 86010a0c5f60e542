"""The test hooks in icv_conv_params.plan above the public bits: they force a tile or a pipeline shape of the
tensor-core kernels, so that every one of them also runs on problems small enough for the CPU oracle."""

TILES = ["128x64_c2x2", "128x128_c2x2", "256x64_c4x1", "256x64_c4x2", "64x64_c2x2", "256x128_c4x2", "128x128_c4x2"]
GATHER_TILES = (0, 1, 3, 4)          # tiles the gathering kernel (and the plain GEMM) is built for


def tile(index: int) -> int:
    return (index + 1) << 8


def ring(depth: int) -> int:
    return depth << 12


def per_cu(n: int) -> int:
    return n << 16


KCB64 = 1 << 18


def group(taps: int) -> int:
    return taps << 20
