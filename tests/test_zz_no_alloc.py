"""The entry point that allocates nothing: icv_conv2d_nhwc_im2col_static against icv_conv2d_nhwc_im2col.

Same kernels, the patch matrix in the library's own device buffer instead of a caller's workspace: the outputs must be
bit-identical.  Two calls in a row, the second with a smaller input, so stale contents of the shared buffer would show.
"""
import numpy as np
import pytest
import torch

from paper_1907_02129_amd import binding as icv
from paper_1907_02129_amd.workloads import ConvShape, make_tensors

pytestmark = pytest.mark.gpu
GATHER = icv.PLAN_GATHER          # a plan whose packed filter the ablation's plain GEMM reads


def _both_ways(s):
    x, w = make_tensors(s)
    xd = icv.to_device(x)
    buf = icv.prepare(s, icv.to_device(w), plan=GATHER)
    assert 0 < icv.im2col_bytes(buf.p) <= icv.static_workspace_bytes()
    ws = torch.empty(icv.im2col_bytes(buf.p), dtype=torch.uint8, device="cuda:0")
    want = torch.full_like(buf.output, -7)
    icv.conv2d_nhwc_im2col(buf.p, xd, buf.packed, ws, want)
    got = torch.full_like(buf.output, -9)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    icv.conv2d_nhwc_im2col_static(buf.p, xd, buf.packed, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return want, got


def test_static_workspace_variant_matches_the_workspace_variant_twice():
    icv.load_library()
    assert icv.static_workspace_bytes() == 16 << 20
    big = ConvShape("na_big", 3, 29, 31, 64, 96, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=401)
    small = ConvShape("na_small", 1, 9, 11, 32, 40, 3, 3, SY=2, SX=1, PT=1, PL=1, PB=1, PR=1, dtype="u8i8", zero_point=128, seed=402)
    for s in (big, small):
        print("no-alloc", s.name, flush=True)
        want, got = _both_ways(s)
        assert torch.equal(want, got), s.name
        assert not torch.equal(got, torch.full_like(got, -9))


def test_static_workspace_variant_rejects_what_does_not_fit():
    icv.load_library()
    s = ConvShape("na_huge", 32, 56, 56, 64, 64, 3, 3, PT=1, PL=1, PB=1, PR=1, seed=403)
    p = icv.make_params(s, plan=GATHER)
    assert icv.im2col_bytes(p) > icv.static_workspace_bytes()
    out = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(icv.IcvError) as e:
        icv.conv2d_nhwc_im2col_static(p, out, out, out)
    assert e.value.status == icv.ICV_ERR_UNSUPPORTED
    # a plan without ablation (filter in registers) is refused the same way
    p2 = icv.make_params(s.with_(N=1, Hin=20, Win=20), plan=icv.PLAN_FILTER_REGS)
    with pytest.raises(icv.IcvError) as e:
        icv.conv2d_nhwc_im2col_static(p2, out, out, out)
    assert e.value.status == icv.ICV_ERR_UNSUPPORTED
