// Tensor-core Indirect GEMM with the filter held in registers: the host side of the launch.  The kernel is in
// icv_igemm_freg_kernel.h; its instantiations are compiled in one translation unit per dtype and output stage
// (icv_igemm_freg_*.hip).
#include "icv_igemm_freg_kernel.h"

namespace icv {

int launch_freg_bf16(const Geometry&, const FregArgs&, int64_t grid, size_t lds, int T, int KS, hipStream_t);
int launch_freg_bf16_fused(const Geometry&, const FregArgs&, int64_t grid, size_t lds, int T, int KS, hipStream_t);
int launch_freg_u8(const Geometry&, const FregArgs&, int64_t grid, size_t lds, int T, int KS, hipStream_t);
int launch_freg_u8_fused(const Geometry&, const FregArgs&, int64_t grid, size_t lds, int T, int KS, hipStream_t);
int launch_freg_f32(const Geometry&, const FregArgs&, int64_t grid, size_t lds, int T, int KS, hipStream_t);
int launch_freg_f32_fused(const Geometry&, const FregArgs&, int64_t grid, size_t lds, int T, int KS, hipStream_t);

// ------------------------------------------------------------------ launch
size_t freg_lds_bytes(int T, int KS, int PBK, int ring_rows)
{
    const size_t pitch = (size_t)(KS * 2 + 1) * 16;
    const size_t zero_off = (size_t)ring_rows * pitch;
    const size_t slot_off = (zero_off + pitch + 1023) / 1024 * 1024;
    return slot_off + 2 * (size_t)freg_slot_bytes(T, PBK);
}

bool freg_shape_supported(int T, int KS) { return (T == 9 && (KS == 2 || KS == 4 || KS == 8)) || (T == 25 && KS == 2); }

int launch_igemm_freg(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, void* out, hipStream_t s)
{
    if (g.kind != PLAN_MFMA_FREG || g.MR != 32) return ICV_ERR_UNSUPPORTED;
    const int KS = g.KCB / 32, T = g.T;
    if (!freg_shape_supported(T, KS)) return ICV_ERR_UNSUPPORTED;
    FregArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.a = (const uint8_t*)input;
    a.w = (const uint8_t*)packed;
    a.rec = (const int4*)ind;
    a.ent = (const uint16_t*)(a.rec + g.img_tiles);
    a.out = out;
    a.q = make_range_geom(p->Hin, p->Win, g.Hout, g.Wout, p->SY, p->SX, p->DY, p->DX, p->PT, p->PL, p->R, p->S);
    a.M = g.M;
    a.K = p->K; a.out_stride = g.out_stride;
    a.stride_bytes = g.in_stride * g.elem_bytes;
    a.last_pixel = (int32_t)((int64_t)p->N * p->Hin * p->Win - 1);
    a.n_blocks = (uint32_t)g.m_tiles;
    a.buf_blocks = (uint32_t)g.img_tiles;
    a.img_pixels = g.per_image ? (uint32_t)((int64_t)p->Hin * p->Win) : 0u;
    a.img_rows = (uint32_t)g.img_rows;
    a.by_buf = make_fast_div(a.buf_blocks);
    a.ent_bytes = (uint32_t)((size_t)g.img_tiles * T * 64);
    a.ring_rows = g.freg_ring;
    a.ep = g.ep;
    a.zero_fill = p->dtype == ICV_U8I8 ? 0x01010101u * (uint32_t)p->input_zero_point : 0u;
    const int WN = g.freg_wn, PBK = (4 / WN) * g.freg_mb;
    a.n_cg = (int32_t)g.n_tiles;
    // One workgroup per compute unit; the column groups share them.  A row range is at least one block.
    const int cus = device_cu_count();
    int64_t ranges = cus / a.n_cg;
    if (ranges < 1) ranges = 1;
    if (ranges > (int64_t)a.n_blocks) ranges = a.n_blocks;
    int64_t grid = ranges * a.n_cg;
    a.xcd_mode = 0;
    if (ranges % 8 == 0) a.xcd_mode = 1;          // grid / 8 workgroups per XCD, a whole number of row ranges each
    a.n_ranges = (int32_t)ranges;
    a.ranges_per_xcd = (int32_t)(ranges / 8);
    a.range_q = (uint32_t)(a.n_blocks / ranges);
    a.range_rem = (uint32_t)(a.n_blocks % ranges);
    a.cg_shift = -1;
    for (int sh = 0; sh < 16; sh++)
        if ((1 << sh) == a.n_cg) a.cg_shift = sh;
    const size_t lds = freg_lds_bytes(T, KS, PBK, a.ring_rows);
    if (lds > kLdsPerCu || (a.ring_rows & (a.ring_rows - 1)) || a.ring_rows < 64) return ICV_ERR_UNSUPPORTED;
    switch (p->dtype * 2 + (g.ep_plain ? 0 : 1)) {
    case ICV_BF16 * 2: return launch_freg_bf16(g, a, grid, lds, T, KS, s);
    case ICV_BF16 * 2 + 1: return launch_freg_bf16_fused(g, a, grid, lds, T, KS, s);
    case ICV_U8I8 * 2: return launch_freg_u8(g, a, grid, lds, T, KS, s);
    case ICV_U8I8 * 2 + 1: return launch_freg_u8_fused(g, a, grid, lds, T, KS, s);
    case ICV_F32 * 2: return launch_freg_f32(g, a, grid, lds, T, KS, s);
    case ICV_F32 * 2 + 1: return launch_freg_f32_fused(g, a, grid, lds, T, KS, s);
    }
    return ICV_ERR_UNSUPPORTED;
}

}  // namespace icv
