// Host side of libicv.so: argument validation, geometry / plan selection and the C entry points.
#include "icv_internal.h"
#include "icv_pixel_range.h"

namespace icv {

static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

// Tile variants of the tensor-core kernel: workgroup tile MR x NR, split over a WM x WN grid of
// wavefronts.  Index + 1 is what icv_conv_params::plan selects.
const TileVariant kTileVariants[] = {
    {128, 64, 2, 2, "128x64_c2x2"},
    {128, 128, 2, 2, "128x128_c2x2"},
    {256, 64, 4, 1, "256x64_c4x1"},
    {256, 64, 4, 2, "256x64_c4x2"},
    {64, 64, 2, 2, "64x64_c2x2"},
    {256, 128, 4, 2, "256x128_c4x2"},
    {128, 128, 4, 2, "128x128_c4x2"},
};
const int kNumTileVariants = (int)(sizeof(kTileVariants) / sizeof(kTileVariants[0]));

static int64_t out_extent(int64_t in, int64_t lo, int64_t hi, int64_t dil, int64_t k, int64_t stride)
{
    const int64_t span = in + lo + hi - dil * (k - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

// bytes of the packed filter proper (the uint8 tensor-core plans append the filter sums, Geometry::wsum_offset)
static size_t packed_filter_base_bytes(const icv_conv_params* p, const Geometry& g)
{
    if (g.kind == PLAN_MFMA_LOWC) return (size_t)g.n_tiles * g.NR * g.KCB;
    return (size_t)g.n_tiles * g.NR * g.T * p->C * g.elem_bytes;
}

int64_t tile_span_bound(const icv_conv_params* p, int64_t Hout, int64_t Wout, int64_t rows)
{
    // Pixel index of entry (m, tap) before clipping: q(m) + ky*DY*Win + kx*DX with
    // q(m) = (n*Hin + oy*SY - PT)*Win + ox*SX - PL.  Along consecutive m, q moves by SX inside an output row, by
    // `rw` at the end of a row and by `iw` at the end of an image; max q - min q over a window is at most the sum
    // of the absolute steps.  Clipped (padding) entries only remove pixels from the set.
    const int64_t Win = p->Win, Hin = p->Hin, SX = p->SX, SY = p->SY;
    const int64_t rw = SY * Win - (Wout - 1) * SX;
    const int64_t iw = Hin * Win - (Hout - 1) * SY * Win - (Wout - 1) * SX;
    const int64_t arw = rw < 0 ? -rw : rw, aiw = iw < 0 ? -iw : iw;
    int64_t nrw = 0, niw = 0;
    if (rows >= 2) {
        nrw = (rows - 2) / Wout + 1;
        niw = (rows - 2) / (Hout * Wout) + 1;
        if (nrw > rows - 1) nrw = rows - 1;
        if (niw > rows - 1) niw = rows - 1;
    }
    const int64_t walk = SX * (rows - 1) + nrw * (arw > SX ? arw - SX : 0) + niw * (aiw > SX ? aiw - SX : 0);
    // The closed-form window ends of icv_pixel_range.h are clamped into the image, which can move them away from the
    // unclipped positions when the padding exceeds the kernel's reach: the lower end by at most `lo`, the upper by `hi`.
    const int64_t x0max = (Wout - 1) * SX - p->PL, x1min = (int64_t)(p->S - 1) * p->DX - p->PL;
    int64_t lo = x0max - (Win - 1), hi = -x1min;
    const int64_t below = ((Hout - 1) * SY - p->PT) * Win + x0max - Hin * Win + 1;
    const int64_t above = ((int64_t)p->PT - (int64_t)(p->R - 1) * p->DY) * Win - x1min;
    lo = lo > below ? lo : below;
    hi = hi > above ? hi : above;
    return walk + (int64_t)(p->R - 1) * p->DY * Win + (int64_t)(p->S - 1) * p->DX + 1 + (lo > 0 ? lo : 0) + (hi > 0 ? hi : 0);
}

static const char* kGenericNames[3] = {"generic_f32", "generic_bf16", "generic_u8i8"};
static const char* kLowcNames[2] = {"mfma_bf16_lowc_64x64", "mfma_i8_lowc_64x64"};
// filter in registers: [dtype][column blocks per workgroup 1, 2, 4][row blocks per wavefront and pass 1, 2]
static const char* kFregNames[3][3][2] = {
    {{"mfma_f32_freg_w1m1", "mfma_f32_freg_w1m2"}, {"mfma_f32_freg_w2m1", "mfma_f32_freg_w2m2"},
     {"mfma_f32_freg_w4m1", "mfma_f32_freg_w4m2"}},
    {{"mfma_bf16_freg_w1m1", "mfma_bf16_freg_w1m2"}, {"mfma_bf16_freg_w2m1", "mfma_bf16_freg_w2m2"},
     {"mfma_bf16_freg_w4m1", "mfma_bf16_freg_w4m2"}},
    {{"mfma_i8_freg_w1m1", "mfma_i8_freg_w1m2"}, {"mfma_i8_freg_w2m1", "mfma_i8_freg_w2m2"},
     {"mfma_i8_freg_w4m1", "mfma_i8_freg_w4m2"}},
};
// [dtype][tile]; the pixel-range kernel has every tile, the gathering kernel (and the plain GEMM it doubles as)
// those with an empty name missing
static const char* kPatchNames[3][7] = {
    {"mfma_bf16_128x64_c2x2_patch", "mfma_bf16_128x128_c2x2_patch", "mfma_bf16_256x64_c4x1_patch", "mfma_bf16_256x64_c4x2_patch",
     "mfma_bf16_64x64_c2x2_patch", "mfma_bf16_256x128_c4x2_patch", "mfma_bf16_128x128_c4x2_patch"},
    {"mfma_i8_128x64_c2x2_patch", "mfma_i8_128x128_c2x2_patch", "mfma_i8_256x64_c4x1_patch", "mfma_i8_256x64_c4x2_patch",
     "mfma_i8_64x64_c2x2_patch", "mfma_i8_256x128_c4x2_patch", "mfma_i8_128x128_c4x2_patch"},
    {"mfma_f32_128x64_c2x2_patch", "", "mfma_f32_256x64_c4x1_patch", "", "mfma_f32_64x64_c2x2_patch", "", "mfma_f32_128x128_c4x2_patch"},
};
static const char* kGemmNames[3][7] = {
    {"gemm_bf16_128x64_c2x2_p4", "gemm_bf16_128x128_c2x2_p4", "", "gemm_bf16_256x64_c4x2_p8", "gemm_bf16_64x64_c2x2_p4", "", ""},
    {"gemm_i8_128x64_c2x2_p4", "gemm_i8_128x128_c2x2_p4", "", "gemm_i8_256x64_c4x2_p8", "gemm_i8_64x64_c2x2_p4", "", ""},
    {"gemm_f32_128x64_c2x2_p4", "gemm_f32_128x128_c2x2_p4", "", "gemm_f32_256x64_c4x2_p8", "gemm_f32_64x64_c2x2_p4", "", ""},
};
static const char* kMfmaNames[3][7] = {
    {"mfma_bf16_128x64_c2x2_p4", "mfma_bf16_128x128_c2x2_p4", "", "mfma_bf16_256x64_c4x2_p8", "mfma_bf16_64x64_c2x2_p4", "", ""},
    {"mfma_i8_128x64_c2x2_p4", "mfma_i8_128x128_c2x2_p4", "", "mfma_i8_256x64_c4x2_p8", "mfma_i8_64x64_c2x2_p4", "", ""},
    {"mfma_f32_128x64_c2x2_p4", "mfma_f32_128x128_c2x2_p4", "", "mfma_f32_256x64_c4x2_p8", "mfma_f32_64x64_c2x2_p4", "", ""},
};


int make_geometry(const icv_conv_params* p, Geometry* g)
{
    if (!p || !g) return ICV_ERR_INVALID_ARG;
    if (p->N < 1 || p->Hin < 1 || p->Win < 1 || p->C < 1 || p->K < 1 || p->R < 1 || p->S < 1) return ICV_ERR_INVALID_ARG;
    if (p->SY < 1 || p->SX < 1 || p->DY < 1 || p->DX < 1) return ICV_ERR_INVALID_ARG;
    if (p->PT < 0 || p->PL < 0 || p->PB < 0 || p->PR < 0) return ICV_ERR_INVALID_ARG;
    if (p->dtype != ICV_F32 && p->dtype != ICV_BF16 && p->dtype != ICV_U8I8) return ICV_ERR_INVALID_ARG;
    if (p->in_pixel_stride < 0 || p->out_pixel_stride < 0) return ICV_ERR_INVALID_ARG;
    if (p->in_pixel_stride != 0 && p->in_pixel_stride < p->C) return ICV_ERR_INVALID_ARG;
    if (p->out_pixel_stride != 0 && p->out_pixel_stride < p->K) return ICV_ERR_INVALID_ARG;
    if (p->dtype == ICV_U8I8 && (p->input_zero_point < 0 || p->input_zero_point > 255)) return ICV_ERR_INVALID_ARG;
    // plan (icv.h): bits 0-2 algorithm, bit 3 batch-independent buffer; the test hooks of icv_internal.h above them
    const int algo = p->plan & 7, plan_per_image = (p->plan >> 3) & 1;
    const int hook_tile = (p->plan >> 8) & 15, plan_ring = (p->plan >> 12) & 15, plan_per_cu = (p->plan >> 16) & 3,
              plan_kcb = (p->plan >> 18) & 3, plan_group = (p->plan >> 20) & 7;
    if (p->plan < 0 || p->plan >= (1 << 23) || (p->plan & 0xF0) != 0 || algo > ICV_PLAN_FILTER_REGS ||
        hook_tile > kNumTileVariants || (hook_tile && algo == ICV_PLAN_VECTOR_ALU) || plan_ring == 1 || plan_ring > 12 ||
        plan_per_cu > 2 || plan_kcb > 2)
        return ICV_ERR_INVALID_ARG;
    // 0: the library chooses; 1: rows gathered per kernel element; 2: the tile's pixel range in LDS; 3: filter in registers
    const int plan_staging = algo == ICV_PLAN_GATHER ? 1 : (algo == ICV_PLAN_WINDOW ? 2 : (algo == ICV_PLAN_FILTER_REGS ? 3 : 0));
    const int plan_kernel = algo == ICV_PLAN_VECTOR_ALU ? 1 : (hook_tile ? hook_tile + 1 : 0);

    const int64_t Hout = out_extent(p->Hin, p->PT, p->PB, p->DY, p->R, p->SY);
    const int64_t Wout = out_extent(p->Win, p->PL, p->PR, p->DX, p->S, p->SX);
    if (Hout < 1 || Wout < 1) return ICV_ERR_INVALID_ARG;
    // entries are int32 byte offsets into the input tensor, so it must be smaller than 2 GiB
    {
        const int64_t esz = p->dtype == ICV_F32 ? 4 : (p->dtype == ICV_BF16 ? 2 : 1);
        const int64_t stride = p->in_pixel_stride ? p->in_pixel_stride : p->C;
        if ((int64_t)p->N * p->Hin * p->Win * stride * esz >= (1ll << 31)) return ICV_ERR_INVALID_ARG;
    }
    const int64_t M = (int64_t)p->N * Hout * Wout;
    const int64_t T = (int64_t)p->R * p->S;
    if (M >= (1ll << 31) || T > 4096 || M * T >= (1ll << 40)) return ICV_ERR_INVALID_ARG;
    if ((int64_t)T * p->C >= (1ll << 31)) return ICV_ERR_INVALID_ARG;

    g->Hout = (int32_t)Hout;
    g->Wout = (int32_t)Wout;
    g->M = M;
    g->T = (int32_t)T;
    g->elem_bytes = p->dtype == ICV_F32 ? 4 : (p->dtype == ICV_BF16 ? 2 : 1);
    g->in_stride = p->in_pixel_stride ? p->in_pixel_stride : p->C;
    g->out_stride = p->out_pixel_stride ? p->out_pixel_stride : p->K;
    g->patch_rows = 0;
    g->zero_row_number = 0;
    g->cc_major = 0;
    g->group = plan_group;
    g->gemm_on_input = 0;
    g->ep.bias = nullptr; g->ep.scale = 1.0f; g->ep.relu = 0; g->ep.out_kind = ICV_OUT_ACC; g->ep.out_zero_point = 0;
    g->ep.wsum = nullptr; g->ep.zp_shift = 0;
    g->ep_plain = true;

    // ---- plan: which kernel, which tile
    const int64_t row_bytes = (int64_t)p->C * g->elem_bytes;        // bytes of one gathered A row
    const int64_t stride_bytes = (int64_t)g->in_stride * g->elem_bytes;
    // fp32 tensors (section 3.1's own precision) run on the matrix cores through the pixel-range kernel (four of its
    // tiles) and the gathering kernel / plain GEMM
    const bool f32 = p->dtype == ICV_F32;
    bool mfma_ok = row_bytes % 64 == 0 && stride_bytes % 16 == 0;
    if (plan_kernel == 1) mfma_ok = false;                                      // forced vector-ALU kernel
    int variant = -1;
    int patch_rows = 0, patch_kcb = 0;
    // LDS-resident pixel range: worthwhile when several kernel elements re-read the rows, possible when the pixel
    // stride is a power of two (entry -> LDS row is a shift) and two patch buffers fit beside the other buffers
    auto try_patch = [&](int v, bool need_two = false) {
        if (plan_staging == 1 || T < 4 || !patch_variant_supported(v) || (f32 && !patch_variant_supported_f32(v))) return false;
        if ((stride_bytes & (stride_bytes - 1)) != 0) return false;
        const TileVariant& tv = kTileVariants[v];
        if ((int64_t)tv.MR * T * 2 > 24 * 1024) return false;     // two tiles' row numbers (uint16) stay in LDS
        const int64_t rows = tile_span_bound(p, Hout, Wout, tv.MR);
        const int ent_copies = (int)((tv.MR * T * 2 + 1023) / 1024);
        const int kcb_max = (row_bytes % 128 == 0 && plan_kcb != 1) ? 128 : 64;
        for (int kcb = kcb_max; kcb >= 64; kcb -= 64) {
            const int64_t cap_units = (rows * kcb + 1023) / 1024;
            if (cap_units >= 4096) continue;
            // one workgroup per compute unit with double buffers, or two with single buffers (64-wide tiles and
            // the tiles with four consumer wavefronts)
            const bool fits_one = !need_two && patch_lds_bytes(tv.NR, kcb, 2, (int)cap_units, ent_copies, 2) <= 160 * 1024;
            const bool fits_two = (tv.NR == 64 || tv.WM * tv.WN == 4) && plan_per_cu != 1 &&
                                  patch_lds_bytes(tv.NR, kcb, 2, (int)cap_units, ent_copies, 1) <= 80 * 1024;
            if (fits_two || fits_one) {
                variant = v; patch_rows = (int)rows; patch_kcb = kcb;
                return true;
            }
        }
        return false;
    };
    // Measured on MI355X.  64-wide filters: 256 x 64 tiles (four consumer wavefronts with 64 x 64 blocks: one LDS
    // fragment read per MFMA instead of three per two), two workgroups per compute unit when the single-buffer
    // layout fits half the LDS.  Wider filters: 256 x 128 tiles of 64 x 64 wavefront blocks when every compute unit
    // still gets a tile, else 128 x 128 tiles.  A grid that leaves compute units idle costs more than a smaller
    // tile's lower efficiency (one 128 x 128 tile keeps a compute unit busy as long as two 128 x 64 tiles keep two),
    // so the tile is halved until the grid fills the chip: 128 x 64, then 64 x 64.  128-byte stages when the patch
    // fits, else 64-byte ones (the launcher then puts several kernel elements into a stage).
    // A batch-independent buffer must have the same layout for every N, so its tile is chosen as for a batch
    // that fills the chip.
    const int64_t kCus = 256;
    auto tiles_of = [&](int64_t mr, int64_t nr) { return ((M + mr - 1) / mr) * ((p->K + nr - 1) / nr); };
    // candidates from the largest tile down; the first whose grid fills the chip is the preferred one
    int order[5], n_order = 0;
    if (p->K <= 64) {
        order[n_order++] = 2;                                                        // 256 x 64, 64 x 64 blocks
        order[n_order++] = 3;                                                        // 256 x 64, 64 x 32 blocks
    } else {
        // 256 x 128 when every compute unit gets one -- but not when some get a second one and others none
        // (between one and two rounds): 128 x 128 tiles then spread the same work more evenly (measured)
        const int64_t t6 = tiles_of(256, 128);
        if (!plan_per_image && t6 >= kCus && !(t6 > kCus && t6 <= 2 * kCus)) order[n_order++] = 5;     // 256 x 128
        order[n_order++] = 6;                                                        // 128 x 128, 32 x 64 blocks
        order[n_order++] = 1;                                                        // 128 x 128, 64 x 64 blocks
    }
    order[n_order++] = 0;                                                            // 128 x 64
    order[n_order++] = 4;                                                            // 64 x 64
    int first = 0;
    if (!plan_per_image) {
        auto fills = [&](int v) {
            const TileVariant& tv = kTileVariants[v];
            // 128 x 128 tiles run one workgroup per compute unit and want one and a half rounds before their higher
            // efficiency pays (measured); 64-wide ones run two side by side
            return tiles_of(tv.MR, tv.NR) * 2 >= (tv.MR == 128 && tv.NR == 128 ? 3 * kCus : 2 * kCus);
        };
        while (first < n_order - 1 && !fills(order[first])) ++first;
    }
    const bool forced = plan_staging == 2;
    if (mfma_ok) {
        if (plan_kernel >= 2) {
            variant = plan_kernel - 2;
            if (!try_patch(variant) && forced) return ICV_ERR_UNSUPPORTED;
        } else {
            // the pixel-range kernel with the preferred tile, else with the next smaller one that fits its LDS
            // (128 x 128: four consumer wavefronts with 64 x 64 blocks when two such workgroups share a compute
            // unit, else eight with 32 x 64 blocks -- measured)
            int i = first;
            while (i < n_order && !(order[i] == 6 && try_patch(1, true)) && !try_patch(order[i])) ++i;
            if (i == n_order) {
                if (plan_staging == 2) return ICV_ERR_UNSUPPORTED;
                // rows gathered per kernel element: 128 x 128 as 2 x 2 wavefronts (measured), 256-row tiles only
                // when a tile's entries fit their LDS budget
                variant = order[first];
            }
        }
        if (!patch_rows) {
            // the gathering kernel has four of the tiles: 128 x 128 as 2 x 2 wavefronts (measured), 256 x 64 with
            // eight producer wavefronts, and 256-row tiles only when a tile's entries fit their LDS budget
            if (variant == 5 || variant == 6) variant = 1;
            if (variant == 2) variant = 3;
            if (variant == 3 && (int64_t)256 * T * 4 > 24 * 1024) variant = 0;
            // large kernels (7x7): 128-row tiles' entries do not fit either, 64-row tiles' do -- unless a tile was asked for
            if (plan_kernel < 2 && (variant == 0 || variant == 1) && (int64_t)128 * T * 4 > 24 * 1024) variant = 4;
        }
        // a workgroup keeps two tiles' worth of entries in LDS: 2 * MR*T int32 (plus padding)
        if (mfma_ok && !patch_rows && (int64_t)kTileVariants[variant].MR * T * 4 > 24 * 1024) mfma_ok = false;
    }
    // Filter in registers, input window in an LDS ring: wherever the kernel applies -- kernel sizes and row widths it
    // is instantiated for, a window of two passes that fits LDS, 16-bit pixel numbers per 32-row block.  Measured
    // against the pixel-range kernel on grids of 3x3 (64 and 128 bf16 channels, 128 and 256 uint8 channels) and 5x5
    // problems from one 7x7 image to batch 64 of 56x56, 32 to 256 output channels: 5 to 130 % faster on all but a
    // handful, which are level (within 3 %).
    int freg_wn = 0, freg_mb = 0, freg_ring = 0;
    if (plan_kernel == 0 && (plan_staging == 3 || plan_staging == 0) && row_bytes % 32 == 0 &&
        stride_bytes % 16 == 0 && freg_shape_supported((int)T, (int)(row_bytes / 32)) &&
        tile_span_bound(p, Hout, Wout, 32) < 65535) {
        const int wn = p->K <= 32 ? 1 : (p->K <= 64 ? 2 : 4);
        for (int mb = 2; mb >= 1 && !freg_mb; --mb) {
            const int pbk = (4 / wn) * mb;
            const int64_t need = tile_span_bound(p, Hout, Wout, 2 * pbk * 32) + 16;     // + what a 1 KB copy overshoots
            int64_t ring = 64;
            while (ring < need) ring *= 2;
            if (ring > (1 << 20) || freg_lds_bytes((int)T, (int)(row_bytes / 32), pbk, (int)ring) > 160 * 1024) continue;
            freg_wn = wn; freg_mb = mb; freg_ring = (int)ring;
        }
        if (!freg_mb && plan_staging == 3) return ICV_ERR_UNSUPPORTED;
    } else if (plan_staging == 3) {
        return ICV_ERR_UNSUPPORTED;
    }
    // very short rows (first-layer convolutions): the whole reduction of a tile is gathered at once
    const bool lowc_ok = p->dtype != ICV_F32 && plan_kernel == 0 &&
                         (row_bytes == 8 || row_bytes == 16 || row_bytes == 32) && stride_bytes % row_bytes == 0 &&
                         T * row_bytes <= 608;
    g->freg_wn = freg_wn; g->freg_mb = freg_mb; g->freg_ring = freg_ring;
    if (freg_mb) {
        g->kind = PLAN_MFMA_FREG;
        g->variant = -1;
        g->MR = 32;
        g->NR = 32 * freg_wn;
        g->KCB = (int32_t)row_bytes;
        g->ring = 0;
        g->blocks_per_cu = 0;
        g->stages_per_tap = 1;
        g->taps_per_stage = 1;
        g->n_stages = g->T;
        g->zero_row_number = 0xFFFFu;
        g->name = kFregNames[p->dtype][freg_wn == 4 ? 2 : freg_wn - 1][freg_mb - 1];
    } else if (lowc_ok) {
        g->kind = PLAN_MFMA_LOWC;
        g->variant = -1;
        g->MR = 64;
        g->NR = 64;
        g->KCB = (int32_t)((T * row_bytes + 31) / 32 * 32);
        g->ring = 0;
        g->blocks_per_cu = 0;
        g->stages_per_tap = 1;
        g->taps_per_stage = g->T;
        g->n_stages = 1;
        g->name = kLowcNames[p->dtype == ICV_U8I8 ? 1 : 0];
        // compact entries (16-bit pixel numbers inside the tile's range) when every tile's range is short enough;
        // plan "rows gathered per kernel element" keeps the int32 offsets, for comparison
        const int64_t span = tile_span_bound(p, Hout, Wout, 64);
        if (plan_staging != 1 && span < 65535 && stride_bytes < (1 << 24)) {
            g->patch_rows = (int32_t)span;
            g->zero_row_number = 65535u;
        }
    } else if (mfma_ok) {
        const TileVariant& tv = kTileVariants[variant];
        g->kind = PLAN_MFMA;
        g->variant = variant;
        g->MR = tv.MR;
        g->NR = tv.NR;
        g->KCB = row_bytes % 128 == 0 ? 128 : 64;
        if (plan_kcb == 1) g->KCB = 64;
        if (patch_rows) g->KCB = patch_kcb;
        g->patch_rows = patch_rows;
        // the zero row sits after the patch buffer, whose size is whole 1 KB pieces
        g->zero_row_number = patch_rows ? (uint32_t)((((int64_t)patch_rows * g->KCB + 1023) / 1024) * 1024 / g->KCB) : 0u;
        g->cc_major = patch_rows ? 1 : 0;
        g->ring = plan_ring;
        g->blocks_per_cu = plan_per_cu;
        g->stages_per_tap = (int32_t)(row_bytes / g->KCB);
        g->taps_per_stage = 1;
        g->n_stages = g->T * g->stages_per_tap;
        const int name_row = f32 ? 2 : (p->dtype == ICV_U8I8 ? 1 : 0);
        g->name = (patch_rows ? kPatchNames : kMfmaNames)[name_row][variant];
        // Section 3.2, closing paragraph: a 1x1 stride-1 convolution needs no im2col, the plain GEMM primitive has
        // the edge there and switching between the two primitives by convolution parameters is advised.  Its A matrix is the input tensor; the indirection buffer is built but not read.
        if (T == 1 && p->SY == 1 && p->SX == 1 && p->PT == 0 && p->PL == 0 && p->PB == 0 && p->PR == 0 &&
            plan_staging != 1) {
            g->gemm_on_input = 1;
            g->name = kGemmNames[name_row][variant];
        }
    } else {
        g->kind = PLAN_GENERIC;
        g->variant = -1;
        g->MR = 64;
        g->NR = 64;
        g->KCB = 0;
        g->ring = 0;
        g->blocks_per_cu = 0;
        g->stages_per_tap = 1;
        g->taps_per_stage = 1;
        g->n_stages = g->T;
        g->name = kGenericNames[p->dtype];
    }
    // the GEMM on the input tensor reads no entries, so it keeps the plain tiling
    g->per_image = plan_per_image && !g->gemm_on_input ? 1 : 0;
    g->img_rows = g->per_image ? Hout * Wout : M;
    g->img_tiles = (g->img_rows + g->MR - 1) / g->MR;
    g->image_bytes = g->per_image ? (int64_t)p->Hin * p->Win * stride_bytes : 0;
    g->m_tiles = g->per_image ? g->img_tiles * p->N : g->img_tiles;
    g->n_tiles = (p->K + g->NR - 1) / g->NR;
    // uint8 on the tensor cores: the filter sums of the zero-point term (EpilogueArgs) follow the packed filter
    g->wsum_offset = p->dtype == ICV_U8I8 && g->kind != PLAN_GENERIC ? (int64_t)((packed_filter_base_bytes(p, *g) + 15) / 16 * 16) : -1;
    return ICV_OK;
}

static bool aligned16(const void* ptr) { return ((uintptr_t)ptr & 15u) == 0; }

// Workspace of icv_conv2d_nhwc_im2col_static: part of the device image, so no call ever allocates it.  Every GPU the
// library runs on holds its own copy at its own address; in host code the array's name is only a handle for
// hipGetSymbolAddress, never an address to pass to a kernel.
constexpr size_t kStaticWorkspaceBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

static int static_workspace(void** out)
{
    static void* address[64] = {};        // per device ordinal; a race between threads stores the same value twice
    int dev = 0;
    ICV_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return ICV_ERR_UNSUPPORTED;
    if (!address[dev]) {
        void* ptr = nullptr;
        ICV_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return ICV_ERR_HIP;
        address[dev] = ptr;
    }
    *out = address[dev];
    return ICV_OK;
}

// The ablation path has no indirection buffer, so it tiles the whole batch as one image.  The tile, stage width and
// stage order stay those of the problem's own plan (batch-independent buffer or not), because the packed filter the
// caller passes was laid out by icv_pack_filter for exactly that plan.
static int make_ablation_geometry(const icv_conv_params* p, Geometry* g)
{
    const int st = make_geometry(p, g);
    if (st != ICV_OK) return st;
    // the packed filter of the filter-in-registers plan is laid out for that kernel alone; the ablation takes a plan
    // whose filter and tile the plain GEMM kernel reads (ICV_PLAN_GATHER always is one)
    if (g->kind == PLAN_MFMA_FREG) return ICV_ERR_UNSUPPORTED;
    if (g->kind == PLAN_MFMA && !kGemmNames[0][g->variant][0]) return ICV_ERR_UNSUPPORTED;      // a tile the GEMM lacks
    g->per_image = 0;
    g->img_rows = g->M;
    g->img_tiles = (g->M + g->MR - 1) / g->MR;
    g->m_tiles = g->img_tiles;
    g->image_bytes = 0;
    return ICV_OK;
}

}  // namespace icv

using namespace icv;

extern "C" {

int icv_output_size(const icv_conv_params* p, int32_t* Hout, int32_t* Wout)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (Hout) *Hout = g.Hout;
    if (Wout) *Wout = g.Wout;
    return ICV_OK;
}

size_t icv_indirection_bytes(const icv_conv_params* p)
{
    Geometry g;
    if (make_geometry(p, &g) != ICV_OK) return 0;
    const size_t n = (size_t)g.img_tiles * g.MR * g.T;
    // compact forms (block form of the filter-in-registers plan, range form of the pixel-range plans): a 16-byte
    // record per block or row tile, then 16-bit entries; else int32 entries
    if (g.kind == PLAN_MFMA_FREG || g.patch_rows) return (size_t)g.img_tiles * 16 + n * sizeof(uint16_t);
    return n * sizeof(int32_t);
}

size_t icv_packed_filter_bytes(const icv_conv_params* p)
{
    Geometry g;
    if (make_geometry(p, &g) != ICV_OK) return 0;
    if (g.wsum_offset >= 0) return (size_t)g.wsum_offset + ((size_t)p->K * 4 + 15) / 16 * 16;
    return packed_filter_base_bytes(p, g);
}

size_t icv_zero_row_bytes(const icv_conv_params* p)
{
    Geometry g;
    if (make_geometry(p, &g) != ICV_OK) return 0;
    return (((size_t)p->C * g.elem_bytes) + 15) / 16 * 16;
}

size_t icv_im2col_bytes(const icv_conv_params* p)
{
    Geometry g;
    if (make_ablation_geometry(p, &g) != ICV_OK) return 0;
    // rows padded to whole tiles so the GEMM kernel may read (and discard) the rows past M
    if (g.kind == PLAN_MFMA_LOWC) return (size_t)g.m_tiles * g.MR * g.KCB;
    return (size_t)g.m_tiles * g.MR * g.T * p->C * g.elem_bytes;
}

int64_t icv_indirection_index(const icv_conv_params* p, int64_t m, int32_t tap)
{
    Geometry g;
    if (make_geometry(p, &g) != ICV_OK) return -1;
    if (m < 0 || m >= g.img_tiles * g.MR || tap < 0 || tap >= g.T) return -1;
    return (m / g.MR) * ((int64_t)g.T * g.MR) + (int64_t)tap * g.MR + m % g.MR;
}

int icv_get_indirection_layout(const icv_conv_params* p, icv_indirection_layout* L)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!L) return ICV_ERR_INVALID_ARG;
    L->tile_rows = g.MR;
    L->tiles = g.img_tiles;
    if (g.kind == PLAN_MFMA_FREG) {
        L->entry_bytes = 2; L->zero_code = 0xFFFF; L->record_bytes = 16;
        L->records_at = 0; L->entries_at = g.img_tiles * 16; L->int32_entries_at = -1;
    } else if (g.patch_rows) {
        L->entry_bytes = 2; L->zero_code = (int32_t)g.zero_row_number; L->record_bytes = 16;
        L->records_at = 0; L->entries_at = g.img_tiles * 16; L->int32_entries_at = -1;
    } else {
        L->entry_bytes = 4; L->zero_code = 0; L->record_bytes = 0;
        L->int32_entries_at = 0; L->records_at = -1; L->entries_at = 0;
    }
    return ICV_OK;
}

int icv_row_pixel_range(const icv_conv_params* p, int64_t m0, int64_t m1, int64_t* first, int64_t* last)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (m0 < 0 || m1 < m0 || m1 >= g.M || !first || !last) return ICV_ERR_INVALID_ARG;
    const RangeGeom q = make_range_geom(p->Hin, p->Win, g.Hout, g.Wout, p->SY, p->SX, p->DY, p->DX, p->PT, p->PL, p->R, p->S);
    *first = lowest_pixel_from(q, decompose(q, (uint32_t)m0));
    *last = highest_pixel_upto(q, decompose(q, (uint32_t)m1));
    return ICV_OK;
}

int64_t icv_tile_span_bound(const icv_conv_params* p, int32_t rows)
{
    Geometry g;
    if (make_geometry(p, &g) != ICV_OK || rows < 1) return -1;
    return tile_span_bound(p, g.Hout, g.Wout, rows);
}

int icv_init_zero_row(const icv_conv_params* p, void* zero_row, void* stream)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!zero_row || !aligned16(zero_row)) return ICV_ERR_INVALID_ARG;
    return launch_zero_row(p, g, zero_row, (hipStream_t)stream);
}

int icv_pack_filter(const icv_conv_params* p, const void* filter_krsc, void* packed, void* stream)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!filter_krsc || !packed || !aligned16(packed) || !aligned16(filter_krsc)) return ICV_ERR_INVALID_ARG;
    return launch_pack_filter(p, g, filter_krsc, packed, (hipStream_t)stream);
}

int icv_setup_indirection(const icv_conv_params* p, void* indirection, void* stream)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!indirection || !aligned16(indirection)) return ICV_ERR_INVALID_ARG;
    return launch_build_indirection(p, g, (int32_t*)indirection, (hipStream_t)stream);
}

static int conv_common(const icv_conv_params* p, Geometry g, const void* a, const void* packed,
                       const int32_t* ind, const void* zero_row, void* out, bool a_direct, hipStream_t s)
{
    if (g.wsum_offset >= 0 && p->input_zero_point != 128) {
        // zero point other than 128: the output stage adds (128 - zp) * (the channel's filter sum)
        g.ep.wsum = (const int32_t*)((const uint8_t*)packed + g.wsum_offset);
        g.ep.zp_shift = 128 - p->input_zero_point;
        g.ep_plain = false;
    }
    if (g.kind == PLAN_MFMA_FREG) return a_direct ? ICV_ERR_UNSUPPORTED : launch_igemm_freg(p, g, a, packed, ind, out, s);
    if (g.kind == PLAN_MFMA && g.patch_rows && !a_direct) return launch_igemm_patch(p, g, a, packed, ind, out, s);
    if (g.kind == PLAN_MFMA)
        return launch_igemm_mfma(p, g, a, packed, ind, zero_row, out,
                                 a_direct ? A_DENSE_WORKSPACE : (g.gemm_on_input ? A_DENSE_INPUT : A_GATHERED), s);
    if (g.kind == PLAN_MFMA_LOWC) return launch_igemm_lowc(p, g, a, packed, ind, zero_row, out, a_direct, s);
    return launch_igemm_generic(p, g, a, packed, ind, zero_row, out, a_direct, s);
}

int icv_conv2d_nhwc(const icv_conv_params* p, const void* input, const void* packed_filter,
                    const void* indirection, const void* zero_row, void* output, void* stream)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!input || !packed_filter || !indirection || !zero_row || !output) return ICV_ERR_INVALID_ARG;
    if (!aligned16(input) || !aligned16(packed_filter) || !aligned16(indirection) || !aligned16(zero_row) ||
        !aligned16(output))
        return ICV_ERR_INVALID_ARG;
    return conv_common(p, g, input, packed_filter, (const int32_t*)indirection, zero_row, output, false,
                       (hipStream_t)stream);
}

int icv_conv2d_nhwc_fused(const icv_conv_params* p, const void* input, const void* packed_filter,
                          const void* indirection, const void* zero_row, const icv_epilogue* ep, void* output,
                          void* stream)
{
    Geometry g;
    const int st = make_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!input || !packed_filter || !indirection || !zero_row || !output || !ep) return ICV_ERR_INVALID_ARG;
    if (!aligned16(input) || !aligned16(packed_filter) || !aligned16(indirection) || !aligned16(zero_row) ||
        !aligned16(output))
        return ICV_ERR_INVALID_ARG;
    if (ep->relu != 0 && ep->relu != 1) return ICV_ERR_INVALID_ARG;
    if (ep->bias && ((uintptr_t)ep->bias & 3u)) return ICV_ERR_INVALID_ARG;
    const bool quantised = p->dtype == ICV_U8I8;
    if (ep->out_type != ICV_OUT_ACC && ep->out_type != (quantised ? ICV_OUT_U8 : ICV_OUT_BF16)) return ICV_ERR_INVALID_ARG;
    if (ep->out_type == ICV_OUT_U8 &&
        (!(ep->out_scale > 0.0f) || !(ep->out_scale < 3.0e38f) || ep->out_zero_point < 0 || ep->out_zero_point > 255))
        return ICV_ERR_INVALID_ARG;
    g.ep.bias = ep->bias;
    g.ep.scale = ep->out_scale;
    g.ep.relu = ep->relu;
    g.ep.out_kind = ep->out_type;
    g.ep.out_zero_point = ep->out_zero_point;
    g.ep_plain = !ep->bias && !ep->relu && ep->out_type == ICV_OUT_ACC;
    return conv_common(p, g, input, packed_filter, (const int32_t*)indirection, zero_row, output, false,
                       (hipStream_t)stream);
}

int icv_im2col(const icv_conv_params* p, const void* input, void* im2col_ws, void* stream)
{
    Geometry g;
    const int st = make_ablation_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!input || !im2col_ws || !aligned16(input) || !aligned16(im2col_ws)) return ICV_ERR_INVALID_ARG;
    return launch_im2col(p, g, input, im2col_ws, (hipStream_t)stream);
}

int icv_gemm_nhwc(const icv_conv_params* p, const void* im2col_ws, const void* packed_filter, void* output,
                  void* stream)
{
    Geometry g;
    const int st = make_ablation_geometry(p, &g);
    if (st != ICV_OK) return st;
    if (!im2col_ws || !packed_filter || !output) return ICV_ERR_INVALID_ARG;
    if (!aligned16(im2col_ws) || !aligned16(packed_filter) || !aligned16(output)) return ICV_ERR_INVALID_ARG;
    return conv_common(p, g, im2col_ws, packed_filter, nullptr, nullptr, output, true, (hipStream_t)stream);
}

int icv_conv2d_nhwc_im2col(const icv_conv_params* p, const void* input, const void* packed_filter,
                           void* im2col_ws, void* output, void* stream)
{
    const int st = icv_im2col(p, input, im2col_ws, stream);
    if (st != ICV_OK) return st;
    return icv_gemm_nhwc(p, im2col_ws, packed_filter, output, stream);
}

size_t icv_static_workspace_bytes(void) { return kStaticWorkspaceBytes; }

int icv_conv2d_nhwc_im2col_static(const icv_conv_params* p, const void* input, const void* packed_filter,
                                  void* output, void* stream)
{
    const size_t need = icv_im2col_bytes(p);
    if (need == 0) {
        Geometry g;
        const int st = make_geometry(p, &g);
        return st != ICV_OK ? st : ICV_ERR_UNSUPPORTED;
    }
    if (need > kStaticWorkspaceBytes) return ICV_ERR_UNSUPPORTED;
    void* ws = nullptr;
    const int st = static_workspace(&ws);
    if (st != ICV_OK) return st;
    return icv_conv2d_nhwc_im2col(p, input, packed_filter, ws, output, stream);
}

const char* icv_plan_name(const icv_conv_params* p)
{
    Geometry g;
    if (make_geometry(p, &g) != ICV_OK) return "";
    return g.name;
}

const char* icv_status_string(int status)
{
    switch (status) {
        case ICV_OK: return "ok";
        case ICV_ERR_INVALID_ARG: return "invalid argument";
        case ICV_ERR_UNSUPPORTED: return "unsupported problem";
        case ICV_ERR_HIP: return "HIP call failed";
        default: return "unknown status";
    }
}

int icv_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
