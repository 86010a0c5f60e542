// Internal declarations shared by the translation units of libicv.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "icv.h"

namespace icv {

// Which inner kernel serves a problem.
enum PlanKind : int32_t {
    PLAN_INVALID = 0,
    PLAN_GENERIC = 1,   // vector-ALU kernel, any C, any dtype
    PLAN_MFMA = 2,      // tensor-core indirect GEMM, C a multiple of the k-granule
    PLAN_MFMA_LOWC = 3, // tensor-core indirect GEMM for pixel rows of 8, 16 or 32 bytes (first-layer convolutions)
    PLAN_MFMA_FREG = 4  // tensor-core indirect GEMM with the filter in registers and the input window in an LDS ring
};

// Output stage of icv_conv2d_nhwc_fused, as the kernels see it (icv_epilogue with the bias pointer typed by use).
struct EpilogueArgs {
    const void* bias;          // K floats (float paths) or K int32 (u8i8); null: none
    float scale;               // requantisation scale (uint8 output)
    int32_t relu;              // 0 / 1
    int32_t out_kind;          // ICV_OUT_ACC / ICV_OUT_BF16 / ICV_OUT_U8
    int32_t out_zero_point;
    // uint8 activations with a zero point other than 128: the tensor-core kernels multiply (x - 128) * w (one XOR turns
    // a uint8 into that signed byte), and sum (x - zp) * w = sum (x - 128) * w + (128 - zp) * sum w, so the output
    // stage adds zp_shift * wsum[channel]: wsum holds each output channel's filter sum (icv_pack_filter writes it
    // behind the packed filter), zp_shift = 128 - zp.  Padding reads the zero row, which holds zp, and so contributes
    // (zp - 128) * w + (128 - zp) * w = 0.  Null / 0 otherwise.
    const int32_t* wsum;
    int32_t zp_shift;
};

// One output element through the output stage; `v` already includes the channel's bias (the caller reads it once
// per column, see output_bias).  `idx` counts elements of the output type.  All branches are uniform.
__device__ inline void emit_output(void* out, int64_t idx, float v, const EpilogueArgs& e)
{
    if (e.relu) v = v > 0.0f ? v : 0.0f;      // a select, and only with ReLU: a NaN accumulator stays NaN otherwise
    if (e.out_kind == ICV_OUT_BF16) ((__bf16*)out)[idx] = (__bf16)v;     // hardware conversion: nearest, ties to even
    else ((float*)out)[idx] = v;
}

__device__ inline void emit_output(void* out, int64_t idx, int32_t v, const EpilogueArgs& e)
{
    if (e.relu) v = v > 0 ? v : 0;
    if (e.out_kind == ICV_OUT_U8) {
        // clamp(rint((float)v * scale) + zero point, 0, 255); single-precision product, ties to even
        float r = rintf(__fmul_rn((float)v, e.scale));
        r = fminf(fmaxf(r, -1e9f), 1e9f);
        int32_t q = (int32_t)r + e.out_zero_point;
        q = q < 0 ? 0 : (q > 255 ? 255 : q);
        ((uint8_t*)out)[idx] = (uint8_t)q;
    } else {
        ((int32_t*)out)[idx] = v;
    }
}

// bias of output channel `col` in the accumulator's type (0 without a bias or past the last channel)
template <typename T>
__device__ inline T output_bias(const EpilogueArgs& e, int32_t col, int32_t K)
{
    T b = e.bias && col < K ? ((const T*)e.bias)[col] : (T)0;
    if (e.wsum && col < K) b += (T)(e.zp_shift * e.wsum[col]);
    return b;
}

// Geometry derived once per call from icv_conv_params (host side).
struct Geometry {
    int32_t Hout, Wout;
    int64_t M;            // N*Hout*Wout, GEMM rows
    int32_t T;            // R*S kernel elements ("taps")
    int32_t elem_bytes;   // input / filter element size
    int32_t in_stride;    // elements between input pixels
    int32_t out_stride;   // elements between output pixels
    // plan
    int32_t kind;         // PlanKind
    int32_t variant;      // index into the tile-variant table (MFMA kinds)
    int32_t MR, NR;       // workgroup tile: rows (output pixels) x columns (output channels)
    int32_t KCB;          // bytes of one A/B row per pipeline stage | LOWC: padded reduction bytes per row
    int32_t stages_per_tap;  // C*elem_bytes / KCB (MFMA)        | 1
    int32_t taps_per_stage;  // 1                                | KCB / 8 (LOWC)
    int32_t n_stages;        // pipeline stages in the reduction
    int64_t m_tiles, n_tiles; // row tiles the kernels walk, column tiles
    // Row tiles never straddle an "image" of img_rows output pixels: with a batch-independent indirection buffer an
    // image is one batch element (img_rows = Hout*Wout, the buffer describes img_tiles tiles and the kernels add
    // batch index * image_bytes to what the entries name), otherwise the whole batch is a single image of M rows.
    int32_t per_image;
    int64_t img_tiles, img_rows, image_bytes;
    int32_t ring;            // forced LDS ring depth (0: launcher decides)
    int32_t blocks_per_cu;   // forced co-resident workgroups per CU (0: launcher decides)
    int32_t gemm_on_input;   // 1: 1x1 stride-1 unpadded convolution run as a plain GEMM on the input tensor
    int32_t group;           // forced kernel elements per pipeline stage of the pixel-range kernel (0: launcher decides)
    int32_t patch_rows;      // > 0: the tile's input pixel range is kept in LDS, this many pixel rows reserved
                             // (short-row plan: > 0 when the buffer also holds the compact 16-bit entries)
    uint32_t zero_row_number;   // what the 16-bit entries hold for the zero row
    int32_t cc_major;        // 1: stage = chunk * T + tap (channel chunks outermost), 0: stage = tap * chunks + chunk
    // filter-in-registers plan: column blocks per workgroup (1, 2, 4), row blocks per wavefront and pass, ring rows
    int32_t freg_wn, freg_mb, freg_ring;
    const char* name;
    EpilogueArgs ep;         // output stage of this call (plain: no bias, no ReLU, accumulator type)
    bool ep_plain;
    int64_t wsum_offset;  // uint8 tensor-core plans: byte offset of the K filter sums in the packed-filter buffer, else -1
};

// Upper bound on the number of consecutive input pixels spanned by the valid indirection entries of any
// `rows` consecutive output pixels.
int64_t tile_span_bound(const icv_conv_params* p, int64_t Hout, int64_t Wout, int64_t rows);

// Fills g; returns ICV_OK / ICV_ERR_INVALID_ARG / ICV_ERR_UNSUPPORTED.
int make_geometry(const icv_conv_params* p, Geometry* g);

void set_hip_error(hipError_t e);

#define ICV_HIP_CHECK(expr)                        \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) {                    \
            ::icv::set_hip_error(e_);              \
            return ICV_ERR_HIP;                    \
        }                                          \
    } while (0)

// Kernel launchers (each returns an icv_status).
int launch_zero_row(const icv_conv_params* p, const Geometry& g, void* zero_row, hipStream_t s);
int launch_pack_filter(const icv_conv_params* p, const Geometry& g, const void* filt, void* packed, hipStream_t s);
int launch_build_indirection(const icv_conv_params* p, const Geometry& g, int32_t* ind, hipStream_t s);
int launch_im2col(const icv_conv_params* p, const Geometry& g, const void* input, void* ws, hipStream_t s);

// a_direct = false: rows of A come from the indirection buffer (the method);
// a_direct = true : A is the dense [M][T*C] patch matrix with constant row stride (ablation GEMM).
// The tensor-core kernel has a third mode: the input tensor itself as the dense matrix (1x1, stride 1, no padding).
enum AMode : int { A_GATHERED = 0, A_DENSE_WORKSPACE = 1, A_DENSE_INPUT = 2 };
int launch_igemm_mfma(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, const void* zero_row, void* out, int a_mode, hipStream_t s);
int launch_igemm_patch(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                       const int32_t* ind, void* out, hipStream_t s);
bool patch_variant_supported(int variant);
bool patch_variant_supported_f32(int variant);      // the tiles the pixel-range kernel has for fp32 tensors
int launch_igemm_freg(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, void* out, hipStream_t s);
bool freg_shape_supported(int T, int KS);
size_t freg_lds_bytes(int T, int KS, int PBK, int ring_rows);
size_t patch_lds_bytes(int NR, int KCB, int ring, int cap_units, int ent_copies, int nbuf);
int launch_igemm_lowc(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, const void* zero_row, void* out, bool a_direct, hipStream_t s);
int launch_igemm_generic(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                         const int32_t* ind, const void* zero_row, void* out, bool a_direct, hipStream_t s);

// Tile variants of the tensor-core kernel (host-visible table).
struct TileVariant {
    int32_t MR, NR, WM, WN;
    const char* tag;
};
// Test hooks in icv_conv_params::plan above the public bits (icv.h says they must be 0; the library's own tests set
// them to run every tile and pipeline shape on problems small enough for the CPU oracle): bits 8-11 tile
// (1 + index into kTileVariants), bits 12-15 LDS ring depth of the gathering kernel (2..12), bits 16-17 workgroups
// per compute unit (1, 2), bits 18-19 stage width (1: 64 bytes, 2: 128 bytes), bits 20-22 kernel elements per
// pipeline stage of the pixel-range kernel.
extern const TileVariant kTileVariants[];
extern const int kNumTileVariants;

}  // namespace icv
