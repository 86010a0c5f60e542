// Vector-ALU indirect GEMM: serves fp32 and every shape the tensor-core kernels do not take (C not a
// multiple of the MFMA k-granule, unaligned pixel strides, zero points other than 128).
//
// It is Listing 3 with one output element per thread: for each kernel element load the row pointer from
// the indirection buffer (entry = byte offset from the input base; < 0 -> the zero row), take the C-long dot product with the filter row,
// accumulate.  A block is 4 output pixels x 64 output channels; the 64 lanes of a wavefront share the
// A row (a broadcast read) and read neighbouring filter elements (the filter is packed with the output channels innermost).
#include <type_traits>
#include "icv_internal.h"

namespace icv {

struct GenericArgs {
    const void* a;         // input tensor, or the im2col matrix when a_direct
    const void* w;         // [T * C][K padded]
    const int32_t* ind;    // [m tile][tap][64]
    const void* zero_row;
    void* out;
    int64_t M;
    int32_t K, T, C, in_stride, out_stride, zero_point, a_direct;
    int64_t img_rows, image_bytes;
    int64_t kp;            // K padded: filter elements between two reduction indices
    EpilogueArgs ep;
};

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(uint16_t bf16_bits) { return __uint_as_float((uint32_t)bf16_bits << 16); }

template <typename TIn, typename TW, typename TAcc>
__global__ __launch_bounds__(256) void k_igemm_generic(GenericArgs g)
{
    const int64_t m = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int32_t oc = blockIdx.y * 64 + (threadIdx.x & 63);
    if (m >= g.M || oc >= g.K) return;
    const TIn* in = (const TIn*)g.a;
    const TW* w = (const TW*)g.w + oc;
    // batch-independent buffer: the entries are those of pixel m % img_rows, the rows they name lie in batch
    // element m / img_rows (img_rows = M and image_bytes = 0 otherwise)
    const int64_t img = m / g.img_rows, mi = m - img * g.img_rows;
    const int32_t* ent = g.a_direct ? nullptr : g.ind + (mi >> 6) * ((int64_t)g.T * 64) + (mi & 63);
    const uint8_t* a_img = (const uint8_t*)in + img * g.image_bytes;
    TAcc acc = 0;
    for (int32_t t = 0; t < g.T; t++) {
        const TIn* row;
        if (g.a_direct) {
            row = in + (m * g.T + t) * (int64_t)g.C;
        } else {
            const int32_t e = ent[(int64_t)t * 64];
            row = e < 0 ? (const TIn*)g.zero_row : (const TIn*)(a_img + e);   // byte offset entry
        }
        const TW* wr = w + (int64_t)t * g.C * g.kp;
        for (int32_t c = 0; c < g.C; c++) {
            if constexpr (std::is_integral<TAcc>::value) {
                acc += ((int32_t)row[c] - g.zero_point) * (int32_t)wr[c * g.kp];
            } else {
                acc = fmaf(to_float(row[c]), to_float(wr[c * g.kp]), acc);
            }
        }
    }
    emit_output(g.out, m * g.out_stride + oc, acc + output_bias<TAcc>(g.ep, oc, g.K), g.ep);
}

int launch_igemm_generic(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                         const int32_t* ind, const void* zero_row, void* out, bool a_direct, hipStream_t s)
{
    GenericArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.a = input; a.w = packed; a.ind = ind; a.zero_row = zero_row; a.out = out;
    a.M = g.M; a.K = p->K; a.T = g.T; a.C = p->C;
    a.in_stride = g.in_stride; a.out_stride = g.out_stride;
    a.zero_point = p->dtype == ICV_U8I8 ? p->input_zero_point : 0;
    a.a_direct = a_direct ? 1 : 0;
    a.img_rows = a_direct ? g.M : g.img_rows;
    a.image_bytes = a_direct ? 0 : g.image_bytes;
    a.kp = g.n_tiles * g.NR;
    a.ep = g.ep;
    const int64_t gx = (g.M + 3) / 4;
    if (gx > 0x7fffffffll || g.n_tiles > 65535) return ICV_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)gx, (unsigned)g.n_tiles);
    if (p->dtype == ICV_F32)
        hipLaunchKernelGGL((k_igemm_generic<float, float, float>), grid, dim3(256), 0, s, a);
    else if (p->dtype == ICV_BF16)
        hipLaunchKernelGGL((k_igemm_generic<uint16_t, uint16_t, float>), grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL((k_igemm_generic<uint8_t, int8_t, int32_t>), grid, dim3(256), 0, s, a);
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

}  // namespace icv
