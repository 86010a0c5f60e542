// Measured tensor-core ceiling of the device the library runs on: a loop of MFMAs on register operands only, four
// independent accumulator blocks per wavefront, one to four wavefronts per SIMD.  No memory is read or written, so
// the rate is what the matrix cores deliver at the clock the device actually sustains under this load -- the
// yardstick beside the data-sheet peak for the Indirect GEMM kernels' "fraction of peak" (section 3.1 reports the
// primitive against what the machine's GEMM reaches, not against a data sheet).
#include "icv_internal.h"
#include "icv_mfma_common.h"

namespace icv {

// VARIED = false: every MFMA multiplies the same two constant operands (1.0, small integers) -- nothing toggles but
// the accumulators' low bits.  VARIED = true: four A and four B operands of pseudo-random values (bfloat16 in
// +-[0.5, 2), random bytes), a different pair in every MFMA -- the switching activity of real tensors, which costs
// power and, on a device that runs at its power limit, clock.
template <bool I8, bool VARIED>
__global__ __launch_bounds__(256) void k_mfma_only(int iters, float* sink)
{
    using acc_t = typename Acc<I8>::type;
    acc_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[i][r] = 0;
    uint4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        if (VARIED) {
            uint32_t h = (uint32_t)(threadIdx.x + 256u * blockIdx.x) * 2654435761u + (uint32_t)i * 0x9E3779B9u;
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) {
                h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
                // bfloat16 pairs: sign, exponent 126 or 127 (0x3F00 / 0x3F80 with the mantissa's top bit), 7 mantissa bits
                v[j] = I8 ? h : ((h & 0x80FF80FFu) | 0x3F003F00u);
            }
            a[i] = make_uint4(v[0], v[1], v[2], v[3]);
            b[i] = make_uint4(v[4], v[5], v[6], v[7]);
        } else {
            const uint32_t av = I8 ? 0x01020301u * (threadIdx.x & 3) : 0x3f803f80u;   // small integers / 1.0 in bfloat16
            const uint32_t bv = I8 ? 0x01010101u : 0x3f803f80u;
            a[i] = make_uint4(av, av, av, av);
            b[i] = make_uint4(bv, bv, bv, bv);
        }
    }
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int v = 0; v < 4; v++)
#pragma unroll
            for (int u = 0; u < 4; u++) acc[u] = mfma32<I8>(a[(u + v) & 3], b[v], acc[u]);
    }
    float t = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) t += (float)acc[i][r];
    if (t == -1.5f && sink) sink[0] = t;  // never true in practice, and no sink is passed: keeps the loop alive, writes nothing
}

}  // namespace icv

using namespace icv;

extern "C" int icv_measure_mfma_peak(int32_t dtype, int32_t waves_per_simd, int32_t varied_operands, double* ops_per_second,
                                     void* stream)
{
    if (!ops_per_second || (dtype != ICV_BF16 && dtype != ICV_U8I8) || waves_per_simd < 1 || waves_per_simd > 4 ||
        (varied_operands != 0 && varied_operands != 1))
        return ICV_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int iters = 8000;
    const int blocks = device_cu_count() * waves_per_simd;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ICV_HIP_CHECK(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return ICV_ERR_HIP;
    }
    int st = ICV_OK;
    float best_ms = 0.f;
    for (int rep = 0; rep < 4 && st == ICV_OK; rep++) {          // the first launch also warms the clock up
        hipError_t err = hipEventRecord(e0, s);
        if (err == hipSuccess) {
            auto kern = dtype == ICV_U8I8 ? (varied_operands ? k_mfma_only<true, true> : k_mfma_only<true, false>)
                                          : (varied_operands ? k_mfma_only<false, true> : k_mfma_only<false, false>);
            hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), 0, s, iters, (float*)nullptr);
            err = hipGetLastError();
        }
        if (err == hipSuccess) err = hipEventRecord(e1, s);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
        if (err != hipSuccess) { set_hip_error(err); st = ICV_ERR_HIP; break; }
        if (rep > 0 && (best_ms == 0.f || ms < best_ms)) best_ms = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != ICV_OK) return st;
    // one MFMA of a wavefront is a 32 x 32 x 16 (bf16) or 32 x 32 x 32 (int8) block product
    const double ops = (double)blocks * 4 /*wavefronts*/ * iters * 4 * (dtype == ICV_U8I8 ? 65536.0 : 32768.0);
    *ops_per_second = ops / ((double)best_ms * 1e-3);
    return ICV_OK;
}
