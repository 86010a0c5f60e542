// Device helpers shared by the tensor-core Indirect GEMM kernels (MFMA wrappers, global -> LDS copies, manual
// vmcnt waits, the persistent workgroups' tile lists).
#pragma once
#include <type_traits>
#include "icv_internal.h"

namespace icv {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));

template <bool I8>
struct Acc {
    using type = f32x16_t;
};
template <>
struct Acc<true> {
    using type = i32x16_t;
};

template <bool I8>
__device__ inline typename Acc<I8>::type mfma32(const uint4& a, const uint4& b, typename Acc<I8>::type c)
{
    if constexpr (I8) {
        i32x4_t av = {(int)(a.x ^ 0x80808080u), (int)(a.y ^ 0x80808080u), (int)(a.z ^ 0x80808080u),
                      (int)(a.w ^ 0x80808080u)};
        i32x4_t bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w};
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
}

// The same 16-byte fragments holding fp32 (section 3.1's own precision): four floats per lane and matrix, multiplied
// as four 32x32x2 products.  Product j pairs element j of the lower half-wavefront (reduction index 4*piece + j, piece
// even) with element j of the upper one (piece odd); the operands of A and B are paired alike, so the sum over the
// four products is the sum over the eight reduction indices the two pieces hold.
__device__ inline f32x16_t mfma32_f32(const uint4& a, const uint4& b, f32x16_t c)
{
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), c, 0, 0, 0);
    return c;
}

// 16-byte global -> LDS copy without a register stop: lane l of the wavefront writes LDS bytes
// [lds_base + 16*l, +16).  Inline assembly on purpose: the compiler does not see a memory instruction, so it
// inserts no waits of its own for it, and the producers count outstanding copies themselves (wait_vmcnt).
// A producer issues no other vector-memory instruction while copies are in flight.
// M0 is written here without being listed as clobbered: the compiler treats it as a reserved register (naming it in
// the clobber list is diagnosed as such), never keeps a value in it across other code, and writes it itself right
// before each of its own instructions that read it.
__device__ inline void copy16_global_to_lds(const void* gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "memory");
}

// Same copy with the address split into a uniform 64-bit base and a per-lane unsigned 32-bit byte offset, which
// keeps the per-lane address arithmetic in 32 bits.
__device__ inline void copy16_global_to_lds(const void* sbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_base)
                 : "memory");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// Wait until at most `stages` x LP of this wavefront's copies are outstanding (copies retire in order).
template <int LP>
__device__ inline void wait_all_but_stages(int stages)
{
    switch (stages) {
        case 0: wait_vmcnt<0>(); break;
        case 1: wait_vmcnt<LP>(); break;
        case 2: wait_vmcnt<2 * LP>(); break;
        case 3: wait_vmcnt<3 * LP>(); break;
        case 4: wait_vmcnt<(4 * LP <= 63 ? 4 * LP : 63)>(); break;
        case 5: wait_vmcnt<(5 * LP <= 63 ? 5 * LP : 63)>(); break;
        default: wait_vmcnt<(6 * LP <= 63 ? 6 * LP : 63)>(); break;
    }
}

// Epilogue of the tensor-core kernels: a wavefront's MB x NB accumulator blocks -> output[row][col].  Register r
// of lane l of a block holds row 8*(r/4) + 4*(l>>5) + (r&3), column l&31; m_base / n_base are this lane's row
// and column of register 0 of block (0, 0).
//   FUSED = false: raw accumulators.  Whole tiles take unguarded non-temporal stores (the output is written once
//                  and not read again by this kernel), tail tiles guarded ones.
//   FUSED = true : the output stage of icv_conv2d_nhwc_fused (bias, ReLU, narrow output types).  A separate
//                  instantiation: its per-element work would otherwise raise the plain kernel's register use
//                  enough to lose the second co-resident workgroup.
template <bool FUSED, int KIND, int MB, int NB, typename ACC, typename OUT_ACC>
__device__ inline void store_tile_as(void* outp, const ACC (&acc)[MB][NB], int64_t M, int32_t K, int64_t out_stride,
                                     int64_t m_base, int32_t n_base, bool whole, const EpilogueArgs& ep)
{
    using store_t = typename std::conditional<KIND == ICV_OUT_BF16, __bf16,
                    typename std::conditional<KIND == ICV_OUT_U8, uint8_t, OUT_ACC>::type>::type;
    store_t* out = (store_t*)outp;
    const float scale = ep.scale;
    const int32_t zero_point = ep.out_zero_point;
    auto convert = [=](OUT_ACC v) -> store_t {
        if constexpr (KIND == ICV_OUT_BF16) {
            return (__bf16)v;                                  // hardware conversion: nearest, ties to even
        } else if constexpr (KIND == ICV_OUT_U8) {
            float f = rintf(__fmul_rn((float)v, scale));       // single-precision product, ties to even
            f = fminf(fmaxf(f, -1e9f), 1e9f);
            int32_t q = (int32_t)f + zero_point;
            return (uint8_t)(q < 0 ? 0 : (q > 255 ? 255 : q));
        } else {
            return v;
        }
    };
    // ReLU as a select that runs only when asked for: without it a NaN accumulator stays NaN on every path
    const bool relu = FUSED && ep.relu;
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < NB; j++) {
            const int32_t col = n_base + j * 32;
            OUT_ACC bias = 0;
            if constexpr (FUSED) bias = output_bias<OUT_ACC>(ep, col, K);
            if (whole) {
                store_t* o = out + (m_base + i * 32) * out_stride + col;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    OUT_ACC v = (OUT_ACC)acc[i][j][r];
                    if constexpr (FUSED) { v += bias; if (relu) v = v > (OUT_ACC)0 ? v : (OUT_ACC)0; }
                    __builtin_nontemporal_store(convert(v), &o[(int64_t)(8 * (r >> 2) + (r & 3)) * out_stride]);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int64_t row = m_base + i * 32 + 8 * (r >> 2) + (r & 3);
                    OUT_ACC v = (OUT_ACC)acc[i][j][r];
                    if constexpr (FUSED) { v += bias; if (relu) v = v > (OUT_ACC)0 ? v : (OUT_ACC)0; }
                    if (row < M && col < K) out[row * out_stride + col] = convert(v);
                }
            }
        }
}

template <bool FUSED, bool I8, int MB, int NB, typename ACC>
__device__ inline void store_tile(void* out, const ACC (&acc)[MB][NB], int64_t M, int32_t K, int64_t out_stride,
                                  int64_t m_base, int32_t n_base, bool whole, const EpilogueArgs& ep)
{
    using out_acc_t = typename std::conditional<I8, int32_t, float>::type;
    if constexpr (!FUSED) {
        store_tile_as<false, ICV_OUT_ACC, MB, NB, ACC, out_acc_t>(out, acc, M, K, out_stride, m_base, n_base, whole, ep);
    } else if constexpr (I8) {
        if (ep.out_kind == ICV_OUT_U8) store_tile_as<true, ICV_OUT_U8, MB, NB, ACC, out_acc_t>(out, acc, M, K, out_stride, m_base, n_base, whole, ep);
        else store_tile_as<true, ICV_OUT_ACC, MB, NB, ACC, out_acc_t>(out, acc, M, K, out_stride, m_base, n_base, whole, ep);
    } else {
        if (ep.out_kind == ICV_OUT_BF16) store_tile_as<true, ICV_OUT_BF16, MB, NB, ACC, out_acc_t>(out, acc, M, K, out_stride, m_base, n_base, whole, ep);
        else store_tile_as<true, ICV_OUT_ACC, MB, NB, ACC, out_acc_t>(out, acc, M, K, out_stride, m_base, n_base, whole, ep);
    }
}

// Tile list of a persistent workgroup.  Workgroups are dealt round-robin to the 8 XCDs (block b runs on
// XCD b % 8).  In XCD mode XCD x owns the contiguous tile range [first, first + count) and its G/8 workgroups
// take tiles first + i, first + i + G/8, ... ; otherwise block b takes b, b + G, ...
struct TileList {
    int64_t first, step, count;   // tiles first + k*step for k < count
};

__device__ inline TileList my_tiles(int64_t total64, int xcd_mode)
{
    // 32-bit arithmetic (the host keeps the tile count below 2^31): this runs before a workgroup's first load is
    // issued, and a 64-bit division is a few hundred instructions there
    const uint32_t total = (uint32_t)total64, b = blockIdx.x, G = gridDim.x;
    TileList t;
    if (xcd_mode) {
        const uint32_t chunk = total >> 3, rem = total & 7, x = b & 7;
        const uint32_t start = x * chunk + (x < rem ? x : rem);
        const uint32_t len = chunk + (x < rem ? 1 : 0);
        const uint32_t i = b >> 3, step = G >> 3;
        t.step = step;
        t.first = start + i;
        // one tile per workgroup is the common case (the grid is sized for it): no division then
        t.count = i >= len ? 0 : (i + step >= len ? 1 : (len - i + step - 1) / step);
    } else {
        t.step = G;
        t.first = b;
        t.count = b >= total ? 0 : (b + G >= total ? 1 : (total - b + G - 1) / G);
    }
    return t;
}

inline int device_cu_count()
{
    static int cached[64] = {0};      // per device ordinal; filled on first use, the value never changes
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

constexpr size_t kLdsPerCu = 160 * 1024;

// Lets `kern` use the whole LDS of a compute unit as dynamic shared memory.  The attribute belongs to the
// (kernel, device) pair, so the caller keeps one flag array per kernel instantiation; the call is idempotent and a
// race between threads only repeats it.
constexpr int kMaxDevices = 64;
inline int allow_full_lds(const void* kern, bool (&done)[kMaxDevices])
{
    int dev = 0;
    const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices;
    if (known && done[dev]) return ICV_OK;
    ICV_HIP_CHECK(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCu));
    if (known) done[dev] = true;
    return ICV_OK;
}

}  // namespace icv
