// Tensor-core Indirect GEMM for gfx950 (section 2.2, Listing 3, re-designed around MFMA).
//
// A workgroup of four wavefronts owns an MR x NR output tile (MR output pixels x NR output channels, the
// paper's micro-kernel tile scaled to a compute unit).  As in Listing 3 the reduction is two nested loops:
// the outer one walks the R*S kernel elements and fetches the MR row pointers of the tile from the
// indirection buffer, the inner one walks the C channels.  One pipeline stage covers one kernel element and
// KCB bytes of its channels:
//
//   A stage tile: MR gathered rows x KCB bytes.  Each row is read from the input tensor (or the zero row)
//                 with coalesced 16-byte loads, lanes running along the channels first, and laid into LDS.
//   B stage tile: NR filter rows x KCB bytes, one contiguous block of the pre-packed filter.
//
// Both tiles keep the reduction dimension contiguous, which is exactly the operand layout of
// v_mfma_f32_32x32x16_bf16 / v_mfma_i32_32x32x32_i8: lane l supplies 16 contiguous bytes of row (l & 31),
// byte offset 16*(l >> 5) inside a 32-byte k-step.  LDS rows are XOR-swizzled in 16-byte units so that the
// ds_read_b128 fragment reads of 32 different rows spread over all banks.
//
// Pipeline: global loads of stage s+1 are issued into registers before the MFMAs of stage s and written to
// the other LDS buffer after them; one barrier per stage.  The tile's indirection entries (MR * T int32,
// contiguous thanks to the [tile][tap][row] order) are copied to LDS once at the start, so the
// pointer -> data dependency never waits on HBM inside the loop.
//
// uint8 activations: MFMA multiplies signed bytes, so every A fragment is XORed with 0x80, which turns
// x into x - 128 exactly; the zero row (filled with the zero point 128) becomes a row of zeros.
#include <type_traits>
#include "icv_internal.h"

namespace icv {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));

struct IgemmArgs {
    const uint8_t* a;         // input tensor | im2col matrix
    const uint8_t* zero_row;
    const uint8_t* w;         // packed filter [n tile][stage][NR][KCB]
    const int32_t* ind;       // [m tile][tap][MR]
    void* out;
    int64_t M;
    int64_t row_stride_bytes;  // input pixel stride | im2col row stride
    int32_t K, T, out_stride;
    int32_t stages_per_tap, n_stages;
    int32_t n_tiles;
};

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

template <bool I8, int MR, int NR, int WM, int WN, int KCB, bool DIRECT>
__global__ __launch_bounds__(256) void k_igemm_mfma(IgemmArgs g)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    constexpr int Q = KCB / 16;          // 16-byte chunks per row per stage
    constexpr int P = 256 / KCB;         // rows per 256 bytes of LDS
    constexpr int ROWS_PER_PASS = 256 / Q;
    constexpr int A_VEC = MR / ROWS_PER_PASS;
    constexpr int B_VEC = NR / ROWS_PER_PASS;
    constexpr int MRW = MR / WM, NRW = NR / WN;
    constexpr int MB = MRW / 32, NB = NRW / 32;
    constexpr int KSTEPS = KCB / 32;
    static_assert(A_VEC >= 1 && B_VEC >= 1 && MB >= 1 && NB >= 1, "tile too small");
    using acc_t = typename Acc<I8>::type;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* ldsA = lds;                          // [2][MR*KCB]
    uint8_t* ldsB = lds + 2 * MR * KCB;           // [2][NR*KCB]
    int32_t* ldsE = (int32_t*)(lds + 2 * (MR + NR) * KCB);   // [T][MR]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t bid = blockIdx.x;
    const int32_t nt = (int32_t)(bid % g.n_tiles);
    const int64_t mt = bid / g.n_tiles;

    // ---- tile's indirection entries -> LDS (Listing 3 reads them in exactly this order)
    if constexpr (!DIRECT) {
        const int4* src = (const int4*)(g.ind + mt * ((int64_t)g.T * MR));
        const int n4 = g.T * MR / 4;
        for (int i = tid; i < n4; i += 256) ((int4*)ldsE)[i] = src[i];
        __syncthreads();
    }

    // ---- per-thread load slots
    const int chunk = tid % Q;
    const int row0 = tid / Q;
    uint32_t a_lds_off[A_VEC], b_lds_off[B_VEC];
#pragma unroll
    for (int j = 0; j < A_VEC; j++) {
        const int row = row0 + j * ROWS_PER_PASS;
        a_lds_off[j] = row * KCB + ((chunk ^ ((row / P) % Q)) << 4);
    }
#pragma unroll
    for (int j = 0; j < B_VEC; j++) {
        const int row = row0 + j * ROWS_PER_PASS;
        b_lds_off[j] = row * KCB + ((chunk ^ ((row / P) % Q)) << 4);
    }
    const uint8_t* wtile = g.w + ((int64_t)nt * g.n_stages) * (NR * KCB) + tid * 16;
    const uint8_t* a_direct_base = g.a + (mt * MR + row0) * g.row_stride_bytes + chunk * 16;

    uint4 ra[A_VEC], rb[B_VEC];
    auto gload = [&](int s) {
        const int tap = s / g.stages_per_tap;
        const int cc = s - tap * g.stages_per_tap;
#pragma unroll
        for (int j = 0; j < A_VEC; j++) {
            const uint8_t* src;
            if constexpr (DIRECT) {
                src = a_direct_base + (int64_t)(j * ROWS_PER_PASS) * g.row_stride_bytes + (int64_t)s * KCB;
            } else {
                const int32_t e = ldsE[tap * MR + row0 + j * ROWS_PER_PASS];
                const uint8_t* rowp = e < 0 ? g.zero_row : g.a + (int64_t)e * g.row_stride_bytes;
                src = rowp + cc * KCB + chunk * 16;
            }
            ra[j] = *(const uint4*)src;
        }
        const uint8_t* ws = wtile + (int64_t)s * (NR * KCB);
#pragma unroll
        for (int j = 0; j < B_VEC; j++) rb[j] = *(const uint4*)(ws + j * 4096);
    };
    auto lstore = [&](int buf) {
        uint8_t* A = ldsA + buf * (MR * KCB);
        uint8_t* B = ldsB + buf * (NR * KCB);
#pragma unroll
        for (int j = 0; j < A_VEC; j++) *(uint4*)(A + a_lds_off[j]) = ra[j];
#pragma unroll
        for (int j = 0; j < B_VEC; j++) *(uint4*)(B + b_lds_off[j]) = rb[j];
    };

    // ---- fragment read offsets (per lane)
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int swz = (lrow / P) % Q;          // tile bases are multiples of 32 rows, and 32 % (P*Q) == 0
    const uint32_t a_frag_base = (wm * MRW + lrow) * KCB;
    const uint32_t b_frag_base = (wn * NRW + lrow) * KCB;

    acc_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < NB; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0;

    gload(0);
    lstore(0);
    __syncthreads();

    for (int s = 0; s < g.n_stages; s++) {
        const int buf = s & 1;
        const bool more = s + 1 < g.n_stages;
        if (more) gload(s + 1);
        const uint8_t* A = ldsA + buf * (MR * KCB);
        const uint8_t* B = ldsB + buf * (NR * KCB);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ks++) {
            const uint32_t coff = (uint32_t)(((2 * ks + lhalf) ^ swz) << 4);
            uint4 af[MB], bf[NB];
#pragma unroll
            for (int i = 0; i < MB; i++) af[i] = *(const uint4*)(A + a_frag_base + i * 32 * KCB + coff);
#pragma unroll
            for (int j = 0; j < NB; j++) bf[j] = *(const uint4*)(B + b_frag_base + j * 32 * KCB + coff);
#pragma unroll
            for (int i = 0; i < MB; i++)
#pragma unroll
                for (int j = 0; j < NB; j++) acc[i][j] = mfma32<I8>(af[i], bf[j], acc[i][j]);
        }
        if (more) lstore(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator register r of lane l holds row 8*(r/4) + 4*(l>>5) + (r&3), column l&31
    using out_t = typename std::conditional<I8, int32_t, float>::type;
    out_t* out = (out_t*)g.out;
    const int64_t m_base = mt * MR + wm * MRW + 4 * lhalf;
    const int32_t n_base = nt * NR + wn * NRW + lrow;
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < NB; j++) {
            const int32_t col = n_base + j * 32;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int64_t row = m_base + i * 32 + 8 * (r >> 2) + (r & 3);
                if (row < g.M && col < g.K) out[row * g.out_stride + col] = acc[i][j][r];
            }
        }
}

// ------------------------------------------------------------------ launch
template <bool I8, int MR, int NR, int WM, int WN, int KCB, bool DIRECT>
static int launch_one(const IgemmArgs& a, int64_t blocks, size_t lds_bytes, hipStream_t s)
{
    auto kern = k_igemm_mfma<I8, MR, NR, WM, WN, KCB, DIRECT>;
    if (lds_bytes > 64 * 1024) {
        static bool raised = false;   // idempotent attribute; a race only repeats the call
        if (!raised) {
            ICV_HIP_CHECK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                              160 * 1024));
            raised = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), lds_bytes, s, a);
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

template <bool I8, int MR, int NR, int WM, int WN>
static int launch_tile(const Geometry& g, const IgemmArgs& a, int64_t blocks, bool direct, hipStream_t s)
{
    const size_t ent = direct ? 0 : (size_t)g.T * MR * 4;
    const size_t lds = (size_t)2 * (MR + NR) * g.KCB + ent;
    if (lds > 160 * 1024) return ICV_ERR_UNSUPPORTED;
    if (g.KCB == 128) {
        return direct ? launch_one<I8, MR, NR, WM, WN, 128, true>(a, blocks, lds, s)
                      : launch_one<I8, MR, NR, WM, WN, 128, false>(a, blocks, lds, s);
    }
    return direct ? launch_one<I8, MR, NR, WM, WN, 64, true>(a, blocks, lds, s)
                  : launch_one<I8, MR, NR, WM, WN, 64, false>(a, blocks, lds, s);
}

template <bool I8>
static int launch_dtype(const Geometry& g, const IgemmArgs& a, int64_t blocks, bool direct, hipStream_t s)
{
    switch (g.variant) {
        case 0: return launch_tile<I8, 128, 64, 2, 2>(g, a, blocks, direct, s);
        case 1: return launch_tile<I8, 128, 128, 2, 2>(g, a, blocks, direct, s);
        case 2: return launch_tile<I8, 128, 64, 4, 1>(g, a, blocks, direct, s);
        case 3: return launch_tile<I8, 256, 64, 4, 1>(g, a, blocks, direct, s);
        case 4: return launch_tile<I8, 256, 128, 2, 2>(g, a, blocks, direct, s);
        case 5: return launch_tile<I8, 64, 64, 2, 2>(g, a, blocks, direct, s);
        default: return ICV_ERR_UNSUPPORTED;
    }
}

int launch_igemm_mfma(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, const void* zero_row, void* out, bool a_direct, hipStream_t s)
{
    // the host-side table and the instantiations above must describe the same tiles
    const TileVariant& tv = kTileVariants[g.variant];
    if (tv.MR != g.MR || tv.NR != g.NR) return ICV_ERR_UNSUPPORTED;
    IgemmArgs a;
    a.a = (const uint8_t*)input;
    a.zero_row = (const uint8_t*)zero_row;
    a.w = (const uint8_t*)packed;
    a.ind = ind;
    a.out = out;
    a.M = g.M;
    a.row_stride_bytes = a_direct ? (int64_t)g.T * p->C * g.elem_bytes : (int64_t)g.in_stride * g.elem_bytes;
    a.K = p->K; a.T = g.T; a.out_stride = g.out_stride;
    a.stages_per_tap = g.stages_per_tap; a.n_stages = g.n_stages;
    a.n_tiles = (int32_t)g.n_tiles;
    const int64_t blocks = g.m_tiles * g.n_tiles;
    if (blocks > 0x7fffffffll) return ICV_ERR_UNSUPPORTED;
    return p->dtype == ICV_U8I8 ? launch_dtype<true>(g, a, blocks, a_direct, s)
                                : launch_dtype<false>(g, a, blocks, a_direct, s);
}

}  // namespace icv
