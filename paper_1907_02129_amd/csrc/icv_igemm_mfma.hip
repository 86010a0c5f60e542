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

// 16-byte global -> LDS copy without a register stop (global_load_lds_dwordx4): lane l of the wavefront
// writes LDS bytes [lds_base + 16*l, +16).  Written as inline assembly on purpose: the compiler does not see
// a memory instruction, so it inserts no waits of its own for it, and the kernel counts outstanding copies
// itself with wait_vmcnt<>.  While such copies are in flight the kernel issues no other vector-memory
// instruction, which keeps the compiler's own counter bookkeeping valid.
__device__ inline void copy16_global_to_lds(const void* gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "memory", "m0");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// XCD-aware block -> tile map.  Workgroups are dealt round-robin to the 8 XCDs (block b lands on XCD b % 8),
// each with its own L2.  Giving every XCD one contiguous range of tiles keeps neighbouring row tiles --
// which for a 3x3 kernel share most of their input rows -- and all column tiles of a row tile in one L2.
__device__ inline int64_t xcd_tile(int64_t b, int64_t n_blocks)
{
    const int64_t chunk = n_blocks >> 3, rem = n_blocks & 7, x = b & 7;
    return x * chunk + (x < rem ? x : rem) + (b >> 3);
}

template <bool I8, int MR, int NR, int WM, int WN, int KCB, int NSTAGE, bool DIRECT>
__global__ __launch_bounds__(256) void k_igemm_mfma(IgemmArgs g)
{
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring depth");
    constexpr int Q = KCB / 16;          // 16-byte chunks per row per stage
    constexpr int P = 256 / KCB;         // rows per 256 bytes of LDS
    constexpr int RPB = 1024 / KCB;      // rows one wavefront-wide copy (64 x 16 B) covers
    constexpr int A_VEC = MR * KCB / 4096;   // copies per wavefront per stage, A tile
    constexpr int B_VEC = NR * KCB / 4096;   // ... B tile
    constexpr int L = A_VEC + B_VEC;
    constexpr int MRW = MR / WM, NRW = NR / WN;
    constexpr int MB = MRW / 32, NB = NRW / 32;
    constexpr int KSTEPS = KCB / 32;
    constexpr int SLOT = (MR + NR) * KCB;    // bytes of one ring slot: A tile then B tile
    static_assert(A_VEC >= 1 && B_VEC >= 1 && MB >= 1 && NB >= 1, "tile too small");
    static_assert((NSTAGE - 1) * L <= 63, "vmcnt is a 6-bit counter");
    using acc_t = typename Acc<I8>::type;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int32_t* ldsE = (int32_t*)(lds + NSTAGE * SLOT);          // [T][MR]
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int64_t tile = xcd_tile(blockIdx.x, gridDim.x);
    const int32_t nt = (int32_t)(tile % g.n_tiles);
    const int64_t mt = tile / g.n_tiles;

    // ---- tile's indirection entries -> LDS (Listing 3 reads them in exactly this order)
    if constexpr (!DIRECT) {
        const int4* src = (const int4*)(g.ind + mt * ((int64_t)g.T * MR));
        const int n4 = g.T * MR / 4;
        for (int i = tid; i < n4; i += 256) ((int4*)ldsE)[i] = src[i];
        __syncthreads();
    }

    // ---- copy slots of this lane: wavefront w moves 1 KB blocks b = w, w+4, ... of a stage tile; block b is
    // rows [b*RPB, +RPB); lane l fills LDS chunk (l % Q) of row b*RPB + l/Q, which must hold source chunk
    // (l % Q) ^ swizzle(row).  swizzle(row) = (row / P) % Q is the same for every block of a wavefront.
    const int lrow_in_blk = lane / Q;
    const int row0 = wave * RPB + lrow_in_blk;                 // first row this lane copies (A and B alike)
    const int src_chunk_off = ((lane % Q) ^ ((row0 / P) % Q)) << 4;
    const uint8_t* wsrc = g.w + ((int64_t)nt * g.n_stages) * (NR * KCB) + row0 * KCB + src_chunk_off;
    const uint8_t* a_direct_src = g.a + (mt * MR + row0) * g.row_stride_bytes + src_chunk_off;
    const uint32_t lds_wave = lds_base + wave * 1024;

    auto issue = [&](int s) {
        const uint32_t slot = lds_wave + (uint32_t)(s % NSTAGE) * SLOT;
        const int tap = s / g.stages_per_tap;
        const int cc = s - tap * g.stages_per_tap;
        const uint8_t* asrc[A_VEC];      // all addresses first: the copies below are opaque to the scheduler
#pragma unroll
        for (int j = 0; j < A_VEC; j++) {
            if constexpr (DIRECT) {
                asrc[j] = a_direct_src + (int64_t)(j * 4 * RPB) * g.row_stride_bytes + (int64_t)s * KCB;
            } else {
                const int32_t e = ldsE[tap * MR + row0 + j * 4 * RPB];
                const uint8_t* rowp = e < 0 ? g.zero_row : g.a + (int64_t)e * g.row_stride_bytes;
                asrc[j] = rowp + cc * KCB + src_chunk_off;
            }
        }
#pragma unroll
        for (int j = 0; j < A_VEC; j++) copy16_global_to_lds(asrc[j], slot + j * 4096);
        const uint8_t* ws = wsrc + (int64_t)s * (NR * KCB);
#pragma unroll
        for (int j = 0; j < B_VEC; j++) copy16_global_to_lds(ws + j * (4 * RPB * KCB), slot + MR * KCB + j * 4096);
    };

    // ---- fragment read offsets (per lane)
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int swz = (lrow / P) % Q;          // tile bases are multiples of 32 rows, and 32 % (P*Q) == 0
    const uint32_t a_frag_base = (wm * MRW + lrow) * KCB;
    const uint32_t b_frag_base = MR * KCB + (wn * NRW + lrow) * KCB;

    acc_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < NB; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0;

    const int n_stages = g.n_stages;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; s++)
        if (s < n_stages) issue(s);

    for (int s = 0; s < n_stages; s++) {
        // stage s has landed once at most the copies of the (up to NSTAGE-2) younger stages are outstanding
        if (s + NSTAGE - 2 < n_stages) wait_vmcnt<(NSTAGE - 2) * L>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();        // every wavefront's part of stage s is in LDS, and all are done with s-1
        if (s + NSTAGE - 1 < n_stages) issue(s + NSTAGE - 1);      // refills the slot stage s-1 used
        const uint8_t* S = lds + (s % NSTAGE) * SLOT;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ks++) {
            const uint32_t coff = (uint32_t)(((2 * ks + lhalf) ^ swz) << 4);
            uint4 af[MB], bf[NB];
#pragma unroll
            for (int i = 0; i < MB; i++) af[i] = *(const uint4*)(S + a_frag_base + i * 32 * KCB + coff);
#pragma unroll
            for (int j = 0; j < NB; j++) bf[j] = *(const uint4*)(S + b_frag_base + j * 32 * KCB + coff);
#pragma unroll
            for (int i = 0; i < MB; i++)
#pragma unroll
                for (int j = 0; j < NB; j++) acc[i][j] = mfma32<I8>(af[i], bf[j], acc[i][j]);
        }
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
constexpr int kRingDepth = 3;

template <bool I8, int MR, int NR, int WM, int WN, int KCB, bool DIRECT>
static int launch_one(const IgemmArgs& a, int64_t blocks, size_t lds_bytes, hipStream_t s)
{
    auto kern = k_igemm_mfma<I8, MR, NR, WM, WN, KCB, kRingDepth, DIRECT>;
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
    const size_t lds = (size_t)kRingDepth * (MR + NR) * g.KCB + ent;
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
