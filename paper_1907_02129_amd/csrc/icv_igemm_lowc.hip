// Tensor-core Indirect GEMM for very few input channels (first-layer convolutions: C*sizeof(element) of
// 8, 16 or 32 bytes per pixel row).
//
// With so short rows one kernel element is less than an MFMA k-step, so the two nested loops of Listing 3
// (kernel elements outside, channels inside) are flattened: the reduction index is k = tap*C + c, the whole
// reduction of a tile (R*S*C elements, zero-padded to a multiple of the 32-byte k-step) is gathered into LDS at
// once, one U-byte load per (output pixel, kernel element) through the indirection buffer, and the tile is then
// multiplied in one sweep of MFMAs.  The packed filter slice of the workgroup's columns stays in LDS for
// all the row tiles the (persistent) workgroup walks, because it is no larger than the gathered A tile.  A
// workgroup takes as many 32-column blocks as fit its LDS budget (all of K for the usual first layers), so the
// rows, whose gather is the expensive part, are fetched once and not once per column tile.
//
// The entries are read in their compact form when the set-up phase wrote one: per row tile a range record with
// the smallest valid byte offset, and per entry a 16-bit pixel number relative to it (0xFFFF = zero row), half
// the bytes of the int32 offsets; with so few channels the entries are the larger part of what a tile reads.
//
// LDS rows are padded by 16 bytes (odd number of 16-byte units per row) instead of swizzled: ds_write_b64
// from the gather and ds_read_b128 for the fragments are then both spread over the banks.
#include "icv_mfma_common.h"

namespace icv {

struct LowcArgs {
    const uint8_t* a;
    const uint8_t* zero_row;
    const uint8_t* w;       // packed filter [n tile][64][KP]
    const int32_t* ind;     // [m tile][tap][64], byte offsets, negative = zero row
    const int4* ranges;     // compact form: per row tile {smallest valid byte offset, ...}, or null
    const uint16_t* rows;   // compact form: [m tile][tap][64] pixel numbers from that offset on, 0xFFFF = zero row
    void* out;
    int64_t M, m_tiles;
    int64_t image_bytes;    // batch-independent buffer: bytes between batch elements of the input (else 0)
    uint32_t img_tiles, img_rows;  // row tiles and output pixels per image (one image = the whole batch otherwise)
    int32_t K, T, out_stride, n_tiles;
    int32_t KP;             // padded reduction bytes per row, multiple of 32
    int32_t stride_bytes;   // bytes between input pixels
    int32_t col_blocks;     // 32-column blocks per workgroup (blockIdx.y selects the group)
    int32_t k_rows;         // rows of the packed filter (K padded to 64)
    int32_t direct;         // 1: `a` is the dense patch matrix [rows][KP] of the ablation path
    uint32_t zero_fill;     // four bytes of the zero row: zeros, or the zero point of uint8 activations
    EpilogueArgs ep;
};

// register type of one gathered piece (native vectors: arrays of them are kept in registers)
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <int U>
struct Piece;
template <>
struct Piece<8> { using type = u32x2_t; };
template <>
struct Piece<16> { using type = u32x4_t; };
template <>
struct Piece<32> { using type = u32x4_t; };   // moved as two 16-byte halves

// A team of 4 wavefronts per tile of 64 rows x (32 * col_blocks) columns; its 32 x 32 blocks are dealt out to the
// wavefronts in turn.  A workgroup is TEAMS such teams that share the filter slice in LDS and each own a gathered
// tile: per tile a wavefront runs a chain of dependent steps (entries -> rows -> LDS -> fragments -> MFMA -> stores)
// that nothing overlaps but other wavefronts, and the filter slice is half the LDS a lone team needs, so sharing it
// is what lets 16 instead of 8 wavefronts work on a compute unit.  All teams pass the same barriers (there is one
// kind of barrier), so they walk their tiles in lock step.
constexpr int kMaxColBlocks = 8;                              // 32-column blocks of a workgroup (256 columns)
constexpr int kMaxBlocksPerWave = 2 * kMaxColBlocks / 4;      // its 32 x 32 blocks, dealt to four wavefronts

template <bool I8, int U, bool FUSED, int TEAMS>
__global__ __launch_bounds__(256 * TEAMS) void k_igemm_lowc(LowcArgs g)
{
    constexpr int MR = 64;
    using acc_t = typename std::conditional<I8, i32x16_t, f32x16_t>::type;
    using out_t = typename std::conditional<I8, int32_t, float>::type;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int pitch = g.KP + 16;
    const int col0 = blockIdx.y * g.col_blocks * 32;                       // first column of this workgroup
    int n_cols = g.k_rows - col0;                                          // packed filter rows from there on
    if (n_cols > g.col_blocks * 32) n_cols = g.col_blocks * 32;
    const int n_blocks = 2 * (n_cols / 32);                                // 32 x 32 blocks of the tile
    const int team = TEAMS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8);
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in the team
    uint8_t* ldsB = lds;                                                    // [32 * col_blocks][pitch], shared
    uint8_t* ldsA = lds + (g.col_blocks * 32 + team * MR) * pitch;          // [MR][pitch], the team's own
    const EpilogueArgs ep = g.ep;

    // ---- filter slice of this workgroup's columns -> LDS, once
    {
        const uint8_t* src = g.w + (int64_t)col0 * g.KP;
        const int vec_per_row = g.KP / 16;
        for (int v = threadIdx.x; v < n_cols * vec_per_row; v += 256 * TEAMS) {
            const int row = v / vec_per_row, c = v - row * vec_per_row;
            *(uint4*)(ldsB + row * pitch + c * 16) = *(const uint4*)(src + (int64_t)row * g.KP + c * 16);
        }
    }
    // zero the k padding of the A rows once (those columns are never written by the gather)
    {
        const int pad_from = g.T * U;             // multiple of 8
        const int pad8 = (g.KP - pad_from) / 8;
        for (int v = tid; v < MR * pad8; v += 256) {
            const int row = v / pad8, c = v - row * pad8;
            *(uint2*)(ldsA + row * pitch + pad_from + c * 8) = make_uint2(0, 0);
        }
    }

    const int lrow = lane & 31, lhalf = lane >> 5;
    const int ksteps = g.KP / 32;
    const bool compact = g.rows != nullptr;
    const bool per_image = g.image_bytes != 0;          // else one "image" is the whole batch: no divisions per tile

    // Entries of a batch of kernel elements of row tile mt: thread -> row tid % 64, elements tap0, tap0 + 4, ...
    // (the 64 entries of an element are contiguous).  A batch is 16 elements, or 8 of the 32-byte rows.
    constexpr int NB = U == 32 ? 8 : 16;
    constexpr int NV = U == 32 ? 2 * NB : NB;             // 16-byte (8-byte for U = 8) registers of a batch
    using piece_t = typename Piece<U>::type;
    const int n_taps = g.direct ? 0 : g.T;
    uint8_t* dstrow = ldsA + (tid & 63) * pitch;
    // (compact form: turned into byte offsets here, with the tile's first offset from its range record)
    auto load_entries = [&](int64_t mt, int tap0, int32_t (&e)[NB]) __attribute__((always_inline)) {
        const uint32_t bt = (uint32_t)mt % g.img_tiles;                                                     // tile of the buffer
        if (compact) {
            const uint16_t* ent = g.rows + bt * ((int64_t)g.T * MR) + (tid & 63);
            const int32_t first = g.ranges[bt].x;
#pragma unroll
            for (int j = 0; j < NB; j++) {
                const int tap = tap0 + 4 * j;
                const uint32_t r = tap < n_taps ? ent[tap * MR] : 0xFFFFu;
                e[j] = r == 0xFFFFu ? INT32_MIN : first + (int32_t)(r * (uint32_t)g.stride_bytes);
            }
        } else {
            const int32_t* ent = g.ind + bt * ((int64_t)g.T * MR) + (tid & 63);
#pragma unroll
            for (int j = 0; j < NB; j++) {
                const int tap = tap0 + 4 * j;
                e[j] = tap < n_taps ? ent[tap * MR] : INT32_MIN;
            }
        }
    };
    // the rows a batch of entries names -> registers (elements past the last one read the zero row and are dropped)
    auto gather = [&](int64_t mt, const int32_t (&e)[NB], piece_t (&v)[NV]) __attribute__((always_inline)) {
        const uint8_t* a_img = g.a + ((uint32_t)mt / g.img_tiles) * g.image_bytes;     // the batch element of this tile
#pragma unroll
        for (int j = 0; j < NB; j++) {
            const uint8_t* src = e[j] < 0 ? g.zero_row : a_img + (uint32_t)e[j];
            if constexpr (U == 32) {
                v[2 * j] = *(const piece_t*)src;
                v[2 * j + 1] = *(const piece_t*)(src + 16);
            } else {
                v[j] = *(const piece_t*)src;
            }
        }
    };
    auto to_lds = [&](int tap0, const piece_t (&v)[NV]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NB; j++) {
            const int tap = tap0 + 4 * j;
            if (tap < n_taps) {
                if constexpr (U == 32) {
                    *(piece_t*)(dstrow + tap * 32) = v[2 * j];
                    *(piece_t*)(dstrow + tap * 32 + 16) = v[2 * j + 1];
                } else {
                    *(piece_t*)(dstrow + tap * U) = v[j];
                }
            }
        }
    };
    auto multiply_and_store = [&](int64_t mt) __attribute__((always_inline)) {
        const uint32_t img = per_image ? (uint32_t)mt / g.img_tiles : 0u;                               // batch element
        const uint32_t t_img = (uint32_t)mt - img * g.img_tiles;                                        // row tile in it
        const int64_t img_row0 = (int64_t)img * g.img_rows;
        const bool whole_rows = (t_img + 1) * MR <= g.img_rows;
        // 32 x 32 block b of the tile: rows 32 * (b & 1), columns 32 * (b >> 1).  Written without a loop over the
        // blocks on purpose: before a loop that stores, the compiler waits for every outstanding load, which would
        // expose the latency of the rows of the next tiles that are in flight at this point.
#pragma unroll
        for (int u = 0; u < kMaxBlocksPerWave; u++) {
            const int b = wave + 4 * u;
            if (b >= n_blocks) break;
            const int rb = b & 1, cb = b >> 1;
            const uint8_t* a_frag = ldsA + (rb * 32 + lrow) * pitch + lhalf * 16;
            const uint8_t* b_frag = ldsB + (cb * 32 + lrow) * pitch + lhalf * 16;
            acc_t block[1][1];
            acc_t& acc = block[0][0];
#pragma unroll
            for (int r = 0; r < 16; r++) acc[r] = 0;
            for (int ks = 0; ks < ksteps; ks++) {
                const uint4 av = *(const uint4*)(a_frag + ks * 32);
                const uint4 bv = *(const uint4*)(b_frag + ks * 32);
                if constexpr (I8) {
                    i32x4_t ai = {(int)(av.x ^ 0x80808080u), (int)(av.y ^ 0x80808080u), (int)(av.z ^ 0x80808080u),
                                  (int)(av.w ^ 0x80808080u)};
                    i32x4_t bi = {(int)bv.x, (int)bv.y, (int)bv.z, (int)bv.w};
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(ai, bi, acc, 0, 0, 0);
                } else {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av),
                                                                  __builtin_bit_cast(bf16x8_t, bv), acc, 0, 0, 0);
                }
            }
            const int64_t m_base = img_row0 + (int64_t)t_img * MR + rb * 32 + 4 * lhalf;
            const int32_t col = col0 + cb * 32 + lrow;
            // register r of lane l holds row 8*(r/4) + 4*(l>>5) + (r&3), column l&31
            const bool whole = whole_rows && col0 + (cb + 1) * 32 <= g.K;
            store_tile<FUSED, I8, 1, 1>(g.out, block, img_row0 + g.img_rows, g.K, g.out_stride, m_base, col, whole, ep);
        }
    };

    const int64_t G = gridDim.x;
    if (!g.direct && compact && n_taps <= 4 * NB) {
        // One batch of compact entries covers the tile (the usual case).  The kernel is bound by instruction issue
        // and by the latency of its two dependent global loads (entries, then the rows they name), so this path
        // keeps both short: the wavefront's kernel elements tap0, tap0 + 4, ... are wavefront-uniform (scalar
        // branches and addresses), a row is loaded from base + 32-bit offset whether its entry is valid or not and
        // replaced by the zero pattern afterwards (what the zero row holds: zeros, or the zero point for uint8).
        const int tap0 = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int nb = (n_taps - tap0 + 3) / 4;                    // kernel elements of this wavefront, <= NB
        const uint32_t stride = (uint32_t)g.stride_bytes;
        const uint32_t zfill = g.zero_fill;
        // entries (16-bit) and the byte offset they count from
        auto load_rows16 = [&](int64_t mt, uint32_t (&r)[NB], int32_t& first) __attribute__((always_inline)) {
            const uint32_t bt = per_image ? (uint32_t)mt % g.img_tiles : (uint32_t)mt;                   // tile of the buffer
            const uint16_t* ent = g.rows + bt * ((int64_t)g.T * MR) + tap0 * MR + (tid & 63);
            first = g.ranges[bt].x;
#pragma unroll
            for (int j = 0; j < NB; j++)
                if (j < nb) r[j] = ent[4 * j * MR];
        };
        auto gather16 = [&](int64_t mt, const uint32_t (&r)[NB], int32_t first, piece_t (&v)[NV], uint32_t& zmask)
                            __attribute__((always_inline)) {
            const uint8_t* base = g.a + (per_image ? (uint32_t)mt / g.img_tiles : 0u) * g.image_bytes + first;   // wavefront-uniform
            zmask = 0;
#pragma unroll
            for (int j = 0; j < NB; j++)
                if (j < nb) {
                    const bool z = r[j] == 0xFFFFu;
                    zmask |= (z ? 1u : 0u) << j;
                    const uint32_t off = z ? 0u : __umul24(r[j], stride);      // offset 0 is the tile's first valid pixel
                    if constexpr (U == 32) {
                        v[2 * j] = *(const piece_t*)(base + off);
                        v[2 * j + 1] = *(const piece_t*)(base + off + 16);
                    } else {
                        v[j] = *(const piece_t*)(base + off);
                    }
                }
        };
        auto to_lds16 = [&](const piece_t (&v)[NV], uint32_t zmask) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < NB; j++)
                if (j < nb) {
                    const bool z = (zmask >> j) & 1u;
                    uint8_t* d = dstrow + (tap0 + 4 * j) * U;
                    if constexpr (U == 32) {
                        *(piece_t*)d = z ? (piece_t)zfill : v[2 * j];
                        *(piece_t*)(d + 16) = z ? (piece_t)zfill : v[2 * j + 1];
                    } else {
                        *(piece_t*)d = z ? (piece_t)zfill : v[j];
                    }
                }
        };
        piece_t v[NV];
        uint32_t r[NB];
        uint32_t zmask = 0;
        int32_t first = 0;
        const int64_t m_tiles = g.m_tiles;
        // team q of workgroup b takes tiles b * TEAMS + q + k * Gt; every team runs the steps of the team with the most
        // tiles (team 0), idle in those it has no tile for, so that all meet at the barriers
        const int64_t Gt = G * TEAMS;
        const int64_t t0 = (int64_t)blockIdx.x * TEAMS;
        const int64_t steps = t0 < m_tiles ? (m_tiles - t0 + Gt - 1) / Gt : 0;
        int64_t t = t0 + team;
        if (t < m_tiles) {
            load_rows16(t, r, first);
            gather16(t, r, first, v, zmask);
            if (t + Gt < m_tiles) load_rows16(t + Gt, r, first);
        }
        // v holds the rows of tile t; while t is multiplied and stored, the rows of tile t + Gt are on their way to
        // registers and the entries of tile t + 2 Gt are being read
        for (int64_t k = 0; k < steps; k++, t += Gt) {
            const bool live = t < m_tiles;
            __syncthreads();      // previous tile's fragment reads are done (first pass: filter and padding are in)
            if (live) to_lds16(v, zmask);
            __syncthreads();
            if (t + Gt < m_tiles) {
                gather16(t + Gt, r, first, v, zmask);
                if (t + 2 * Gt < m_tiles) load_rows16(t + 2 * Gt, r, first);
            }
            if (live) multiply_and_store(t);
        }
        return;
    }
    if constexpr (TEAMS > 1) return;      // the paths below are single-team (their loops end at different times)

    for (int64_t mt = blockIdx.x; mt < g.m_tiles; mt += G) {
        __syncthreads();      // previous tile's fragment reads are done (first pass: filter and padding are in)
        if (g.direct) {
            const uint8_t* src = g.a + mt * MR * (int64_t)g.KP;
            const int vec_per_row = g.KP / 16;
            for (int v = tid; v < MR * vec_per_row; v += 256) {
                const int row = v / vec_per_row, c = v - row * vec_per_row;
                *(uint4*)(ldsA + row * pitch + c * 16) = *(const uint4*)(src + (int64_t)row * g.KP + c * 16);
            }
        }
        // gather, batch by batch: all entries of a batch are in registers before the rows they name are loaded,
        // and all rows before anything goes to LDS, so the dependent loads of the elements overlap
        for (int tap0 = tid >> 6; tap0 < n_taps; tap0 += 4 * NB) {
            int32_t e[NB];
            piece_t v[NV];
            load_entries(mt, tap0, e);
            gather(mt, e, v);
            to_lds(tap0, v);
        }
        __syncthreads();
        multiply_and_store(mt);
    }
}

int launch_igemm_lowc(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, const void* zero_row, void* out, bool a_direct, hipStream_t s)
{
    LowcArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.a = (const uint8_t*)input;
    a.zero_row = (const uint8_t*)zero_row;
    a.w = (const uint8_t*)packed;
    a.ind = ind;
    a.out = out;
    a.M = g.M; a.m_tiles = g.m_tiles;
    a.image_bytes = a_direct ? 0 : g.image_bytes;
    a.img_tiles = (uint32_t)(a_direct ? g.m_tiles : g.img_tiles);
    a.img_rows = (uint32_t)(a_direct ? g.M : g.img_rows);
    a.K = p->K; a.T = g.T; a.out_stride = g.out_stride; a.n_tiles = (int32_t)g.n_tiles;
    a.KP = g.KCB;
    a.direct = a_direct ? 1 : 0;
    a.ep = g.ep;
    a.zero_fill = p->dtype == ICV_U8I8 ? 0x01010101u * (uint32_t)p->input_zero_point : 0u;
    a.stride_bytes = g.in_stride * g.elem_bytes;
    // the compact entries (range records, then 16-bit pixel numbers) follow the int32 entries in the buffer
    a.ranges = nullptr; a.rows = nullptr;
    if (!a_direct && g.patch_rows) {
        a.ranges = (const int4*)ind;      // range records, then the 16-bit entries
        a.rows = (const uint16_t*)(a.ranges + g.img_tiles);
    }
    // 32-column blocks per workgroup: as many as fit beside the 64 gathered rows in half a compute unit's LDS
    // (two workgroups per compute unit), spread evenly over the groups
    a.k_rows = (int32_t)g.n_tiles * 64;
    const int pitch = a.KP + 16;
    const int kb_total = (p->K + 31) / 32;
    int cb_max = (80 * 1024 / pitch - 64) / 32;
    if (cb_max < 1) return ICV_ERR_UNSUPPORTED;
    if (cb_max > kMaxColBlocks) cb_max = kMaxColBlocks;
    if (cb_max > kb_total) cb_max = kb_total;
    const int groups = (kb_total + cb_max - 1) / cb_max;
    a.col_blocks = (kb_total + groups - 1) / groups;
    if (groups > 65535) return ICV_ERR_UNSUPPORTED;
    const int unit = p->C * g.elem_bytes;
    const bool i8 = p->dtype == ICV_U8I8;
    // Teams per workgroup: the path that gathers a whole tile from compact entries in one batch runs several teams
    // on one filter slice (four for the 8-byte rows, two for the wider ones, whose batches need twice the
    // registers), one workgroup per compute unit; every other path runs single teams, two workgroups per compute unit.
    const size_t b_bytes = (size_t)32 * a.col_blocks * pitch, a_bytes = (size_t)64 * pitch;
    const int batch_taps = unit == 32 ? 32 : 64;
    int teams = 1;
    if (!a_direct && a.rows && g.T <= batch_taps) {
        const int fit = (int)((kLdsPerCu - b_bytes) / a_bytes);
        const int want = unit == 8 ? 4 : 2;
        teams = fit >= want ? want : (fit >= 2 ? 2 : 1);
    }
    const size_t lds_bytes = b_bytes + teams * a_bytes;
    const int cus = device_cu_count();
    int64_t gx = (int64_t)cus * (teams > 1 ? 1 : 2) / groups;      // workgroups, shared among the column groups
    if (gx < 1) gx = 1;
    if (gx * teams > g.m_tiles) gx = (g.m_tiles + teams - 1) / teams;
    const dim3 grid((unsigned)gx, (unsigned)groups);
#define ICV_LOWC_LAUNCH_T(I8, U, TEAMS)                                                                         \
    do {                                                                                                        \
        auto kern = g.ep_plain ? k_igemm_lowc<I8, U, false, TEAMS> : k_igemm_lowc<I8, U, true, TEAMS>;          \
        if (lds_bytes > 64 * 1024) {                                                                            \
            static bool raised[2][kMaxDevices] = {};         /* per instantiation and device */                \
            const int st_ = allow_full_lds((const void*)kern, raised[g.ep_plain ? 0 : 1]);                      \
            if (st_ != ICV_OK) return st_;                                                                      \
        }                                                                                                       \
        hipLaunchKernelGGL(kern, grid, dim3(256 * TEAMS), lds_bytes, s, a);                                     \
    } while (0)
#define ICV_LOWC_LAUNCH(I8, U)                                                                                  \
    do {                                                                                                        \
        if (teams == 4) ICV_LOWC_LAUNCH_T(I8, U, 4);                                                            \
        else if (teams == 2) ICV_LOWC_LAUNCH_T(I8, U, 2);                                                       \
        else ICV_LOWC_LAUNCH_T(I8, U, 1);                                                                       \
    } while (0)
    if (unit == 8) { if (i8) ICV_LOWC_LAUNCH(true, 8); else ICV_LOWC_LAUNCH(false, 8); }
    else if (unit == 16) { if (i8) ICV_LOWC_LAUNCH(true, 16); else ICV_LOWC_LAUNCH(false, 16); }
    else if (unit == 32) { if (i8) ICV_LOWC_LAUNCH(true, 32); else ICV_LOWC_LAUNCH(false, 32); }
    else return ICV_ERR_UNSUPPORTED;
#undef ICV_LOWC_LAUNCH
#undef ICV_LOWC_LAUNCH_T
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

}  // namespace icv
