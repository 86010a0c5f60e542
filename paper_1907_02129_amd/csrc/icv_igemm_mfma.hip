// Tensor-core Indirect GEMM for gfx950 (section 2.2, Listing 3, re-designed around MFMA).
//
// Listing 3 is kept as the shape of the computation: an MR x NR output tile (MR output pixels x NR output
// channels, the paper's micro-kernel tile scaled up to a compute unit) accumulates over two nested loops --
// the outer one walks the R*S kernel elements and fetches the tile's MR row pointers from the indirection
// buffer, the inner one walks the C channels of the rows they name.  What changes is how it is executed:
//
//  * Persistent workgroups.  The grid is sized to the chip (one or two workgroups per compute unit) and every
//    workgroup walks a list of tiles.  The stages of all its tiles form one stream, so the next tile's
//    operands are already in flight while the current tile is multiplied and stored; a convolution layer is
//    a few microseconds of work, and per-tile start-up latency would otherwise dominate it.
//  * Producer / consumer wavefronts.  A workgroup is eight wavefronts: four producers move data, four
//    consumers run MFMA and store results.  A pipeline stage covers one kernel element and KCB bytes of its
//    channels:
//       A stage tile: MR gathered rows x KCB bytes, each row read from the input tensor (or the zero row)
//                     with 16-byte pieces, lanes running along the channels first;
//       B stage tile: NR filter rows x KCB bytes, one contiguous block of the pre-packed filter.
//    Producers copy both straight from global memory into a ring of LDS slots (global_load_lds_dwordx4, no
//    register stop) and run up to `ring - 1` stages ahead.  They count their own outstanding copies with
//    s_waitcnt vmcnt; consumers never wait on memory except LDS, and their output stores never delay a load.
//    One s_barrier per stage hands a filled slot to the consumers and a drained one back to the producers.
//  * Both tiles keep the reduction dimension contiguous, which is the operand layout of
//    v_mfma_f32_32x32x16_bf16 / v_mfma_i32_32x32x32_i8: lane l supplies 16 contiguous bytes of row (l & 31),
//    byte offset 16*(l >> 5) inside a 32-byte k-step.  LDS rows are XOR-swizzled in 16-byte units so the
//    ds_read_b128 fragment reads of 32 different rows spread over all banks; the swizzle is applied by
//    choosing which source piece each lane copies, since a wavefront-wide copy fills 1 KB of LDS linearly.
//  * The indirection entries of a tile (MR * T int32, contiguous thanks to the [tile][tap][row] order) are
//    themselves copied to LDS one tile ahead, each producer fetching the quarter of the rows it serves, so the
//    pointer -> data dependency of Listing 3 never waits on HBM inside the loop.
//  * XCD-aware tile order: every XCD (own L2) gets one contiguous range of tiles, and its workgroups sweep it
//    side by side, so neighbouring row tiles -- which share most input rows for a 3x3 kernel -- meet in L2.
//
// uint8 activations: MFMA multiplies signed bytes, so every A fragment is XORed with 0x80, which turns
// x into x - 128 exactly; the zero row (filled with the zero point 128) becomes a row of zeros.
#include "icv_mfma_common.h"

namespace icv {

struct IgemmArgs {
    const uint8_t* a;         // input tensor | im2col matrix
    const uint8_t* zero_row;
    const uint8_t* w;         // packed filter [n tile][stage][NR][KCB]
    const int32_t* ind;       // [m tile][tap][MR]
    void* out;
    int64_t M;
    int64_t row_stride_bytes;  // input pixel stride | im2col row stride
    int64_t total_tiles;       // m_tiles * n_tiles
    int32_t K, T, out_stride;
    int32_t stages_per_tap, n_stages;
    int32_t n_tiles;
    int32_t ring;              // LDS slots in the ring, 2..6
    int32_t ent_copies;        // wavefront-wide copies per producer per tile of entries
    int32_t xcd_mode;          // 1: grid is a multiple of 8 and tiles are dealt per XCD
    int32_t cc_major;          // packed filter stage order: 1 = chunk * T + tap, 0 = tap * stages_per_tap + chunk
    int32_t row_bytes;         // C * element size
    int64_t a_rows;            // rows of the dense matrix that may be read (later rows of a tile re-read the last one)
    int64_t image_bytes;       // batch-independent buffer: bytes between batch elements of the input (else 0)
    uint32_t img_tiles, img_rows;  // row tiles and output pixels per image (one image = the whole batch otherwise)
    EpilogueArgs ep;           // output stage (read by the FUSED instantiations only)
};

template <int DT, int MR, int NR, int WM, int WN, int NP, int KCB, bool DIRECT, bool FUSED>
__global__ __launch_bounds__(64 * (WM * WN + NP)) void k_igemm_mfma(IgemmArgs g)
{
    constexpr int NC = WM * WN;              // consumer wavefronts; NP producer wavefronts follow them
    constexpr int Q = KCB / 16;              // 16-byte chunks per row per stage
    constexpr int P = 256 / KCB;             // rows per 256 bytes of LDS
    constexpr int RPB = 1024 / KCB;          // rows one wavefront-wide copy (64 x 16 B) covers
    constexpr int A_VEC = MR * KCB / 1024 / NP;   // copies per producer per stage, A tile (MR/NP of its rows)
    constexpr int B_VEC = NR * KCB / 1024 / NP;   // ... B tile
    constexpr int LP = A_VEC + B_VEC;
    constexpr int MRW = MR / WM, NRW = NR / WN;
    constexpr int MB = MRW / 32, NB = NRW / 32;
    constexpr int KSTEPS = KCB / 32;
    constexpr int SLOT = (MR + NR) * KCB;    // bytes of one ring slot: A tile then B tile
    static_assert(A_VEC >= 1 && B_VEC >= 1 && MB >= 1 && NB >= 1, "tile too small for this wavefront split");
    static_assert(A_VEC * NP * 1024 == MR * KCB && B_VEC * NP * 1024 == NR * KCB, "copies must divide evenly");
    static_assert(4 * LP <= 63, "vmcnt is a 6-bit counter");
    static_assert((MR / NP) % RPB == 0, "a producer's rows are whole copy blocks");
    constexpr bool I8 = DT == ICV_U8I8;      // DT: the icv_dtype of input and filter
    using acc_t = typename Acc<I8>::type;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const int D = g.ring;
    const int ent_base = D * SLOT;                       // [parity][tap][MR] int32, each parity ent_bytes long
    const int ent_bytes = g.ent_copies * 1024;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const TileList tl = my_tiles(g.total_tiles, g.xcd_mode);
    const int n_stages = g.n_stages;
    const int64_t total_stages = tl.count * n_stages;                // same value in every wavefront

    if (wave >= NC) {
        // =============================================================== producer
        const int p = wave - NC;
        const int lrow_in_blk = lane / Q;

        // source piece of each copy: LDS chunk (lane % Q) of row r must hold source chunk (lane % Q) ^ swz(r)
        int a_lane_off[A_VEC];       // byte offset inside the KCB bytes of the row
        int a_row[A_VEC];            // row of the tile this lane copies
#pragma unroll
        for (int j = 0; j < A_VEC; j++) {
            a_row[j] = (p * A_VEC + j) * RPB + lrow_in_blk;
            a_lane_off[j] = ((lane % Q) ^ ((a_row[j] / P) % Q)) << 4;
        }
        int b_src_off[B_VEC];
#pragma unroll
        for (int j = 0; j < B_VEC; j++) {
            const int row = (p * B_VEC + j) * RPB + lrow_in_blk;
            b_src_off[j] = row * KCB + (((lane % Q) ^ ((row / P) % Q)) << 4);
        }

        // entries of my k-th tile -> ENT[k & 1]; the T*MR int32 are one contiguous run, the producers share it
        // in 1 KB pieces.  A piece issued here is complete, and visible to every wavefront, once its issuer has
        // passed ring-1 more stage waits and barriers; the host keeps ring - 1 <= n_stages, so that is always
        // before the first stage of tile k is copied.
        auto fetch_entries = [&](int64_t k) {
            if constexpr (!DIRECT) {
                if (k >= tl.count) return;
                const int64_t mt = (uint32_t)((tl.first + k * tl.step) / g.n_tiles) % g.img_tiles;      // tile of the buffer
                const int32_t* src = g.ind + mt * ((int64_t)g.T * MR);
                const uint32_t dst = lds_base + ent_base + (uint32_t)(k & 1) * ent_bytes;
                const int n_chunks = g.T * MR / 4;
                for (int u = p; u < g.ent_copies; u += NP) {
                    const int c = u * 64 + lane;
                    if (c < n_chunks) copy16_global_to_lds(src + c * 4, dst + u * 1024);
                }
            }
        };

        // Copy cursor.  A stage is handled in two steps: `prepare` turns its indirection entries into source
        // addresses (kept in registers), `issue` fires the copies.  The addresses of the next stage are prepared
        // right after the copies of the current one were issued, so that work overlaps with the memory pipeline
        // draining instead of delaying the next burst of copies.  Everything that only changes per tile or per
        // kernel element is carried along incrementally.
        int64_t ik = 0;          // tile index in my list (of the stage to prepare next)
        int is = 0;              // stage within the tile
        int itap = 0, icc = 0;   // kernel element and channel chunk of stage `is`
        int islot = 0;           // ring slot the next issued stage goes to
        const uint8_t* wstage = nullptr;     // B tile of the stage to prepare, before the per-lane offset
        const uint8_t* adirect[A_VEC];       // DIRECT: the rows of the tile this lane copies from (clamped to the matrix)
        const uint8_t* a_img = g.a;          // the batch element the tile's entries refer to
        auto enter_tile = [&]() {
            if (ik >= tl.count) return;
            const int64_t tile = tl.first + ik * tl.step;
            const int32_t nt = (int32_t)(tile % g.n_tiles);
            const int64_t mt = tile / g.n_tiles;
            a_img = g.a + ((uint32_t)mt / g.img_tiles) * g.image_bytes;
            wstage = g.w + ((int64_t)nt * n_stages) * (NR * KCB);
            if constexpr (DIRECT) {
#pragma unroll
                for (int j = 0; j < A_VEC; j++) {
                    const int64_t row = mt * MR + a_row[j];
                    adirect[j] = g.a + (row < g.a_rows ? row : g.a_rows - 1) * g.row_stride_bytes;
                }
            }
        };
        enter_tile();

        const uint8_t* asrc[A_VEC];          // prepared source addresses of the next stage to issue
        const uint8_t* bsrc = nullptr;
        bool prepared = false;
        auto prepare = [&]() {
            prepared = ik < tl.count;
            if (!prepared) return;
            if constexpr (DIRECT) {
                // byte offset of this stage inside a patch-matrix row ([tap][C])
                const int64_t koff = g.cc_major ? (int64_t)(is % g.T) * g.row_bytes + (int64_t)(is / g.T) * KCB
                                                : (int64_t)is * KCB;
#pragma unroll
                for (int j = 0; j < A_VEC; j++)
                    asrc[j] = adirect[j] + koff + a_lane_off[j];
            } else {
                const int32_t* ent = (const int32_t*)(lds + ent_base + (int)(ik & 1) * ent_bytes) + itap * MR;
                int32_t e[A_VEC];
#pragma unroll
                for (int j = 0; j < A_VEC; j++) e[j] = ent[a_row[j]];     // all LDS reads first
                const uint8_t* zsrc = g.zero_row + icc * KCB;
                const uint8_t* abase = a_img + icc * KCB;
#pragma unroll
                for (int j = 0; j < A_VEC; j++) {
                    // entry = byte offset of the pixel row from the input base; negative = the zero row
                    const uint32_t off = (uint32_t)(e[j] + a_lane_off[j]);
                    asrc[j] = e[j] < 0 ? zsrc + a_lane_off[j] : abase + off;
                }
            }
            bsrc = wstage;
            wstage += NR * KCB;
            if (++icc == g.stages_per_tap) { icc = 0; ++itap; }
            if (++is == n_stages) {
                // every stage of tile ik has its addresses: its entry buffer is free for the tile after next
                is = 0; itap = 0; icc = 0;
                fetch_entries(ik + 2);
                ++ik;
                enter_tile();
            }
        };
        auto issue = [&]() {
            if (!prepared) return;
            const uint32_t slot = lds_base + (uint32_t)islot * SLOT;
#pragma unroll
            for (int j = 0; j < A_VEC; j++) copy16_global_to_lds(asrc[j], slot + (p * A_VEC + j) * 1024);
#pragma unroll
            for (int j = 0; j < B_VEC; j++)
                copy16_global_to_lds(bsrc + b_src_off[j], slot + MR * KCB + (p * B_VEC + j) * 1024);
            islot = islot + 1 == D ? 0 : islot + 1;
        };

        fetch_entries(0);
        fetch_entries(1);
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();         // entries of the first two tiles are visible to all producers
        prepare();
        for (int q = 0; q < D - 1; q++) { issue(); prepare(); }
        for (int64_t q = 0; q < total_stages; q++) {
            // stage q has landed once only the copies of younger stages (at most D-2 of them) are outstanding
            const int64_t younger = total_stages - 1 - q;
            wait_all_but_stages<LP>(younger < D - 2 ? (int)younger : D - 2);
            __builtin_amdgcn_s_barrier();     // hand stage q to the consumers; they are done with stage q-1
            issue();                          // stage q + D - 1 refills the slot stage q - 1 used
            prepare();                        // addresses of stage q + D, while those copies are in flight
        }
        wait_vmcnt<0>();
    } else {
        // =============================================================== consumer
        const int wm = wave / WN, wn = wave % WN;
        const int lrow = lane & 31, lhalf = lane >> 5;
        const int swz = (lrow / P) % Q;          // tile bases are multiples of 32 rows, and 32 % (P*Q) == 0
        const uint32_t a_frag_base = (wm * MRW + lrow) * KCB;
        const uint32_t b_frag_base = MR * KCB + (wn * NRW + lrow) * KCB;
        using out_t = typename std::conditional<I8, int32_t, float>::type;

        __builtin_amdgcn_s_barrier();         // pairs with the producers' start-up barrier
        int slot = 0;
        for (int64_t k = 0; k < tl.count; k++) {
            acc_t acc[MB][NB];
#pragma unroll
            for (int i = 0; i < MB; i++)
#pragma unroll
                for (int j = 0; j < NB; j++)
#pragma unroll
                    for (int r = 0; r < 16; r++) acc[i][j][r] = 0;

            for (int s = 0; s < n_stages; s++) {
                __builtin_amdgcn_s_barrier();
                const uint8_t* S = lds + slot * SLOT;
                slot = slot + 1 == D ? 0 : slot + 1;
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
                        for (int j = 0; j < NB; j++) {
                            if constexpr (DT == ICV_F32) acc[i][j] = mfma32_f32(af[i], bf[j], acc[i][j]);
                            else acc[i][j] = mfma32<I8>(af[i], bf[j], acc[i][j]);
                        }
                }
            }

            // epilogue: accumulator register r of lane l holds row 8*(r/4) + 4*(l>>5) + (r&3), column l&31
            const int64_t tile = tl.first + k * tl.step;
            const int32_t nt = (int32_t)(tile % g.n_tiles);
            const int64_t mt = tile / g.n_tiles;
            const uint32_t img = (uint32_t)mt / g.img_tiles, t_img = (uint32_t)mt - img * g.img_tiles;      // batch element, row tile in it
            const int64_t img_row0 = (int64_t)img * g.img_rows;
            const int64_t m_base = img_row0 + (int64_t)t_img * MR + wm * MRW + 4 * lhalf;
            const int32_t n_base = nt * NR + wn * NRW + lrow;
            const bool whole = (t_img + 1) * MR <= g.img_rows && (nt + 1) * NR <= g.K;     // no row or column tail
            store_tile<FUSED, I8, MB, NB>(g.out, acc, img_row0 + g.img_rows, g.K, g.out_stride, m_base, n_base, whole, g.ep);
        }
    }
}

// ------------------------------------------------------------------ launch
template <int DT, int MR, int NR, int WM, int WN, int NP, int KCB, bool DIRECT, bool FUSED>
static int launch_one(const Geometry& g, IgemmArgs a, hipStream_t s)
{
    constexpr int threads = 64 * (WM * WN + NP);
    auto kern = k_igemm_mfma<DT, MR, NR, WM, WN, NP, KCB, DIRECT, FUSED>;
    constexpr size_t slot = (size_t)(MR + NR) * KCB;
    a.ent_copies = DIRECT ? 0 : (int32_t)(((size_t)g.T * MR * 4 + 1023) / 1024);
    const size_t ent = (size_t)2 * a.ent_copies * 1024;
    // ring depth and workgroups per CU: two co-resident workgroups when each can still have >= 3 slots,
    // otherwise one workgroup with as deep a ring as fits (at most 6 slots).  The ring never runs further
    // ahead than one tile's worth of stages (ring - 1 <= n_stages): the entry prefetch relies on it.
    int per_cu = g.blocks_per_cu, ring = g.ring;
    if (per_cu == 0) per_cu = (threads <= 512 && kLdsPerCu / 2 >= ent + 3 * slot) ? 2 : 1;
    if (threads > 512) per_cu = 1;
    const size_t budget = kLdsPerCu / per_cu;
    if (budget < ent + 2 * slot) return ICV_ERR_UNSUPPORTED;
    const int fit = (int)((budget - ent) / slot);
    if (ring == 0) ring = fit;
    if (ring > fit) ring = fit;
    if (ring > 6) ring = 6;
    if (ring > g.n_stages + 1) ring = g.n_stages + 1;
    if (ring < 2) return ICV_ERR_UNSUPPORTED;
    a.ring = ring;
    const size_t lds_bytes = ent + (size_t)ring * slot;

    // One workgroup per tile when the tiles fit the chip's slots, else as many as there are slots.  The XCD-aware
    // tile order needs a multiple of 8 workgroups: rounded UP to it when every tile can have its own workgroup (the
    // surplus ones find no tile and leave) -- rounding down would give a few workgroups a second tile and double
    // the kernel's duration.
    const int64_t slots = (int64_t)device_cu_count() * per_cu;
    int64_t grid = slots < a.total_tiles ? slots : a.total_tiles;
    a.xcd_mode = 0;
    if (slots >= 8 && a.total_tiles >= 8) {
        const int64_t up = (a.total_tiles + 7) / 8 * 8, down = slots - slots % 8;
        grid = up < down ? up : down;
        a.xcd_mode = 1;
    }
    if (lds_bytes > 64 * 1024) {
        static bool raised[kMaxDevices] = {};      // one array per instantiation of this function template
        const int st = allow_full_lds((const void*)kern, raised);
        if (st != ICV_OK) return st;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(threads), lds_bytes, s, a);
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

// picks the DIRECT (dense A) and FUSED (output stage) instantiation
template <int DT, int MR, int NR, int WM, int WN, int NP, int KCB>
static int launch_pick(const Geometry& g, const IgemmArgs& a, bool direct, hipStream_t s)
{
    if (direct)
        return g.ep_plain ? launch_one<DT, MR, NR, WM, WN, NP, KCB, true, false>(g, a, s)
                          : launch_one<DT, MR, NR, WM, WN, NP, KCB, true, true>(g, a, s);
    return g.ep_plain ? launch_one<DT, MR, NR, WM, WN, NP, KCB, false, false>(g, a, s)
                      : launch_one<DT, MR, NR, WM, WN, NP, KCB, false, true>(g, a, s);
}

template <int DT, int MR, int NR, int WM, int WN, int NP>
static int launch_tile(const Geometry& g, const IgemmArgs& a, bool direct, hipStream_t s)
{
    if (g.KCB == 128) {
        return launch_pick<DT, MR, NR, WM, WN, NP, 128>(g, a, direct, s);
    }
    if constexpr (NR * 64 / 1024 >= NP) {      // a 64-byte stage of the B tile must still split over the copying wavefronts
        return launch_pick<DT, MR, NR, WM, WN, NP, 64>(g, a, direct, s);
    } else {
        return launch_pick<DT, MR, NR, WM, WN, 4, 64>(g, a, direct, s);
    }
}

template <int DT>
static int launch_dtype(const Geometry& g, const IgemmArgs& a, bool direct, hipStream_t s)
{
    switch (g.variant) {
        case 0: return launch_tile<DT, 128, 64, 2, 2, 4>(g, a, direct, s);
        case 1: return launch_tile<DT, 128, 128, 2, 2, 4>(g, a, direct, s);
        case 3: return launch_tile<DT, 256, 64, 4, 2, 8>(g, a, direct, s);
        case 4: return launch_tile<DT, 64, 64, 2, 2, 4>(g, a, direct, s);
        default: return ICV_ERR_UNSUPPORTED;
    }
}

int launch_igemm_mfma(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                      const int32_t* ind, const void* zero_row, void* out, int a_mode, hipStream_t s)
{
    // A dense A matrix is either the im2col workspace (rows of T*C elements, padded to whole tiles) or, for a
    // 1x1 stride-1 unpadded convolution, the input tensor itself (M rows of in_pixel_stride elements).
    const bool a_direct = a_mode != A_GATHERED, on_input = a_mode == A_DENSE_INPUT;
    // the host-side table and the instantiations above must describe the same tiles
    const TileVariant& tv = kTileVariants[g.variant];
    if (tv.MR != g.MR || tv.NR != g.NR) return ICV_ERR_UNSUPPORTED;
    IgemmArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.a = (const uint8_t*)input;
    a.zero_row = (const uint8_t*)zero_row;
    a.w = (const uint8_t*)packed;
    a.ind = ind;
    a.out = out;
    a.M = g.M;
    a.row_stride_bytes = a_direct && !on_input ? (int64_t)g.T * p->C * g.elem_bytes : (int64_t)g.in_stride * g.elem_bytes;
    a.a_rows = on_input ? g.M : g.m_tiles * g.MR;
    a.image_bytes = a_direct ? 0 : g.image_bytes;
    a.img_tiles = (uint32_t)(a_direct ? g.m_tiles : g.img_tiles);
    a.img_rows = (uint32_t)(a_direct ? g.M : g.img_rows);
    a.total_tiles = g.m_tiles * g.n_tiles;
    if (a.total_tiles >= (1ll << 31)) return ICV_ERR_UNSUPPORTED;      // the kernels count tiles in 32 bits
    a.K = p->K; a.T = g.T; a.out_stride = g.out_stride;
    a.stages_per_tap = g.stages_per_tap; a.n_stages = g.n_stages;
    a.n_tiles = (int32_t)g.n_tiles;
    a.ring = 0; a.ent_copies = 0; a.xcd_mode = 0;
    a.cc_major = g.cc_major; a.row_bytes = p->C * g.elem_bytes;
    a.ep = g.ep;
    if (p->dtype == ICV_F32) return launch_dtype<ICV_F32>(g, a, a_direct, s);
    return p->dtype == ICV_U8I8 ? launch_dtype<ICV_U8I8>(g, a, a_direct, s) : launch_dtype<ICV_BF16>(g, a, a_direct, s);
}

}  // namespace icv
