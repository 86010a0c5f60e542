// Tensor-core Indirect GEMM with the gathered rows kept in LDS across kernel elements.
//
// Listing 3 reads, for every kernel element, the MR rows its indirection entries name.  For a convolution the
// R*S entries of neighbouring output pixels name mostly the same input pixels (the second performance factor
// section 3 lists: rows contributing to different output pixels are read from the same location); here that
// re-use is made explicit.  The valid entries of a tile of MR consecutive output pixels all fall into one short
// range of consecutive input pixels, so that range ("patch") is copied to LDS once per tile and channel chunk,
// and every kernel element then takes its MR rows from the patch.  The set-up phase prepares this next to the
// int32 entries: per tile a range record {first byte offset, pixel count}, and the tile's entries rewritten as
// 16-bit LDS row numbers,
//
//     row number of entry e  =  (e - first offset of the tile) / pixel stride      (zero row: the row after the patch)
//
// which is what the kernel reads: half the bytes of the entries, and no subtraction, shift or select per lookup.
//
// The loop nest is Listing 3's with the channel chunks outermost (chunk, kernel element, channels of the chunk);
// only the filter tile of a stage (NR rows x KCB bytes, contiguous in the packed filter) still streams through a
// small LDS ring.  Compared with gathering the rows of every kernel element separately this moves R*S times
// fewer input bytes into LDS, and LDS bandwidth -- fragment reads plus fills -- is what bounds these kernels.
//
// Execution model (same as the streamed kernel): persistent workgroups, NC consumer wavefronts running MFMA and
// NP producer wavefronts issuing global -> LDS copies, one s_barrier per stage, producers counting their own
// outstanding copies with s_waitcnt vmcnt.  Per stage every producer issues a share of the next patch and of the
// next tile's entries, then its part of the filter tile of stage q + ring - 1; the wait before stage q is "at
// most the filter copies of ring - 2 stages outstanding", which is conservative for the shares in between.
//
// Patch rows are XOR-swizzled like the stage tiles of the streamed kernel (LDS row r holds source piece
// c ^ swz(r) at piece c), the consumer applies swz(r) of the row its entry names.
#include "icv_mfma_common.h"

namespace icv {

struct PatchArgs {
    const uint8_t* a;          // input tensor
    const uint8_t* w;          // packed filter [n tile][channel chunk][tap][NR][KCB]
    const uint16_t* rows;      // [m tile][tap][MR]: the entries as LDS row numbers of the tile's patch (set-up makes them)
    const int4* ranges;        // per m tile: {first byte offset, pixel rows, 0, 0}
    void* out;
    int64_t M;
    int64_t total_tiles;       // m_tiles * n_tiles
    int64_t image_bytes;       // batch-independent buffer: bytes between batch elements of the input (else 0)
    uint32_t img_tiles, img_rows;   // row tiles and output pixels per image (one image = the whole batch otherwise)
    int32_t stride_bytes, stride_shift;   // bytes between input pixels, a power of two
    int32_t K, T, NCC, out_stride, n_tiles;
    int32_t ring;              // filter slots in the ring
    int32_t G;                 // kernel elements per pipeline stage (divides T): one barrier per G filter tiles
    int32_t TS;                // T / G: stages per channel chunk (from the host, a division less at start-up)
    int32_t ent_copies;        // 1 KB pieces of one tile's row numbers
    int32_t cap_units;         // 1 KB pieces of one patch buffer (the zero row follows them)
    int32_t a_share, e_share;  // copies per producer per stage: next patch, next entries
    int32_t nbuf;              // 2: the next patch and entries load while the current ones are used; 1: one buffer,
                               //    loaded between patches (for two workgroups per compute unit, which cover
                               //    each other's load bubbles)
    int32_t xcd_mode;
    uint32_t zero_fill;        // four bytes of the zero row: zeros, or the zero point of uint8 activations
    EpilogueArgs ep;           // output stage (read by the FUSED instantiations only)
};

template <int DT, int MR, int NR, int WM, int WN, int NP, int KCB, bool FUSED>
__global__ __launch_bounds__(64 * (WM * WN + NP)) void k_igemm_patch(PatchArgs g)
{
    constexpr int NC = WM * WN;
    constexpr int Q = KCB / 16;              // 16-byte pieces per row per stage
    constexpr int P = 256 / KCB;             // rows per 256 bytes of LDS
    constexpr int RPB = 1024 / KCB;          // rows one wavefront-wide copy covers
    constexpr int B_VEC = NR * KCB / 1024 / NP;
    constexpr int MRW = MR / WM, NRW = NR / WN;
    constexpr int MB = MRW / 32, NB = NRW / 32;
    constexpr int KSTEPS = KCB / 32;
    constexpr int BS = NR * KCB;             // bytes of one filter-tile slot
    static_assert(B_VEC >= 1 && B_VEC * NP * 1024 == NR * KCB, "filter tile must split over the producers");
    static_assert(MB >= 1 && NB >= 1, "tile too small for this wavefront split");
    constexpr bool I8 = DT == ICV_U8I8;      // DT: the icv_dtype of input and filter
    using acc_t = typename Acc<I8>::type;
    using out_t = typename std::conditional<I8, int32_t, float>::type;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const int D = g.ring;
    const int pbytes = (g.cap_units + 1) * 1024;          // patch buffer: cap_units pieces, then the zero row
    const int zoff = g.cap_units * 1024;
    const int G = g.G;
    const int slot_bytes = G * BS;                        // one stage: the filter tiles of G kernel elements
    const int patch_base = D * slot_bytes;
    const bool single = g.nbuf == 1;
    const uint32_t bufmask = single ? 0u : 1u;            // buffer of patch / tile number x: x & bufmask
    const int ent_base = patch_base + g.nbuf * pbytes;
    const int ent_bytes = g.ent_copies * 1024;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const TileList tl = my_tiles(g.total_tiles, g.xcd_mode);
    const int T = g.T, NCC = g.NCC;
    const int TS = g.TS;                                  // stages per channel chunk
    const int n_st = NCC * TS;                            // stages per tile, stage = chunk * TS + tap / G
    const int64_t total_stages = tl.count * n_st;

    const int lrow_in_blk = lane / Q, lchunk = lane % Q;
    const uint32_t n_tiles = (uint32_t)g.n_tiles;
    // (the common cases -- one column tile, a whole-batch buffer -- skip the integer divisions: each is a few
    // dozen scalar instructions on the start-up path)
    const bool one_col = n_tiles == 1, per_image = g.image_bytes != 0;
    auto m_tile_of = [&](int k) {                                                               // global row tile
        const uint32_t t = (uint32_t)(tl.first + k * tl.step);
        return one_col ? t : t / n_tiles;
    };
    auto buf_tile_of = [&](int k) { return per_image ? m_tile_of(k) % g.img_tiles : m_tile_of(k); };    // ... in the buffer
    auto image_of = [&](int k) { return per_image ? m_tile_of(k) / g.img_tiles : 0u; };                  // batch element
    auto n_tile_of = [&](int k) { return one_col ? 0u : (uint32_t)(tl.first + k * tl.step) % n_tiles; };
    const int count = (int)tl.count;
    // range record {first byte offset, pixel rows} of my k-th tile, read through the constant address space:
    // a scalar load, which neither touches the vector-memory counter the copies are tracked with nor makes the
    // compiler wait on it
    auto load_range = [&](int k) {
        int2 r = make_int2(0, 1);
        if (k < count) {
            typedef const int32_t __attribute__((address_space(4))) * const_int_ptr;
            const_int_ptr rec = (const_int_ptr)(uintptr_t)(g.ranges + buf_tile_of(k));
            r = make_int2(rec[0], rec[1]);
        }
        return r;
    };
    // piece u of a patch: LDS rows u*RPB .. +RPB hold pixels first + row (clamped to the tile's range, so the
    // read stays inside the tensor), channel chunk cc, piece c of row r taken from source piece c ^ swz(r)
    auto copy_patch_piece = [&](int u, const uint8_t* src, int nrows, uint32_t dst) {
        const uint32_t r = (uint32_t)(u * RPB + lrow_in_blk);
        const uint32_t rc = r < (uint32_t)nrows ? r : (uint32_t)nrows - 1;
        const uint32_t off = (rc << g.stride_shift) + ((lchunk ^ ((r / P) % Q)) << 4);
        copy16_global_to_lds(src, off, dst + u * 1024);
    };
    // piece u of a tile's row numbers (T * MR uint16, contiguous)
    const int ent_chunks = T * MR / 8;
    auto copy_ent_piece = [&](int u, const uint16_t* src, uint32_t par) {
        if (u < g.ent_copies) {
            const int c = u * 64 + lane;
            if (c < ent_chunks) copy16_global_to_lds(src, (uint32_t)c * 16u, lds_base + ent_base + par * ent_bytes + u * 1024);
        }
    };


    // ---- start-up, all wavefronts: the first tile's entries, the filter stages the ring runs ahead by, and the first
    // patch.  Everything but the patch is issued before the tile's range record (a dependent scalar load) is needed.
    if (count > 0) {
        constexpr int NW = NC + NP;
        const uint32_t mt = buf_tile_of(0);
        for (int u = wave; u < g.ent_copies; u += NW) copy_ent_piece(u, g.rows + (int64_t)mt * T * MR, 0);
        // stages 0 .. D-2 are contiguous in the packed filter and in the ring (the host keeps D - 1 <= stages per tile)
        const uint8_t* w0 = g.w + (int64_t)n_tile_of(0) * n_st * slot_bytes;
        const int b_pieces = (D - 1) * slot_bytes / 1024;
        for (int u = wave; u < b_pieces; u += NW) {
            const int row = u * RPB + lrow_in_blk;
            copy16_global_to_lds(w0, (uint32_t)(row * KCB + ((lchunk ^ ((row / P) % Q)) << 4)), lds_base + u * 1024);
        }
        const int2 rng0 = load_range(0);
        int units = (rng0.y + RPB - 1) / RPB;
        if (units > g.cap_units) units = g.cap_units;
        for (int u = wave; u < units; u += NW)
            copy_patch_piece(u, g.a + (int64_t)image_of(0) * g.image_bytes + rng0.x, rng0.y, lds_base + patch_base);
    }

    if (wave >= NC) {
        // =============================================================== producer
        // The per-stage body below is the critical path of a stage whenever the consumers have little to do (one
        // wavefront issues an instruction every few cycles only), so everything that can be is precomputed,
        // uniform values stay in scalar registers, and per-lane addresses are 32-bit offsets from uniform bases.
        const int p = wave - NC;
        uint32_t b_src_off[B_VEC];
#pragma unroll
        for (int j = 0; j < B_VEC; j++) {
            const int row = (p * B_VEC + j) * RPB + lrow_in_blk;
            b_src_off[j] = row * KCB + ((lchunk ^ ((row / P) % Q)) << 4);
        }
        // filter cursor: the next stage to issue is stage bs of my tile bk, into slot bslot; a stage's G filter
        // tiles are contiguous in the packed filter
        int bk = 0, bs = 0, bslot = 0;
        const uint8_t* wsrc = g.w + (int64_t)(count > 0 ? n_tile_of(0) : 0) * n_st * slot_bytes;
        auto issue_b = [&](bool copy) {
            if (bk >= count) return;
            if (copy) {
                uint32_t dst = lds_base + (uint32_t)bslot * slot_bytes + p * B_VEC * 1024;
                for (int t = 0; t < G; t++) {
#pragma unroll
                    for (int j = 0; j < B_VEC; j++) copy16_global_to_lds(wsrc, b_src_off[j], dst + j * 1024);
                    wsrc += BS;
                    dst += BS;
                }
            } else {
                wsrc += slot_bytes;
            }
            bslot = bslot + 1 == D ? 0 : bslot + 1;
            if (++bs == n_st) {
                bs = 0;
                if (++bk < count) wsrc = g.w + (int64_t)n_tile_of(bk) * n_st * slot_bytes;
            }
        };
        for (int q = 0; q < D - 1; q++) issue_b(false);     // those stages were copied at start-up
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();         // first tile's entries, patch and filter stages are in LDS

        // Shares go out before the stage's filter tiles.  Copies retire in order, so "at most ALLOWED <= (ring-2) *
        // G * B_VEC copies outstanding" then implies: the filter tiles issued ring-1 stages ago have landed, and so
        // has every share issued ring-1 or more stages ago -- which is why shares stop ring-1 stages before their
        // data is needed.  s_waitcnt takes an immediate, so the loop is instantiated for a few allowances and the
        // largest one not above the exact value is used (waiting for more than necessary is always safe).
        const int a_last = TS - D + 1, e_last = n_st - D + 1;     // last stage of a patch / tile that still carries a share
        auto run = [&](auto allowed_c) {
            constexpr int ALLOWED = decltype(allowed_c)::value;
            int younger = (int)total_stages - 1;                  // stages after the one being handed over
            int2 rng_k = load_range(0), rng_k1 = load_range(1);
            for (int k = 0; k < count; k++) {
                const bool next_tile = k + 1 < count;
                const uint32_t mt1 = next_tile ? buf_tile_of(k + 1) : 0;
                const uint8_t* a_k = g.a + (int64_t)image_of(k) * g.image_bytes;                        // this tile's image
                const uint8_t* a_k1 = g.a + (int64_t)(next_tile ? image_of(k + 1) : 0) * g.image_bytes;  // the next tile's
                const uint16_t* ent_src = g.rows + (int64_t)mt1 * T * MR;
                const uint32_t ent_par = (uint32_t)(k + 1) & bufmask;
                int s = 0;
                for (int cc = 0; cc < NCC; cc++) {
                    // the patch after this one: (k, cc+1) or (k+1, 0); its buffer was last read in the patch before this one
                    const bool same_tile = cc + 1 < NCC;
                    const int2 rng = same_tile ? rng_k : rng_k1;
                    const bool next_patch = same_tile || next_tile;
                    const uint8_t* psrc = (same_tile ? a_k : a_k1) + rng.x + (same_tile ? cc + 1 : 0) * KCB;
                    int units = next_patch ? (rng.y + RPB - 1) / RPB : 0;
                    if (units > g.cap_units) units = g.cap_units;
                    const uint32_t pdst = lds_base + patch_base + ((uint32_t)(k * NCC + cc + 1) & bufmask) * pbytes;
                    for (int ts = 0; ts < TS; ts++, s++) {
                        // one buffer: a patch's first stage also waits for the bulk load issued just before it;
                        // the last stages: nothing useful is in flight behind them
                        if (younger >= D - 2 && !(single && ts == 0)) wait_vmcnt<ALLOWED>();
                        else wait_vmcnt<0>();
                        --younger;
                        __builtin_amdgcn_s_barrier();     // hand this stage to the consumers; they are done with the one before
                        if (!single && ts <= a_last) {
                            int u = ts * g.a_share * NP + p;
                            for (int j = 0; j < g.a_share; j++, u += NP)
                                if (u < units) copy_patch_piece(u, psrc, rng.y, pdst);
                        }
                        if (!single && next_tile && s <= e_last) {
                            int u = s * g.e_share * NP + p;
                            for (int j = 0; j < g.e_share; j++, u += NP) copy_ent_piece(u, ent_src, ent_par);
                        }
                        issue_b(true);
                    }
                    if (single) {
                        // the consumers are done with this patch (and, after a tile's last one, with its entries):
                        // load the next ones into the same buffers
                        __builtin_amdgcn_s_barrier();
                        for (int u = p; u < units; u += NP) copy_patch_piece(u, psrc, rng.y, pdst);
                        if (!same_tile && next_tile)
                            for (int u = p; u < g.ent_copies; u += NP) copy_ent_piece(u, ent_src, ent_par);
                    }
                }
                rng_k = rng_k1;
                rng_k1 = load_range(k + 2);
            }
        };
        {
            const int exact = (D - 2) * G * B_VEC;
            if (exact >= 32) run(std::integral_constant<int, 32>());
            else if (exact >= 24) run(std::integral_constant<int, 24>());
            else if (exact >= 16) run(std::integral_constant<int, 16>());
            else if (exact >= 12) run(std::integral_constant<int, 12>());
            else if (exact >= 8) run(std::integral_constant<int, 8>());
            else if (exact >= 6) run(std::integral_constant<int, 6>());
            else if (exact >= 4) run(std::integral_constant<int, 4>());
            else if (exact >= 3) run(std::integral_constant<int, 3>());
            else if (exact >= 2) run(std::integral_constant<int, 2>());
            else if (exact >= 1) run(std::integral_constant<int, 1>());
            else run(std::integral_constant<int, 0>());
        }
        wait_vmcnt<0>();
    } else {
        // =============================================================== consumer
        const int wm = wave / WN, wn = wave % WN;
        const int lrow = lane & 31, lhalf = lane >> 5;
        const int bswz = (lrow / P) % Q;
        const uint32_t b_frag_base = (wn * NRW + lrow) * KCB;

        // the zero row of both patch buffers (zeros, or the zero point of uint8 activations)
        {
            const uint32_t zv = g.zero_fill;
            for (int i = tid; i < g.nbuf * 256; i += 64 * NC)
                *(uint32_t*)(lds + patch_base + (i >> 8) * pbytes + zoff + (i & 255) * 4) = zv;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        wait_vmcnt<0>();                      // this wavefront's share of the start-up copies
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

            const uint16_t* ent = (const uint16_t*)(lds + ent_base + (int)((uint32_t)k & bufmask) * ent_bytes) + wm * MRW + lrow;
            // The rows of kernel element tap+1 are looked up while the MFMAs of tap run: the row numbers and the
            // patch are in LDS for the whole tile, only the filter tile behind the next barrier is not.
            uint32_t abase[MB], aswz[MB];        // LDS address of the patch row per 32-row block, and the row's swizzle
            auto locate = [&](const uint32_t (&r)[MB], uint32_t pb) {
#pragma unroll
                for (int i = 0; i < MB; i++) {
                    abase[i] = pb + r[i] * KCB;            // the zero row is simply the row after the patch
                    aswz[i] = ((r[i] / P) % Q) << 4;
                }
            };
            for (int cc = 0; cc < NCC; cc++) {
                const uint32_t pb = patch_base + ((uint32_t)(k * NCC + cc) & bufmask) * pbytes;
                const uint32_t pb_next = patch_base + ((uint32_t)(k * NCC + cc + 1) & bufmask) * pbytes;
                const uint16_t* entp = ent;                // row numbers of the kernel element being multiplied
                for (int ts = 0; ts < TS; ts++) {
                    __builtin_amdgcn_s_barrier();
                    if (cc == 0 && ts == 0) {
                        // first stage of the tile: its row numbers only became visible with this barrier
                        uint32_t r0[MB];
#pragma unroll
                        for (int i = 0; i < MB; i++) r0[i] = ent[i * 32];
                        locate(r0, pb);
                    }
                    const uint8_t* S = lds + slot * slot_bytes;
                    slot = slot + 1 == D ? 0 : slot + 1;
                    for (int t = 0; t < G; t++) {
                        // entries of the next kernel element; after a chunk's last one the next chunk starts over at
                        // element 0 in the other patch buffer (after the tile's last one the result is not used)
                        const bool last = ts == TS - 1 && t == G - 1;
                        const uint16_t* entn = last ? ent : entp + MR;
                        uint32_t en[MB];
#pragma unroll
                        for (int i = 0; i < MB; i++) en[i] = entn[i * 32];
#pragma unroll
                        for (int ks = 0; ks < KSTEPS; ks++) {
                            const uint32_t piece = (uint32_t)(2 * ks + lhalf) << 4;
                            uint4 af[MB], bf[NB];
#pragma unroll
                            for (int i = 0; i < MB; i++) af[i] = *(const uint4*)(lds + abase[i] + (piece ^ aswz[i]));
#pragma unroll
                            for (int j = 0; j < NB; j++)
                                bf[j] = *(const uint4*)(S + b_frag_base + j * 32 * KCB + (piece ^ (uint32_t)(bswz << 4)));
#pragma unroll
                            for (int i = 0; i < MB; i++)
#pragma unroll
                                for (int j = 0; j < NB; j++) {
                                    if constexpr (DT == ICV_F32) acc[i][j] = mfma32_f32(af[i], bf[j], acc[i][j]);
                                    else acc[i][j] = mfma32<I8>(af[i], bf[j], acc[i][j]);
                                }
                        }
                        locate(en, last ? pb_next : pb);
                        entp = entn;
                        S += BS;
                    }
                }
                if (single) __builtin_amdgcn_s_barrier();     // done reading this patch: the producers may refill its buffer
            }

            // epilogue: accumulator register r of lane l holds row 8*(r/4) + 4*(l>>5) + (r&3), column l&31
            const int64_t tile = tl.first + k * tl.step;
            const int32_t nt = (int32_t)(tile % g.n_tiles);
            const uint32_t mt = (uint32_t)(tile / g.n_tiles);
            const uint32_t img = mt / g.img_tiles, t_img = mt - img * g.img_tiles;     // batch element, row tile in it
            const int64_t img_row0 = (int64_t)img * g.img_rows;
            const int64_t m_base = img_row0 + (int64_t)t_img * MR + wm * MRW + 4 * lhalf;
            const int32_t n_base = nt * NR + wn * NRW + lrow;
            const bool whole = (t_img + 1) * MR <= g.img_rows && (nt + 1) * NR <= g.K;     // no row or column tail
            store_tile<FUSED, I8, MB, NB>(g.out, acc, img_row0 + g.img_rows, g.K, g.out_stride, m_base, n_base, whole, g.ep);
        }
    }
}

// ------------------------------------------------------------------ launch
size_t patch_lds_bytes(int NR, int KCB, int ring, int cap_units, int ent_copies, int nbuf)
{
    // `ring` counts filter tiles (slots times kernel elements per slot)
    return (size_t)ring * NR * KCB + (size_t)nbuf * (cap_units + 1) * 1024 + (size_t)nbuf * ent_copies * 1024;
}

template <int DT, int MR, int NR, int WM, int WN, int NP, int KCB, bool FUSED>
static int launch_one(const Geometry& g, PatchArgs a, hipStream_t s)
{
    constexpr int threads = 64 * (WM * WN + NP);
    auto kern = k_igemm_patch<DT, MR, NR, WM, WN, NP, KCB, FUSED>;
    a.ent_copies = (int32_t)(((size_t)a.T * MR * 2 + 1023) / 1024);
    a.cap_units = (int32_t)(((size_t)g.patch_rows * KCB + 1023) / 1024);
    // Kernel elements per stage: a stage should hold enough MFMAs (16 per consumer wavefront) to amortise its
    // barrier and the producers' bookkeeping; G divides T.
    constexpr int mfma_per_tap = (MR / WM / 32) * (NR / WN / 32) * (KCB / 32);
    int G = g.group;
    if (G == 0) {
        for (G = 1; G < a.T && (a.T % G || G * mfma_per_tap < 16); ++G) {}
    }
    if (G > a.T) G = a.T;
    // Two workgroups per compute unit (64-wide tiles and tiles with four consumer wavefronts, when they fit; or on
    // request): each gets half the LDS and a single patch / entry buffer, and covers the other's load bubbles,
    // start-up and epilogue.  Otherwise one workgroup with double buffers.
    // Ring depth.  A copy takes on the order of a microsecond from issue to completion under load, a stage far
    // less, and a stage's filter tiles must be issued ring - 1 stages ahead: as deep as fits (LDS, enough stages
    // left to spread the shares over), at most 8; when LDS is short, kernel elements per stage go before depth.
    const int G0 = G;
    int per_cu = g.blocks_per_cu ? g.blocks_per_cu : (NR == 64 || WM * WN == 4 ? 2 : 1);
    int ring = 0;
    for (; per_cu >= 1; --per_cu) {
        a.nbuf = per_cu == 2 ? 1 : 2;
        const size_t budget = kLdsPerCu / per_cu;
        for (G = G0; G >= 1; --G) {
            if (a.T % G) continue;
            const int TS = a.T / G, n_st = a.NCC * TS;
            for (ring = g.ring ? g.ring : 8; ring >= 2; --ring) {
                if (n_st - ring + 2 < 1 || (a.nbuf == 2 && TS - ring + 2 < 1)) continue;
                if (patch_lds_bytes(NR, KCB, ring * G, a.cap_units, a.ent_copies, a.nbuf) > budget) continue;
                break;
            }
            if (ring >= 2) break;      // measured: more kernel elements per stage beat a deeper ring
        }
        if (G >= 1 && ring >= 2) break;
    }
    if (per_cu < 1) return ICV_ERR_UNSUPPORTED;
    {
        const int TS = a.T / G, n_st = a.NCC * TS;
        a.a_share = a.nbuf == 2 ? (a.cap_units + NP * (TS - ring + 2) - 1) / (NP * (TS - ring + 2)) : 0;
        a.e_share = a.nbuf == 2 ? (a.ent_copies + NP * (n_st - ring + 2) - 1) / (NP * (n_st - ring + 2)) : 0;
    }
    a.G = G;
    a.TS = a.T / G;
    a.ring = ring;
    const size_t lds_bytes = patch_lds_bytes(NR, KCB, ring * G, a.cap_units, a.ent_copies, a.nbuf);

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

template <int DT, int MR, int NR, int WM, int WN>
static int launch_tile(const Geometry& g, const PatchArgs& a, hipStream_t s)
{
    if (g.KCB == 128)
        return g.ep_plain ? launch_one<DT, MR, NR, WM, WN, 4, 128, false>(g, a, s)
                          : launch_one<DT, MR, NR, WM, WN, 4, 128, true>(g, a, s);
    return g.ep_plain ? launch_one<DT, MR, NR, WM, WN, 4, 64, false>(g, a, s)
                      : launch_one<DT, MR, NR, WM, WN, 4, 64, true>(g, a, s);
}

template <int DT>
static int launch_dtype(const Geometry& g, const PatchArgs& a, hipStream_t s)
{
    switch (g.variant) {
        case 0: return launch_tile<DT, 128, 64, 2, 2>(g, a, s);
        case 2: return launch_tile<DT, 256, 64, 4, 1>(g, a, s);
        case 4: return launch_tile<DT, 64, 64, 2, 2>(g, a, s);
        case 6: return launch_tile<DT, 128, 128, 4, 2>(g, a, s);
        default: break;
    }
    if constexpr (DT != ICV_F32) {      // fp32 tensors have the four tiles above
        switch (g.variant) {
            case 1: return launch_tile<DT, 128, 128, 2, 2>(g, a, s);
            case 3: return launch_tile<DT, 256, 64, 4, 2>(g, a, s);
            case 5: return launch_tile<DT, 256, 128, 4, 2>(g, a, s);
            default: break;
        }
    }
    return ICV_ERR_UNSUPPORTED;
}

bool patch_variant_supported(int variant) { return variant >= 0 && variant < kNumTileVariants; }
bool patch_variant_supported_f32(int variant) { return variant == 0 || variant == 2 || variant == 4 || variant == 6; }

int launch_igemm_patch(const icv_conv_params* p, const Geometry& g, const void* input, const void* packed,
                       const int32_t* ind, void* out, hipStream_t s)
{
    const TileVariant& tv = kTileVariants[g.variant];
    if (tv.MR != g.MR || tv.NR != g.NR || !g.patch_rows) return ICV_ERR_UNSUPPORTED;
    const int64_t stride_bytes = (int64_t)g.in_stride * g.elem_bytes;
    int shift = 0;
    while ((1ll << shift) < stride_bytes) ++shift;
    if ((1ll << shift) != stride_bytes) return ICV_ERR_UNSUPPORTED;
    PatchArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.a = (const uint8_t*)input;
    a.w = (const uint8_t*)packed;
    // the buffer: int32 entries, then the tiles' range records, then the entries as 16-bit patch row numbers
    a.ranges = (const int4*)ind;      // range records, then the 16-bit entries
    a.rows = (const uint16_t*)(a.ranges + g.img_tiles);
    a.image_bytes = g.image_bytes;
    a.img_tiles = (uint32_t)g.img_tiles;
    a.img_rows = (uint32_t)g.img_rows;
    a.out = out;
    a.M = g.M;
    a.total_tiles = g.m_tiles * g.n_tiles;
    if (a.total_tiles >= (1ll << 31)) return ICV_ERR_UNSUPPORTED;      // the kernels count tiles in 32 bits
    a.stride_bytes = (int32_t)stride_bytes; a.stride_shift = shift;
    a.K = p->K; a.T = g.T; a.NCC = g.stages_per_tap; a.out_stride = g.out_stride;
    a.n_tiles = (int32_t)g.n_tiles;
    a.ep = g.ep;
    a.zero_fill = p->dtype == ICV_U8I8 ? 0x01010101u * (uint32_t)p->input_zero_point : 0u;
    a.ring = 0; a.G = 1; a.ent_copies = 0; a.cap_units = 0; a.a_share = 0; a.e_share = 0; a.nbuf = 2; a.xcd_mode = 0;
    if (p->dtype == ICV_F32) return launch_dtype<ICV_F32>(g, a, s);
    return p->dtype == ICV_U8I8 ? launch_dtype<ICV_U8I8>(g, a, s) : launch_dtype<ICV_BF16>(g, a, s);
}

}  // namespace icv
