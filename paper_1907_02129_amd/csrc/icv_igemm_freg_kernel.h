// Tensor-core Indirect GEMM with the filter held in registers and the input streamed through an LDS ring.
//
// Listing 3's loop nest (row block, kernel element, channels) is kept; what is chosen for gfx950 is where the two
// operands live while a workgroup walks its share of the output:
//
//  * B, the filter.  A wavefront owns one block of 32 output channels and keeps that block's whole filter --
//    R*S*C elements per channel, already in the operand layout of v_mfma_*_32x32x* -- in its registers for the
//    lifetime of the kernel: T*KS fragments of four registers (T = R*S kernel elements, KS 32-byte steps per pixel
//    row; 288 registers for a 3x3 kernel on 256-byte rows).  A compute unit's register file is three times its LDS;
//    with one wavefront per SIMD the filter of a convolution layer fits there, is loaded once, and costs no LDS
//    space, no LDS bandwidth and no synchronisation afterwards (section 3.1: the filter never changes, so it can be
//    repacked once into whatever layout the kernel reads best).
//  * A, the rows the indirection entries name.  The workgroup walks a contiguous range of output pixels, 32-row
//    blocks grouped into passes.  The valid entries of consecutive output pixels name a window of consecutive input
//    pixels that only moves forward (icv_pixel_range.h), so that window is kept in LDS as a ring of pixel rows: each
//    input pixel is fetched from memory once per workgroup and then read by all R*S kernel elements of all the
//    output pixels it contributes to (the re-use that section 3 lists as the method's second performance factor,
//    organised explicitly).  The indirection buffer holds, per row block, a base pixel and per (row, kernel element) a
//    16-bit pixel number counted from it (0xFFFF: the zero row, section 2.3); the kernel turns an entry into a ring
//    row with one add and one mask.  Padding entries read a row of zeros kept after the ring.
//
// Four wavefronts, one per SIMD, WN column blocks x WM row groups; a pass is WM*MB row blocks.  All four take part in
// copying the window of the NEXT pass (global -> LDS without a register stop) at the start of a pass, multiply the
// current pass out of LDS, wait for their own copies, store the pass's outputs, and meet at the only barrier of the
// pass.  The stores are not waited for until the end of the following pass, and the copies have a whole pass to
// land, so loads, MFMAs and stores of neighbouring passes overlap inside one workgroup.
//
// uint8 activations: every A fragment is XORed with 0x80 (x -> x - 128 as a signed byte); the zero row holds 0x80.
#pragma once
#include "icv_mfma_common.h"
#include <utility>
#include "icv_pixel_range.h"

namespace icv {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

struct FregArgs {
    const uint8_t* a;          // input tensor
    const uint8_t* w;          // packed filter [column block][fragment][lane][16 bytes]
    const int4* rec;           // per row block: {base byte offset, 0, base pixel, 0}
    const uint16_t* ent;       // [row block][kernel element][32]: pixel number from the block's base, 0xFFFF = zero row
    void* out;
    RangeGeom q;
    int64_t M;
    int32_t K, out_stride;
    int32_t stride_bytes;      // bytes between input pixels
    int32_t last_pixel;        // N*Hin*Win - 1
    uint32_t n_blocks;         // row blocks of 32 output pixels
    uint32_t buf_blocks;       // row blocks the buffer describes: n_blocks, or those of one image (batch-independent buffer)
    uint32_t img_pixels;       // batch-independent buffer: input pixels per image (its records count from image 0); else 0
    uint32_t img_rows;         // batch-independent buffer: output pixels per image (an image is buf_blocks blocks, the last
                               // one partly empty when this is not a multiple of 32); else unused
    FastDiv by_buf;            // division by buf_blocks
    uint32_t range_q, range_rem;   // n_blocks / n_ranges and the remainder: the first range_rem ranges get one block more
    int32_t cg_shift;          // log2(n_cg), or -1 when n_cg is not a power of two
    int32_t ranges_per_xcd;    // XCD mode: n_ranges / 8
    uint32_t ent_bytes;        // bytes of the entries (copies are clamped to them)
    int32_t n_cg;              // column groups of WN column blocks
    int32_t n_ranges;          // row ranges: workgroups per column group
    int32_t xcd_mode;          // 1: XCD x (workgroups x, x + 8, ...) owns a contiguous run of row ranges, all column groups
    int32_t ring_rows;         // pixel rows of the ring, a power of two and a multiple of 64
    uint32_t zero_fill;        // four bytes of the zero row: zeros, or the zero point of uint8 activations
    EpilogueArgs ep;
};

// One 16-byte A fragment times one 16-byte B fragment per lane: a 32x32x32 product of bytes, a 32x32x16 product of
// bfloat16, or -- fp32 tensors, section 3.1's own precision -- four 32x32x2 products (icv_mfma_common.h).
template <int DT>
__device__ inline typename Acc<DT == ICV_U8I8>::type mfma_frag(const u32x4_t& a, const u32x4_t& b, typename Acc<DT == ICV_U8I8>::type c)
{
    if constexpr (DT == ICV_U8I8) {
        const u32x4_t ax = a ^ 0x80808080u;
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4_t, ax), __builtin_bit_cast(i32x4_t, b), c, 0, 0, 0);
    } else if constexpr (DT == ICV_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    } else {
        return mfma32_f32(__builtin_bit_cast(uint4, a), __builtin_bit_cast(uint4, b), c);
    }
}

// A pointer the compiler can prove to be wavefront-uniform (the copies take their base address in scalar registers).
template <typename P>
__device__ inline const P* uniform_ptr(const P* p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (const P*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), as straight-line code whatever the size of f:
// the reduction below indexes registers with the step number, so it must never remain a loop (an unroll pragma is a
// request that the compiler's size threshold may turn into a partial unroll, and the registers into scratch memory).
template <typename F, int... I>
__device__ __forceinline__ void static_steps_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>()), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_steps(F&& f)
{
    static_steps_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>());
}

constexpr int freg_slot_bytes(int T, int PBK) { return 1024 + (PBK * T * 64 + 1023) / 1024 * 1024; }

template <int DT, int T, int KS, int WN, int MB, bool FUSED>
__global__ __launch_bounds__(256) void k_igemm_freg(FregArgs g)
{
    constexpr bool I8 = DT == ICV_U8I8;      // DT: the icv_dtype of input and filter
    constexpr int WM = 4 / WN;
    constexpr int PBK = WM * MB;             // row blocks per pass
    constexpr int NF = T * KS;               // filter fragments per column block
    constexpr int PP = KS * 2 + 1;           // 16-byte pieces per ring row: the pixel's KS*32 bytes and one of padding,
    constexpr int PITCH = PP * 16;           //   which spreads the fragment reads of 16 consecutive rows over all banks
    constexpr int SLOT = freg_slot_bytes(T, PBK);     // one pass's block records (1 KB) and entries
    constexpr int ECOP = (SLOT - 1024) / 1024;
    using acc_t = typename Acc<I8>::type;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t ring_rows = (uint32_t)g.ring_rows, ring_mask = ring_rows - 1;
    const uint32_t ring_chunks = ring_rows * PP;                  // 16-byte pieces of the ring, a multiple of 64
    const uint32_t zero_off = ring_chunks * 16;                   // the zero row
    const uint32_t slot_off = (zero_off + PITCH + 1023) / 1024 * 1024;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, lhalf = lane >> 5;
    const uint8_t* const a_base = uniform_ptr(g.a);
    const int4* const rec_base = uniform_ptr(g.rec);
    const uint16_t* const ent_base = uniform_ptr(g.ent);

    // ---- this workgroup's column group and row range (the host passes the quotients: a division costs this lone
    // wavefront a few hundred cycles, and everything before the first copy is start-up latency)
    uint32_t cg, range;
    {
        const uint32_t b = blockIdx.x, i = g.xcd_mode ? b >> 3 : b;
        uint32_t j;
        if (g.cg_shift >= 0) {
            cg = i & ((1u << g.cg_shift) - 1u);
            j = i >> g.cg_shift;
        } else {
            j = i / (uint32_t)g.n_cg;
            cg = i - j * (uint32_t)g.n_cg;
        }
        range = g.xcd_mode ? (b & 7u) * (uint32_t)g.ranges_per_xcd + j : j;
    }
    if (range >= (uint32_t)g.n_ranges) return;                    // the whole workgroup, before any barrier
    // the first range_rem ranges have range_q + 1 row blocks, the others range_q
    const uint32_t rb_lo = range * g.range_q + (range < g.range_rem ? range : g.range_rem);
    const uint32_t rb_hi = rb_lo + g.range_q + (range < g.range_rem ? 1u : 0u);
    const int n_pass = (int)((rb_hi - rb_lo + PBK - 1) / PBK);
    const uint32_t M = (uint32_t)g.M;
    // Output pixels of a row block.  With a whole-batch buffer block b holds pixels 32 b ... 32 b + 31 (the last block
    // of the batch fewer).  With a batch-independent buffer every image starts a block of its own: block b is block
    // b % buf_blocks of image b / buf_blocks, and the last block of an image is partly empty unless the image is a
    // multiple of 32 pixels (its empty rows have zero-row entries and are never stored).
    auto first_row = [&](uint32_t b) -> uint32_t {
        if (!g.img_pixels) return b * 32u;
        const uint32_t n = fast_div(b, g.by_buf);
        return n * g.img_rows + (b - n * g.buf_blocks) * 32u;
    };
    auto end_row = [&](uint32_t b) -> uint32_t {           // one past the last output pixel of block b
        if (!g.img_pixels) return (b + 1u) * 32u < M ? (b + 1u) * 32u : M;
        const uint32_t n = fast_div(b, g.by_buf);
        const uint32_t e = (b - n * g.buf_blocks + 1u) * 32u;
        return n * g.img_rows + (e < g.img_rows ? e : g.img_rows);
    };
    const int32_t origin = lowest_pixel_from(g.q, decompose(g.q, first_row(rb_lo)));   // pixel of ring row 0

    // copies that must have been issued before pass k is multiplied: everything up to the highest pixel its rows name
    auto copies_upto_pass = [&](int k) -> uint32_t {
        uint32_t blk_end = rb_lo + (uint32_t)(k + 1) * PBK;
        if (blk_end > rb_hi) blk_end = rb_hi;
        const int32_t top = highest_pixel_upto(g.q, decompose(g.q, end_row(blk_end - 1u) - 1u));
        const uint32_t pixels = top >= origin ? (uint32_t)(top - origin) + 1u : 1u;
        return (pixels * PP + 63u) / 64u;
    };
    // Ring copies.  Copy u fills ring pieces 64u .. 64u + 63 (one wavefront-wide 1 KB copy); this wavefront issues
    // u = wave, wave + 4, ...  Its state is carried from copy to copy with adds and compares only: the LDS address, and
    // per lane the pixel (counted from the origin) and the piece of that pixel's row the lane moves.
    const uint32_t ring_bytes = ring_chunks * 16u;
    uint32_t cu = (uint32_t)wave;
    uint32_t cdst = lds_base + (uint32_t)wave * 1024u;
    uint32_t cps = ((uint32_t)wave * 64u + (uint32_t)lane) / PP;
    uint32_t cpiece = ((uint32_t)wave * 64u + (uint32_t)lane) % PP;
    auto copy_next = [&]() {
        uint32_t pix = (uint32_t)origin + cps;
        if (pix > (uint32_t)g.last_pixel) pix = (uint32_t)g.last_pixel;      // never read past the tensor
        const uint32_t piece = cpiece > PP - 2 ? PP - 2 : cpiece;            // the padding piece repeats the last one
        copy16_global_to_lds(a_base, pix * (uint32_t)g.stride_bytes + piece * 16u,
                             (uint32_t)__builtin_amdgcn_readfirstlane((int)cdst));
        cu += 4u;
        cdst += 4096u;
        if (cdst >= lds_base + ring_bytes) cdst -= ring_bytes;
        cps += 256u / PP;
        cpiece += 256u % PP;
        if (cpiece >= (uint32_t)PP) { cpiece -= PP; cps += 1u; }
    };
    // block records and entries of pass k -> its slot
    auto copy_entries = [&](int k) {
        const uint32_t slot = (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + slot_off + (uint32_t)(k & 1) * SLOT));
        const uint32_t blk0 = rb_lo + (uint32_t)k * PBK;
        // block number in the buffer: a batch-independent buffer holds the blocks of one image, and an image is a
        // whole number of blocks
        auto in_buffer = [&](uint32_t blk) {
            if (blk > g.n_blocks - 1) blk = g.n_blocks - 1;
            return g.img_pixels ? blk - fast_div(blk, g.by_buf) * g.buf_blocks : blk;
        };
        if (wave == 0) {
            if (lane < PBK) copy16_global_to_lds(rec_base, in_buffer(blk0 + (uint32_t)lane) * 16u, slot);
        }
#pragma unroll
        for (int e = 0; e < ECOP; e++)
            if (((e + 1) & 3) == wave) {
                const uint32_t o = (uint32_t)e * 1024u + (uint32_t)lane * 16u;      // byte of the pass's entries
                uint32_t off;
                if (g.img_pixels) {
                    // the pass's blocks need not follow each other in the buffer (the next image starts over at block 0);
                    // a block's entries are T * 64 bytes, a multiple of the 16 bytes a lane moves
                    const uint32_t b = o / (uint32_t)(T * 64);
                    off = in_buffer(blk0 + b) * (uint32_t)(T * 64) + (o - b * (uint32_t)(T * 64));
                } else {
                    off = blk0 * (uint32_t)(T * 64) + o;
                }
                if (off > g.ent_bytes - 16u) off = g.ent_bytes - 16u;
                copy16_global_to_lds(ent_base, off, slot + 1024u + (uint32_t)e * 1024u);
            }
    };

    // ---- start-up: the windows of the first two passes and the zero row.  The filter is not loaded here: see below.
    uint32_t upto_next = copies_upto_pass(n_pass > 1 ? 1 : 0);
    copy_entries(0);
    if (n_pass > 1) copy_entries(1);
    while (cu < upto_next) copy_next();
    const int c = wave % WN, h = wave / WN;
    // The kernel elements are walked in an order rotated by the row range: the sum does not care, and the workgroups
    // -- which all read the same filter at the same time -- then ask the L2 channels for different lines at any one
    // moment instead of queueing on the same ones.
    int tap_of[T];
    {
        const int rot = (int)(range % (uint32_t)T);
#pragma unroll
        for (int j = 0; j < T; j++) tap_of[j] = j + rot < T ? j + rot : j + rot - T;
    }
    u32x4_t B[NF];
    const u32x4_t* const wp = (const u32x4_t*)(g.w + ((size_t)(cg * WN + c) * NF) * 1024) + lane;
    auto load_filter = [&](int f) { B[f] = wp[(tap_of[f / KS] * KS + f % KS) * 64]; };
    for (int i = tid; i < PITCH / 4; i += 256) *(uint32_t*)(lds + zero_off + i * 4) = g.zero_fill;
    // Fused output stage: a lane's output channel is the same in every pass, so its bias is read once, here, where the
    // start-up wait covers the load (read at the stores it would cost every pass a trip to L2), and added to the
    // accumulators before they are handed to the output stage, which then gets no bias pointer.
    using out_acc_t = typename std::conditional<I8, int32_t, float>::type;
    out_acc_t lane_bias = 0;
    EpilogueArgs ep = g.ep;
    if constexpr (FUSED) {
        lane_bias = output_bias<out_acc_t>(g.ep, (int32_t)(cg * WN + c) * 32 + lrow, g.K);
        ep.bias = nullptr;
        ep.wsum = nullptr;         // (the zero-point term is part of lane_bias)
    }
    if (n_pass > 2) upto_next = copies_upto_pass(2);
    wait_vmcnt<0>();
    __syncthreads();

    const int32_t col = (int32_t)(cg * WN + c) * 32 + lrow;
    // One pass.  `first` (a compile-time tag) selects the copy of the body that runs once, for pass 0: it loads the
    // filter fragments FD steps ahead of their first use, so the filter -- the largest thing a workgroup reads,
    // through a 64 byte per clock L1 -- arrives spread over the first pass instead of delaying its start.  That copy
    // issues no ring copies (the second pass's window was requested at start-up): the compiler's waits for the filter
    // loads count every vector-memory operation of the wavefront, and a copy from HBM between them would stall the MFMAs.
    constexpr int FD = 10;
    auto run_pass = [&](int k, auto first, auto blocks_per_wave) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first)::value;
        constexpr int MBE = decltype(blocks_per_wave)::value;      // MB, or 1 for a short last pass (see below)
        // the next pass's window: its copies land while this pass is multiplied (their ring rows and entry slot were
        // last read in the pass before this one, which every wavefront has left); the entries now, the ring copies one
        // at a time between the MFMA steps below, where their address arithmetic costs nothing
        const uint32_t upto = !FIRST && k + 1 < n_pass ? upto_next : 0u;
        if (!FIRST && k + 1 < n_pass) copy_entries(k + 1);
        if constexpr (FIRST) {
#pragma unroll
            for (int f = 0; f < FD && f < NF; f++) load_filter(f);
        }

        const uint8_t* slot = lds + slot_off + (k & 1) * SLOT;
        const uint16_t* ent = (const uint16_t*)(slot + 1024) + (h * MBE) * (T * 32) + lrow;
        int32_t delta[MBE];
#pragma unroll
        for (int i = 0; i < MBE; i++) {
            delta[i] = *(const int32_t*)(slot + (h * MBE + i) * 16 + 8) - origin;
            if (g.img_pixels) {
                // the record counts pixels from its image's first one: add the images before it
                uint32_t b = rb_lo + (uint32_t)k * PBK + (uint32_t)(h * MBE + i);
                if (b > g.n_blocks - 1) b = g.n_blocks - 1;
                delta[i] += (int32_t)(fast_div(b, g.by_buf) * g.img_pixels);
            }
        }

        acc_t acc[MBE][1];
#pragma unroll
        for (int i = 0; i < MBE; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][0][r] = 0;

        // The reduction as one unrolled sequence of NF steps (step st: kernel element tap_of[st / KS], 32-byte piece
        // st % KS of its rows).  The wavefront is alone on its SIMD, so the latencies are hidden by software
        // pipelining: a kernel element's row numbers are read LA + 1 steps before its first step, turned into LDS
        // addresses PF + 1 steps before it, the A fragments are read PF steps ahead, and only then come the step's
        // MFMAs.  The scheduling barriers keep the compiler from folding that order back into load-wait-multiply.
        constexpr int PF = 3, LA = 6;
        uint32_t e16[T][MBE], addr[T][MBE];                    // few of them are live at any time
        u32x4_t af[PF + 1][MBE];
        auto read_rows = [&](int j) {
#pragma unroll
            for (int i = 0; i < MBE; i++) e16[j][i] = ent[(i * T + tap_of[j]) * 32];
        };
        auto locate = [&](int j) {
#pragma unroll
            for (int i = 0; i < MBE; i++) {
                const uint32_t row = (e16[j][i] + (uint32_t)delta[i]) & ring_mask;
                addr[j][i] = (e16[j][i] == 0xFFFFu ? zero_off : __umul24(row, (uint32_t)PITCH)) + (uint32_t)lhalf * 16u;
            }
        };
        auto read_frags = [&](int st) {
#pragma unroll
            for (int i = 0; i < MBE; i++) af[st % (PF + 1)][i] = *(const u32x4_t*)(lds + addr[st / KS][i] + (st % KS) * 32);
        };
        // before the first step: the rows of the kernel elements whose fragments are read within the first PF + 1
        // steps are located here, those read within the first LA + 1 steps have their row numbers requested
#pragma unroll
        for (int j = 0; j * KS < LA + 1 && j < T; j++) read_rows(j);
#pragma unroll
        for (int j = 0; j * KS < PF + 1 && j < T; j++) locate(j);
#pragma unroll
        for (int st = 0; st < PF && st < NF; st++) read_frags(st);
        __builtin_amdgcn_sched_barrier(0);
        static_steps<NF>([&](auto step) __attribute__((always_inline)) {
            constexpr int st = decltype(step)::value;
            if (st + PF < NF) read_frags(st + PF);
            if constexpr (FIRST) {
                if (st + FD < NF) load_filter(st + FD);
            }
#pragma unroll
            for (int i = 0; i < MBE; i++) acc[i][0] = mfma_frag<DT>(af[st % (PF + 1)][i], B[st], acc[i][0]);
            // book-keeping behind the MFMAs, where it is free: the kernel element whose fragments the NEXT step starts
            // to read is located now, row numbers are requested LA - PF steps before they are located
            constexpr int jl = (st + 1 + PF) / KS, jr = (st + 1 + LA) / KS;
            if ((st + 1 + PF) % KS == 0 && jl < T && jl * KS >= PF + 1) locate(jl);
            if ((st + 1 + LA) % KS == 0 && jr < T && jr * KS >= LA + 1) read_rows(jr);
            if (!FIRST && st % 2 == 1 && cu < upto) copy_next();
            if (st == NF / 2 && k + 2 < n_pass && (!FIRST || n_pass > 2)) upto_next = copies_upto_pass(k + 2);
            __builtin_amdgcn_sched_barrier(0);
        });
        while (cu < upto) copy_next();                      // a window that jumped (an image boundary) has more

        // my copies for the next pass (issued during this one) and the stores of the pass before this one
        wait_vmcnt<0>();
        const uint32_t blk = rb_lo + (uint32_t)k * PBK + (uint32_t)(h * MBE);
        const bool k_whole = (int32_t)(cg * WN + c + 1) * 32 <= g.K;
        if constexpr (FUSED) {
#pragma unroll
            for (int i = 0; i < MBE; i++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][0][r] += lane_bias;
        }
        if (blk < rb_hi && !g.img_pixels) {
            uint32_t m_end = rb_hi * 32u;
            if (m_end > M) m_end = M;
            const int64_t m_base = (int64_t)blk * 32 + 4 * lhalf;
            const bool whole = (blk + MBE) * 32u <= m_end && k_whole;
            store_tile<FUSED, I8, MBE, 1>(g.out, acc, (int64_t)m_end, g.K, g.out_stride, m_base, col, whole, ep);
        } else if (blk < rb_hi) {
            // batch-independent buffer: consecutive blocks need not hold consecutive output pixels
#pragma unroll
            for (int i = 0; i < MBE; i++)
                if (blk + (uint32_t)i < rb_hi) {
                    const uint32_t m0 = first_row(blk + (uint32_t)i), m1 = end_row(blk + (uint32_t)i);
                    acc_t one[1][1];
                    one[0][0] = acc[i][0];
                    store_tile<FUSED, I8, 1, 1>(g.out, one, (int64_t)m1, g.K, g.out_stride, (int64_t)m0 + 4 * lhalf, col,
                                                m1 - m0 == 32u && k_whole, ep);
                }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // A last pass with no more row blocks than row groups (WM) runs with one block per wavefront, the blocks dealt to
    // the row groups one each: half the multiplications of a full pass for a range that ends just behind a pass
    // boundary (3136 row blocks on 256 compute units are 12 for most workgroups and 13 for some).
    const bool short_tail = MB > 1 && (rb_hi - rb_lo) - (uint32_t)(n_pass - 1) * PBK <= (uint32_t)WM;
    using full_t = std::integral_constant<int, MB>;
    using one_t = std::integral_constant<int, 1>;
    if (n_pass == 1 && short_tail) run_pass(0, std::true_type(), one_t());
    else run_pass(0, std::true_type(), full_t());
    // The filter registers are final from here on.  Passing them through an empty statement tells the compiler that
    // none of their loads is outstanding any more (the loop below then carries no wait for them) and says where each
    // fragment lives: 4 * NF registers do not fit the 256 vector registers beside everything else, so all but the
    // first FV fragments are kept in the accumulation registers, from which the MFMAs read them directly.
    constexpr int FV = NF <= 36 ? NF : (NF <= 56 ? 28 : 20);
#pragma unroll
    for (int f = 0; f < NF; f++) {
        if (f < FV) asm volatile("" : "+v"(B[f]));
        else asm volatile("" : "+a"(B[f]));
    }
    const int n_full = short_tail ? n_pass - 1 : n_pass;
    for (int k = 1; k < n_full; k++) run_pass(k, std::false_type(), full_t());
    if (short_tail && n_pass > 1) run_pass(n_pass - 1, std::false_type(), one_t());
}

// ------------------------------------------------------------------ launch of one instantiation
template <int DT, int T, int KS, int WN, int MB, bool FUSED>
static int launch_one(const FregArgs& a, int64_t grid, size_t lds_bytes, hipStream_t s)
{
    auto kern = k_igemm_freg<DT, T, KS, WN, MB, FUSED>;
    if (lds_bytes > 64 * 1024) {
        static bool raised[kMaxDevices] = {};      // one array per instantiation of this function template
        const int st = allow_full_lds((const void*)kern, raised);
        if (st != ICV_OK) return st;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds_bytes, s, a);
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

template <int DT, bool FUSED, int T, int KS>
static int launch_shape(const Geometry& g, const FregArgs& a, int64_t grid, size_t lds, hipStream_t s)
{
#define ICV_FREG_CASE(WN_, MB_) \
    if (g.freg_wn == WN_ && g.freg_mb == MB_) return launch_one<DT, T, KS, WN_, MB_, FUSED>(a, grid, lds, s);
    ICV_FREG_CASE(4, 2)
    ICV_FREG_CASE(4, 1)
    ICV_FREG_CASE(2, 2)
    ICV_FREG_CASE(2, 1)
    ICV_FREG_CASE(1, 2)
    ICV_FREG_CASE(1, 1)
#undef ICV_FREG_CASE
    return ICV_ERR_UNSUPPORTED;
}

// Every instantiation of one (dtype, output stage) pair: one translation unit each, so that they compile side by side.
template <int DT, bool FUSED>
static int launch_freg_instances(const Geometry& g, const FregArgs& a, int64_t grid, size_t lds, int T, int KS, hipStream_t s)
{
#define ICV_FREG_SHAPE(T_, KS_) \
    if (T == T_ && KS == KS_) return launch_shape<DT, FUSED, T_, KS_>(g, a, grid, lds, s);
    ICV_FREG_SHAPE(9, 8)
    ICV_FREG_SHAPE(9, 4)
    ICV_FREG_SHAPE(9, 2)
    ICV_FREG_SHAPE(25, 2)
#undef ICV_FREG_SHAPE
    return ICV_ERR_UNSUPPORTED;
}

}  // namespace icv
