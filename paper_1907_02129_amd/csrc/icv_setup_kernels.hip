// Set-up kernels: zero row, filter pre-pack, indirection build, and the im2col of the ablation path.
#include "icv_internal.h"
#include "icv_pixel_range.h"

namespace icv {

// ------------------------------------------------------------------ zero row (section 2.3)
__global__ void k_fill_bytes(uint8_t* dst, int n, uint8_t v)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

int launch_zero_row(const icv_conv_params* p, const Geometry& g, void* zero_row, hipStream_t s)
{
    const int n = (int)((((size_t)p->C * g.elem_bytes) + 15) / 16 * 16);
    const uint8_t v = p->dtype == ICV_U8I8 ? (uint8_t)p->input_zero_point : 0;
    hipLaunchKernelGGL(k_fill_bytes, dim3((n + 255) / 256), dim3(256), 0, s, (uint8_t*)zero_row, n, v);
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

// ------------------------------------------------------------------ filter pre-pack
// Source  [K][T][C] elements.
// Packed  [n_tile][stage][NR][KCB bytes], stage = (tap, C-chunk), or (C-chunk, tap) for the plans that keep the
//         tile's pixel range in LDS: the tile one pipeline stage of the GEMM kernel copies into LDS is one
//         contiguous block.  Rows past K are zero.
// One thread moves 16 bytes (KCB and C*elem are multiples of 16 for the tensor-core plans); the generic
// plan (KCB == 0) transposes to [T * C][K padded] and moves single elements.
struct PackArgs {
    const uint8_t* src;
    uint8_t* dst;
    int32_t K, T, CB;  // CB = C * elem bytes
    int32_t NR, KCB, stages_per_tap, n_stages;
    int32_t cc_major;   // stage = chunk * T + tap instead of tap * stages_per_tap + chunk
    int64_t total_vec;  // number of 16-byte vectors in dst
};

__global__ void k_pack_filter_vec(PackArgs a)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= a.total_vec) return;
    const int32_t q = a.KCB / 16;  // vectors per row per stage
    const int32_t chunk = (int32_t)(v % q);
    int64_t r = v / q;
    const int32_t row = (int32_t)(r % a.NR);
    r /= a.NR;
    const int32_t stage = (int32_t)(r % a.n_stages);
    const int32_t ntile = (int32_t)(r / a.n_stages);
    const int32_t tap = a.cc_major ? stage % a.T : stage / a.stages_per_tap;
    const int32_t cc = a.cc_major ? stage / a.T : stage % a.stages_per_tap;
    const int32_t oc = ntile * a.NR + row;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (oc < a.K)
        val = *(const uint4*)(a.src + ((int64_t)oc * a.T + tap) * a.CB + (int64_t)cc * a.KCB + chunk * 16);
    *(uint4*)(a.dst + v * 16) = val;
}

// Vector-ALU plan: [R*S*C][K padded], output channels innermost, so that the 64 lanes of a wavefront (64 neighbouring
// output channels) read one contiguous run per reduction index.  One thread per element; channels past K are zero.
template <typename T>
__global__ void k_pack_filter_transposed(const T* src, T* dst, int K, int64_t red, int64_t kp)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= red * kp) return;
    const int64_t r = i / kp, oc = i - r * kp;
    dst[i] = oc < K ? src[oc * red + r] : (T)0;
}

// Low-C plan: [n tile][64][KP]; row oc is the filter's own [R][S][C] run followed by zeros up to KP bytes.
__global__ void k_pack_filter_lowc(const uint8_t* src, uint8_t* dst, int K, int row_bytes, int KP, int64_t total_rows)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // one thread per 8 bytes
    const int per_row = KP / 8;
    if (i >= total_rows * per_row) return;
    const int64_t row = i / per_row;
    const int b = (int)(i - row * per_row) * 8;
    uint2 v = make_uint2(0, 0);
    if (row < K && b < row_bytes) v = *(const uint2*)(src + row * (int64_t)row_bytes + b);
    *(uint2*)(dst + row * (int64_t)KP + b) = v;
}

// Filter-in-registers plan: [block of 32 output channels][fragment = tap * KS + step][lane][16 bytes], the operand
// layout of the 32x32 MFMAs -- lane l holds bytes 32*step + 16*(l >> 5) .. +16 of kernel element `tap` of channel
// 32*block + (l & 31) -- so that a wavefront loads a fragment with one coalesced 1 KB read.  Channels past K are zero.
__global__ void k_pack_filter_frag(const uint8_t* src, uint8_t* dst, int K, int T, int KS, int64_t total_vec)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= total_vec) return;
    const int lane = (int)(v & 63);
    const int64_t fi = v >> 6;
    const int f = (int)(fi % (T * KS));
    const int cb = (int)(fi / (T * KS));
    const int tap = f / KS, ks = f - tap * KS;
    const int oc = cb * 32 + (lane & 31);
    uint4 val = make_uint4(0, 0, 0, 0);
    if (oc < K) val = *(const uint4*)(src + ((int64_t)oc * T + tap) * (KS * 32) + ks * 32 + (lane >> 5) * 16);
    *(uint4*)(dst + v * 16) = val;
}

// uint8 tensor-core plans: sums[k] = sum over the R*S*C filter elements of output channel k (the zero-point term of
// EpilogueArgs).  One wavefront per channel.
__global__ __launch_bounds__(256) void k_filter_channel_sums(const int8_t* filt_krsc, int32_t* sums, int K, int64_t per_channel)
{
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (k >= K) return;
    const int8_t* w = filt_krsc + (int64_t)k * per_channel;
    int32_t acc = 0;
    for (int64_t i = lane; i < per_channel; i += 64) acc += (int32_t)w[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) sums[k] = acc;
}

int launch_pack_filter(const icv_conv_params* p, const Geometry& g, const void* filt, void* packed, hipStream_t s)
{
    const int64_t CB = (int64_t)p->C * g.elem_bytes;
    if (g.wsum_offset >= 0) {
        hipLaunchKernelGGL(k_filter_channel_sums, dim3((unsigned)((p->K + 3) / 4)), dim3(256), 0, s, (const int8_t*)filt,
                           (int32_t*)((uint8_t*)packed + g.wsum_offset), p->K, (int64_t)g.T * p->C);
        ICV_HIP_CHECK(hipGetLastError());
    }
    if (g.kind == PLAN_MFMA_FREG) {
        const int KS = g.KCB / 32;
        const int64_t col_blocks = g.n_tiles * (g.NR / 32);
        const int64_t total = col_blocks * g.T * KS * 64;
        hipLaunchKernelGGL(k_pack_filter_frag, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const uint8_t*)filt, (uint8_t*)packed, p->K, g.T, KS, total);
        ICV_HIP_CHECK(hipGetLastError());
        return ICV_OK;
    }
    if (g.kind == PLAN_MFMA_LOWC) {
        const int64_t rows = g.n_tiles * g.NR, threads = rows * (g.KCB / 8);
        hipLaunchKernelGGL(k_pack_filter_lowc, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                           (const uint8_t*)filt, (uint8_t*)packed, p->K, (int)(g.T * CB), g.KCB, rows);
        ICV_HIP_CHECK(hipGetLastError());
        return ICV_OK;
    }
    if (g.kind == PLAN_MFMA) {
        PackArgs a{};      // every field starts at zero; the ones this call uses are set below
        a.src = (const uint8_t*)filt;
        a.dst = (uint8_t*)packed;
        a.K = p->K; a.T = g.T; a.CB = (int32_t)CB;
        a.NR = g.NR; a.KCB = g.KCB; a.stages_per_tap = g.stages_per_tap; a.n_stages = g.n_stages;
        a.cc_major = g.cc_major;
        a.total_vec = g.n_tiles * g.NR * (int64_t)g.T * CB / 16;
        hipLaunchKernelGGL(k_pack_filter_vec, dim3((unsigned)((a.total_vec + 255) / 256)), dim3(256), 0, s, a);
    } else {
        const int64_t red = (int64_t)g.T * p->C, kp = g.n_tiles * g.NR, total = red * kp;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (g.elem_bytes == 4)
            hipLaunchKernelGGL(k_pack_filter_transposed<uint32_t>, grid, dim3(256), 0, s, (const uint32_t*)filt, (uint32_t*)packed, p->K, red, kp);
        else if (g.elem_bytes == 2)
            hipLaunchKernelGGL(k_pack_filter_transposed<uint16_t>, grid, dim3(256), 0, s, (const uint16_t*)filt, (uint16_t*)packed, p->K, red, kp);
        else
            hipLaunchKernelGGL(k_pack_filter_transposed<uint8_t>, grid, dim3(256), 0, s, (const uint8_t*)filt, (uint8_t*)packed, p->K, red, kp);
    }
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

// ------------------------------------------------------------------ indirection build (section 2.3)
// Entry (m, tap): iy = oy*SY + ky*DY - PT, ix = ox*SX + kx*DX - PL (Listing 1's index arithmetic);
// inside the input -> byte offset of pixel (n*Hin + iy)*Win + ix from the input base, else INT32_MIN (the
// zero row).  Physical order [m tile][tap][MR].
// A thread owns four consecutive rows m0..m0+3 of a tile and walks the kernel elements, writing one 16-byte (int32
// entries) or 8-byte (16-bit entries) piece per element: the MR / 4 threads of a tile, neighbours in one wavefront,
// write neighbouring pieces of a (tile, tap) run.
struct IndArgs {
    int32_t* ind;
    int64_t M;
    int32_t Hin, Win, Hout, Wout, R, S, SY, SX, DY, DX, PT, PL, MR, T;
    int32_t stride_bytes;   // bytes between input pixels
    // compact form (plans that read it): range records, 16-bit entries, what those hold for the zero row
    int4* ranges;
    uint16_t* rows16;
    uint32_t zero_row_number;
    uint32_t n_tiles;
    int32_t quad_shift;       // log2(MR / 4)
    int32_t splits;           // threads that share a row quad's kernel elements (grid.y)
    FastDiv by_wout, by_hout, by_s, by_dy, by_dx;
};

template <bool COMPACT>
__global__ __launch_bounds__(256) void k_build_indirection(IndArgs a)
{
    // The kernel is bound by instruction issue, not by the bytes it writes (a wavefront instruction occupies its SIMD
    // for four cycles), so a thread does everything that depends on its rows alone once and then walks all kernel
    // elements (every splits-th one when a small problem is spread over more threads); divisions are multiply-shifts;
    // and a tile's range comes from a closed form instead of a pass over its entries.
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    const uint32_t tile = t >> a.quad_shift, quad = t & ((1u << a.quad_shift) - 1u);
    const int32_t split = (int32_t)blockIdx.y;
    const bool active = tile < a.n_tiles;           // the others still take part in the shuffles below
    const int32_t mr4 = 1 << a.quad_shift;
    const int32_t r = 4 * (int32_t)quad;
    const int64_t m0 = (int64_t)tile * a.MR + r;
    // per row: iy = by + ky*DY, ix = bx + kx*DX, pixel = pb + iy*Win + ix
    int32_t by[4], bx[4], pb[4];
    bool live[4];
    {
        const uint32_t mm = (uint32_t)(active && m0 < a.M ? m0 : 0);
        const uint32_t q = fast_div(mm, a.by_wout);
        int32_t x = (int32_t)(mm - q * (uint32_t)a.Wout);
        const uint32_t nn = fast_div(q, a.by_hout);
        int32_t y = (int32_t)(q - nn * (uint32_t)a.Hout);
        int32_t n = (int32_t)nn;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            by[j] = y * a.SY - a.PT; bx[j] = x * a.SX - a.PL; pb[j] = n * a.Hin * a.Win;
            live[j] = active && m0 + j < a.M;
            if (++x == a.Wout) { x = 0; if (++y == a.Hout) { y = 0; ++n; } }
        }
    }
    int32_t first = 0;           // pixel the compact entries count from
    if constexpr (COMPACT) {
        // The tile's range record: its smallest valid entry and the number of pixels from there to the largest one,
        // {0, 1} without any.  A row's valid kernel elements are a rectangle ky_lo..ky_hi x kx_lo..kx_hi (iy depends
        // on ky alone, ix on kx alone) and the entry grows with both, so the row's extremes sit in two corners.  The
        // MR / 4 threads of a tile are neighbours in one wavefront: the tile's extremes are a few shuffles away.
        int32_t lo = INT32_MAX, hi = -1;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int32_t ky_lo = by[j] < 0 ? (int32_t)fast_div((uint32_t)(-by[j] + a.DY - 1), a.by_dy) : 0;
            const int32_t kx_lo = bx[j] < 0 ? (int32_t)fast_div((uint32_t)(-bx[j] + a.DX - 1), a.by_dx) : 0;
            const int32_t room_y = a.Hin - 1 - by[j], room_x = a.Win - 1 - bx[j];
            int32_t ky_hi = (int32_t)fast_div((uint32_t)(room_y < 0 ? 0 : room_y), a.by_dy);
            int32_t kx_hi = (int32_t)fast_div((uint32_t)(room_x < 0 ? 0 : room_x), a.by_dx);
            ky_hi = ky_hi < a.R - 1 ? ky_hi : a.R - 1;
            kx_hi = kx_hi < a.S - 1 ? kx_hi : a.S - 1;
            const bool any = live[j] && room_y >= 0 && room_x >= 0 && ky_lo <= ky_hi && kx_lo <= kx_hi;
            const int32_t e_lo = pb[j] + (by[j] + ky_lo * a.DY) * a.Win + bx[j] + kx_lo * a.DX;
            const int32_t e_hi = pb[j] + (by[j] + ky_hi * a.DY) * a.Win + bx[j] + kx_hi * a.DX;
            lo = any && e_lo < lo ? e_lo : lo;
            hi = any && e_hi > hi ? e_hi : hi;
        }
        for (int d = mr4 >> 1; d >= 1; d >>= 1) {
            const int32_t lo2 = __shfl_xor(lo, d, 64), hi2 = __shfl_xor(hi, d, 64);
            lo = lo2 < lo ? lo2 : lo;
            hi = hi2 > hi ? hi2 : hi;
        }
        first = hi < 0 ? 0 : lo;
        if (active && quad == 0 && split == 0)
            a.ranges[tile] = make_int4(first * a.stride_bytes, hi < 0 ? 1 : hi - lo + 1, 0, 0);
    }
    if (!active) return;
    // this thread's kernel elements split, split + splits, ... as (ky, kx)
    int32_t ky = (int32_t)fast_div((uint32_t)split, a.by_s), kx = split - ky * a.S;
    const int32_t step_y = (int32_t)fast_div((uint32_t)a.splits, a.by_s), step_x = a.splits - step_y * a.S;
    // Four rows in one output row (the usual case) share iy and step through ix by SX: one pixel number per kernel
    // element and four bounds checks instead of four full evaluations.
    const bool flat = by[3] == by[0] && pb[3] == pb[0] && live[3];
    const int64_t tile_at = (int64_t)tile * ((int64_t)a.T * a.MR) + r;
    uint2* dst16 = COMPACT ? (uint2*)(a.rows16 + tile_at) + (int64_t)split * mr4 : nullptr;
    int4* dst32 = COMPACT ? nullptr : (int4*)(a.ind + tile_at) + (int64_t)split * mr4;
    const int64_t dst_step = (int64_t)a.splits * mr4;
    for (int32_t tap = split; tap < a.T; tap += a.splits) {
        const int32_t dy = ky * a.DY, dx = kx * a.DX;
        int32_t e[4];
        if (flat) {
            const int32_t iy = by[0] + dy, ix0 = bx[0] + dx;
            const bool in_y = (uint32_t)iy < (uint32_t)a.Hin;
            const int32_t pixel0 = pb[0] + iy * a.Win + ix0 - first;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const bool in = in_y && (uint32_t)(ix0 + j * a.SX) < (uint32_t)a.Win;
                if constexpr (COMPACT) e[j] = in ? pixel0 + j * a.SX : (int32_t)a.zero_row_number;
                else e[j] = in ? (pixel0 + j * a.SX) * a.stride_bytes : INT32_MIN;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int32_t iy = by[j] + dy, ix = bx[j] + dx;
                const bool in = live[j] && (uint32_t)iy < (uint32_t)a.Hin && (uint32_t)ix < (uint32_t)a.Win;
                const int32_t pixel = pb[j] + iy * a.Win + ix;
                if constexpr (COMPACT) e[j] = in ? pixel - first : (int32_t)a.zero_row_number;
                else e[j] = in ? pixel * a.stride_bytes : INT32_MIN;         // byte offsets, INT32_MIN for the zero row
            }
        }
        if constexpr (COMPACT) {
            *dst16 = make_uint2((uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16));
            dst16 += dst_step;
        } else {
            *dst32 = make_int4(e[0], e[1], e[2], e[3]);
            dst32 += dst_step;
        }
        kx += step_x; ky += step_y;
        if (kx >= a.S) { kx -= a.S; ++ky; }
    }
}

// Block form (filter-in-registers plan): per block of 32 consecutive output pixels one 16-byte record {base byte
// offset, 0, base pixel, 0} -- the base is the closed-form lower bound of icv_pixel_range.h for the block's first
// pixel, so a kernel can compute it without reading anything -- and per (kernel element, row) the entry as a 16-bit
// pixel number counted from that base, 0xFFFF for the zero row (and for rows past M).  Physical order
// [block][kernel element][32].  A wavefront builds one block: lane -> (kernel element l / 16 of a group of four,
// rows 2 * (l % 16) and the next), so every store instruction writes 256 contiguous bytes.
struct BlockIndArgs {
    int4* rec;
    uint16_t* ent;
    RangeGeom q;
    int64_t M;
    uint32_t n_blocks;
    int32_t T, stride_bytes;
    FastDiv by_s;
};

__global__ __launch_bounds__(256) void k_build_block_indirection(BlockIndArgs a)
{
    const uint32_t blk = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (blk >= a.n_blocks) return;
    const int lane = threadIdx.x & 63;
    const int32_t base = lowest_pixel_from(a.q, decompose(a.q, blk * 32u));
    if (lane == 0) a.rec[blk] = make_int4(base * a.stride_bytes, 0, base, 0);
    const uint32_t m0 = blk * 32u + 2u * (uint32_t)(lane & 15);
    OutPixel o[2];
    bool live[2];
#pragma unroll
    for (int j = 0; j < 2; j++) {
        live[j] = (int64_t)(m0 + j) < a.M;
        o[j] = decompose(a.q, live[j] ? m0 + j : 0u);
    }
    uint32_t* dst = (uint32_t*)(a.ent + (int64_t)blk * a.T * 32) + lane;
    // this lane's kernel elements lane / 16, + 4, ... as (ky, kx), stepped without a division per element
    int32_t ky = (int32_t)fast_div((uint32_t)(lane >> 4), a.by_s), kx = (lane >> 4) - ky * a.q.S;
    const int32_t step_y = (int32_t)fast_div(4u, a.by_s), step_x = 4 - step_y * a.q.S;
    for (int32_t tap = lane >> 4; tap < a.T; tap += 4) {
        uint32_t e[2];
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int32_t iy = o[j].oy * a.q.SY + ky * a.q.DY - a.q.PT;
            const int32_t ix = o[j].ox * a.q.SX + kx * a.q.DX - a.q.PL;
            const bool in = live[j] && (uint32_t)iy < (uint32_t)a.q.Hin && (uint32_t)ix < (uint32_t)a.q.Win;
            e[j] = in ? (uint32_t)((o[j].n * a.q.Hin + iy) * a.q.Win + ix - base) : 0xFFFFu;
        }
        dst[(tap - (lane >> 4)) * 16] = e[0] | (e[1] << 16);
        kx += step_x; ky += step_y;
        if (kx >= a.q.S) { kx -= a.q.S; ++ky; }
    }
}

int launch_build_indirection(const icv_conv_params* p, const Geometry& g, int32_t* ind, hipStream_t s)
{
    if (g.kind == PLAN_MFMA_FREG) {
        BlockIndArgs b{};
        b.rec = (int4*)ind;
        b.ent = (uint16_t*)(b.rec + g.img_tiles);
        b.q = make_range_geom(p->Hin, p->Win, g.Hout, g.Wout, p->SY, p->SX, p->DY, p->DX, p->PT, p->PL, p->R, p->S);
        b.M = g.img_rows;
        b.n_blocks = (uint32_t)g.img_tiles;
        b.T = g.T;
        b.stride_bytes = g.in_stride * g.elem_bytes;
        b.by_s = make_fast_div((uint32_t)p->S);
        hipLaunchKernelGGL(k_build_block_indirection, dim3((unsigned)((g.img_tiles + 3) / 4)), dim3(256), 0, s, b);
        ICV_HIP_CHECK(hipGetLastError());
        return ICV_OK;
    }
    IndArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.ind = ind;
    // a batch-independent buffer holds the entries of one image (batch index 0); img_rows = M otherwise
    a.M = g.img_rows;
    a.Hin = p->Hin; a.Win = p->Win; a.Hout = g.Hout; a.Wout = g.Wout;
    a.R = p->R; a.S = p->S; a.SY = p->SY; a.SX = p->SX; a.DY = p->DY; a.DX = p->DX;
    a.PT = p->PT; a.PL = p->PL; a.MR = g.MR; a.T = g.T;
    a.stride_bytes = g.in_stride * g.elem_bytes;
    if (g.MR != 64 && g.MR != 128 && g.MR != 256) return ICV_ERR_UNSUPPORTED;         // a tile's threads share a wavefront
    a.quad_shift = g.MR == 64 ? 4 : (g.MR == 128 ? 5 : 6);
    const int64_t threads = g.img_tiles << a.quad_shift;
    if (g.img_tiles > 0x7fffffffll || (threads + 255) / 256 > 0x7fffffffll) return ICV_ERR_UNSUPPORTED;
    a.n_tiles = (uint32_t)g.img_tiles;
    // A small problem has fewer row quads than the chip has lanes: the kernel elements of a quad are then shared
    // among several threads, eight elements or more each.
    int64_t splits = (65536 + threads - 1) / threads;
    const int64_t most = (g.T + 7) / 8;
    if (splits > most) splits = most;
    if (splits < 1) splits = 1;
    a.splits = (int32_t)splits;
    const dim3 grid((unsigned)((threads + 255) / 256), (unsigned)splits);
    a.ranges = nullptr; a.rows16 = nullptr; a.zero_row_number = 0;
    a.by_wout = make_fast_div((uint32_t)g.Wout); a.by_hout = make_fast_div((uint32_t)g.Hout);
    a.by_s = make_fast_div((uint32_t)p->S); a.by_dy = make_fast_div((uint32_t)p->DY); a.by_dx = make_fast_div((uint32_t)p->DX);
    if (g.patch_rows) {
        // the buffer holds the range records, then the 16-bit entries
        if (g.zero_row_number > 65535 || g.zero_row_number < (uint32_t)g.patch_rows) return ICV_ERR_UNSUPPORTED;
        a.ranges = (int4*)ind;
        a.rows16 = (uint16_t*)(a.ranges + g.img_tiles);
        a.zero_row_number = g.zero_row_number;
        hipLaunchKernelGGL(k_build_indirection<true>, grid, dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL(k_build_indirection<false>, grid, dim3(256), 0, s, a);
    }
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

// ------------------------------------------------------------------ im2col (ablation; section 1, "GEMM-based algorithms")
// ws[m][tap][C]: the patch of input pixels behind output pixel m copied into row m; taps outside the input
// become zeros (the zero point for u8i8).  Rows past M (tile padding) are filled like padding.
// One thread moves `VB` bytes of one (m, tap) pixel row.
struct Im2colArgs {
    const uint8_t* in;
    uint8_t* ws;
    int64_t M, m_padded;
    int32_t Hin, Win, Hout, Wout, S, SY, SX, DY, DX, PT, PL, T;
    int32_t CB;             // bytes of one pixel row copied (C * elem)
    int64_t stride_bytes;   // input pixel stride in bytes
    uint32_t fill;          // padding pattern, replicated per byte
};

template <int VB>
__global__ __launch_bounds__(256) void k_im2col(Im2colArgs a)
{
    const int32_t vec_per_row = a.CB / VB;
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = a.m_padded * a.T * vec_per_row;
    if (v >= total) return;
    const int32_t c = (int32_t)(v % vec_per_row);
    const int64_t mt = v / vec_per_row;
    const int32_t tap = (int32_t)(mt % a.T);
    const int64_t m = mt / a.T;
    const int32_t ky = tap / a.S, kx = tap - ky * a.S;
    const int32_t ox = (int32_t)(m % a.Wout);
    const int64_t q = m / a.Wout;
    const int32_t oy = (int32_t)(q % a.Hout);
    const int32_t n = (int32_t)(q / a.Hout);
    const int32_t iy = oy * a.SY + ky * a.DY - a.PT;
    const int32_t ix = ox * a.SX + kx * a.DX - a.PL;
    const bool in = m < a.M && (uint32_t)iy < (uint32_t)a.Hin && (uint32_t)ix < (uint32_t)a.Win;
    uint8_t* d = a.ws + v * VB;
    if constexpr (VB == 16) {
        uint4 val = make_uint4(a.fill, a.fill, a.fill, a.fill);
        if (in) val = *(const uint4*)(a.in + (((int64_t)n * a.Hin + iy) * a.Win + ix) * a.stride_bytes + c * 16);
        *(uint4*)d = val;
    } else {
        for (int b = 0; b < VB; b++)
            d[b] = in ? a.in[(((int64_t)n * a.Hin + iy) * a.Win + ix) * a.stride_bytes + c * VB + b]
                      : (uint8_t)(a.fill & 0xff);
    }
}

// Low-C plan: rows of KP bytes, [tap][C] followed by zeros; one thread per 8 bytes.
__global__ __launch_bounds__(256) void k_im2col_lowc(Im2colArgs a, int KP)
{
    const int per_row = KP / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.m_padded * per_row) return;
    const int64_t m = i / per_row;
    const int b = (int)(i - m * per_row) * 8;
    const int32_t tap = b / a.CB, within = b - tap * a.CB;
    uint2 val = make_uint2(0, 0);
    if (tap < a.T) {
        const int32_t ky = tap / a.S, kx = tap - ky * a.S;
        const int32_t ox = (int32_t)(m % a.Wout);
        const int64_t q = m / a.Wout;
        const int32_t oy = (int32_t)(q % a.Hout);
        const int32_t n = (int32_t)(q / a.Hout);
        const int32_t iy = oy * a.SY + ky * a.DY - a.PT;
        const int32_t ix = ox * a.SX + kx * a.DX - a.PL;
        const bool in = m < a.M && (uint32_t)iy < (uint32_t)a.Hin && (uint32_t)ix < (uint32_t)a.Win;
        val = make_uint2(a.fill, a.fill);
        if (in) val = *(const uint2*)(a.in + (((int64_t)n * a.Hin + iy) * a.Win + ix) * a.stride_bytes + within);
    }
    *(uint2*)(a.ws + i * 8) = val;
}

int launch_im2col(const icv_conv_params* p, const Geometry& g, const void* input, void* ws, hipStream_t s)
{
    Im2colArgs a{};      // every field starts at zero; the ones this call uses are set below
    a.in = (const uint8_t*)input;
    a.ws = (uint8_t*)ws;
    a.M = g.M; a.m_padded = g.m_tiles * g.MR;
    a.Hin = p->Hin; a.Win = p->Win; a.Hout = g.Hout; a.Wout = g.Wout;
    a.S = p->S; a.SY = p->SY; a.SX = p->SX; a.DY = p->DY; a.DX = p->DX; a.PT = p->PT; a.PL = p->PL; a.T = g.T;
    a.CB = p->C * g.elem_bytes;
    a.stride_bytes = (int64_t)g.in_stride * g.elem_bytes;
    const uint32_t zp = p->dtype == ICV_U8I8 ? (uint32_t)p->input_zero_point : 0u;
    a.fill = zp * 0x01010101u;
    if (g.kind == PLAN_MFMA_LOWC) {
        const int64_t threads = a.m_padded * (g.KCB / 8);
        hipLaunchKernelGGL(k_im2col_lowc, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, a, g.KCB);
        ICV_HIP_CHECK(hipGetLastError());
        return ICV_OK;
    }
    const bool vec16 = a.CB % 16 == 0 && a.stride_bytes % 16 == 0;
    const int vb = vec16 ? 16 : g.elem_bytes;
    const int64_t total = a.m_padded * a.T * (a.CB / vb);
    const dim3 grid((unsigned)((total + 255) / 256));
    if (vec16) hipLaunchKernelGGL(k_im2col<16>, grid, dim3(256), 0, s, a);
    else if (vb == 4) hipLaunchKernelGGL(k_im2col<4>, grid, dim3(256), 0, s, a);
    else if (vb == 2) hipLaunchKernelGGL(k_im2col<2>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(k_im2col<1>, grid, dim3(256), 0, s, a);
    ICV_HIP_CHECK(hipGetLastError());
    return ICV_OK;
}

}  // namespace icv
