/*
 * icv -- Indirect Convolution for AMD MI355X (gfx950).  C ABI of libicv.so.
 *
 * The library implements the hot path of the Indirect Convolution algorithm
 * (M. Dukhan, arXiv 1907.02129): an indirection buffer that names, for every
 * output pixel and kernel element, the input pixel row to read (section 2.3),
 * and an Indirect GEMM that accumulates output tiles over R*S*C by gathering
 * rows of A through that buffer (section 2.2, Listing 3), so that no im2col
 * matrix is ever written.
 *
 * Conventions that hold for every entry point
 *  - Tensors: input NHWC, output NHWC, filter [K][R][S][C] (Listing 1).
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    allocates no memory, keeps no state between calls and is re-entrant.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work on it and return without synchronising.
 *  - Return value: ICV_OK or a negative icv_status; nothing aborts or throws.
 *    Invalid arguments are detected on the host before anything is launched.
 *  - Base pointers must be 16-byte aligned and pixel strides must make every
 *    pixel row start 16-byte aligned (bf16 / u8i8 tensor-core paths).
 */
#ifndef ICV_H
#define ICV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported from libicv.so (everything else in the library has hidden visibility) */
#define ICV_API __attribute__((visibility("default")))

typedef enum {
    ICV_OK = 0,
    ICV_ERR_INVALID_ARG = -1, /* null pointer, non-positive extent, misalignment, index overflow */
    ICV_ERR_UNSUPPORTED = -2, /* a valid problem this build has no kernel for */
    ICV_ERR_HIP = -3          /* a HIP call failed; see icv_last_hip_error() */
} icv_status;

/* Element types: input/filter -> accumulator/output. */
typedef enum {
    ICV_F32 = 0,  /* float  x float    -> float  (MFMA when C is a multiple of 16, else vector ALU) */
    ICV_BF16 = 1, /* bf16   x bf16     -> float  (MFMA, fp32 accumulate)                 */
    ICV_U8I8 = 2  /* uint8  x int8     -> int32  (MFMA, out = sum (x - zero_point) * w)  */
} icv_dtype;

/*
 * Problem statement, in the symbols of Listing 1 and section 2.3.
 * Output extent (the paper leaves it undefined; the customary floor formula):
 *   Hout = floor((Hin + PT + PB - DY*(R-1) - 1) / SY) + 1, Wout alike with PL, PR, DX, S, SX.
 * A tap (ky,kx) of output pixel (oy,ox) reads input pixel
 *   iy = oy*SY + ky*DY - PT,  ix = ox*SX + kx*DX - PL
 * (the listing prints PL in the y formula and PT in the x formula; top pads y and
 * left pads x here), or the zero row when that lies outside the input.
 */
typedef struct icv_conv_params {
    int32_t N, Hin, Win, C, K, R, S;
    int32_t SY, SX, DY, DX;
    int32_t PT, PL, PB, PR;    /* implicit zero padding: top, left, bottom, right */
    int32_t in_pixel_stride;   /* elements between input pixels;  0 means C (section 2.3: input rows may be strided) */
    int32_t out_pixel_stride;  /* elements between output pixels; 0 means K (ldc of Listing 3)                 */
    int32_t dtype;             /* icv_dtype */
    int32_t input_zero_point;  /* ICV_U8I8 only: the value the zero row holds, 0..255.  Any value runs on the tensor
                                  cores: they multiply (x - 128) * w, and the kernels add (128 - zero point) times
                                  the output channel's filter sum, which icv_pack_filter computes once */
    int32_t plan;              /* 0: the library chooses.  Else one ICV_PLAN_* algorithm (bits 0-2), optionally or-ed
                                  with ICV_PLAN_PER_IMAGE; all other bits must be 0.  All set-up calls and the conv
                                  call of one problem must use the same value. */
} icv_conv_params;

/* plan, bits 0-2: the kernel family that computes the convolution (the library's choice when 0).
 * ICV_ERR_UNSUPPORTED when the family does not cover the problem. */
#define ICV_PLAN_VECTOR_ALU 1   /* fp32 vector-ALU kernel, no tensor cores: every dtype, every shape */
#define ICV_PLAN_GATHER 2       /* tensor cores; each kernel element's rows fetched through their entries, one
                                   element at a time: the Indirect GEMM of section 2.2 as printed, and the only
                                   family whose packed filter the im2col + GEMM comparison path reads */
#define ICV_PLAN_WINDOW 3       /* tensor cores; the input pixels a row tile names are copied to LDS once and
                                   every kernel element reads them there */
#define ICV_PLAN_FILTER_REGS 4  /* tensor cores; the filter stays in registers and the input slides through LDS
                                   (3x3 on 64-, 128- and 256-byte pixel rows, 5x5 on 64-byte ones) */
/* plan, bit 3: batch-independent indirection buffer.  The buffer then holds the entries of ONE image, offsets
 * relative to that image's first pixel, and row tiles never straddle two images; the kernels add
 * n * Hin*Win*pixel stride for image n.  Section 2.3 lists a change of batch size among the events that force the
 * buffer to be (partly) rebuilt; with this bit none is needed: a buffer built with any N serves every N, and N
 * plays no part in the choice of the tile (the packed filter and zero row do not depend on N either).  The price
 * is a partial last tile per image instead of one per batch. */
#define ICV_PLAN_PER_IMAGE 8


/* Hout, Wout by the formula above.  ICV_ERR_INVALID_ARG when the parameters are not a valid problem. */
ICV_API int icv_output_size(const icv_conv_params* p, int32_t* Hout, int32_t* Wout);

/*
 * Buffer sizes in bytes (0 when the parameters are invalid).
 *  indirection  : one entry per (output pixel, kernel element), M rounded up to whole row tiles, times R*S
 *                 (independent of C, section 1.1; with ICV_PLAN_PER_IMAGE, M is Hout*Wout, one image's output
 *                 pixels, whatever N is).  Entries are int32 byte offsets, or -- for the kernels that keep a
 *                 tile's input pixels in LDS, and the kernel for very short pixel rows -- a 16-byte record per
 *                 row tile followed by uint16 pixel numbers counted from the tile's base; only the form the plan's
 *                 kernel reads is built.  icv_get_indirection_layout describes it.
 *  packed filter: the [K][R][S][C] filter re-laid as the tiles the GEMM kernel reads, K padded to the tile; for
 *                 ICV_U8I8 on the tensor cores followed by K int32 filter sums (the zero-point term, below)
 *  zero row     : C elements (section 2.3's explicit zero vector), rounded up to 16 bytes
 *  im2col       : the [M][R*S*C] patch matrix of the ablation path
 */
ICV_API size_t icv_indirection_bytes(const icv_conv_params* p);
ICV_API size_t icv_packed_filter_bytes(const icv_conv_params* p);
ICV_API size_t icv_zero_row_bytes(const icv_conv_params* p);
ICV_API size_t icv_im2col_bytes(const icv_conv_params* p);

/*
 * Where the entry of output pixel m = (n*Hout + oy)*Wout + ox and kernel element tap = ky*S + kx sits among the
 * entries of the indirection buffer (index in entries, see icv_get_indirection_layout).  The physical order is
 * [row tile][tap][row in tile], the order in which Listing 3 consumes pointers (*ppa++: all rows of the tile for one
 * tap, then the next tap).  Rows past M in the last tile name the zero row.  Returns -1 on invalid arguments.  With
 * ICV_PLAN_PER_IMAGE the buffer describes one image: m = oy*Wout + ox < Hout*Wout.
 */
ICV_API int64_t icv_indirection_index(const icv_conv_params* p, int64_t m, int32_t tap);

/*
 * How icv_setup_indirection lays the buffer out for this problem (section 2.3 fixes what an entry means, not how
 * it is stored).  All offsets are bytes from the start of the buffer.
 *   entry_bytes 4: entries are int32 byte offsets of the pixel row from the input base, INT32_MIN = the zero row.
 *   entry_bytes 2: entries are uint16 pixel numbers counted from their row tile's base, `zero_code` = the zero row;
 *                  every row tile has a 16-byte record {int32 base byte offset, int32 pixels from the base to the
 *                  tile's largest valid entry (0: not recorded), int32 base pixel index (0: not recorded), 0}, and
 *                  entry e names the pixel row at byte offset  base byte offset + e * pixel stride in bytes.
 * `entries_at` / `entry_bytes` describe the form the convolution kernel of this plan reads, the only one built;
 * `int32_entries_at` says where int32 entries start (0 for entry_bytes 4, -1 when they are not built).
 */
typedef struct icv_indirection_layout {
    int32_t tile_rows;         /* output pixels per row tile */
    int32_t entry_bytes;       /* 4 or 2 */
    int32_t zero_code;         /* 2-byte entries: the value that names the zero row */
    int32_t record_bytes;      /* 16 when the tiles have records, else 0 */
    int64_t tiles;             /* row tiles the buffer describes */
    int64_t entries_at;
    int64_t records_at;        /* -1 without records */
    int64_t int32_entries_at;  /* -1 when the int32 form is not built */
} icv_indirection_layout;
ICV_API int icv_get_indirection_layout(const icv_conv_params* p, icv_indirection_layout* layout);

/*
 * Closed-form bounds (host arithmetic) on the input pixels that the valid entries (section 2.3; Listing 1's iy, ix)
 * of output pixels m0..m1 name:
 * *first is not above any of them, *last not below (pixel indices (n*Hin + iy)*Win + ix of the whole tensor).  Both
 * are non-decreasing in m0 and m1, which is what lets a kernel keep a sliding window of input pixels while it walks
 * the output pixels in order.  last - first + 1 <= icv_tile_span_bound(p, m1 - m0 + 1).
 */
ICV_API int icv_row_pixel_range(const icv_conv_params* p, int64_t m0, int64_t m1, int64_t* first, int64_t* last);

/*
 * Upper bound on the number of consecutive input pixels that the valid entries of any `rows` consecutive
 * output pixels span (the entries of neighbouring output pixels overlap, the re-use of input rows that section 3 lists as the method's second performance factor);
 * the library sizes its LDS input patch with it.  Host arithmetic only.  Returns -1 on invalid arguments.
 */
ICV_API int64_t icv_tile_span_bound(const icv_conv_params* p, int32_t rows);

/* Fill the explicit zero vector of section 2.3: zeros, or input_zero_point bytes for ICV_U8I8. */
ICV_API int icv_init_zero_row(const icv_conv_params* p, void* zero_row, void* stream);

/*
 * Repack the filter once, off the timed path (section 3.1, "Implementation": matrix B is repacked into a
 * contiguous region because weights never change at inference time).
 *   filter_krsc: [K][R][S][C] device, packed: icv_packed_filter_bytes() device.
 */
ICV_API int icv_pack_filter(const icv_conv_params* p, const void* filter_krsc, void* packed, void* stream);

/*
 * Build the indirection buffer (section 2.3).  Entry = byte offset of the input pixel's row from the input
 * base, ((n*Hin + iy)*Win + ix) * in_pixel_stride * sizeof(element), or INT32_MIN for "the zero row": the
 * paper's row pointer minus the tensor's base pointer.  Storing offsets keeps the buffer valid when the
 * input or zero-row pointers change (the paper's fourth invalidation rule then never applies); it must be
 * rebuilt only when the shape, stride, dilation, padding, pixel stride, element type or batch size change
 * (with ICV_PLAN_PER_IMAGE not even for the batch size: N is not read).
 * The input tensor must be smaller than 2 GiB (ICV_ERR_INVALID_ARG otherwise).
 *   indirection: icv_indirection_bytes() device.
 */
ICV_API int icv_setup_indirection(const icv_conv_params* p, void* indirection, void* stream);

/*
 * The Indirect GEMM (section 2.2): output = conv(input, filter) with rows of A gathered through the
 * indirection buffer; negative entries read `zero_row`.  alpha = 1, beta = 0: the output is overwritten.
 *   input        : [N][Hin][Win] pixels of in_pixel_stride elements (first C used)
 *   packed_filter: from icv_pack_filter with the same params
 *   indirection  : from icv_setup_indirection with the same params
 *   zero_row     : from icv_init_zero_row.  Its contents must be what that call wrote: the kernels that stage rows
 *                  in LDS keep a copy of that constant row there (zeros, or the zero point) instead of fetching
 *                  this buffer for every padding entry; the other kernels read it as Listing 3 does
 *   output       : [N][Hout][Wout] pixels of out_pixel_stride elements (first K written), float or int32
 */
ICV_API int icv_conv2d_nhwc(const icv_conv_params* p, const void* input, const void* packed_filter,
                    const void* indirection, const void* zero_row, void* output, void* stream);

/*
 * The same convolution with an output stage fused into the kernel's epilogue.  Not part of the paper's
 * algorithm (the paper only lists a bias tensor among the operands of its benchmark, section 3.1); it saves the
 * extra pass over the output that a separate bias / activation / conversion kernel would cost.  Per output
 * channel k:   y = acc + bias[k];   relu: y = max(y, 0);   then, by out_type,
 *   ICV_OUT_ACC : y stored as float (ICV_F32, ICV_BF16) or int32 (ICV_U8I8), as icv_conv2d_nhwc does;
 *   ICV_OUT_BF16: float paths only; y rounded to bfloat16 (nearest, ties to even), 2 bytes per element;
 *   ICV_OUT_U8  : ICV_U8I8 only; q = clamp(rint((float)y * out_scale) + out_zero_point, 0, 255), the product and
 *                 the rounding (ties to even) in single precision, 1 byte per element.
 * `output` is [N][Hout][Wout] pixels of out_pixel_stride elements of that type.  bias: K floats, or K int32 for
 * ICV_U8I8, device memory, 4-byte aligned, or NULL.  ICV_ERR_INVALID_ARG for an out_type that does not fit the
 * dtype, a scale that is not positive and finite, a zero point outside 0..255.
 */
typedef enum icv_out_type { ICV_OUT_ACC = 0, ICV_OUT_BF16 = 1, ICV_OUT_U8 = 2 } icv_out_type;
typedef struct icv_epilogue {
    const void* bias;
    int32_t relu;            /* 0 or 1 */
    int32_t out_type;        /* icv_out_type */
    float out_scale;         /* ICV_OUT_U8 */
    int32_t out_zero_point;  /* ICV_OUT_U8 */
} icv_epilogue;
ICV_API int icv_conv2d_nhwc_fused(const icv_conv_params* p, const void* input, const void* packed_filter,
                          const void* indirection, const void* zero_row, const icv_epilogue* epilogue,
                          void* output, void* stream);

/*
 * Ablation, not the method: the GEMM-based algorithm the paper compares against (section 1, "GEMM-based
 * algorithms"): write the [M][R*S*C] patch matrix (im2col), then a plain constant-stride GEMM with the same
 * tensor-core inner loop.  icv_im2col and icv_gemm_nhwc are its two halves; icv_conv2d_nhwc_im2col runs both.
 */
ICV_API int icv_im2col(const icv_conv_params* p, const void* input, void* im2col_ws, void* stream);
ICV_API int icv_gemm_nhwc(const icv_conv_params* p, const void* im2col_ws, const void* packed_filter, void* output,
                  void* stream);
ICV_API int icv_conv2d_nhwc_im2col(const icv_conv_params* p, const void* input, const void* packed_filter,
                           void* im2col_ws, void* output, void* stream);

/*
 * icv_conv2d_nhwc_im2col for callers that cannot allocate device memory: code under HIP graph capture, serving loops
 * and harnesses that forbid hipMalloc.  The patch matrix goes into a buffer that is part of the library's own device
 * image (icv_static_workspace_bytes() bytes, 16 MiB, per GPU, held until the process ends) instead of a caller's
 * workspace; the call itself allocates nothing and frees nothing.  The kernels and the results are those of
 * icv_conv2d_nhwc_im2col.  ICV_ERR_UNSUPPORTED when icv_im2col_bytes(p) exceeds the buffer (or is 0: a plan without
 * ablation).  All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (different
 * streams, or threads) race on it; calls on one stream are ordered and safe.  Nothing in the buffer needs clearing
 * between calls: every byte a call reads, it has written before.
 */
ICV_API size_t icv_static_workspace_bytes(void);
ICV_API int icv_conv2d_nhwc_im2col_static(const icv_conv_params* p, const void* input, const void* packed_filter,
                                  void* output, void* stream);

/*
 * Measurement aid: the rate, in multiply-add operations times two per second, at which the current device runs a
 * loop of nothing but tensor-core instructions on register operands (dtype ICV_BF16: 32x32x16 bfloat16 blocks,
 * ICV_U8I8: 32x32x32 int8 blocks), `waves_per_simd` (1..4) wavefronts on every SIMD of every compute unit.
 * varied_operands = 0: every instruction multiplies the same two constant operands, the least switching activity
 * the matrix cores can have; 1: pseudo-random operands, a different pair in every instruction, as with real
 * tensors (a device at its power limit holds a lower clock then).  Either is a ceiling the Indirect GEMM kernels'
 * throughput can be set against beside the data-sheet figure, at the clock the device sustains under that load.
 * Takes a few milliseconds, synchronises `stream`, allocates no memory.  Other argument values: ICV_ERR_INVALID_ARG.
 */
ICV_API int icv_measure_mfma_peak(int32_t dtype, int32_t waves_per_simd, int32_t varied_operands, double* ops_per_second,
                                  void* stream);

/* Name of the kernel variant icv_conv2d_nhwc would launch for p (static string; "" when invalid). */
ICV_API const char* icv_plan_name(const icv_conv_params* p);

ICV_API const char* icv_status_string(int status);
/* hipError_t of the last failed HIP call on this thread (0 when none). */
ICV_API int icv_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ICV_H */
