// Closed-form bounds on the input pixels that the indirection entries of a run of consecutive output pixels name
// (host and device).
//
// Entry (m, tap) of the indirection buffer (section 2.3) names input pixel
//     (n*Hin + iy)*Win + ix,   iy = oy*SY + ky*DY - PT,  ix = ox*SX + kx*DX - PL        (Listing 1's indices)
// when (iy, ix) lies inside the image, else the zero row.  For one kernel element the valid entries grow strictly
// with m; so the valid entries of output pixels m0..m1 all lie between a lower bound that depends on m0 alone and an
// upper bound that depends on m1 alone.  Both are non-decreasing in m, which is what lets a kernel walk the output
// pixels in order with a sliding window of input pixels, and start copying that window before it has read a
// single entry.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define ICV_HD __host__ __device__
#else
#define ICV_HD
#endif

namespace icv {

// Division of a non-negative number below 2^31 by an invariant divisor, as a multiplication and a shift: with
// sh = ceil(log2 d) and mul = ceil(2^(31 + sh) / d) (which fits 32 bits), floor(n / d) = (n * mul) >> (31 + sh) exactly.
// The kernels divide output pixel numbers by Wout and Hout before they can issue their first load, and a hardware
// division is some thirty dependent instructions.
struct FastDiv {
    uint32_t mul, shift, d;
};

inline FastDiv make_fast_div(uint32_t d)
{
    FastDiv f;
    uint32_t sh = 0;
    while ((1ull << sh) < d) ++sh;
    f.mul = (uint32_t)(((1ull << (31 + sh)) + d - 1) / d);
    f.shift = 31 + sh;
    f.d = d;
    return f;
}

ICV_HD inline uint32_t fast_div(uint32_t n, const FastDiv& f) { return (uint32_t)(((uint64_t)n * f.mul) >> f.shift); }

struct RangeGeom {
    int32_t Hin, Win, Hout, Wout, SY, SX, DY, DX, PT, PL, R, S;
    FastDiv by_wout, by_hout;
};

inline RangeGeom make_range_geom(int32_t Hin, int32_t Win, int32_t Hout, int32_t Wout, int32_t SY, int32_t SX, int32_t DY,
                                 int32_t DX, int32_t PT, int32_t PL, int32_t R, int32_t S)
{
    return RangeGeom{Hin, Win, Hout, Wout, SY, SX, DY, DX, PT, PL, R, S, make_fast_div((uint32_t)Wout), make_fast_div((uint32_t)Hout)};
}

struct OutPixel {
    int32_t n, oy, ox;
};

ICV_HD inline OutPixel decompose(const RangeGeom& q, uint32_t m)
{
    const uint32_t row = fast_div(m, q.by_wout);
    OutPixel o;
    o.ox = (int32_t)(m - row * (uint32_t)q.Wout);
    o.n = (int32_t)fast_div(row, q.by_hout);
    o.oy = (int32_t)(row - (uint32_t)o.n * (uint32_t)q.Hout);
    return o;
}

// A pixel index that no valid entry of output pixel `o`, or of any later output pixel, lies below.
ICV_HD inline int32_t lowest_pixel_from(const RangeGeom& q, const OutPixel& o)
{
    const int32_t img = o.n * q.Hin * q.Win;
    const int32_t iy = o.oy * q.SY - q.PT;
    int32_t ix = o.ox * q.SX - q.PL;
    if (iy < 0) return img;                               // the kernel still starts above the image
    if (iy > q.Hin - 1) return img + q.Hin * q.Win - 1;   // ... below it: nothing of this image is named from here on
    ix = ix < 0 ? 0 : (ix > q.Win - 1 ? q.Win - 1 : ix);
    return img + iy * q.Win + ix;
}

// A pixel index that no valid entry of output pixel `o`, or of any earlier output pixel, lies above.
ICV_HD inline int32_t highest_pixel_upto(const RangeGeom& q, const OutPixel& o)
{
    const int32_t img = o.n * q.Hin * q.Win;
    const int32_t iy = o.oy * q.SY + (q.R - 1) * q.DY - q.PT;
    int32_t ix = o.ox * q.SX + (q.S - 1) * q.DX - q.PL;
    if (iy > q.Hin - 1) return img + q.Hin * q.Win - 1;
    if (iy < 0) return img;                               // nothing of this image has been named yet
    ix = ix < 0 ? 0 : (ix > q.Win - 1 ? q.Win - 1 : ix);
    return img + iy * q.Win + ix;
}

}  // namespace icv
