// 8-point inverse DCT and the colour conversion, fp32 (paper, Section 4.3; the transform is the
// inverse of the type-II DCT named in Section 2).  Host/device.
#pragma once
#include "jpgd_common.h"

namespace jpgd {

// x_n = 1/2 * sum_k c_k X_k cos((2n+1) k pi / 16), c_0 = 1/sqrt(2), c_k = 1 otherwise.
// Even/odd split: x_n = e_n + o_n, x_{7-n} = e_n - o_n for n = 0..3; the even half is a 4-point
// transform split once more, the odd half a 4x4 product with cos(j pi/16)/2, j = 1,3,5,7.
JPGD_HD void idct8(float& v0, float& v1, float& v2, float& v3, float& v4, float& v5, float& v6, float& v7) {
    const float c1 = 0.49039264020161522f;  // cos(1 pi/16)/2
    const float c2 = 0.46193976625564337f;  // cos(2 pi/16)/2
    const float c3 = 0.41573480615127262f;
    const float c4 = 0.35355339059327379f;  // cos(4 pi/16)/2 = 1/(2 sqrt 2)
    const float c5 = 0.27778511650980114f;
    const float c6 = 0.19134171618254489f;
    const float c7 = 0.09754516100806417f;
    float a0 = (v0 + v4) * c4, a1 = (v0 - v4) * c4;
    float b0 = v2 * c2 + v6 * c6, b1 = v2 * c6 - v6 * c2;
    float e0 = a0 + b0, e3 = a0 - b0, e1 = a1 + b1, e2 = a1 - b1;
    float o0 = v1 * c1 + v3 * c3 + v5 * c5 + v7 * c7;
    float o1 = v1 * c3 - v3 * c7 - v5 * c1 - v7 * c5;
    float o2 = v1 * c5 - v3 * c1 + v5 * c7 + v7 * c3;
    float o3 = v1 * c7 - v3 * c5 + v5 * c3 - v7 * c1;
    v0 = e0 + o0; v7 = e0 - o0;
    v1 = e1 + o1; v6 = e1 - o1;
    v2 = e2 + o2; v5 = e2 - o2;
    v3 = e3 + o3; v4 = e3 - o3;
}

// The first input of idct8 reaches every output multiplied by 1/(2 sqrt 2): adding 128 * 2 sqrt 2 to it adds the
// level shift of 128 to all eight outputs.
constexpr float kLevelShiftDc = 362.03867196751236f;

// Float to 8-bit sample, written into byte `byte` (0..3) of `word`: nearest integer, ties to the even one,
// limited to [0, 255] (NaN gives 0).  On the device this is one instruction, v_cvt_pk_u8_f32, which also does the
// packing of four samples into the 32-bit words the pixel kernel stores.  A tie is rounded down where rounding
// half up would round up, in one of two cases; unrounded samples are sums of products of floats and all but
// never ties, and one level is the bar for pixels.
JPGD_HD uint32_t pack_u8(float v, uint32_t byte, uint32_t word) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_cvt_pk_u8_f32(v, byte, word);
#else
    float r = v != v ? 0.0f : __builtin_rintf(v);  // the default rounding mode: nearest, ties to even
    r = r < 0.0f ? 0.0f : (r > 255.0f ? 255.0f : r);
    const uint32_t sh = 8u * (byte & 3u);
    return (word & ~(0xFFu << sh)) | ((uint32_t)r << sh);
#endif
}

// JFIF YCbCr -> RGB: what one chroma sample (level shift applied: 128 = neutral) adds to the luma sample of every
// pixel it covers, R = Y + r, G = Y + g, B = Y + b.  Computed once per chroma sample, not per pixel.
struct ChromaTerms {
    float r, g, b;
};
JPGD_HD ChromaTerms chroma_terms(float cb, float cr) {
    ChromaTerms t;
    t.r = __builtin_fmaf(1.402f, cr, -1.402f * 128.0f);
    t.g = __builtin_fmaf(-0.344136f, cb, __builtin_fmaf(-0.714136f, cr, (0.344136f + 0.714136f) * 128.0f));
    t.b = __builtin_fmaf(1.772f, cb, -1.772f * 128.0f);
    return t;
}

// zig-zag position -> row*8 + col, from walking the anti-diagonals (kept as a literal so that it can
// sit in constant memory; tests/ regenerate it from the walk and compare)
#define JPGD_ZIGZAG_LITERAL                                                                                     \
    {0,  1,  8,  16, 9,  2,  3,  10, 17, 24, 32, 25, 18, 11, 4,  5,  12, 19, 26, 33, 40, 48,                     \
     41, 34, 27, 20, 13, 6,  7,  14, 21, 28, 35, 42, 49, 56, 57, 50, 43, 36, 29, 22, 15, 23,                     \
     30, 37, 44, 51, 58, 59, 52, 45, 38, 31, 39, 46, 53, 60, 61, 54, 47, 55, 62, 63}

}  // namespace jpgd
