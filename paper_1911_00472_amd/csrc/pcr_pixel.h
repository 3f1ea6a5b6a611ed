// De-quantised coefficients -> samples -> RGB, compiled for host and device.
// The inverse DCT is the 8x8 IDCT of the JPEG standard (A.3.3) evaluated separably in fp32
// with an even/odd split of the 8-point transform; colour is the JFIF YCbCr -> RGB matrix;
// chroma is replicated; one rounding at the very end (round half up, clamp to [0,255]).
#pragma once
#include "pcr_common.h"

namespace pcr {

// out[x] = sum_u a(u) in[u] cos((2x+1) u pi / 16), a(0) = 1/(2 sqrt 2), a(u>0) = 1/2
PCR_HD void idct8(const float in[8], float out[8]) {
    const float c1 = 0.98078528040323044913f, c2 = 0.92387953251128675613f, c3 = 0.83146961230254523708f,
                c4 = 0.70710678118654752440f, c5 = 0.55557023301960222474f, c6 = 0.38268343236508977173f,
                c7 = 0.19509032201612826785f;
    float s0 = 0.5f * c4 * in[0], s4 = 0.5f * c4 * in[4];
    float a = s0 + s4, b = s0 - s4;
    float h2 = 0.5f * in[2], h6 = 0.5f * in[6];
    float p = h2 * c2 + h6 * c6, q = h2 * c6 - h6 * c2;
    float e0 = a + p, e1 = b + q, e2 = b - q, e3 = a - p;
    float h1 = 0.5f * in[1], h3 = 0.5f * in[3], h5 = 0.5f * in[5], h7 = 0.5f * in[7];
    float o0 = h1 * c1 + h3 * c3 + h5 * c5 + h7 * c7;
    float o1 = h1 * c3 - h3 * c7 - h5 * c1 - h7 * c5;
    float o2 = h1 * c5 - h3 * c1 + h5 * c7 + h7 * c3;
    float o3 = h1 * c7 - h3 * c5 + h5 * c3 - h7 * c1;
    out[0] = e0 + o0; out[7] = e0 - o0;
    out[1] = e1 + o1; out[6] = e1 - o1;
    out[2] = e2 + o2; out[5] = e2 - o2;
    out[3] = e3 + o3; out[4] = e3 - o3;
}

// v (finite) clamped to [0, 255].  On the device the median of (v, 0, 255) is one instruction; written with compares it
// is four, and the pixel kernels clamp every sample.
PCR_HD float clamp255(float v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(v, 0.f, 255.f);
#else
    return v < 0.f ? 0.f : (v > 255.f ? 255.f : v);
#endif
}

PCR_HD uint8_t round_u8(float v) {
    v = __builtin_floorf(v + 0.5f);
    return (uint8_t)(v < 0.f ? 0.f : (v > 255.f ? 255.f : v));
}

PCR_HD void ycc_to_rgb(float Y, float Cb, float Cr, uint8_t* o) {
    Cb -= 128.f; Cr -= 128.f;
    o[0] = round_u8(Y + 1.402f * Cr);
    o[1] = round_u8(Y - 0.344136f * Cb - 0.714136f * Cr);
    o[2] = round_u8(Y + 1.772f * Cb);
}

}  // namespace pcr
