// Host-side helpers of the C ABI: float parameters of a quantised model -> integers (I-ViT, arXiv 2207.01405:
// Sec. 3.1 Eq. 6, the dyadic number of Sec. 3.2, I_0 of Algorithm 1).  No device code in this file.
#include <cmath>
#include <cstdint>

#include "../../include/ivit.h"

namespace {
inline int bitlen(uint32_t v) { int n = 0; while (v) { ++n; v >>= 1; } return n; }
}  // namespace

extern "C" {

int ivit_quantize_symmetric(const float* r, int64_t n, float m, int32_t k, int8_t* q, float* scale) {
    if (n < 0) return IVIT_ERR_SHAPE;
    if (!(m > 0.0f) || !std::isfinite(m) || k < 2 || k > 8) return IVIT_ERR_PARAM;
    if (n > 0 && (!r || !q)) return IVIT_ERR_NULL;
    const int32_t qmax = (1 << (k - 1)) - 1;
    const double S = (double)m / (double)qmax;
    if (scale) *scale = (float)S;
    for (int64_t i = 0; i < n; ++i) {
        const double t = (double)r[i] / S;
        double v = std::round(t);                      // nearest, ties away from zero
        if (!(v == v)) v = 0.0;
        v = v < -qmax ? -qmax : (v > qmax ? qmax : v);
        q[i] = (int8_t)v;
    }
    return IVIT_OK;
}

int ivit_dyadic_from_float(double x, int32_t bits, ivit_dyadic* out) {
    if (!out) return IVIT_ERR_NULL;
    if (!(x > 0.0) || !std::isfinite(x) || bits < 2 || bits > 31) return IVIT_ERR_PARAM;
    int e;
    std::frexp(x, &e);                                 // x = f 2^e, 0.5 <= f < 1: floor(log2 x) = e - 1
    int c = bits - e;                                  // bits - 1 - floor(log2 x)
    if (c > 46) c = 46;
    if (c < 1) c = 1;
    double b = std::round(std::ldexp(x, c));
    if (b >= std::ldexp(1.0, bits) && c > 1) { --c; b = std::round(std::ldexp(x, c)); }   // rounding carried into bit `bits`
    if (b > 2147483647.0) return IVIT_ERR_PARAM;
    if (b < 1.0) b = 1.0;
    out->b = (int32_t)b;
    out->c = c;
    return IVIT_OK;
}

int ivit_shift_params_from_scale(double s, int32_t width, int32_t m_bits, int32_t k_out, ivit_shift_params* out) {
    if (!out) return IVIT_ERR_NULL;
    if (!(s > 0.0) || !std::isfinite(s) || width < 2 || width > 16) return IVIT_ERR_PARAM;
    if (k_out < 2 || k_out > 8 || m_bits < k_out - 1 || m_bits > 31) return IVIT_ERR_PARAM;
    double i0d = std::round(1.0 / s);
    if (i0d < 1.0) i0d = 1.0;
    if (i0d >= std::ldexp(1.0, width)) return IVIT_ERR_PARAM;
    const int32_t i0 = (int32_t)i0d;
    out->i0 = i0;
    out->n_shift = width - bitlen((uint32_t)i0);
    out->m_bits = m_bits;
    out->k_out = k_out;
    return IVIT_OK;
}

}  // extern "C"
