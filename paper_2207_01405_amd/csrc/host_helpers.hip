// Host-side helpers of the C ABI: float parameters of a quantised model -> integers (I-ViT, arXiv 2207.01405:
// Sec. 3.1 Eq. 6, the dyadic number of Sec. 3.2, I_0 of Algorithm 1).  No device code in this file.
#include <algorithm>
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

// Token-index table of (shifted-)window attention on a g x g token grid kept in raster order: the image is shifted
// cyclically by -shift along both axes and cut into window x window windows in raster order; entry [w][t] is the raster
// position, in the unshifted image, of token t (raster order inside the window) of window w.
int ivit_swin_window_index(int32_t g, int32_t window, int32_t shift, int32_t* index) {
    if (g < 1 || window < 1 || g % window != 0 || g > 4096) return IVIT_ERR_SHAPE;
    if (shift < 0 || shift >= window) return IVIT_ERR_PARAM;
    if (!index) return IVIT_ERR_NULL;
    const int n = g / window, T = window * window;
    for (int wy = 0; wy < n; ++wy)
        for (int wx = 0; wx < n; ++wx)
            for (int iy = 0; iy < window; ++iy)
                for (int ix = 0; ix < window; ++ix) {
                    const int sy = (wy * window + iy + shift) % g, sx = (wx * window + ix + shift) % g;
                    index[(wy * n + wx) * T + iy * window + ix] = sy * g + sx;
                }
    return IVIT_OK;
}

// Mask of shifted-window attention for the same layout: along each axis a position p of the shifted image lies in one of
// three bands (p < g - window: windows the shift did not split; p < g - shift: the part of the last window that did not
// wrap; else the part that wrapped around); two tokens of a window are masked (1) when their bands differ on either axis.
int ivit_swin_shift_mask(int32_t g, int32_t window, int32_t shift, int8_t* mask) {
    if (g < 1 || window < 1 || g % window != 0 || g > 4096) return IVIT_ERR_SHAPE;
    if (shift < 0 || shift >= window) return IVIT_ERR_PARAM;
    if (!mask) return IVIT_ERR_NULL;
    const int n = g / window, T = window * window;
    auto band = [&](int p) { return p < g - window ? 0 : (p < g - shift ? 1 : 2); };
    for (int wy = 0; wy < n; ++wy)
        for (int wx = 0; wx < n; ++wx) {
            int8_t* m = mask + (int64_t)(wy * n + wx) * T * T;
            for (int i = 0; i < T; ++i)
                for (int j = 0; j < T; ++j) {
                    const int yi = wy * window + i / window, xi = wx * window + i % window;
                    const int yj = wy * window + j / window, xj = wx * window + j % window;
                    m[i * T + j] = (band(yi) != band(yj) || band(xi) != band(xj)) ? 1 : 0;
                }
        }
    return IVIT_OK;
}

int ivit_ilayernorm_limits(int32_t C, int32_t f_bits, int32_t c_shift, int32_t* gamma_max, int32_t* beta_max) {
    if (C < 4 || C > 2048 || (C & 3)) return IVIT_ERR_SHAPE;
    if (f_bits < 1 || f_bits > 20 || c_shift < 1 || c_shift > 31) return IVIT_ERR_PARAM;
    if (!gamma_max || !beta_max) return IVIT_ERR_NULL;
    // |x - mean| f <= 2 sqrt(C) 2^F for every row: sum (x - mean)^2 < C (var + 1), std >= max(1, floor(sqrt(var))),
    // whose ratio peaks at var = 3, and f <= 2^F / std.  s = ceil(sqrt(4 C)).
    int64_t s = (int64_t)std::sqrt(4.0 * C);
    while (s * s < 4LL * C) ++s;
    while ((s - 1) * (s - 1) >= 4LL * C) --s;
    const int64_t U = s << f_bits;
    const int64_t half = 1LL << (c_shift - 1);
    const int64_t bmax = std::min<int64_t>(1LL << 30, (1LL << 31) - 1 - half);
    const int64_t room = (1LL << 31) - 1 - bmax - half;
    int64_t g = room > 0 ? room / U : 0;
    if (g > (1 << 15) - 1) g = (1 << 15) - 1;              // the first product is a 24-bit multiply: 255 |gamma| < 2^23
    *gamma_max = (int32_t)g;
    *beta_max = (int32_t)bmax;
    return IVIT_OK;
}

}  // extern "C"
