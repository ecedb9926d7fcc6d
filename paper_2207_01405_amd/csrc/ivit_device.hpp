// Device-side integer primitives shared by the gfx950 kernels.
//
// Everything here is exact integer arithmetic following I-ViT (arXiv 2207.01405):
// dyadic requantisation (Sec. 3.2, Eq. 8-10), ShiftExp and IntDiv (Sec. 3.3,
// Eq. 13-16, Algorithm 1), ShiftGELU (Sec. 3.4, Algorithm 2) and the fixed-count
// integer square root of I-LayerNorm (Sec. 3.5, Eq. 20).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ivit {

struct ShiftParams { int32_t i0, n_shift, m_bits, k_out; };
struct Dyadic { int32_t b, c; };

constexpr int kWave = 64;

__device__ __forceinline__ int32_t clamp8(int32_t v) { return min(max(v, -127), 127); }

// 64-bit minimum / maximum as a compare and a select (the min / max templates of the HIP headers, instantiated for
// int64_t, go through double precision).
__device__ __forceinline__ int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }
__device__ __forceinline__ int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

// (b v + rnd 2^(c-1)) >> c with the full 64-bit product; any 1 <= c <= 62.  rnd = 1: round(b v / 2^c) half up (Eq. 8
// realised as Eq. 10, the reading used throughout); rnd = 0: the bare shift of Eq. 10 as printed, floor(b v / 2^c).
__device__ __forceinline__ int64_t rnd_shift64(int32_t v, int32_t b, int32_t c, int32_t rnd = 1) {
    int64_t p = (int64_t)v * (int64_t)b;
    return (p + ((int64_t)rnd << (c - 1))) >> c;
}

__device__ __forceinline__ int32_t clamp8_64(int64_t v) {
    v = v < -127 ? -127 : v;
    v = v > 127 ? 127 : v;
    return (int32_t)v;
}

__device__ __forceinline__ int32_t requant64(int32_t v, int32_t b, int32_t c, int32_t rnd = 1) {
    return clamp8_64(rnd_shift64(v, b, c, rnd));
}

// round(b v / 2^c) when 1 <= c <= 31 and 1 <= b <= 2^c (a rescale by at most 1, so the result fits 32 bits):
// one 64-bit multiply-add, then the 32 result bits are cut out of the 64-bit value.
__device__ __forceinline__ bool dyadic_fits32(int32_t b, int32_t c) {
    return c >= 1 && c <= 31 && b >= 1 && (uint32_t)b <= (1u << c);
}
__device__ __forceinline__ int32_t rnd_shift_fit32(int32_t v, int32_t b, int32_t c, int32_t rnd = 1) {
    const int64_t p = (int64_t)v * b + (int64_t)((uint32_t)rnd << (c - 1));
    return (int32_t)__builtin_amdgcn_alignbit((uint32_t)(p >> 32), (uint32_t)p, c);
}

// floor(a / b) for b > 0 and any sign of a.
__device__ __forceinline__ int32_t floordiv(int32_t a, int32_t b) {
    int32_t q = a / b;
    return q - ((a % b != 0) && (a < 0));
}

// floor(v / x) for 1 <= x and v < 2^22: the quotient from a single-precision reciprocal is off by at most one,
// which one multiply and two compares repair (the general unsigned division does the same with more steps).  An
// implementation of integer division, not arithmetic of the method.
__device__ __forceinline__ uint32_t div_small(uint32_t v, uint32_t x) {
    uint32_t q = (uint32_t)((float)v * __builtin_amdgcn_rcpf((float)x));
    const int32_t r = (int32_t)(v - q * x);
    q += (r >= (int32_t)x);
    q -= (r < 0);
    return q;
}

// The same repair works whenever the QUOTIENT is small (below 2^18, say), whatever the size of v < 2^31: the estimate
// is then still within one of the quotient, and the remainder is formed exactly in 32 bits.
__device__ __forceinline__ uint32_t div_small_quotient(uint32_t v, uint32_t x) { return div_small(v, x); }

// floor(n / c) for c >= 1 and |n| < 2^22, through the unsigned form: floor(n / c) = -ceil(-n / c) for n < 0.
__device__ __forceinline__ int32_t floordiv_small(int32_t n, int32_t c) {
    const uint32_t a = n < 0 ? (uint32_t)(-n + c - 1) : (uint32_t)n;
    const int32_t q = (int32_t)div_small(a, (uint32_t)c);
    return n < 0 ? -q : q;
}

// ShiftExp (Sec. 3.3, Eq. 13-15, Algorithm 1) of an argument I <= 0: the value E with (S / 2^N) E ~ exp(S I).
// t = -(I + (I >> 1) - (I >> 4)) >= 0 is the magnitude of I log2(e) in units of S; it splits as t = q I_0 + r with
// 0 <= r < I_0: q whole powers of two to shift out, and the fraction -r / I_0, whose power of two is taken as
// 1 - r / (2 I_0), i.e. the integer I_0 - ceil(r / 2).  The left pre-shift N comes first so that q > N shifts the
// value out instead of asking for a negative shift count.
__device__ __forceinline__ uint32_t shiftexp(int32_t I, int32_t i0, int32_t n_shift) {
    const uint32_t t = (uint32_t)(-(I + (I >> 1) - (I >> 4)));
    const uint32_t q = t < (1u << 22) ? div_small(t, (uint32_t)i0) : t / (uint32_t)i0;
    const uint32_t r = t - q * (uint32_t)i0;
    return q > 31 ? 0u : ((((uint32_t)i0 - ((r + 1) >> 1)) << n_shift) >> q);
}

// IntDiv (Eq. 16) with the reciprocal floor(2^M / sum) already formed; M <= 31 and e <= sum, so the
// product is at most 2^31 and fits 32 unsigned bits.
__device__ __forceinline__ uint32_t intdiv_apply(uint32_t inv, uint32_t e, int32_t m_bits, int32_t k_out) {
    return (inv * e) >> (m_bits - (k_out - 1));
}

__device__ __forceinline__ uint32_t recip_pow2(uint32_t sum, int32_t m_bits) {
    return (1u << m_bits) / sum;              // m_bits <= 31
}

// The same value for 2^9 <= sum < 2^24 (a row sum of ShiftExp values: the maximum's term alone is I_0 << N): the
// quotient is below 2^23, a single-precision estimate of it is off by at most one, and the remainder
// 2^M - q sum, exact in 32-bit wrap-around arithmetic, repairs it.  Other sums take the general division.
__device__ __forceinline__ uint32_t recip_pow2_small(uint32_t sum, int32_t m_bits) {
    if (sum < (1u << 9) || sum >= (1u << 24)) return (1u << m_bits) / sum;
    const uint32_t num = 1u << m_bits;
    uint32_t q = (uint32_t)((float)num * __builtin_amdgcn_rcpf((float)sum));
    const int32_t r = (int32_t)(num - q * sum);
    q += (r >= (int32_t)sum);
    q -= (r < 0);
    return q;
}

// ShiftGELU on one int8 value (Sec. 3.4, Eq. 17-18, Algorithm 2), the maximum of the algorithm taken per element:
// x sigmoid(1.702 x) with the sigmoid as a ratio of two exponentials whose arguments are both <= 0.  With
// t = I + (I >> 1) + (I >> 3) + (I >> 4) (1.702 I in integers) these are min(t, 0) and min(-t, 0); IntDiv (Eq. 16) turns
// their ratio into k_out - 1 fraction bits.  Returns I * I_div, |result| <= 127 * 2^(k_out-1).
__device__ __forceinline__ int32_t shiftgelu_raw(int32_t I, ShiftParams p) {
    const int32_t t = I + (I >> 1) + (I >> 3) + (I >> 4);
    const uint32_t e_num = shiftexp(min(t, 0), p.i0, p.n_shift);
    const uint32_t e_one = shiftexp(min(-t, 0), p.i0, p.n_shift);
    return I * (int32_t)intdiv_apply(recip_pow2(e_num + e_one, p.m_bits), e_num, p.m_bits, p.k_out);
}

// Low 32 bits of the product of the low 24 bits of a and b, as the one full-rate instruction.  Written out because the
// compiler falls back to the quarter-rate 32-bit multiply when an operand's range was established in another block.
// (The compiler inserts no wait states for what an asm statement reads: the operands must come from ordinary vector
// instructions or loads, not directly from a dot-product, matrix or transcendental instruction.)
__device__ __forceinline__ uint32_t mul_u24(uint32_t a, uint32_t b) {
    uint32_t r;
    asm("v_mul_u32_u24 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// The same for signed factors: low 32 bits of the product of the sign-extended low 24 bits of a and b.
__device__ __forceinline__ int32_t mul_i24(int32_t a, int32_t b) {
    int32_t r;
    asm("v_mul_i32_i24 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Tenth iterate of I <- (I + floor(v / I)) >> 1 from I = 2^floor(bitlen(v) / 2) (Eq. 20); 0 for v = 0.
constexpr uint32_t isqrt10_steps(uint32_t v) {
    if (v == 0) return 0;
    uint32_t bits = 0;
    for (uint32_t t = v; t; t >>= 1) ++bits;
    uint32_t x = 1u << (bits >> 1);
    for (int it = 0; it < 10; ++it) x = (x + v / x) >> 1;
    return x;
}
// The iteration settles on floor(sqrt v) long before the tenth step (from that start, for v < 2^32), unless v + 1 is
// a square, v = m^2 - 1: there it alternates between m - 1 and m for ever, and which of the two the tenth iterate is
// depends on how many steps it took to get there.  For the variances of int8 rows (v <= 255^2) the answer per m is this
// table, bit m of it set when the tenth iterate of m^2 - 1 is m; the compiler evaluates the iteration itself to fill it.
struct Isqrt10Table {
    uint32_t w[8];
    constexpr Isqrt10Table() : w{} {
        for (uint32_t m = 2; m < 256; ++m)
            if (isqrt10_steps(m * m - 1) == m) w[m >> 5] |= 1u << (m & 31);
    }
};
__device__ __forceinline__ uint32_t isqrt10(uint32_t v) {
    if (v > 255u * 255u) {                                      // (beyond what an int8 row can give: the iteration as it stands)
        uint32_t x = 1u << ((32 - __clz(v)) >> 1);
#pragma unroll 1
        for (int it = 0; it < 10; ++it) {
            const uint32_t xn = (x + v / x) >> 1;               // x stays >= 1 for v >= 1
            if (xn == x) break;                                 // a fixed point: every later iterate equals it
            x = xn;
        }
        return x;
    }
    // v <= 255^2: floor(sqrt v) from the single-precision square root (exact to within one for such v), repaired
    constexpr Isqrt10Table T{};
    uint32_t s = (uint32_t)__builtin_sqrtf((float)v);
    s -= (s * s > v);
    s += ((s + 1) * (s + 1) <= v);
    const uint32_t m = s + 1;                                   // v == m^2 - 1 <=> v == s^2 + 2 s
    const bool osc = (v == s * s + 2 * s) & (s >= 1);
    const uint32_t bit = (T.w[m >> 5 & 7] >> (m & 31)) & 1u;
    return osc ? s + bit : s;
}

// Reductions over the 64 lanes of a wavefront; every lane gets the result.  Inside each row of 16 lanes four DPP
// exchanges (lane pairs, quad pairs, half-row mirror, row mirror: all of them read existing lanes, so "bound_ctrl with
// old = 0" only serves to let the compiler fold the move into the operation); the four row results are then combined
// through scalar registers.  To be called where all 64 lanes are active (an inactive source lane would read as 0).
template <int CTRL>
__device__ __forceinline__ int32_t dpp_i32(int32_t v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ int32_t wave_max(int32_t v) {
    v = max(v, dpp_i32<0xB1>(v));
    v = max(v, dpp_i32<0x4E>(v));
    v = max(v, dpp_i32<0x141>(v));
    v = max(v, dpp_i32<0x140>(v));
    return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
__device__ __forceinline__ int32_t wave_sum(int32_t v) {
    v += dpp_i32<0xB1>(v);
    v += dpp_i32<0x4E>(v);
    v += dpp_i32<0x141>(v);
    v += dpp_i32<0x140>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

// All-reduce over the four rows of 16 lanes of a wavefront (lanes l, l + 16, l + 32, l + 48), every lane getting the
// result, without a trip through LDS: v_permlane16_swap exchanges the odd rows of its first operand with the even rows
// of its second, v_permlane32_swap the upper half of the first with the lower half of the second; given two copies of
// v, each leaves a lane's own value and its partner's side by side.
template <class OP>
__device__ __forceinline__ int32_t rows_allreduce(int32_t v, OP op) {
    const auto a = __builtin_amdgcn_permlane16_swap((uint32_t)v, (uint32_t)v, false, false);
    v = op((int32_t)a[0], (int32_t)a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap((uint32_t)v, (uint32_t)v, false, false);
    return op((int32_t)b[0], (int32_t)b[1]);
}

}  // namespace ivit
