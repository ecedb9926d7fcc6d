// Row-wise integer operators for gfx950: I-LayerNorm (Sec. 3.5, Eq. 19-20), Shiftmax (Sec. 3.3,
// Algorithm 1) and ShiftGELU (Sec. 3.4, Algorithm 2) of I-ViT (arXiv 2207.01405).
//
// All three are bound by HBM traffic (one int8 read and one int8 write per element), so the kernels
// are organised around coalesced dword / 16-byte accesses and wavefront-wide reductions; the scalar
// per-row work (integer mean, variance, the ten-step square root, the two reciprocals) is done once per row.
#include <algorithm>

#include "ivit_kernels.hpp"

namespace ivit {

int num_cus() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            return 256;
    }
    return n;
}

// ------------------------------------------------------------------------------------------------
// I-LayerNorm.  One wavefront per row; lane l owns dwords l, l + 64, ... of the row (4 channels each),
// so gamma / beta for those channels stay in registers across all rows the wave processes.
// The sum of squared deviations uses the exact integer identity
//   sum (x - m)^2 = sum x^2 - 2 m sum x + C m^2,
// which lets both sums come from one pass with 4-way int8 dot products.
template <int NT>
__global__ __launch_bounds__(256) void ilayernorm_kernel(const int8_t* __restrict__ x,
                                                         const int32_t* __restrict__ gamma_q,
                                                         const int32_t* __restrict__ beta_q,
                                                         int8_t* __restrict__ y, int64_t rows, int C,
                                                         int f_bits, int c_shift) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int ndw = C >> 2;
    const int32_t half = 1 << (c_shift - 1);

    int32_t g[NT][4], bt[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int idx = lane + 64 * t;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            g[t][e] = idx < ndw ? gamma_q[4 * idx + e] : 0;
            bt[t][e] = idx < ndw ? (int32_t)((uint32_t)beta_q[4 * idx + e] + (uint32_t)half) : 0;
        }
    }

    for (int64_t row = wave; row < rows; row += nwaves) {
        const uint32_t* xr = reinterpret_cast<const uint32_t*>(x + row * C);
        uint32_t xv[NT];
        int32_t s = 0, ss = 0;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int idx = lane + 64 * t;
            xv[t] = idx < ndw ? xr[idx] : 0u;
            s = __builtin_amdgcn_sdot4((int)xv[t], 0x01010101, s, false);
            ss = __builtin_amdgcn_sdot4((int)xv[t], (int)xv[t], ss, false);
        }
        s = wave_sum(s);
        ss = wave_sum(ss);
        const int32_t mean = floordiv(s + (C >> 1), C);
        const int32_t sq = ss - 2 * mean * s + C * mean * mean;      // sum of squared deviations, >= 0
        const uint32_t var = (uint32_t)sq / (uint32_t)C;
        const uint32_t sd = max(isqrt10(var), 1u);
        const int32_t f = (int32_t)((1u << f_bits) / sd);
        uint32_t* yr = reinterpret_cast<uint32_t*>(y + row * C);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int idx = lane + 64 * t;
            uint32_t out = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t xe = (int32_t)(int8_t)(xv[t] >> (8 * e));
                const int32_t dg = mul_i24(xe - mean, g[t][e]);                   // |.| < 2^23: 24-bit factors, see below
                const int32_t v = __mul24(dg, f) + bt[t][e];
                out |= ((uint32_t)clamp8(v >> c_shift) & 0xffu) << (8 * e);
            }
            if (idx < ndw) yr[idx] = out;
        }
    }
}

// I-LayerNorm, tiled form for C a multiple of 16 with 64 <= C <= GBN (1024, or 2048 for the few wide rows of patch merging).  A workgroup takes R = RP * J
// consecutive rows, where CPR = C / 16 threads cover one row with 16 bytes each and RP = 256 / CPR rows are
// covered per pass.  Thread (rgrp, cc) keeps chunk cc of rows rgrp, rgrp + RP, ... in registers, so gamma / beta
// of its 16 channels are loaded once.  The per-row scalar work (integer mean, variance, ten-step square
// root, reciprocal) would idle 63 of 64 lanes if done per wavefront, so the 4-way dot-product partial sums
// go through LDS and every thread then does the scalar work of a DIFFERENT row.
template <int J, int GBN = 1024>
__global__ __launch_bounds__(256) void ilayernorm_tiled_kernel(const int8_t* __restrict__ x,
                                                               const int32_t* __restrict__ gamma_q,
                                                               const int32_t* __restrict__ beta_q,
                                                               int8_t* __restrict__ y, int64_t rows, int C,
                                                               int f_bits, int c_shift) {
    typedef int v4i __attribute__((ext_vector_type(4)));
    // (sum x, sum x^2) of one 16-byte chunk, laid out [pass][chunk][row of the pass] so that the threads that add up
    // the rows (consecutive rows, the same chunk at a time) read consecutive words: no bank conflicts there
    __shared__ int2 part[J * 256];
    __shared__ int2 stat[J * 64];                  // [row in workgroup]: (mean, f)
    const int tid = threadIdx.x;
    const int CPR = C >> 4, RP = 256 / CPR, R = RP * J;
    const bool active = tid < RP * CPR;
    const int rgrp = tid / CPR, cc = tid - rgrp * CPR;
    const int64_t row0 = (int64_t)blockIdx.x * R;
    const int32_t half = 1 << (c_shift - 1);

    v4i xv[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int64_t row = row0 + j * RP + rgrp;
        xv[j] = v4i{0, 0, 0, 0};
        if (active && row < rows) xv[j] = *reinterpret_cast<const v4i*>(x + row * C + 16 * cc);
    }
    // gamma and beta + 2^(c-1) go through LDS: read once per workgroup with coalesced loads instead of 128 bytes per
    // thread; each thread picks up its 16 channels after the first barrier
    // (the 16 channels of a chunk are 20 words apart, so that the threads of a row, which read theirs at the same
    // time, meet no bank twice)
    constexpr int GBP = GBN / 16 * 20;
    __shared__ __align__(16) int32_t gb[2 * GBP];
    for (int i = tid; i < C; i += 256) {
        gb[(i >> 4) * 20 + (i & 15)] = gamma_q[i];
        gb[GBP + (i >> 4) * 20 + (i & 15)] = (int32_t)((uint32_t)beta_q[i] + (uint32_t)half);
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
        int32_t s = 0, ss = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            s = __builtin_amdgcn_sdot4(xv[j][d], 0x01010101, s, false);
            ss = __builtin_amdgcn_sdot4(xv[j][d], xv[j][d], ss, false);
        }
        if (active) part[j * 256 + cc * RP + rgrp] = make_int2(s, ss);
    }
    __syncthreads();
    for (int r = tid; r < R; r += 256) {           // one row per thread: r = j * RP + rgrp
        const int j = r / RP, rg = r - j * RP;
        const int2* p = &part[j * 256 + rg];
        int32_t s = 0, ss = 0;
        for (int c = 0; c < CPR; ++c) { s += p[c * RP].x; ss += p[c * RP].y; }
        // (|sum x| <= 128 C < 2^19, the variance is at most 255^2 and f at most 2^20: the three divisions are of the
        // kind one reciprocal and a repair step settle)
        const int32_t mean = floordiv_small(s + (C >> 1), C);
        const int32_t sq = ss - 2 * mean * s + C * mean * mean;      // sum of squared deviations (exact)
        const uint32_t var = div_small_quotient((uint32_t)sq, (uint32_t)C);
        const uint32_t sd = max(isqrt10(var), 1u);
        stat[r] = make_int2(mean, (int32_t)div_small(1u << f_bits, sd));
    }
    __syncthreads();
    int32_t g[16], bt[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const v4i gv = *reinterpret_cast<const v4i*>(&gb[(active ? 20 * cc : 0) + 4 * q]);
        const v4i bv = *reinterpret_cast<const v4i*>(&gb[GBP + (active ? 20 * cc : 0) + 4 * q]);
#pragma unroll
        for (int e = 0; e < 4; ++e) { g[4 * q + e] = gv[e]; bt[4 * q + e] = bv[e]; }
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int64_t row = row0 + j * RP + rgrp;
        const int2 mf = stat[j * RP + rgrp];
        uint32_t outw[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t o = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t xe = (int32_t)(int8_t)((uint32_t)xv[j][d] >> (8 * e));
                // |x - mean| <= 255, |gamma_q| < 2^15 and f <= 2^20: both products have 24-bit factors, so the
                // full-rate 24-bit multiply (low 32 bits of the product) gives what the 32-bit one would
                const int32_t dg = mul_i24(xe - mf.x, g[4 * d + e]);                 // |.| < 2^23
                const int32_t v = __mul24(dg, mf.y) + bt[4 * d + e];
                o |= ((uint32_t)clamp8(v >> c_shift) & 0xffu) << (8 * e);
            }
            outw[d] = o;
        }
        if (active && row < rows)
            *reinterpret_cast<uint4*>(y + row * C + 16 * cc) = make_uint4(outw[0], outw[1], outw[2], outw[3]);
    }
}

hipError_t launch_ilayernorm(hipStream_t s, const int8_t* x, const int32_t* gamma_q, const int32_t* beta_q,
                             int8_t* y, int64_t rows, int C, int f_bits, int c_shift) {
    if (rows == 0) return hipSuccess;
    if ((C & 15) == 0 && C >= 64 && C <= 2048 && (((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma_q | (uintptr_t)beta_q) & 15) == 0) {
        // rows per workgroup = (256 / (C / 16)) * J
        const int rp = 256 / (C >> 4);
        // the smallest J whose workgroups are all resident at once (8 per CU): one round of the three dependent phases
        const int64_t resident = (int64_t)num_cus() * 8;
        int J = 1;
        while (J < 8 && (rows + rp * J - 1) / (rp * J) > resident) J <<= 1;
        while (J > 1 && rp * J > 256) J >>= 1;       // at most one row of scalar work per thread (narrow rows: C < 128)
        const int64_t grid = (rows + rp * J - 1) / (rp * J);
        if (grid <= 0x7fffffffLL) {
            TraceScope trace(s, KIND_ILAYERNORM, 0, 2 * rows * C + 8LL * C);
            const dim3 g((unsigned)grid), b(256);
            if (C > 1024) {
                switch (J) {
                    case 8: hipLaunchKernelGGL((ilayernorm_tiled_kernel<8, 2048>), g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                    case 4: hipLaunchKernelGGL((ilayernorm_tiled_kernel<4, 2048>), g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                    case 2: hipLaunchKernelGGL((ilayernorm_tiled_kernel<2, 2048>), g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                    default: hipLaunchKernelGGL((ilayernorm_tiled_kernel<1, 2048>), g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                }
                return hipGetLastError();
            }
            switch (J) {
                case 8: hipLaunchKernelGGL(ilayernorm_tiled_kernel<8>, g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                case 4: hipLaunchKernelGGL(ilayernorm_tiled_kernel<4>, g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                case 2: hipLaunchKernelGGL(ilayernorm_tiled_kernel<2>, g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
                default: hipLaunchKernelGGL(ilayernorm_tiled_kernel<1>, g, b, 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
            }
            return hipGetLastError();
        }
    }
    const int64_t want = (rows + 3) / 4;
    const int grid = (int)std::min<int64_t>(want, (int64_t)num_cus() * 16);
    const int nt = (C / 4 + 63) / 64;
    TraceScope trace(s, KIND_ILAYERNORM, 0, 2 * rows * C + 8LL * C);
    switch (nt) {
        case 1: hipLaunchKernelGGL(ilayernorm_kernel<1>, dim3(grid), dim3(256), 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
        case 2: hipLaunchKernelGGL(ilayernorm_kernel<2>, dim3(grid), dim3(256), 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
        case 3: hipLaunchKernelGGL(ilayernorm_kernel<3>, dim3(grid), dim3(256), 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
        case 4: hipLaunchKernelGGL(ilayernorm_kernel<4>, dim3(grid), dim3(256), 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
        case 5: case 6: hipLaunchKernelGGL(ilayernorm_kernel<6>, dim3(grid), dim3(256), 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;
        default: hipLaunchKernelGGL(ilayernorm_kernel<8>, dim3(grid), dim3(256), 0, s, x, gamma_q, beta_q, y, rows, C, f_bits, c_shift); break;   // C <= 2048
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Shiftmax.  One wavefront per row, lane l owns columns l, l + 64, ...  ShiftExp only ever sees
// Delta = value - max in [-508, 0] (int8 input plus int8 bias), so each workgroup tabulates it once in LDS.
template <int NT>
__global__ __launch_bounds__(256) void shiftmax_kernel(const int8_t* __restrict__ x, const int8_t* __restrict__ bias,
                                                       int H, int T, int8_t* __restrict__ y, int64_t rows,
                                                       int cols, int ld, ShiftParams p) {
    __shared__ uint16_t lut[512];
    for (int i = threadIdx.x; i < 512; i += 256) lut[i] = (uint16_t)shiftexp(-i, p.i0, p.n_shift);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int sh = p.m_bits - (p.k_out - 1);
    const uint32_t top = (1u << (p.k_out - 1)) - 1u;
    for (int64_t row = wave; row < rows; row += nwaves) {
        const int8_t* xr = x + row * ld;
        const int8_t* br = bias ? bias + (((row / T) % H) * (int64_t)T + (row % T)) * cols : nullptr;
        int32_t v[NT];
        int32_t mx = INT32_MIN;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int j = lane + 64 * t;
            v[t] = INT32_MIN;
            if (j < cols) {
                v[t] = xr[j];
                if (br) v[t] += br[j];
                mx = max(mx, v[t]);
            }
        }
        mx = wave_max(mx);
        uint32_t e[NT];
        int32_t sum = 0;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int j = lane + 64 * t;
            e[t] = j < cols ? lut[mx - v[t]] : 0u;
            sum += (int32_t)e[t];
        }
        sum = wave_sum(sum);
        const uint32_t inv = (1u << p.m_bits) / (uint32_t)sum;
        int8_t* yr = y + row * cols;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int j = lane + 64 * t;
            if (j < cols) yr[j] = (int8_t)min((inv * e[t]) >> sh, top);
        }
    }
}

// Shiftmax without bias for 16 <= cols <= 16 * LPR: LPR (4, 8 or 16) adjacent lanes share a row and every lane owns
// 16 consecutive bytes of it, read and written as one 16-byte access at byte granularity (rows need no alignment).
// The last lane of a row is moved back so that it ends at the row's end; the bytes it has in common with its
// neighbour give the same results and only have to be left out of the row sum.  All arithmetic on the 16 bytes is
// done on packed words: with the sign bits flipped the bytes order as unsigned numbers, the maximum is taken on
// 16-bit pairs, and max - value needs no borrow between bytes, so one subtraction yields four table indices.
// Reductions over the LPR lanes are DPP permutations (quad exchange, then mirrored halves of 8 and 16 lanes).
typedef uint32_t u32x4_unaligned __attribute__((ext_vector_type(4), aligned(1)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v) {
    // every pattern used below reads an existing lane, so "old = 0, bound_ctrl" changes nothing except that the compiler
    // can then fold the move into the max / add that consumes it
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int LPR, class OP>
__device__ __forceinline__ uint32_t group_allreduce(uint32_t v, OP op) {
    v = op(v, dpp<0xB1>(v));                         // quad_perm [1,0,3,2]
    v = op(v, dpp<0x4E>(v));                         // quad_perm [2,3,0,1]
    if (LPR >= 8) v = op(v, dpp<0x141>(v));          // row_half_mirror: quads 0 <-> 1, 2 <-> 3
    if (LPR >= 16) v = op(v, dpp<0x140>(v));         // row_mirror: halves of the 16 lanes
    return v;
}

// DUP: the number of leading bytes of a row's last lane that belong to its neighbour, 16 ceil(cols / 16) - cols,
// when it is one of the instantiated values (0; 11 for 197 columns; 15 for 49 and 65), else -1 = taken at run time.
template <int LPR, int UNR, int FAST, int DUP>
__global__ __launch_bounds__(256) void shiftmax_vec_kernel(const int8_t* __restrict__ x, int8_t* __restrict__ y,
                                                           int64_t rows, int cols, int ld, ShiftParams p) {
    __shared__ uint16_t lut[256];                    // ShiftExp(-delta), delta = max - value in [0, 255]
    lut[threadIdx.x] = (uint16_t)shiftexp(-(int)threadIdx.x, p.i0, p.n_shift);
    __syncthreads();
    const int j = threadIdx.x % LPR;                 // lane within the row
    const int nl = (cols + 15) >> 4;                 // lanes of a row that own bytes
    const int off = min(16 * j, cols - 16);          // lanes past the end repeat the last one and store nothing
    const bool owner = j < nl;
    const bool last = j == nl - 1;
    const int dup = DUP >= 0 ? DUP : 16 * (nl - 1) - (cols - 16);   // leading bytes of the last lane that its neighbour owns
    const int sh = p.m_bits - (p.k_out - 1);
    constexpr int RPP = 256 / LPR;                   // rows the workgroup covers per pass
    const int rl = threadIdx.x / LPR;                // this thread's row within a pass
    auto umax = [](uint32_t a, uint32_t b) { return max(a, b); };
    auto uadd = [](uint32_t a, uint32_t b) { return a + b; };
    // A workgroup takes UNR RPP consecutive rows per step, all of its UNR loads requested before the first is used.  The
    // grid has one workgroup per step, so the workgroups in flight sweep memory as one compact window (measured on
    // 1 GiB of 197-byte rows: 5.2 TB/s, against 4.8 TB/s for 32 persistent workgroups per compute unit striding over
    // the rows, and 4.5 TB/s with non-temporal accesses on top of that).  The row offset of a step is a uniform 64-bit
    // product plus this thread's constant part: no per-thread 64-bit multiplies.
    const int64_t xlast = (rows - 1) * ld + off, xt = (int64_t)rl * ld + off, yt = (int64_t)rl * cols + off;
    for (int64_t f0 = (int64_t)blockIdx.x * (UNR * RPP); f0 < rows; f0 += (int64_t)gridDim.x * (UNR * RPP)) {
        u32x4_unaligned in[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t r = f0 + u * RPP + rl;                       // a slot past the end repeats the last row
            in[u] = *reinterpret_cast<const u32x4_unaligned*>(x + (r < rows ? (f0 + u * RPP) * ld + xt : xlast));
        }
        const int64_t yo = f0 * cols + yt, ys = (int64_t)RPP * cols;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t r = f0 + u * RPP + rl;
            uint32_t xf[4];
            u16x2 m2 = {0, 0};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                xf[d] = in[u][d] ^ 0x80808080u;
                const uint32_t lo = xf[d] & 0x00ff00ffu, hi = (xf[d] >> 8) & 0x00ff00ffu;
                m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(u16x2, lo));
                m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(u16x2, hi));
            }
            const uint32_t mx = group_allreduce<LPR>(max((uint32_t)m2[0], (uint32_t)m2[1]), umax);
            const uint32_t mrep = __builtin_amdgcn_perm(mx, mx, 0u);  // the maximum (< 256) in all four bytes
            uint32_t e[16];
            uint32_t full = 0, tail = 0;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const uint32_t delta = mrep - xf[k >> 2];                // bytewise, no borrows: every byte <= max
                e[k] = lut[(delta >> (8 * (k & 3))) & 0xffu];
                full += e[k];
                if (k >= dup) tail += e[k];                              // known at compile time when DUP >= 0
            }
            const uint32_t mine = owner ? (last ? tail : full) : 0u;
            const uint32_t sum = group_allreduce<LPR>(mine, uadd);
            const uint32_t inv = recip_pow2_small(sum, p.m_bits);
            uint32_t out[4];
            const uint32_t invs = FAST ? inv << (32 - sh) : inv;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t w = 0;
                if (FAST == 2) {
                    // M - (k_out - 1) = 24: inv < 2^24, e < 2^16 and inv e <= 2^31, so the quotient is the top byte of one
                    // 24-bit multiply
                    uint32_t pr[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) pr[b] = mul_u24(inv, e[4 * d + b]);
                    w = __builtin_amdgcn_perm(pr[1], pr[0], 0x0c0c0703u) | __builtin_amdgcn_perm(pr[3], pr[2], 0x07030c0cu);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const uint32_t ek = e[4 * d + b];
                        const uint32_t q = FAST ? __umulhi(invs, ek) : (inv * ek) >> sh;
                        w |= q << (8 * b);                               // q <= 2^(k_out-1) fits a byte
                    }
                }
                out[d] = w - ((w >> (p.k_out - 1)) & 0x01010101u);       // bytewise min(q, 2^(k_out-1) - 1)
            }
            if (owner && r < rows) {
                u32x4_unaligned o = {out[0], out[1], out[2], out[3]};
                *reinterpret_cast<u32x4_unaligned*>(y + yo + u * ys) = o;
            }
        }
    }
}

template <int LPR>
static void launch_shiftmax_vec(hipStream_t s, const int8_t* x, int8_t* y, int64_t rows, int cols, int ld, ShiftParams p) {
    constexpr int UNR = 4;
    const int64_t per_wg = (256 / LPR) * UNR;
    const int grid = (int)std::min<int64_t>((rows + per_wg - 1) / per_wg, 0x7fffffffLL);
    // inv << (32 - sh) must fit 32 bits: inv <= 2^M / (I_0 << N) < 2^sh needs I_0 << N > 2^(k_out - 1); sh >= 1
    const int sh = p.m_bits - (p.k_out - 1);
    const bool fast = sh >= 1 && ((int64_t)p.i0 << p.n_shift) > ((int64_t)1 << (p.k_out - 1));
    const int dup = 16 * ((cols + 15) / 16) - cols;
    const dim3 g(grid), b(256);
#define IVIT_SM(FAST_, DUP_) hipLaunchKernelGGL((shiftmax_vec_kernel<LPR, UNR, FAST_, DUP_>), g, b, 0, s, x, y, rows, cols, ld, p)
    if (fast && sh == 24) {
        if (dup == 0) IVIT_SM(2, 0); else if (dup == 11) IVIT_SM(2, 11); else if (dup == 15) IVIT_SM(2, 15); else IVIT_SM(2, -1);
    } else if (fast) {
        IVIT_SM(1, -1);
    } else {
        IVIT_SM(0, -1);
    }
#undef IVIT_SM
}

hipError_t launch_shiftmax(hipStream_t s, const int8_t* x, const int8_t* bias, int H, int T, int8_t* y,
                           int64_t rows, int cols, int ld, ShiftParams p) {
    if (rows == 0) return hipSuccess;
    const int64_t want = (rows + 3) / 4;
    const int grid = (int)std::min<int64_t>(want, (int64_t)num_cus() * 16);
    const int nt = (cols + 63) / 64;
    TraceScope trace(s, KIND_SHIFTMAX, 0, rows * cols * (bias ? 3LL : 2LL));
    if (!bias && cols >= 16 && cols <= 256) {
        if (cols <= 64) launch_shiftmax_vec<4>(s, x, y, rows, cols, ld, p);
        else if (cols <= 128) launch_shiftmax_vec<8>(s, x, y, rows, cols, ld, p);
        else launch_shiftmax_vec<16>(s, x, y, rows, cols, ld, p);
        return hipGetLastError();
    }
    if (nt <= 1) hipLaunchKernelGGL(shiftmax_kernel<1>, dim3(grid), dim3(256), 0, s, x, bias, H, T, y, rows, cols, ld, p);
    else if (nt <= 2) hipLaunchKernelGGL(shiftmax_kernel<2>, dim3(grid), dim3(256), 0, s, x, bias, H, T, y, rows, cols, ld, p);
    else if (nt <= 4) hipLaunchKernelGGL(shiftmax_kernel<4>, dim3(grid), dim3(256), 0, s, x, bias, H, T, y, rows, cols, ld, p);
    else if (nt <= 8) hipLaunchKernelGGL(shiftmax_kernel<8>, dim3(grid), dim3(256), 0, s, x, bias, H, T, y, rows, cols, ld, p);
    else hipLaunchKernelGGL(shiftmax_kernel<16>, dim3(grid), dim3(256), 0, s, x, bias, H, T, y, rows, cols, ld, p);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// ShiftGELU.  A pure function of one int8 value, so each workgroup tabulates all 256 results in LDS
// (raw int16 product, or the int8 value after the dyadic rescale) and the body is a table lookup.
template <bool RAW, bool VEC>
__global__ __launch_bounds__(256) void shiftgelu_kernel(const int8_t* __restrict__ x, int8_t* __restrict__ y8,
                                                        int16_t* __restrict__ y16, int64_t n, ShiftParams p,
                                                        Dyadic rq) {
    __shared__ int16_t lut[256];
    {
        const int32_t I = (int32_t)(int8_t)threadIdx.x;       // table index = the value's low byte
        const int32_t g = shiftgelu_raw(I, p);
        lut[threadIdx.x] = RAW ? (int16_t)g : (int16_t)requant64(g, rq.b, rq.c);
    }
    __syncthreads();
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    if (VEC && !RAW) {
        const int64_t nv = n >> 4;
        const uint4* xv = reinterpret_cast<const uint4*>(x);
        uint4* yv = reinterpret_cast<uint4*>(y8);
        for (int64_t i = tid; i < nv; i += nthreads) {
            const uint4 a = xv[i];
            uint32_t in[4] = {a.x, a.y, a.z, a.w}, out[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t o = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) o |= ((uint32_t)lut[(in[d] >> (8 * e)) & 0xffu] & 0xffu) << (8 * e);
                out[d] = o;
            }
            yv[i] = make_uint4(out[0], out[1], out[2], out[3]);
        }
        for (int64_t i = (nv << 4) + tid; i < n; i += nthreads) y8[i] = (int8_t)lut[(uint8_t)x[i]];
    } else {
        for (int64_t i = tid; i < n; i += nthreads) {
            const int16_t v = lut[(uint8_t)x[i]];
            if (RAW) y16[i] = v; else y8[i] = (int8_t)v;
        }
    }
}

hipError_t launch_shiftgelu(hipStream_t s, const int8_t* x, int8_t* y8, int16_t* y16, int64_t n,
                            ShiftParams p, Dyadic out_rq) {
    if (n == 0) return hipSuccess;
    const bool raw = y16 != nullptr;
    const bool vec = !raw && (((uintptr_t)x | (uintptr_t)y8) & 15) == 0;
    const int64_t per_block = vec ? 256 * 16 : 256 * 4;
    const int grid = (int)std::min<int64_t>((n + per_block - 1) / per_block, (int64_t)num_cus() * 16);
    TraceScope trace(s, KIND_SHIFTGELU, 0, n * (raw ? 3LL : 2LL));
    if (raw) hipLaunchKernelGGL((shiftgelu_kernel<true, false>), dim3(grid), dim3(256), 0, s, x, y8, y16, n, p, out_rq);
    else if (vec) hipLaunchKernelGGL((shiftgelu_kernel<false, true>), dim3(grid), dim3(256), 0, s, x, y8, y16, n, p, out_rq);
    else hipLaunchKernelGGL((shiftgelu_kernel<false, false>), dim3(grid), dim3(256), 0, s, x, y8, y16, n, p, out_rq);
    return hipGetLastError();
}

// ShiftGELU with the maximum of Algorithm 2 taken over each row (the alternative reading of max(I_p)): m = max(0,
// max_j I_p[j]).  Given m, the result is a function of the int8 input alone, so each wavefront (one row at a time)
// finds m with one pass over its registers, tabulates the 256 results for this m in LDS (four entries per lane:
// ShiftExp of I_p - m, IntDiv with a 64-bit reciprocal since this form needs M above 31, requantisation) and
// looks every element up.  Entries for inputs above the maximum cannot occur and are skipped.
constexpr int RM_ROWS = 8;                                   // consecutive rows per wavefront
template <int NT>
__global__ __launch_bounds__(256) void shiftgelu_rowmax_kernel(const int8_t* __restrict__ x, int8_t* __restrict__ y,
                                                               int64_t rows, int cols, ShiftParams p, Dyadic rq) {
    __shared__ int8_t lut_all[4][256];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int8_t* lut = lut_all[wv];
    const int64_t wave = (int64_t)blockIdx.x * 4 + wv;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int ndw = cols >> 2;
    const int sh = p.m_bits - (p.k_out - 1);
    auto ip_of = [](int32_t I) { return I + (I >> 1) + (I >> 3) + (I >> 4); };
    const double two_m = (double)((uint64_t)1 << p.m_bits);
    int32_t table_mx = INT32_MIN;                                // row maximum the wavefront's table was built for (none yet)
    // a wavefront takes RM_ROWS consecutive rows at a time: step `it` is row it % RM_ROWS of its (it / RM_ROWS)-th group
    for (int64_t it = 0;; ++it) {
        const int64_t row = (wave + (it / RM_ROWS) * nwaves) * RM_ROWS + it % RM_ROWS;
        if (row >= rows) break;                                  // rows only grow with `it`
        const uint32_t* xr = reinterpret_cast<const uint32_t*>(x + row * cols);
        uint32_t xv[NT];
        // the maximum is taken on sign-flipped bytes, two at a time as packed 16-bit lanes (even and odd bytes)
        u16x2 m2 = {0, 0};
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int idx = lane + 64 * t;
            xv[t] = idx < ndw ? xr[idx] : 0x80808080u;           // padding: -128, never the maximum of a real row
            const uint32_t xf = xv[t] ^ 0x80808080u;
            m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(u16x2, xf & 0x00ff00ffu));
            m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(u16x2, (xf >> 8) & 0x00ff00ffu));
        }
        // I_p is increasing in I: the row maximum of I_p is I_p(max I)
        const int32_t mx = wave_max((int32_t)max((uint32_t)m2[0], (uint32_t)m2[1])) - 128;
        // the table depends on the row only through its maximum: a row with the maximum of the wavefront's previous row
        // (saturated activations: often 127) reuses that row's table
        const bool rebuild = mx != table_mx;
        table_mx = mx;
        const int32_t m = max(ip_of(mx), 0);
        const uint32_t e2 = shiftexp(-m, p.i0, p.n_shift);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (!rebuild) break;
            const int32_t I = (int32_t)(int8_t)(lane + 64 * k);  // the value whose low byte is the table index
            int32_t out = 0;
            if (I <= mx) {
                const uint32_t e1 = shiftexp(ip_of(I) - m, p.i0, p.n_shift);
                const uint32_t sum = e1 + e2;                    // at most 2^31
                // floor(2^M / sum), M <= 46, through one double-precision division: the quotient is correctly rounded
                // and, when it is not an integer, lies at least 1 / sum below the next one, which is more than half
                // a unit in the last place of any quotient up to 2^52; so the truncation is the exact floor
                const uint64_t inv = sum ? (uint64_t)(two_m / (double)sum) : 0;
                const uint64_t dv = (inv * e1) >> sh;
                out = requant64(I * (int32_t)dv, rq.b, rq.c);
            }
            lut[lane + 64 * k] = (int8_t)out;
        }
        __builtin_amdgcn_wave_barrier();                         // LDS serves a wavefront's accesses in order: the reads below see the table
        uint32_t* yr = reinterpret_cast<uint32_t*>(y + row * cols);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int idx = lane + 64 * t;
            uint32_t o = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) o |= ((uint32_t)(uint8_t)lut[(xv[t] >> (8 * e)) & 0xffu]) << (8 * e);
            if (idx < ndw) yr[idx] = o;
        }
        __builtin_amdgcn_wave_barrier();                         // next row's table is written after these reads were issued
    }
}

hipError_t launch_shiftgelu_rowmax(hipStream_t s, const int8_t* x, int8_t* y, int64_t rows, int cols, ShiftParams p,
                                   Dyadic rq) {
    if (rows == 0) return hipSuccess;
    // one workgroup per 4 RM_ROWS consecutive rows: the workgroups in flight cover a compact window of memory
    const int grid = (int)std::min<int64_t>((rows + 4 * RM_ROWS - 1) / (4 * RM_ROWS), 0x7fffffffLL);
    const int nt = (cols / 4 + 63) / 64;
    TraceScope trace(s, KIND_SHIFTGELU, 0, 2 * rows * cols);
#define IVIT_RM(NT_) hipLaunchKernelGGL(shiftgelu_rowmax_kernel<NT_>, dim3(grid), dim3(256), 0, s, x, y, rows, cols, p, rq)
    if (nt <= 1) IVIT_RM(1); else if (nt <= 2) IVIT_RM(2); else if (nt <= 4) IVIT_RM(4); else if (nt <= 6) IVIT_RM(6);
    else if (nt <= 8) IVIT_RM(8); else if (nt <= 12) IVIT_RM(12); else IVIT_RM(16);
#undef IVIT_RM
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Token assembly of the embedding layer: class token, patch tokens and position embedding, each int8 at its own
// scale, brought to the token scale by two dyadic rescales and added (the residual-add rule of Eq. 1-2 applied to
// the embedding sum).  One thread per 16 bytes of an output row; C % 16 == 0.
template <bool FAST>
__global__ __launch_bounds__(256) void embed_tokens_kernel(const int8_t* __restrict__ patch_tok, const int8_t* __restrict__ cls,
                                                           const int8_t* __restrict__ pos, Dyadic tq, Dyadic pq,
                                                           int8_t* __restrict__ tokens, int64_t n_pieces, int P, int C) {
    typedef int v4i __attribute__((ext_vector_type(4)));
    const int cpr = C >> 4, T = P + 1;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_pieces; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / cpr;
        const int cc = (int)(i - row * cpr);
        const int64_t b = row / T;
        const int t = (int)(row - b * T);
        const int8_t* src = t == 0 ? cls + 16 * cc : patch_tok + ((b * P + (t - 1)) * C + 16 * cc);
        const v4i sv = *reinterpret_cast<const v4i*>(src);
        const v4i pv = *reinterpret_cast<const v4i*>(pos + (int64_t)t * C + 16 * cc);
        v4i ov;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int32_t a = (int32_t)(int8_t)((uint32_t)sv[d] >> (8 * e));
                const int32_t q = (int32_t)(int8_t)((uint32_t)pv[d] >> (8 * e));
                const int32_t v = FAST ? clamp8(rnd_shift_fit32(a, tq.b, tq.c) + rnd_shift_fit32(q, pq.b, pq.c))
                                       : clamp8_64(rnd_shift64(a, tq.b, tq.c) + rnd_shift64(q, pq.b, pq.c));
                w |= ((uint32_t)v & 0xffu) << (8 * e);
            }
            ov[d] = (int)w;
        }
        *reinterpret_cast<v4i*>(tokens + row * C + 16 * cc) = ov;
    }
}

hipError_t launch_embed_tokens(hipStream_t s, const int8_t* patch_tok, const int8_t* cls, const int8_t* pos, Dyadic tok_rq,
                               Dyadic pos_rq, int8_t* tokens, int B, int P, int C) {
    const int64_t n_pieces = (int64_t)B * (P + 1) * (C >> 4);
    if (n_pieces == 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((n_pieces + 255) / 256, (int64_t)num_cus() * 32);
    auto fits = [](Dyadic d) { return d.c >= 1 && d.c <= 31 && d.b >= 1 && (uint32_t)d.b <= (1u << d.c); };
    TraceScope trace(s, KIND_EMBED, 0, (int64_t)B * (2 * P + 1) * C + (int64_t)(P + 2) * C);
    if (fits(tok_rq) && fits(pos_rq))
        hipLaunchKernelGGL(embed_tokens_kernel<true>, dim3(grid), dim3(256), 0, s, patch_tok, cls, pos, tok_rq, pos_rq, tokens, n_pieces, P, C);
    else
        hipLaunchKernelGGL(embed_tokens_kernel<false>, dim3(grid), dim3(256), 0, s, patch_tok, cls, pos, tok_rq, pos_rq, tokens, n_pieces, P, C);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Patch merging of the hierarchical windowed models, the data movement only: the four tokens of each 2 x 2
// neighbourhood of a g x g token grid are concatenated, in the order of (row, column) offsets (0,0), (1,0), (0,1),
// (1,1), into one row of 4C bytes.  One thread per 16 bytes of output.
__global__ __launch_bounds__(256) void patch_merge_gather_kernel(const int8_t* __restrict__ x, int8_t* __restrict__ y,
                                                                 int64_t n_pieces, int g, int C) {
    typedef int v4i __attribute__((ext_vector_type(4)));
    const int cpr = C >> 4, g2 = g >> 1;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_pieces; i += (int64_t)gridDim.x * 256) {
        const int64_t orow = i / (4 * cpr);
        const int j = (int)(i - orow * (4 * cpr));
        const int q = j / cpr, cc = j - q * cpr;
        const int64_t b = orow / ((int64_t)g2 * g2);
        const int rem = (int)(orow - b * g2 * g2);
        const int yy = rem / g2, xx = rem - yy * g2;
        const int64_t irow = (b * g + 2 * yy + (q & 1)) * g + 2 * xx + (q >> 1);
        *reinterpret_cast<v4i*>(y + orow * 4 * C + (int64_t)16 * j) = *reinterpret_cast<const v4i*>(x + irow * C + 16 * cc);
    }
}

hipError_t launch_patch_merge_gather(hipStream_t s, const int8_t* x, int8_t* y, int B, int g, int C) {
    const int64_t n_pieces = (int64_t)B * (g / 2) * (g / 2) * 4 * (C >> 4);
    if (n_pieces == 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((n_pieces + 255) / 256, (int64_t)num_cus() * 32);
    TraceScope trace(s, KIND_PATCH_MERGE, 0, 2 * n_pieces * 16);
    hipLaunchKernelGGL(patch_merge_gather_kernel, dim3(grid), dim3(256), 0, s, x, y, n_pieces, g, C);
    return hipGetLastError();
}

// Average pooling over the tokens of an image as a dyadic rescale of the token sum: one thread per four channels of
// an image walks the T rows (consecutive threads read consecutive dwords of a row).
__global__ __launch_bounds__(256) void mean_pool_kernel(const int8_t* __restrict__ x, int8_t* __restrict__ y, int64_t n_words,
                                                        int T, int C, Dyadic rq) {
    const int wpr = C >> 2;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * 256) {
        const int64_t b = i / wpr;
        const int wd = (int)(i - b * wpr);
        const uint32_t* src = reinterpret_cast<const uint32_t*>(x + b * T * C) + wd;
        int32_t acc[4] = {0, 0, 0, 0};
        int t = 0;
        for (; t + 8 <= T; t += 8) {               // eight independent loads in flight
            uint32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(t + u) * wpr];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += (int32_t)(int8_t)(v[u] >> (8 * e));
        }
        for (; t < T; ++t) {
            const uint32_t v = src[(int64_t)t * wpr];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += (int32_t)(int8_t)(v >> (8 * e));
        }
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) w |= ((uint32_t)requant64(acc[e], rq.b, rq.c) & 0xffu) << (8 * e);
        reinterpret_cast<uint32_t*>(y)[i] = w;
    }
}

hipError_t launch_mean_pool(hipStream_t s, const int8_t* x, int8_t* y, int B, int T, int C, Dyadic rq) {
    const int64_t n_words = (int64_t)B * (C >> 2);
    if (n_words == 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((n_words + 255) / 256, (int64_t)num_cus() * 32);
    TraceScope trace(s, KIND_MEAN_POOL, 0, (int64_t)B * (T + 1) * C);
    hipLaunchKernelGGL(mean_pool_kernel, dim3(grid), dim3(256), 0, s, x, y, n_words, T, C, rq);
    return hipGetLastError();
}

}  // namespace ivit
