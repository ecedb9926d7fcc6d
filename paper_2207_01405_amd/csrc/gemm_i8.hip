// int8 x int8 -> int32 Dense / MatMul on the gfx950 matrix cores with the dyadic requantisation of
// I-ViT (arXiv 2207.01405, Sec. 3.2, Eq. 7-10) fused into the epilogue, optionally with the residual
// add of Eq. 1-2 or with ShiftGELU (Sec. 3.4, Algorithm 2) and its rescale.
//
// Layout of one workgroup (256 threads = 4 wavefronts as 2 x 2): a BM x BN = 128 x 128 output tile,
// K consumed in steps of 64 bytes through double-buffered LDS tiles.  Each wavefront owns 64 tokens x
// 64 channels = 4 x 4 tiles of v_mfma_i32_16x16x64_i8.  The weights are the MFMA "A" operand (rows =
// output channels) and the activations the "B" operand (columns = tokens), so an accumulator lane holds
// four consecutive channels of one token; a permutation of the channel rows when the weight tile is
// written to LDS makes the 16 accumulator registers of a token tile 16 consecutive channels, which are
// requantised, packed and stored as one 16-byte write per token.
#include "ivit_kernels.hpp"

namespace ivit {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LROW = BK + 16;                 // LDS row pitch in bytes: 16 rows of 16-byte reads hit distinct banks

enum Epilogue { EPI_PLAIN = 0, EPI_RESIDUAL = 1, EPI_GELU = 2 };

struct GemmParams {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N; int K; int tiles_n;
};

// Row of the 64-row weight slab in LDS that holds channel offset n (0..63) of the slab: MFMA tile ct,
// row 4g + r of the slab holds channel 16g + 4ct + r.
__device__ __forceinline__ int slab_row(int n) { return ((n >> 2) & 3) * 16 + (n >> 4) * 4 + (n & 3); }

template <int EPI>
__global__ __launch_bounds__(256) void gemm_i8_kernel(GemmParams P) {
    __shared__ __align__(16) int8_t Xs[2][BM * LROW];
    __shared__ __align__(16) int8_t Ws[2][BN * LROW];
    __shared__ int8_t gelu_lut[256];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    const int wm = (wv >> 1) * 64, wn = (wv & 1) * 64;          // wave's token / channel offset in the tile
    const int64_t m0 = (int64_t)(blockIdx.x / P.tiles_n) * BM;
    const int n0 = (int)(blockIdx.x % P.tiles_n) * BN;
    const int K = P.K, N = P.N;
    const int64_t M = P.M;

    if (EPI == EPI_GELU) {
        const int32_t I = (int32_t)(int8_t)tid;
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c);
    }

    // global -> LDS staging: thread t moves 16 bytes of rows t/4 and t/4 + 64 of each operand tile
    const int ld_row = tid >> 2, ld_k = (tid & 3) * 16;
    const int8_t* xg[2]; const int8_t* wg[2];
    int xs_off[2], ws_off[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = ld_row + 64 * p;
        const int64_t xm = min<int64_t>(m0 + r, M - 1);
        const int wnn = min(n0 + r, N - 1);
        xg[p] = P.x + xm * K + ld_k;
        wg[p] = P.w + (int64_t)wnn * K + ld_k;
        xs_off[p] = r * LROW + ld_k;
        ws_off[p] = ((r & 64) + slab_row(r & 63)) * LROW + ld_k;
    }

    v4i acc[4][4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        int32_t bv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ch = min(n0 + wn + 16 * lg + 4 * ct + r, N - 1);
            bv[r] = P.bias ? P.bias[ch] : 0;
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[ct][tt] = v4i{bv[0], bv[1], bv[2], bv[3]};
    }

    v4i xr[2], wr[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {                                 // K may be shorter than one 64-byte step
        xr[p] = ld_k < K ? *reinterpret_cast<const v4i*>(xg[p]) : v4i{0, 0, 0, 0};
        wr[p] = ld_k < K ? *reinterpret_cast<const v4i*>(wg[p]) : v4i{0, 0, 0, 0};
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        *reinterpret_cast<v4i*>(&Xs[0][xs_off[p]]) = xr[p];
        *reinterpret_cast<v4i*>(&Ws[0][ws_off[p]]) = wr[p];
    }
    __syncthreads();

    const int nk = K / BK;                    // full 64-byte steps; a 16/32/48-byte remainder is handled below
    const int krem = K - nk * BK;
    const int steps = nk + (krem ? 1 : 0);
    for (int kb = 0; kb < steps; ++kb) {
        const int cur = kb & 1;
        const bool more = kb + 1 < steps;
        if (more) {
            const int koff = (kb + 1) * BK;
            const bool in = koff + ld_k < K;                      // the last step may be partial: pad with zeros
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                xr[p] = in ? *reinterpret_cast<const v4i*>(xg[p] + koff) : v4i{0, 0, 0, 0};
                wr[p] = in ? *reinterpret_cast<const v4i*>(wg[p] + koff) : v4i{0, 0, 0, 0};
            }
        }
        v4i a[4], b[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
            a[ct] = *reinterpret_cast<const v4i*>(&Ws[cur][(wn + 16 * ct + li) * LROW + 16 * lg]);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
            b[tt] = *reinterpret_cast<const v4i*>(&Xs[cur][(wm + 16 * tt + li) * LROW + 16 * lg]);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
                acc[ct][tt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[ct], b[tt], acc[ct][tt], 0, 0, 0);
        if (more) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                *reinterpret_cast<v4i*>(&Xs[cur ^ 1][xs_off[p]]) = xr[p];
                *reinterpret_cast<v4i*>(&Ws[cur ^ 1][ws_off[p]]) = wr[p];
            }
        }
        __syncthreads();
    }

    // ---- epilogue: lane (li, lg) holds, for token tile tt, channels cbase .. cbase + 15 of token m0 + wm + 16 tt + li
    const int cbase = n0 + wn + 16 * lg;
    uint32_t outw[4][4];                       // [tt][ct]: 4 packed int8 each
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        int32_t qb[4], qc[4];
        bool fast = true;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ch = min(cbase + 4 * ct + r, N - 1);
            qb[r] = P.rq_b[ch];
            qc[r] = P.rq_c[ch];
            fast = fast && qb[r] > 0 && qb[r] < 32768 && qc[r] >= 16 && qc[r] <= 31;
        }
        fast = __all(fast);
        uint32_t resw[4] = {0, 0, 0, 0};
        if (EPI == EPI_RESIDUAL) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int64_t m = m0 + wm + 16 * tt + li;
                const int ch = cbase + 4 * ct;
                if (m < M && ch + 3 < N && (N & 3) == 0) {
                    resw[tt] = *reinterpret_cast<const uint32_t*>(P.residual + m * N + ch);
                } else if (m < M) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (ch + r < N) resw[tt] |= ((uint32_t)(uint8_t)P.residual[m * N + ch + r]) << (8 * r);
                }
            }
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            uint32_t packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int32_t a32 = acc[ct][tt][r];
                int32_t v;
                if (EPI == EPI_RESIDUAL) {
                    const int32_t res = (int32_t)(int8_t)(resw[tt] >> (8 * r));
                    const int64_t t = (fast ? (int64_t)rnd_shift_b15(a32, qb[r], qc[r]) : rnd_shift64(a32, qb[r], qc[r]))
                                    + rnd_shift64(res, P.res_rq.b, P.res_rq.c);
                    v = clamp8_64(t);
                } else {
                    v = fast ? clamp8(rnd_shift_b15(a32, qb[r], qc[r])) : requant64(a32, qb[r], qc[r]);
                    if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                }
                packed |= ((uint32_t)v & 0xffu) << (8 * r);
            }
            outw[tt][ct] = packed;
        }
    }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
        const int64_t m = m0 + wm + 16 * tt + li;
        if (m >= M) continue;
        int8_t* yp = P.y + m * N + cbase;
        if (cbase + 15 < N && (N & 15) == 0) {
            *reinterpret_cast<uint4*>(yp) = make_uint4(outw[tt][0], outw[tt][1], outw[tt][2], outw[tt][3]);
        } else {
#pragma unroll
            for (int c = 0; c < 16; ++c)
                if (cbase + c < N) yp[c] = (int8_t)(outw[tt][c >> 2] >> (8 * (c & 3)));
        }
    }
}

hipError_t launch_linear(hipStream_t s, const LinearArgs& a) {
    if (a.M == 0) return hipSuccess;
    GemmParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.K = a.K;
    P.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles_m = (a.M + BM - 1) / BM;
    const int64_t grid = tiles_m * P.tiles_n;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t bytes = a.M * a.K + (int64_t)a.N * a.K + a.M * a.N * (a.residual ? 2 : 1) + 8LL * a.N + (a.bias ? 4LL * a.N : 0);
    TraceScope trace(s, a.residual ? KIND_GEMM_RESIDUAL : (a.gelu ? KIND_GEMM_GELU : KIND_GEMM), 2 * a.M * a.N * a.K, bytes);
    if (a.residual) hipLaunchKernelGGL(gemm_i8_kernel<EPI_RESIDUAL>, dim3((unsigned)grid), dim3(256), 0, s, P);
    else if (a.gelu) hipLaunchKernelGGL(gemm_i8_kernel<EPI_GELU>, dim3((unsigned)grid), dim3(256), 0, s, P);
    else hipLaunchKernelGGL(gemm_i8_kernel<EPI_PLAIN>, dim3((unsigned)grid), dim3(256), 0, s, P);
    return hipGetLastError();
}

}  // namespace ivit
