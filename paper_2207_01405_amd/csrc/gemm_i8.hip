// int8 x int8 -> int32 Dense / MatMul on the gfx950 matrix cores with the dyadic requantisation of
// I-ViT (arXiv 2207.01405, Sec. 3.2, Eq. 7-10) fused into the epilogue, optionally with the residual
// add of Eq. 1-2 or with ShiftGELU (Sec. 3.4, Algorithm 2) and its rescale.
//
// One workgroup (256 threads = 4 wavefronts as 2 x 2) computes a 128-token x 128-channel output tile.  K is
// consumed in 64-byte steps through two LDS buffers; the global loads of the next TWO steps are in flight
// (in two register sets) while the current step is multiplied, because with K of a few hundred bytes the
// kernel is bound by load latency, not by the matrix cores.  Each wavefront owns 64 tokens x 64 channels =
// 2 x 2 tiles of v_mfma_i32_32x32x32_i8 (the int8 instruction that reaches the matrix-core peak on gfx950).
// The weights are the MFMA "A" operand (rows = output channels) and the activations the "B" operand
// (columns = tokens), so an accumulator lane holds 16 channels of ONE token per tile.  The channel rows are
// permuted when the weight tile is written to LDS so that the 32 accumulator registers of a token are 32
// consecutive channels: they are requantised, packed and stored as two 16-byte writes per token.
// Workgroup ids are remapped so that each XCD (own L2) works on a contiguous range of tiles.
#include "ivit_kernels.hpp"

namespace ivit {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#ifndef IVIT_GEMM_BK
#define IVIT_GEMM_BK 64
#endif
#ifndef IVIT_GEMM_WGS_PER_CU
#define IVIT_GEMM_WGS_PER_CU 2
#endif
constexpr int BM = 128, BN = 128, BK = IVIT_GEMM_BK;
constexpr int CPR = BK / 16;                  // 16-byte chunks per tile row
constexpr int RPP = 256 / CPR;                // tile rows covered by one pass of the 256 threads
constexpr int NLD = BM / RPP;                 // passes (= 16-byte loads per thread and operand) per K step
constexpr int LROW = BK + 16;                 // LDS row pitch (bytes): 32 consecutive rows of 16-byte reads cover all banks
constexpr int NXCD = 8;

enum Epilogue { EPI_PLAIN = 0, EPI_RESIDUAL = 1, EPI_GELU = 2 };

struct GemmParams {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N; int K; int tiles_n; int64_t tiles; int64_t per_xcd;
};

// LDS row (0..63) of channel offset n (0..63) inside a wavefront's 64-channel slab.  MFMA tile ct, row
// i = 8q + 4g + r lands in accumulator register 4q + r of lane group g; storing channel 32g + 16ct + 4q + r
// there gives lane group g the 32 consecutive channels 32g .. 32g + 31 (register index 16ct + 4q + r).
__device__ __forceinline__ int slab_row(int n) {
    return ((n >> 4) & 1) * 32 + ((n >> 2) & 3) * 8 + (n >> 5) * 4 + (n & 3);
}

// Requantise, fuse and store the 2 x 32 outputs of a lane: tokens m, m + 32 and channels n .. n + 31
// (tile-local channel index cl for the staged parameters).  FAST: every channel of the tile has
// 1 <= c <= 31 and b <= 2^c, so the rounded product fits 32 bits.
template <int EPI, bool FAST>
__device__ __forceinline__ void epilogue(const GemmParams& P, const v16i (&acc)[2][2], const int32_t* qb_s,
                                         const int32_t* qc_s, const int8_t* gelu_lut, int64_t m, int n, int cl) {
    const int N = P.N;
    const bool full = (N & 15) == 0 && n + 31 < N;       // all 32 channels exist and rows are 16-byte aligned
    const bool res_fast = dyadic_fits32(P.res_rq.b, P.res_rq.c);
#pragma unroll
    for (int tt = 0; tt < 2; ++tt, m += 32) {
        const bool row_ok = m < P.M;
        uint32_t outw[8];
        uint32_t resw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (EPI == EPI_RESIDUAL && row_ok) {
            const int8_t* rp = P.residual + m * N + n;
            if (full) {
                const uint4 r0 = *reinterpret_cast<const uint4*>(rp), r1 = *reinterpret_cast<const uint4*>(rp + 16);
                resw[0] = r0.x; resw[1] = r0.y; resw[2] = r0.z; resw[3] = r0.w;
                resw[4] = r1.x; resw[5] = r1.y; resw[6] = r1.z; resw[7] = r1.w;
            } else {
                for (int c = 0; c < 32; ++c)
                    if (n + c < N) resw[c >> 2] |= ((uint32_t)(uint8_t)rp[c]) << (8 * (c & 3));
            }
        }
#pragma unroll
        for (int w4 = 0; w4 < 8; ++w4) {               // 4 channels per packed output word
            const v4i qb = *reinterpret_cast<const v4i*>(&qb_s[cl + 4 * w4]);
            const v4i qc = *reinterpret_cast<const v4i*>(&qc_s[cl + 4 * w4]);
            uint32_t packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int32_t a32 = acc[w4 >> 2][tt][4 * (w4 & 3) + r];
                int32_t v;
                if (EPI == EPI_RESIDUAL) {
                    const int32_t res = (int32_t)(int8_t)(resw[w4] >> (8 * r));
                    if (FAST && res_fast) {
                        v = clamp8(rnd_shift_fit32(a32, qb[r], qc[r]) + rnd_shift_fit32(res, P.res_rq.b, P.res_rq.c));
                    } else {
                        const int64_t rr = rnd_shift64(res, P.res_rq.b, P.res_rq.c);
                        v = clamp8_64((FAST ? (int64_t)rnd_shift_fit32(a32, qb[r], qc[r]) : rnd_shift64(a32, qb[r], qc[r])) + rr);
                    }
                } else {
                    v = FAST ? clamp8(rnd_shift_fit32(a32, qb[r], qc[r])) : requant64(a32, qb[r], qc[r]);
                    if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                }
                packed |= ((uint32_t)v & 0xffu) << (8 * r);
            }
            outw[w4] = packed;
            __builtin_amdgcn_sched_barrier(0);          // keep the register footprint of the epilogue small
        }
        if (row_ok) {
            int8_t* yp = P.y + m * N + n;
            if (full) {
                *reinterpret_cast<uint4*>(yp) = make_uint4(outw[0], outw[1], outw[2], outw[3]);
                *reinterpret_cast<uint4*>(yp + 16) = make_uint4(outw[4], outw[5], outw[6], outw[7]);
            } else {
                for (int c = 0; c < 32; ++c)
                    if (n + c < N) yp[c] = (int8_t)(outw[c >> 2] >> (8 * (c & 3)));
            }
        }
    }
}

struct Stage { v4i x[NLD], w[NLD]; };               // one K step of a thread's share of both operand tiles

template <int EPI>
__global__ __launch_bounds__(256, IVIT_GEMM_WGS_PER_CU) void gemm_i8_kernel(GemmParams P) {
    __shared__ __align__(16) int8_t Xs[2][BM * LROW];
    __shared__ __align__(16) int8_t Ws[2][BN * LROW];
    __shared__ __align__(16) int32_t qb_s[BN], qc_s[BN], bias_s[BN];
    __shared__ int8_t gelu_lut[256];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int wm = (wv >> 1) * 64, wn = (wv & 1) * 64;          // wavefront's token / channel offset in the tile

    // each XCD takes a contiguous range of tiles; within it the channel tile index runs fastest
    const int64_t tile = (int64_t)(blockIdx.x % NXCD) * P.per_xcd + blockIdx.x / NXCD;
    if (tile >= P.tiles) return;
    const int64_t m0 = (tile / P.tiles_n) * BM;
    const int n0 = (int)(tile % P.tiles_n) * BN;
    const int K = P.K, N = P.N;
    const int64_t M = P.M;

    // global -> LDS staging: thread t moves 16 bytes (chunk t % CPR) of rows t / CPR + RPP p of each operand tile
    const int ld_row = tid / CPR, ld_k = (tid % CPR) * 16;
    const int8_t* xg[NLD]; const int8_t* wg[NLD];
    int xs_off[NLD], ws_off[NLD];
#pragma unroll
    for (int p = 0; p < NLD; ++p) {
        const int r = ld_row + RPP * p;
        const int64_t xm = min<int64_t>(m0 + r, M - 1);
        const int wnn = min(n0 + r, N - 1);
        xg[p] = P.x + xm * K + ld_k;
        wg[p] = P.w + (int64_t)wnn * K + ld_k;
        xs_off[p] = r * LROW + ld_k;
        ws_off[p] = ((r & 64) + slab_row(r & 63)) * LROW + ld_k;
    }
    const int steps = (K + BK - 1) / BK;      // the last step may be partial (K % 128 != 0): zero padded per 16 bytes
    auto load_stage = [&](Stage& s, int kb) {
        const int koff = kb * BK;
        const bool in = koff + ld_k < K;
#pragma unroll
        for (int p = 0; p < NLD; ++p) {
            s.x[p] = in ? *reinterpret_cast<const v4i*>(xg[p] + koff) : v4i{0, 0, 0, 0};
            s.w[p] = in ? *reinterpret_cast<const v4i*>(wg[p] + koff) : v4i{0, 0, 0, 0};
        }
    };
    auto store_stage = [&](const Stage& s, int buf) {
#pragma unroll
        for (int p = 0; p < NLD; ++p) {
            *reinterpret_cast<v4i*>(&Xs[buf][xs_off[p]]) = s.x[p];
            *reinterpret_cast<v4i*>(&Ws[buf][ws_off[p]]) = s.w[p];
        }
    };

    Stage st0, st1;
    load_stage(st0, 0);
    if (steps > 1) load_stage(st1, 1);

    // per-channel parameters of the tile go to LDS once; the 32-bit requantisation path is taken only if
    // every channel of the tile has 1 <= c <= 31 and 1 <= b <= 2^c (a rescale by at most 1)
    bool chan_fast = true;
    if (tid < BN) {
        const int ch = min(n0 + tid, N - 1);
        const int32_t b = P.rq_b[ch], c = P.rq_c[ch];
        qb_s[tid] = b; qc_s[tid] = c;
        bias_s[tid] = P.bias ? P.bias[ch] : 0;
        chan_fast = dyadic_fits32(b, c);
    }
    if (EPI == EPI_GELU) {
        const int32_t I = (int32_t)(int8_t)tid;
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c);
    }
    store_stage(st0, 0);
    if (steps > 2) load_stage(st0, 2);
    const bool fast = __syncthreads_and(chan_fast) != 0;

    // accumulators start at the bias of their channel: register 16 ct + v of lane group g is channel 32 g + 16 ct + v
    v16i acc[2][2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
        v16i bv;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const v4i t = *reinterpret_cast<const v4i*>(&bias_s[wn + 32 * lg + 16 * ct + 4 * q]);
            bv[4 * q] = t[0]; bv[4 * q + 1] = t[1]; bv[4 * q + 2] = t[2]; bv[4 * q + 3] = t[3];
        }
        acc[ct][0] = bv; acc[ct][1] = bv;
    }

    auto compute = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            v4i a[2], b[2];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
                a[ct] = *reinterpret_cast<const v4i*>(&Ws[buf][(wn + 32 * ct + li) * LROW + 32 * ks + 16 * lg]);
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
                b[tt] = *reinterpret_cast<const v4i*>(&Xs[buf][(wm + 32 * tt + li) * LROW + 32 * ks + 16 * lg]);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
                    acc[ct][tt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[ct], b[tt], acc[ct][tt], 0, 0, 0);
        }
    };

    // step kb is multiplied from LDS buffer kb & 1; step kb + 1 waits in register set (kb + 1) & 1 and is written to
    // the other buffer after the multiply; its register set is then refilled with step kb + 3
    for (int kb = 0; kb < steps; kb += 2) {
        compute(0);
        if (kb + 1 < steps) {
            store_stage(st1, 1);
            if (kb + 3 < steps) load_stage(st1, kb + 3);
        }
        __syncthreads();
        if (kb + 1 >= steps) break;
        compute(1);
        if (kb + 2 < steps) {
            store_stage(st0, 0);
            if (kb + 4 < steps) load_stage(st0, kb + 4);
        }
        __syncthreads();
    }

    // ---- epilogue: lane (li, lg) holds, for token tile tt, channels cl .. cl + 31 (tile-local) of token m0 + wm + 32 tt + li
    const int cl = wn + 32 * lg;
    if (fast) epilogue<EPI, true>(P, acc, qb_s, qc_s, gelu_lut, m0 + wm + li, n0 + cl, cl);
    else epilogue<EPI, false>(P, acc, qb_s, qc_s, gelu_lut, m0 + wm + li, n0 + cl, cl);
}

hipError_t launch_linear(hipStream_t s, const LinearArgs& a) {
    if (a.M == 0) return hipSuccess;
    GemmParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.K = a.K;
    P.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles_m = (a.M + BM - 1) / BM;
    P.tiles = tiles_m * P.tiles_n;
    P.per_xcd = (P.tiles + NXCD - 1) / NXCD;
    const int64_t grid = P.per_xcd * NXCD;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t bytes = a.M * a.K + (int64_t)a.N * a.K + a.M * a.N * (a.residual ? 2 : 1) + 8LL * a.N + (a.bias ? 4LL * a.N : 0);
    TraceScope trace(s, a.residual ? KIND_GEMM_RESIDUAL : (a.gelu ? KIND_GEMM_GELU : KIND_GEMM), 2 * a.M * a.N * a.K, bytes);
    if (a.residual) hipLaunchKernelGGL(gemm_i8_kernel<EPI_RESIDUAL>, dim3((unsigned)grid), dim3(256), 0, s, P);
    else if (a.gelu) hipLaunchKernelGGL(gemm_i8_kernel<EPI_GELU>, dim3((unsigned)grid), dim3(256), 0, s, P);
    else hipLaunchKernelGGL(gemm_i8_kernel<EPI_PLAIN>, dim3((unsigned)grid), dim3(256), 0, s, P);
    return hipGetLastError();
}

}  // namespace ivit
