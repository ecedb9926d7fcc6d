// int8 x int8 -> int32 Dense / MatMul on the gfx950 matrix cores with the dyadic requantisation of
// I-ViT (arXiv 2207.01405, Sec. 3.2, Eq. 7-10) fused into the epilogue, optionally with the residual
// add of Eq. 1-2 or with ShiftGELU (Sec. 3.4, Algorithm 2) and its rescale.
//
// One workgroup (256 threads = 4 wavefronts as 2 x 2) computes a 128-token x 128-channel output tile.  K is
// consumed in 128-byte steps through two LDS buffers; the global loads of the next TWO steps are in flight
// (in two register sets) while the current step is multiplied, because with K of a few hundred bytes the
// kernel is bound by load latency, not by the matrix cores.  Each wavefront owns 64 tokens x 64 channels =
// 2 x 2 tiles of v_mfma_i32_32x32x32_i8 (the int8 instruction that reaches the matrix-core peak on gfx950).
// The weights are the MFMA "A" operand (rows = output channels) and the activations the "B" operand
// (columns = tokens), so an accumulator lane holds 16 channels of ONE token per tile.  The channel rows are
// permuted when the weight tile is written to LDS so that the 32 accumulator registers of a token are 32
// consecutive channels: they are requantised, packed and stored as two 16-byte writes per token.
// Workgroup ids are remapped so that each XCD (own L2) works on a contiguous range of tiles.
#include "ivit_kernels.hpp"
#include <algorithm>
#include <type_traits>

namespace ivit {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 128;
constexpr int TILED_WGS_PER_CU = 2;           // workgroups of the tiled kernel resident per compute unit
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
    int64_t ldx;                         // bytes between rows of x
    int rnd;                             // 1: round to nearest, 0: floor (every requantisation of the epilogue)
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
                        v = clamp8(rnd_shift_fit32(a32, qb[r], qc[r], P.rnd) + rnd_shift_fit32(res, P.res_rq.b, P.res_rq.c, P.rnd));
                    } else {
                        const int64_t rr = rnd_shift64(res, P.res_rq.b, P.res_rq.c, P.rnd);
                        v = clamp8_64((FAST ? (int64_t)rnd_shift_fit32(a32, qb[r], qc[r], P.rnd) : rnd_shift64(a32, qb[r], qc[r], P.rnd)) + rr);
                    }
                } else {
                    v = FAST ? clamp8(rnd_shift_fit32(a32, qb[r], qc[r], P.rnd)) : requant64(a32, qb[r], qc[r], P.rnd);
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
__global__ __launch_bounds__(256, TILED_WGS_PER_CU) void gemm_i8_kernel(GemmParams P) {
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
        const int64_t xm = min64(m0 + r, M - 1);
        const int wnn = min(n0 + r, N - 1);
        xg[p] = P.x + xm * P.ldx + ld_k;
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
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c, P.rnd);
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

// ------------------------------------------------------------------------------------------------
// Weight-stationary kernel for K small enough that a slab of 32 NCB output channels, all of K, stays in LDS.
//
// A workgroup (8 wavefronts, two per SIMD) loads its weight slab once; only this prologue has barriers.  Every
// wavefront then walks over its own groups of 32 tokens, reads their activations straight from global memory into
// registers in the layout of the MFMA "B" operand (no LDS round trip: nobody else needs them) and multiplies them
// with the slab, NCB tiles of v_mfma_i32_32x32x32_i8 per 32 bytes of K.  Within a 128-byte chunk of K a lane reads
// 64 contiguous bytes (lane group g the half g of the chunk) and uses its j-th 16 bytes in the j-th MFMA of the
// chunk; the weight fragments are read from LDS with the same assignment of K bytes to MFMAs, so the contraction
// is unchanged.  Activations move in units of UNIT chunks through two register buffers: while one unit is
// multiplied the loads of the next one (of the next group, at the end of a group) are in flight, which hides the
// memory latency, and the second wavefront of the SIMD feeds the matrix core while this one requantises.
// Slab rows are stored in LDS so that the accumulator registers of a lane are 16 NCB consecutive channels of one
// token (see row_of_channel); results go through a small per-wavefront LDS buffer so that every store instruction
// writes whole output rows.
constexpr int WS_THREADS = 512, WS_WAVES = WS_THREADS / 64, WS_CHUNK = 128;
constexpr int WS_LDS_MAX = 160 * 1024;

struct WsParams {
    GemmParams g;
    int slabs, q, nunits, pitch;        // channel slabs, workgroups per slab, units per group, LDS row pitch
    int64_t groups;                     // groups of 32 tokens
};

// LDS row (within the slab) of slab-local channel n: lane group g owns channels 16 NCB g .. 16 NCB (g + 1) - 1;
// channel 16 NCB g + 16 cb + 4 q + r is row 8 q + 4 g + r of MFMA tile cb, i.e. accumulator register 4 q + r.
template <int NCB>
__device__ __forceinline__ int row_of_channel(int n) {
    const int g = n / (16 * NCB), rem = n % (16 * NCB), cb = rem >> 4, v = rem & 15;
    return 32 * cb + 8 * (v >> 2) + 4 * g + (v & 3);
}

// UNIT: chunks per unit.  PAD: K is not a whole number of units, the rest reads as zero.  EVEN: the number of
// units per group is even, so a group can only end after the second unit of the unrolled pair.
template <int EPI, int NCB, int UNIT, bool PAD, bool EVEN>
__global__ __launch_bounds__(WS_THREADS) void gemm_ws_kernel(WsParams W) {
    extern __shared__ __align__(16) int8_t lds[];
    const GemmParams& P = W.g;
    constexpr int NS = 32 * NCB;                       // channels of a slab
    constexpr int RB = 32 * NCB, SP = RB + 16;         // bytes of an output row of the slab, pitch of its staging copy
    constexpr int XP = WS_CHUNK + 16;                  // pitch of a staged activation chunk (32 tokens x 128 bytes)
    constexpr int STG = 32 * SP > 32 * XP ? 32 * SP : 32 * XP;   // staging bytes per wavefront: output rows, or one chunk
    const int pitch = W.pitch, nunits = W.nunits;
    int8_t* Wl = lds;
    int32_t* qb_s = reinterpret_cast<int32_t*>(lds + (size_t)NS * pitch);
    int32_t* qc_s = qb_s + NS;
    int32_t* bias_s = qc_s + NS;
    int64_t* hb_s = reinterpret_cast<int64_t*>(bias_s + NS);   // bias * b + 2^(c-1): the 64-bit addend of the fast requantisation
    int32_t* lo_s = reinterpret_cast<int32_t*>(hb_s + NS);     // the four tables of the 24-bit requantisation (see below)
    int32_t* hi_s = lo_s + NS;
    int32_t* mb_s = hi_s + NS;
    int32_t* ad_s = mb_s + NS;
    int8_t* gelu_lut = reinterpret_cast<int8_t*>(ad_s + NS);

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    int8_t* stage = gelu_lut + 256 + wv * STG;     // this wavefront's 32 token rows, written and read by it alone
    const int K = P.K, N = P.N;
    const int64_t M = P.M;

    // workgroups of one XCD (block id modulo 8) get consecutive logical ids: the slabs that share a token range, and
    // therefore re-read the same activations, sit on the same L2
    const int G = gridDim.x, xcd = blockIdx.x % NXCD;
    const int L = xcd * (G / NXCD) + min(xcd, G % NXCD) + blockIdx.x / NXCD;
    const int slab = L % W.slabs, wi = L / W.slabs;
    const int n0 = slab * NS;

    // group r + t stride belongs to wavefront r / q of workgroup r % q: when the last round is not full, its groups go
    // to the low wavefronts (distinct SIMDs) of all workgroups instead of to all wavefronts of a few
    const int64_t stride = (int64_t)W.q * WS_WAVES;
    int64_t cgrp = (int64_t)wv * W.q + wi;              // group being multiplied
    int64_t lgrp = cgrp;                                // group and unit of the next load
    int lu = 0;
    const bool has_work = cgrp < W.groups;

    // One unit of activations.  A load instruction reads whole 128-byte lines (8 lanes per token, 8 tokens per
    // instruction, 4 instructions per chunk): lane l gets piece l % 8 of chunk c of tokens 8 t + l / 8, t = 0..3.
    // Scattered 16-byte reads in MFMA layout would cost the texture addresser one cycle per touched line, twice the
    // time; the chunk is brought into MFMA layout through this wavefront's LDS staging rows right before its use.
    // No branches around the loads (the compiler then counts outstanding loads exactly): past the last group the
    // last one is loaded again, and with PAD a piece past the end of the row reads the row's last 16 bytes and is
    // replaced by zero.
    v4i xa[UNIT][4], xb[UNIT][4];
    const int l8 = lane >> 3, p8 = lane & 7;
    auto issue = [&](v4i (&buf)[UNIT][4]) __attribute__((always_inline)) {
        const int64_t g0 = min64(lgrp, W.groups - 1) * 32 + l8;
        const int start = lu * (UNIT * WS_CHUNK) + 16 * p8;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int8_t* row = P.x + min64(g0 + 8 * t, M - 1) * P.ldx;
#pragma unroll
            for (int c = 0; c < UNIT; ++c) {
                const int off = start + c * WS_CHUNK;
                if (PAD) {
                    const v4i v = *reinterpret_cast<const v4i*>(row + min(off, K - 16));
                    buf[c][t] = off < K ? v : v4i{0, 0, 0, 0};
                } else {
                    buf[c][t] = *reinterpret_cast<const v4i*>(row + off);
                }
            }
        }
        if (++lu == nunits) { lu = 0; lgrp += stride; }
    };
    if (has_work) issue(xa);                            // in flight during the prologue
    bool slow_any, wide_any;

    // ---- prologue: the slab (zero padded to whole units and whole slabs), its parameters, the GELU table; all
    // global loads are issued before anything waits for one of them
    {
        int32_t pb = 1, pc = 1, pbias = 0;
        if (tid < NS && n0 + tid < N) {
            pb = P.rq_b[n0 + tid]; pc = P.rq_c[n0 + tid];
            if (P.bias) pbias = P.bias[n0 + tid];
        }
        const int cpr = nunits * UNIT * (WS_CHUNK / 16);   // 16-byte pieces per padded row
        for (int n = tid >> 3; n < NS; n += WS_THREADS / 8)            // 8 lanes read a 128-byte line of a weight row
            for (int ck = tid & 7; ck < cpr; ck += 8) {
                v4i v = {0, 0, 0, 0};
                if (n0 + n < N && 16 * ck < K) v = *reinterpret_cast<const v4i*>(P.w + (int64_t)(n0 + n) * K + 16 * ck);
                *reinterpret_cast<v4i*>(Wl + row_of_channel<NCB>(n) * pitch + 16 * ck) = v;
            }
        if (tid < NS) { qb_s[tid] = pb; qc_s[tid] = pc; bias_s[tid] = pbias; hb_s[tid] = (int64_t)pbias * pb + (int64_t)((uint32_t)P.rnd << ((pc - 1) & 31)); }
        if (EPI == EPI_GELU && tid < 256) {
            const int32_t I = (int32_t)(int8_t)tid;
            gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c, P.rnd);
        }
        // 24-bit requantisation.  With v = dot + bias, the int8 result clamp8((v b + 2^(c-1)) >> c) is the same for all
        // v >= Lp (127) and all v <= Ln (-127), Lp / Ln being the first v that reach +-127; for b < 2^c the result AT Lp
        // and Ln is exactly +-127.  So v is limited to [Ln, Lp] first, after which T = v b + 2^(c-1) lies in
        // (-128 2^c, 128 2^c) and T 2^(24-c) fits 32 bits with the result in its top byte: one median of three against
        // [Ln - bias, Lp - bias], one 24-bit multiply-add by b 2^(24-c) (the addend, taken modulo 2^32, carries bias and
        // rounding), no shift and no final clamp.  Needs c <= 24, b 2^(24-c) < 2^23 and bounds that fit 24 bits;
        // anything else takes the 64-bit paths below.  (Residual layers: the same with wider bounds and the result one
        // bit lower, see below.)
        // Residual layers: the first term only has to be exact within +-(127 + R2), R2 the largest magnitude of the
        // (per-tensor) residual term, because beyond that the clamped sum is +-127 whatever the residual adds.  With
        // R2 <= 128 the limited first term needs nine bits: it is kept one bit lower, in bits 23..31.
        int64_t wlim = 127;
        int sh24 = 24;
        bool chan_24 = true;
        if (EPI == EPI_RESIDUAL) {
            const int64_t br = P.res_rq.b, cr = P.res_rq.c;
            bool res_ok = br >= 1 && br < (1 << 23) && cr >= 1 && cr <= 30;
            if (res_ok) {
                const int64_t hr = (int64_t)P.rnd << (cr - 1);
                const int64_t r2 = max((127 * br + hr) >> cr, -((-128 * br + hr) >> cr));
                res_ok = r2 <= 128;
                wlim = 127 + r2;
            }
            sh24 = 23;
            chan_24 = res_ok;
        }
        if (tid < NS) {
            int32_t lo = 0, hi = 0, mb = 0, ad = 0;
            if (n0 + tid < N && chan_24) {
                chan_24 = pc >= 1 && pc <= sh24 && pb >= 1 && pb < (1 << ((pc - 1) & 31));
                if (chan_24) {
                    // with h the rounding addend (2^(c-1), or 0 for the bare shift): (v b + h) >> c >= W from
                    // v = ceil((W 2^c - h) / b) on, <= -W up to v = -ceil(((W - 1) 2^c + 1 + h) / b)
                    const int64_t half = (int64_t)P.rnd << (pc - 1), two_c = (int64_t)1 << pc;
                    const int64_t Lp = (wlim * two_c - half + pb - 1) / pb;
                    const int64_t Ln = -(((wlim - 1) * two_c + 1 + half + pb - 1) / pb);
                    const int64_t l = Ln - pbias, h = Lp - pbias;
                    chan_24 = l >= -(1 << 23) && h < (1 << 23);
                    lo = (int32_t)l; hi = (int32_t)h; mb = pb << (sh24 - pc);
                    ad = (int32_t)(uint32_t)((uint64_t)((int64_t)pbias * pb + half) << (sh24 - pc));
                }
            }
            lo_s[tid] = lo; hi_s[tid] = hi; mb_s[tid] = mb; ad_s[tid] = ad;
        }
        wide_any = __syncthreads_and(chan_24) == 0;
        const bool chan_fast = tid >= NS || dyadic_fits32(pb, pc);
        slow_any = __syncthreads_and(chan_fast) == 0;
    }
    if (!has_work) return;
    const bool fast = !slow_any && (EPI != EPI_RESIDUAL || dyadic_fits32(P.res_rq.b, P.res_rq.c));
    const bool fast24 = !wide_any;

    // The accumulators hold the bare dot products: the first MFMA group of a token group takes C = 0, and the bias
    // enters through the 64-bit addend of the requantisation (general path: added explicitly).
    v16i acc[NCB];
    const int8_t* wl_lane = Wl + li * pitch + 64 * lg;
    int cu = 0;                                         // unit of the group being multiplied

    // A unit: per chunk 4 groups of NCB MFMAs.  The chunk after the one being multiplied goes through the staging
    // rows meanwhile (LDS executes a wavefront's accesses in order, so the rows can be overwritten as soon as the
    // reads of the previous chunk have been issued), and the weight fragments of an MFMA group are read while the
    // previous group is multiplied.
    int8_t* st_wr = stage + l8 * XP + 16 * p8;          // where this lane's piece of tokens l8 + 8 t goes
    const int8_t* st_rd = stage + li * XP + 64 * lg;    // MFMA layout: token li, bytes 64 lg + 16 j of the chunk
    auto stage_chunk = [&](const v4i (&ch)[4], v4i (&bf)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t) *reinterpret_cast<v4i*>(st_wr + 8 * t * XP) = ch[t];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < 4; ++j) bf[j] = *reinterpret_cast<const v4i*>(st_rd + 16 * j);
        __builtin_amdgcn_wave_barrier();
    };
    auto consume = [&](const v4i (&buf)[UNIT][4]) __attribute__((always_inline)) {
        const int8_t* wp = wl_lane + cu * (UNIT * WS_CHUNK);
        v4i af[2][NCB], bf[2][4];
        stage_chunk(buf[0], bf[0]);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) af[0][cb] = *reinterpret_cast<const v4i*>(wp + cb * 32 * pitch);
#pragma unroll
        for (int n = 0; n < 4 * UNIT; ++n) {
            if ((n & 3) == 0 && (n >> 2) + 1 < UNIT) stage_chunk(buf[(n >> 2) + 1], bf[((n >> 2) + 1) & 1]);
            if (n + 1 < 4 * UNIT) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    af[(n + 1) & 1][cb] = *reinterpret_cast<const v4i*>(wp + cb * 32 * pitch + ((n + 1) >> 2) * WS_CHUNK + 16 * ((n + 1) & 3));
            }
            if (n == 0 && cu == 0) {
                const v16i zero = {};
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0][cb], bf[0][0], zero, 0, 0, 0);
            } else {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[n & 1][cb], bf[(n >> 2) & 1][n & 3], acc[cb], 0, 0, 0);
            }
        }
    };

    // Requantise the 16 NCB channels of this lane's token and store the group's 32 rows.
    auto finish = [&]() __attribute__((always_inline)) {
        const int64_t tok = cgrp * 32 + li;
        const int nl = 16 * NCB * lg;                   // slab-local first channel of the lane
        if (EPI != EPI_RESIDUAL && fast24) {
            // The asm statements below read the accumulators and get no hazard wait states from the compiler: make
            // sure by hand that the last MFMA (16 passes: 18 wait states) has written them, whatever the scheduler
            // placed in between.  Three instructions per token group.
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_nop 7");
            asm volatile("s_nop 7");
            asm volatile("s_nop 3");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                v4i outv;
#pragma unroll
                for (int w4 = 0; w4 < 4; ++w4) {
                    const v4i lo = *reinterpret_cast<const v4i*>(&lo_s[nl + 16 * cb + 4 * w4]);
                    const v4i hi = *reinterpret_cast<const v4i*>(&hi_s[nl + 16 * cb + 4 * w4]);
                    const v4i mb = *reinterpret_cast<const v4i*>(&mb_s[nl + 16 * cb + 4 * w4]);
                    const v4i ad = *reinterpret_cast<const v4i*>(&ad_s[nl + 16 * cb + 4 * w4]);
                    uint32_t o[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // (an asm statement gets no wait states from the compiler: its input must not come from the
                        // instruction just before; the accumulators were written at least one MFMA group earlier)
                        int32_t m;
                        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(m) : "v"(acc[cb][4 * w4 + r]), "v"(lo[r]), "v"(hi[r]));
                        o[r] = (uint32_t)(__mul24(m, mb[r]) + ad[r]);             // result in the top byte
                        if (EPI == EPI_GELU) o[r] = (uint32_t)gelu_lut[o[r] >> 24];   // result in the low byte
                    }
                    // top (GELU: low) bytes of o[0..3] -> one word
                    const uint32_t p01 = __builtin_amdgcn_perm(o[1], o[0], EPI == EPI_GELU ? 0x0c0c0400u : 0x0c0c0703u);
                    const uint32_t p23 = __builtin_amdgcn_perm(o[3], o[2], EPI == EPI_GELU ? 0x04000c0cu : 0x07030c0cu);
                    outv[w4] = (int)(p01 | p23);
                }
                *reinterpret_cast<v4i*>(stage + li * SP + nl + 16 * cb) = outv;
            }
        } else if (EPI == EPI_RESIDUAL && fast24) {
            // first term limited and taken from bits 23..31 of one 24-bit multiply-add (see the prologue), residual term
            // by a second one (|residual| <= 128, b_r < 2^23), then the sum is clamped
            __builtin_amdgcn_sched_barrier(0);          // as above: asm readers of fresh MFMA results
            asm volatile("s_nop 7");
            asm volatile("s_nop 7");
            asm volatile("s_nop 3");
            __builtin_amdgcn_sched_barrier(0);
            const int32_t rb = P.res_rq.b, rc = P.res_rq.c, rh = P.rnd << ((P.res_rq.c - 1) & 31);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const int64_t rt = min64(tok, M - 1);
                const v4i resv = *reinterpret_cast<const v4i*>(P.residual + rt * N + min(n0 + nl + 16 * cb, N - 16));
                v4i outv;
#pragma unroll
                for (int w4 = 0; w4 < 4; ++w4) {
                    const v4i lo = *reinterpret_cast<const v4i*>(&lo_s[nl + 16 * cb + 4 * w4]);
                    const v4i hi = *reinterpret_cast<const v4i*>(&hi_s[nl + 16 * cb + 4 * w4]);
                    const v4i mb = *reinterpret_cast<const v4i*>(&mb_s[nl + 16 * cb + 4 * w4]);
                    const v4i ad = *reinterpret_cast<const v4i*>(&ad_s[nl + 16 * cb + 4 * w4]);
                    uint32_t o[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int32_t m;
                        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(m) : "v"(acc[cb][4 * w4 + r]), "v"(lo[r]), "v"(hi[r]));
                        const int32_t t1 = (__mul24(m, mb[r]) + ad[r]) >> 23;
                        const int32_t res = (int32_t)(int8_t)((uint32_t)resv[w4] >> (8 * r));
                        const int32_t t2 = (__mul24(res, rb) + rh) >> rc;
                        o[r] = (uint32_t)clamp8(t1 + t2);
                    }
                    const uint32_t p01 = __builtin_amdgcn_perm(o[1], o[0], 0x0c0c0400u);
                    const uint32_t p23 = __builtin_amdgcn_perm(o[3], o[2], 0x04000c0cu);
                    outv[w4] = (int)(p01 | p23);
                }
                *reinterpret_cast<v4i*>(stage + li * SP + nl + 16 * cb) = outv;
            }
        } else if (fast) {
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                v4i resv = {0, 0, 0, 0};
                if (EPI == EPI_RESIDUAL) {              // N % 16 == 0: a 16-channel piece is in or out as a whole
                    const int64_t rt = min64(tok, M - 1);
                    resv = *reinterpret_cast<const v4i*>(P.residual + rt * N + min(n0 + nl + 16 * cb, N - 16));
                }
                v4i outv;
#pragma unroll
                for (int w4 = 0; w4 < 4; ++w4) {
                    const v4i qb = *reinterpret_cast<const v4i*>(&qb_s[nl + 16 * cb + 4 * w4]);
                    const v4i qc = *reinterpret_cast<const v4i*>(&qc_s[nl + 16 * cb + 4 * w4]);
                    const v4i h01 = *reinterpret_cast<const v4i*>(&hb_s[nl + 16 * cb + 4 * w4]);
                    const v4i h23 = *reinterpret_cast<const v4i*>(&hb_s[nl + 16 * cb + 4 * w4 + 2]);
                    uint32_t o[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // (dot + bias) * b + 2^(c-1) in one 64-bit multiply-add, then bits c .. c + 31 (rnd_shift_fit32)
                        const v4i& hh = r < 2 ? h01 : h23;
                        const int64_t hb = (int64_t)(((uint64_t)(uint32_t)hh[2 * (r & 1) + 1] << 32) | (uint32_t)hh[2 * (r & 1)]);
                        const int64_t pr = (int64_t)acc[cb][4 * w4 + r] * qb[r] + hb;
                        int32_t v = (int32_t)__builtin_amdgcn_alignbit((uint32_t)(pr >> 32), (uint32_t)pr, qc[r]);
                        if (EPI == EPI_RESIDUAL) {
                            const int32_t res = (int32_t)(int8_t)((uint32_t)resv[w4] >> (8 * r));
                            v += rnd_shift_fit32(res, P.res_rq.b, P.res_rq.c, P.rnd);
                        }
                        v = clamp8(v);
                        if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                        o[r] = (uint32_t)v;
                    }
                    // low bytes of o[0..3] -> one word (byte selectors 0-3 pick from the second operand, 4-7 from the first)
                    const uint32_t lo = __builtin_amdgcn_perm(o[1], o[0], 0x0c0c0400u);
                    const uint32_t hi = __builtin_amdgcn_perm(o[3], o[2], 0x04000c0cu);
                    outv[w4] = (int)(lo | hi);
                }
                *reinterpret_cast<v4i*>(stage + li * SP + nl + 16 * cb) = outv;
            }
        } else {
            // general dyadic pairs (64-bit rounding): one MFMA tile at a time through the staging buffer as int32,
            // in a rolled loop; this path is rare and kept small rather than fast
            int32_t* st32 = reinterpret_cast<int32_t*>(stage);              // [32 tokens][32 channels] fits 32 SP bytes
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const v16i a = acc[cb];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<v4i*>(st32 + li * 32 + 16 * lg + 4 * q) = v4i{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                __builtin_amdgcn_wave_barrier();
#pragma unroll 1
                for (int e = lane; e < 32 * 32; e += 64) {
                    const int t = e >> 5, c = e & 31;   // token row, channel 16 (c / 16) NCB... see below
                    const int g2 = c >> 4, v2 = c & 15;
                    const int nloc = 16 * NCB * g2 + 16 * cb + v2;
                    const int64_t tk = cgrp * 32 + t;
                    const int n = n0 + nloc;
                    if (tk < M && n < N) {
                        const int32_t a32 = st32[t * 32 + c] + bias_s[nloc];
                        int64_t r64 = rnd_shift64(a32, qb_s[nloc], qc_s[nloc], P.rnd);
                        int32_t v;
                        if (EPI == EPI_RESIDUAL) v = clamp8_64(r64 + rnd_shift64(P.residual[tk * N + n], P.res_rq.b, P.res_rq.c, P.rnd));
                        else v = clamp8_64(r64);
                        if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                        P.y[tk * N + n] = (int8_t)v;
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
            return;
        }
        // The lane's 16-byte pieces lie in 32 different rows; written like that every store instruction would touch
        // 32 memory lines.  Through the staging rows each store instruction writes whole rows instead: 2 NCB
        // adjacent lanes cover the 32 NCB bytes of one token.
        __builtin_amdgcn_wave_barrier();
        constexpr int LPR = 2 * NCB, RPI = 64 / LPR;    // lanes per row, rows per store instruction (NCB = 3: 4 lanes idle)
        const int srow = lane / LPR, piece = lane % LPR;
#pragma unroll
        for (int t = 0; t * RPI < 32; ++t) {
            const int row = t * RPI + srow;
            const bool mine = srow < RPI && row < 32;
            const v4i v = *reinterpret_cast<const v4i*>(stage + (mine ? row : 0) * SP + 16 * piece);
            const int64_t tk = cgrp * 32 + row;
            if (mine && tk < M && n0 + 16 * piece < N) *reinterpret_cast<v4i*>(P.y + tk * N + n0 + 16 * piece) = v;
        }
        __builtin_amdgcn_wave_barrier();
    };

    // true when the wavefront has finished its last group
    auto end_of_unit = [&]() __attribute__((always_inline)) -> bool {
        if (++cu < nunits) return false;
        finish();
        cu = 0;
        cgrp += stride;
        return cgrp >= W.groups;
    };

    for (;;) {
        issue(xb);
        consume(xa);
        if (EVEN) ++cu; else if (end_of_unit()) return;
        issue(xa);
        consume(xb);
        if (end_of_unit()) return;
    }
}

// ------------------------------------------------------------------------------------------------
// Kernel for few rows (small batches, the classifier head): latency, not throughput, is what counts there.  One
// workgroup of four wavefronts computes one 32-token x 32-channel tile; the wavefronts split K between them (k-steps
// w, w + 4, ...), read both operands straight from memory in MFMA layout (16 bytes per lane and k-step; nothing is
// staged or reused, the whole problem is a few hundred tiles), add their partial tiles through LDS, and the first
// wavefront requantises with the general 64-bit formulas and writes the 32 x 32 outputs.
constexpr int SM_WAVES = 4, SM_MAXSTEPS = 8;            // k-steps whose loads are in flight together per wavefront

template <int EPI>
__global__ __launch_bounds__(64 * SM_WAVES) void gemm_small_kernel(GemmParams P) {
    __shared__ int32_t part[SM_WAVES - 1][16][64];      // partial tiles of wavefronts 1..3, [register][lane]
    __shared__ int8_t gelu_lut[256];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int K = P.K, N = P.N;
    const int64_t M = P.M;
    const int tiles_n = (N + 31) / 32;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / tiles_n) * 32;
    const int n0 = (int)(tile % tiles_n) * 32;
    if (EPI == EPI_GELU) {
        const int32_t I = (int32_t)(int8_t)tid;
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c, P.rnd);
    }
    // rows past the end repeat the last one (their results are not stored); K % 32 == 16: the upper half of the last step is zero
    const int8_t* xr = P.x + min64(m0 + li, M - 1) * P.ldx + 16 * lg;
    const int8_t* wr = P.w + (int64_t)min(n0 + li, N - 1) * K + 16 * lg;
    const int nsteps = (K + 31) / 32;
    // the first wavefront's requantisation constants are requested before the operands, not after the multiply
    int32_t qb[16], qc[16], qbias[16];
    if (wv == 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int n = min(n0 + 8 * (i >> 2) + 4 * lg + (i & 3), N - 1);
            qb[i] = P.rq_b[n]; qc[i] = P.rq_c[n]; qbias[i] = P.bias ? P.bias[n] : 0;
        }
    }
    v16i acc = {};
    for (int s0 = wv; s0 < nsteps; s0 += SM_WAVES * SM_MAXSTEPS) {
        v4i xf[SM_MAXSTEPS], wf[SM_MAXSTEPS];
#pragma unroll
        for (int u = 0; u < SM_MAXSTEPS; ++u) {
            const int ks = s0 + u * SM_WAVES;
            const bool in = ks < nsteps && 32 * ks + 16 * lg < K;
            const int off = in ? 32 * ks : 0;
            const v4i xv = *reinterpret_cast<const v4i*>(xr + off - (in ? 0 : 16 * lg));
            const v4i wv4 = *reinterpret_cast<const v4i*>(wr + off - (in ? 0 : 16 * lg));
            xf[u] = in ? xv : v4i{0, 0, 0, 0};
            wf[u] = in ? wv4 : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < SM_MAXSTEPS; ++u) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[u], xf[u], acc, 0, 0, 0);
    }
    if (wv > 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) part[wv - 1][i][lane] = acc[i];
    }
    __syncthreads();
    if (wv > 0) return;
    // lane (li, lg): token m0 + li; register i = 4 q + r is channel n0 + 8 q + 4 lg + r
    const int64_t tok = m0 + li;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * q + r;
            const int n = n0 + 8 * q + 4 * lg + r;
            int32_t a = acc[i] + part[0][i][lane] + part[1][i][lane] + part[2][i][lane];
            if (tok < M && n < N) {
                a += qbias[i];
                const int64_t r64 = rnd_shift64(a, qb[i], qc[i], P.rnd);
                int32_t v;
                if (EPI == EPI_RESIDUAL) v = clamp8_64(r64 + rnd_shift64(P.residual[tok * N + n], P.res_rq.b, P.res_rq.c, P.rnd));
                else v = clamp8_64(r64);
                if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                P.y[tok * N + n] = (int8_t)v;
            }
        }
    }
}

static bool ws_plan(const LinearArgs& a, int& ncb, int& unit, int& nunits, int& pitch, size_t& lds_bytes) {
    if ((a.N & 15) != 0 || (a.K & 15) != 0) return false;
    unit = a.K % (3 * WS_CHUNK) == 0 ? 3 : 1;
    nunits = (a.K + unit * WS_CHUNK - 1) / (unit * WS_CHUNK);
    const int kp = nunits * unit * WS_CHUNK;
    pitch = kp + ((kp / 16) % 2 == 0 ? 16 : 32);        // (pitch / 16) odd: 16 lanes x 16 bytes cover all LDS banks
    // 128-channel slabs halve the activation traffic per MFMA; with fewer than six of them the 64-channel slabs'
    // finer work items fill the wavefronts more evenly
    int ncb0 = (a.N + 127) / 128 >= 6 ? 4 : 2;
    // With many token groups per wavefront (65536 rows and more) the rounds are long enough to be counted: a slab
    // width of 128, 96 or 64 channels is picked by rounds x (tiles per unit + fixed work per unit), which puts the
    // widths of the windowed models' first stages (288 = 3 x 96, 96, 576) on 96-channel slabs without empty tiles.
    const int64_t groups = (a.M + 31) / 32;
    if (groups >= 2048) {
        double best = 0.0;
        for (int n = 4; n >= 2; --n) {
            const int slabs = (a.N + 32 * n - 1) / (32 * n);
            const int64_t waves = (int64_t)WS_WAVES * std::max(1, num_cus() / slabs);
            const double cost = (double)((groups + waves - 1) / waves) * (n + 1.2);
            if (n == 4 || cost < best) { best = cost; ncb0 = n; }
        }
    }
    for (ncb = ncb0; ncb >= 2; --ncb) {
        lds_bytes = (size_t)32 * ncb * pitch + 9 * 4 * 32 * ncb + 256 + (size_t)WS_WAVES * std::max(32 * (32 * ncb + 16), 32 * (WS_CHUNK + 16));
        if (lds_bytes <= (size_t)WS_LDS_MAX) return true;
    }
    return false;
}

template <int EPI, int NCB>
static void launch_ws_ncb(hipStream_t s, const WsParams& W, int unit, int grid, size_t lds_bytes) {
    const dim3 g(grid), b(WS_THREADS);
    if (unit == 3 && W.nunits % 2 == 0) hipLaunchKernelGGL((gemm_ws_kernel<EPI, NCB, 3, false, true>), g, b, lds_bytes, s, W);
    else if (unit == 3) hipLaunchKernelGGL((gemm_ws_kernel<EPI, NCB, 3, false, false>), g, b, lds_bytes, s, W);
    else hipLaunchKernelGGL((gemm_ws_kernel<EPI, NCB, 1, true, false>), g, b, lds_bytes, s, W);
}

template <int EPI>
static void launch_ws(hipStream_t s, const WsParams& W, int ncb, int unit, int grid, size_t lds_bytes) {
    if (ncb == 4) launch_ws_ncb<EPI, 4>(s, W, unit, grid, lds_bytes);
    else if (ncb == 3) launch_ws_ncb<EPI, 3>(s, W, unit, grid, lds_bytes);
    else launch_ws_ncb<EPI, 2>(s, W, unit, grid, lds_bytes);
}

hipError_t launch_linear(hipStream_t s, const LinearArgs& a) {
    if (a.M == 0) return hipSuccess;
    GemmParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.K = a.K; P.ldx = a.ldx ? a.ldx : a.K; P.rnd = a.floor_shift ? 0 : 1;
    P.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles_m = (a.M + BM - 1) / BM;
    P.tiles = tiles_m * P.tiles_n;
    P.per_xcd = (P.tiles + NXCD - 1) / NXCD;
    const int64_t grid = P.per_xcd * NXCD;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t bytes = a.M * a.K + (int64_t)a.N * a.K + a.M * a.N * (a.residual ? 2 : 1) + 8LL * a.N + (a.bias ? 4LL * a.N : 0);
    TraceScope trace(s, a.residual ? KIND_GEMM_RESIDUAL : (a.gelu ? KIND_GEMM_GELU : KIND_GEMM), 2 * a.M * a.N * a.K, bytes);
    // few rows: one workgroup per 32 x 32 tile (a.kernel can keep such shapes on the kernels for many rows)
    const int64_t small_tiles = ((a.M + 31) / 32) * ((a.N + 31) / 32);
    // measured on patches-to-logits forwards at batch 1 and 8: up to one tile per CU it always wins (batch 1: DeiT-S 0.77 ->
    // 0.66 ms, ViT-B 1.11 -> 0.74 ms), beyond that only when K is long enough for the split over the four wavefronts to pay
    // (a single image of a wide model: at most 256 rows)
    // (the kernel with the weights in registers, where it takes the layer, is the faster one beyond one tile per CU:
    // 197 x 3072 x 768: 13.2 -> 10.4 us)
    const bool rs_auto = linear_rs_takes(a) && (!a.residual || (a.K == 768 && a.N % 256 == 0));
    const int64_t small_limit = (int64_t)num_cus() * (a.K >= 768 && a.M <= 256 && !rs_auto ? 3 : 1);
    // (K = 1536 with a whole image's rows: the K-split kernel below is faster, 197 x 384 x 1536: 11.1 -> 9.8 us)
    const bool ks_instead = linear_ks_takes(a) && a.M >= 128;
    if (small_tiles <= small_limit && a.kernel == LINEAR_AUTO && !ks_instead) {
        const dim3 g((unsigned)small_tiles), b(64 * SM_WAVES);
        if (a.residual) hipLaunchKernelGGL(gemm_small_kernel<EPI_RESIDUAL>, g, b, 0, s, P);
        else if (a.gelu) hipLaunchKernelGGL(gemm_small_kernel<EPI_GELU>, g, b, 0, s, P);
        else hipLaunchKernelGGL(gemm_small_kernel<EPI_PLAIN>, g, b, 0, s, P);
        return hipGetLastError();
    }
    // weights in registers: K = 192 / 384 / 768, whatever the one-tile-per-workgroup kernel above leaves (197 rows:
    // fc1 11.2 -> 8.8 us at K = 384, 13.2 -> 10.4 us at K = 768; K = 192, 100352 rows: QKV 39.4 -> 28.1 us, fc1
    // 51.1 -> 36.0 us); measured against
    // the kernels below on the DeiT-S and ViT-B shapes it wins on the layers without a residual (QKV 27.1 -> 21.6 us,
    // fc1 35.5 -> 28.2 us at K = 384; 116 -> 82 us and 179 -> 127 us at K = 768).  With a residual its epilogue costs
    // more instructions per output: at K = 384 it loses (projection 15.8 -> 19.6 us), at K = 768 it wins when the
    // channels fill whole 256-channel slabs (N = 768: 52.6 -> 46.9 us at 50432 rows, 15.1 -> 13.6 us at 4100) and
    // loses otherwise (N = 384: 21.1 -> 23.3 us; N = 192: 33.9 -> 34.5 us)
    if (linear_rs_takes(a) && (a.kernel == LINEAR_REG_STATIONARY || (a.kernel == LINEAR_AUTO && rs_auto)))
        return launch_linear_rs(s, a);
    // K = 1536: the same idea with K split over pairs of wavefronts (gemm_ks.hip).  Both also win on few rows, down to
    // what the one-tile-per-workgroup kernel above takes (394 .. 3152 rows: QKV 10.4 -> 8.2 us, fc2 14.4 -> 10.0 us at
    // the 384-wide model's shapes, 13.2 -> 9.8 us and 13.7 -> 10.4 us at the 768-wide model's)
    if (linear_ks_takes(a) && (a.kernel == LINEAR_REG_STATIONARY || a.kernel == LINEAR_AUTO))
        return launch_linear_ks(s, a);
    int ncb, unit, nunits, pitch; size_t lds_bytes;
    const bool ws = ws_plan(a, ncb, unit, nunits, pitch, lds_bytes);
    // rows too long for the weight-stationary kernels: 256 x 128 tiles with both operands streamed (gemm_tl.hip), when
    // there are tiles for half the compute units at least (6272 x 768 x 3072, 150 tiles: 37.8 -> 31.2 us; with fewer
    // tiles a launch is one tile's latency either way).  Its cost per tile outside the k-loop only pays off for long
    // rows: on the 768-wide model it takes the second MLP layer (K = 3072) from 212 to 148 us and loses at K = 768 (QKV
    // 174 against 124 us with the tiled kernel below)
    if (linear_tl_takes(a) && (a.kernel == LINEAR_BIG_TILES ||
                               (a.kernel == LINEAR_AUTO && !ws && a.K >= 2048 && (a.M + 255) / 256 * (a.N / 128) >= num_cus() / 2)))
        return launch_linear_tl(s, a);
    if (ws) {
        WsParams W;
        W.g = P; W.pitch = pitch; W.nunits = nunits;
        W.slabs = (a.N + 32 * ncb - 1) / (32 * ncb);
        W.groups = (a.M + 31) / 32;
        const int64_t want = (W.groups + WS_WAVES - 1) / WS_WAVES;        // workgroups per slab that still get a group
        W.q = (int)std::max<int64_t>(1, std::min<int64_t>(want, num_cus() / W.slabs));
        const int wgrid = W.q * W.slabs;
        if (a.residual) launch_ws<EPI_RESIDUAL>(s, W, ncb, unit, wgrid, lds_bytes);
        else if (a.gelu) launch_ws<EPI_GELU>(s, W, ncb, unit, wgrid, lds_bytes);
        else launch_ws<EPI_PLAIN>(s, W, ncb, unit, wgrid, lds_bytes);
        return hipGetLastError();
    }
    if (a.residual) hipLaunchKernelGGL(gemm_i8_kernel<EPI_RESIDUAL>, dim3((unsigned)grid), dim3(256), 0, s, P);
    else if (a.gelu) hipLaunchKernelGGL(gemm_i8_kernel<EPI_GELU>, dim3((unsigned)grid), dim3(256), 0, s, P);
    else hipLaunchKernelGGL(gemm_i8_kernel<EPI_PLAIN>, dim3((unsigned)grid), dim3(256), 0, s, P);
    return hipGetLastError();
}

}  // namespace ivit
