// int8 x int8 -> int32 Dense / MatMul on the gfx950 matrix cores with the dyadic requantisation of
// I-ViT (arXiv 2207.01405, Sec. 3.2, Eq. 7-10) fused into the epilogue, optionally with the residual
// add of Eq. 1-2 or with ShiftGELU (Sec. 3.4, Algorithm 2) and its rescale.
//
// Persistent, weight-stationary kernel.  The shapes of a ViT encoder have short K (C or 4C bytes) and
// few output tiles per compute unit, so a kernel that starts a workgroup per tile spends most of its
// time on per-workgroup latencies (launch, parameter loads, the first operand loads).  Here a workgroup
// (256 threads = 4 wavefronts as 2 x 2, two workgroups per CU) owns one slab of 128 output channels and
// walks over token tiles of 128 rows:
//  - the slab's parameters (multiplier, shift, bias) and, when K <= 768, the whole weight slab [128, K]
//    are loaded into LDS once per workgroup; for longer K the weights are streamed like the activations;
//  - activations move global -> registers -> LDS in 64-byte K steps through two LDS buffers, with PD steps
//    in flight in registers; the stream of steps runs across tile boundaries, so the loads of the next
//    tile are in flight during the epilogue of the current one;
//  - each wavefront owns 64 tokens x 64 channels = 2 x 2 tiles of v_mfma_i32_32x32x32_i8 (the int8
//    instruction that reaches the matrix-core peak on gfx950).  The weights are the MFMA "A" operand
//    (rows = output channels) and the activations the "B" operand (columns = tokens), so an accumulator
//    lane holds 16 channels of ONE token per tile; the channel rows are permuted when the weights are
//    written to LDS so that the 32 accumulator registers of a token are 32 consecutive channels, which
//    are requantised, packed and stored as two 16-byte writes per token.
// LDS tiles are [128 rows][64 bytes] without padding; the 16-byte chunk index is XOR-swizzled with
// (row / 4) % 4 so that the 16-byte reads of 16 consecutive rows fall into distinct banks.
// Workgroup ids are remapped so that the workgroups of one XCD (own L2) share a band of token tiles.
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "ivit_kernels.hpp"

namespace ivit {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int TILE = BM * BK;                 // bytes of one K step of one operand tile in LDS
constexpr int NXCD = 8;
constexpr int MAX_WRES_STEPS = 12;            // weight slab resident in LDS up to K = 768
#ifndef IVIT_GEMM_PD
#define IVIT_GEMM_PD 4
#endif
constexpr int PD = IVIT_GEMM_PD;              // K steps kept in flight in registers (even)

enum Epilogue { EPI_PLAIN = 0, EPI_RESIDUAL = 1, EPI_GELU = 2 };

struct GemmParams {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N; int K;
    int tiles_m, tiles_n;                     // token tiles, channel slabs
    int q;                                    // workgroups per channel slab (grid = q * tiles_n)
    int steps;                                // K steps of 64 bytes (the last may be partial)
};

// byte offset of 16-byte chunk `chunk` (0..3) of row `row` (0..127) inside a [128][64] LDS tile
__device__ __forceinline__ int swz(int row, int chunk) { return row * BK + ((chunk ^ ((row >> 2) & 3)) << 4); }

// LDS row (0..63) of channel offset n (0..63) inside a wavefront's 64-channel slab.  MFMA tile ct, row
// i = 8q + 4g + r lands in accumulator register 4q + r of lane group g; storing channel 32g + 16ct + 4q + r
// there gives lane group g the 32 consecutive channels 32g .. 32g + 31 (register index 16ct + 4q + r).
__device__ __forceinline__ int slab_row(int n) {
    return ((n >> 4) & 1) * 32 + ((n >> 2) & 3) * 8 + (n >> 5) * 4 + (n & 3);
}

// Requantise, fuse and store the 2 x 32 outputs of a lane: tokens m, m + 32 and channels n .. n + 31
// (tile-local channel index cl for the staged parameters).  FAST: every channel of the slab has
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

struct Stage { v4i x[2], w[2]; };             // one K step of a thread's share of the operand tiles (w: streamed weights only)

template <int EPI, bool WRES>
__global__ __launch_bounds__(256, 2) void gemm_i8_kernel(GemmParams P) {
    extern __shared__ __align__(16) int8_t lds[];
    const int steps = P.steps;
    int8_t* const Xl = lds;                                   // [2][TILE]
    int8_t* const Wl = lds + 2 * TILE;                        // [steps][TILE] (resident) or [2][TILE] (streamed)
    int32_t* const qb_s = reinterpret_cast<int32_t*>(Wl + (WRES ? steps : 2) * TILE);
    int32_t* const qc_s = qb_s + BN;
    int32_t* const bias_s = qc_s + BN;
    int8_t* const gelu_lut = reinterpret_cast<int8_t*>(bias_s + BN);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int li = lane & 31, lg = lane >> 5;
    const int wm = (wv >> 1) * 64, wn = (wv & 1) * 64;          // wavefront's token / channel offset in the tile
    const int K = P.K, N = P.N;
    const int64_t M = P.M;

    // workgroups of one XCD (ids congruent modulo 8) get consecutive logical ids, i.e. a band of token tiles
    int L = blockIdx.x;
    if (gridDim.x % NXCD == 0) L = (blockIdx.x % NXCD) * (gridDim.x / NXCD) + blockIdx.x / NXCD;
    const int slab = L % P.tiles_n, wi = L / P.tiles_n;         // this workgroup: token tiles wi, wi + q, wi + 2q, ...
    const int n0 = slab * BN;
    const int ntiles = wi < P.tiles_m ? (P.tiles_m - wi + P.q - 1) / P.q : 0;
    if (ntiles == 0) return;
    const int total = ntiles * steps;                           // K steps of all tiles, processed as one stream

    // global -> LDS staging: thread t moves 16 bytes (chunk t % 4) of rows t/4 and t/4 + 64 of each operand tile
    const int ld_row = tid >> 2, ld_c = tid & 3, ld_k = ld_c * 16;
    int xs_off[2], ws_off[2];
    const int8_t* wg[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = ld_row + 64 * p;
        xs_off[p] = swz(r, ld_c);
        ws_off[p] = swz((r & 64) + slab_row(r & 63), ld_c);
        wg[p] = P.w + (int64_t)min(n0 + r, N - 1) * K + ld_k;
    }
    int ld_t = 0, ld_kb = 0;                                    // (tile, K step) of the next stage to load
    auto load_stage = [&](Stage& s) {
        const int64_t mt = (int64_t)(wi + ld_t * P.q) * BM;
        const int koff = ld_kb * BK;
        const bool in = koff + ld_k < K;                        // a partial last step is zero padded per 16 bytes
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int64_t xm = min<int64_t>(mt + ld_row + 64 * p, M - 1);
            s.x[p] = in ? *reinterpret_cast<const v4i*>(P.x + xm * K + koff + ld_k) : v4i{0, 0, 0, 0};
            if (!WRES) s.w[p] = in ? *reinterpret_cast<const v4i*>(wg[p] + koff) : v4i{0, 0, 0, 0};
        }
        if (++ld_kb == steps) { ld_kb = 0; ++ld_t; }
    };
    auto store_stage = [&](const Stage& s, int buf) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            *reinterpret_cast<v4i*>(&Xl[buf * TILE + xs_off[p]]) = s.x[p];
            if (!WRES) *reinterpret_cast<v4i*>(&Wl[buf * TILE + ws_off[p]]) = s.w[p];
        }
    };

    Stage st[PD];
#pragma unroll
    for (int j = 0; j < PD; ++j)
        if (j < total) load_stage(st[j]);

    // once per workgroup: per-channel parameters of the slab, the ShiftGELU table, the resident weight slab.
    // The 32-bit requantisation path is taken only if every channel has 1 <= c <= 31 and 1 <= b <= 2^c.
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
    if (WRES) {
        // the slab [128 rows][steps * 4 chunks of 16 bytes]: batches of eight loads in flight per thread
        const int cpr = steps * 4;                              // chunks per weight row, padded to whole K steps
        const int nchunks = BN * cpr;
        for (int c0 = tid; c0 < nchunks; c0 += 256 * 8) {
            v4i v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 256 * u;
                const int r = c / cpr, kc = c - r * cpr;
                v[u] = v4i{0, 0, 0, 0};
                if (c < nchunks && kc * 16 < K)
                    v[u] = *reinterpret_cast<const v4i*>(P.w + (int64_t)min(n0 + r, N - 1) * K + kc * 16);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 256 * u;
                const int r = c / cpr, kc = c - r * cpr;
                if (c < nchunks)
                    *reinterpret_cast<v4i*>(&Wl[(kc >> 2) * TILE + swz((r & 64) + slab_row(r & 63), kc & 3)]) = v[u];
            }
        }
    }
    store_stage(st[0], 0);
    if (PD < total) load_stage(st[0]);
    const bool fast = __syncthreads_and(chan_fast) != 0;

    // accumulators start at the bias of their channel: register 16 ct + v of lane group g is channel 32 g + 16 ct + v
    const int cl = wn + 32 * lg;
    v16i bias_v[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const v4i t = *reinterpret_cast<const v4i*>(&bias_s[cl + 16 * ct + 4 * q4]);
            bias_v[ct][4 * q4] = t[0]; bias_v[ct][4 * q4 + 1] = t[1]; bias_v[ct][4 * q4 + 2] = t[2]; bias_v[ct][4 * q4 + 3] = t[3];
        }
    v16i acc[2][2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) { acc[ct][0] = bias_v[ct]; acc[ct][1] = bias_v[ct]; }

    auto compute = [&](int xbuf, int wbuf) {
        const int8_t* xb = Xl + xbuf * TILE;
        const int8_t* wb = Wl + wbuf * TILE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i a[2], b[2];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
                a[ct] = *reinterpret_cast<const v4i*>(&wb[swz(wn + 32 * ct + li, 2 * ks + lg)]);
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
                b[tt] = *reinterpret_cast<const v4i*>(&xb[swz(wm + 32 * tt + li, 2 * ks + lg)]);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
                    acc[ct][tt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[ct], b[tt], acc[ct][tt], 0, 0, 0);
        }
    };

    // stream step g is multiplied from LDS buffer g & 1 while step g + 1 moves from its register set (g + 1) % PD
    // to the other buffer; that set is then refilled with step g + 1 + PD.  Unrolled by PD (even) so that register
    // sets and buffers are addressed statically.  After the last K step of a tile the tile is finished in place.
    int kb = 0, t = 0;
    for (int g0 = 0; g0 < total; g0 += PD) {
#pragma unroll
        for (int j = 0; j < PD; ++j) {
            const int g = g0 + j;
            if (g >= total) break;
            compute(j & 1, WRES ? kb : (j & 1));
            if (g + 1 < total) {
                store_stage(st[(j + 1) % PD], (j + 1) & 1);
                if (g + 1 + PD < total) load_stage(st[(j + 1) % PD]);
            }
            if (++kb == steps) {
                const int64_t m = (int64_t)(wi + t * P.q) * BM + wm + li;
                if (fast) epilogue<EPI, true>(P, acc, qb_s, qc_s, gelu_lut, m, n0 + cl, cl);
                else epilogue<EPI, false>(P, acc, qb_s, qc_s, gelu_lut, m, n0 + cl, cl);
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) { acc[ct][0] = bias_v[ct]; acc[ct][1] = bias_v[ct]; }
                kb = 0; ++t;
            }
            __syncthreads();
        }
    }
}

static size_t lds_bytes(int steps, bool wres) { return (size_t)(2 + (wres ? steps : 2)) * TILE + 3 * BN * 4 + 256; }

template <int EPI, bool WRES>
static hipError_t launch_variant(hipStream_t s, const GemmParams& P, int grid) {
    const size_t shmem = lds_bytes(P.steps, WRES);
    // (dynamic LDS beyond 64 KB needs no opt-in on this platform; up to 160 KB per workgroup is available)
    hipLaunchKernelGGL((gemm_i8_kernel<EPI, WRES>), dim3(grid), dim3(256), shmem, s, P);
    hipError_t le = hipGetLastError();
    if (le != hipSuccess && getenv("IVIT_LOG")) fprintf(stderr, "ivit: gemm launch failed: %s (grid %d, lds %zu)\n", hipGetErrorString(le), grid, shmem);
    return le;
}

hipError_t launch_linear(hipStream_t s, const LinearArgs& a) {
    if (a.M == 0) return hipSuccess;
    GemmParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.K = a.K;
    P.tiles_n = (a.N + BN - 1) / BN;
    const int64_t tiles_m = (a.M + BM - 1) / BM;
    if (tiles_m > 0x7fffffffLL) return hipErrorInvalidValue;
    P.tiles_m = (int)tiles_m;
    P.steps = (a.K + BK - 1) / BK;
    const bool wres = P.steps <= MAX_WRES_STEPS;
    // two workgroups per CU when their LDS fits twice, else one; q workgroups share a slab
    const int per_cu = 2 * lds_bytes(P.steps, wres) <= 160 * 1024 ? 2 : 1;
    int64_t q = std::max<int64_t>(1, (int64_t)num_cus() * per_cu / P.tiles_n);
    q = std::min<int64_t>(q, tiles_m);
    if (q >= NXCD) q -= q % NXCD;                 // grid a multiple of the XCD count: the id remap applies
    P.q = (int)q;
    const int64_t grid = q * P.tiles_n;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t bytes = a.M * a.K + (int64_t)a.N * a.K + a.M * a.N * (a.residual ? 2 : 1) + 8LL * a.N + (a.bias ? 4LL * a.N : 0);
    TraceScope trace(s, a.residual ? KIND_GEMM_RESIDUAL : (a.gelu ? KIND_GEMM_GELU : KIND_GEMM), 2 * a.M * a.N * a.K, bytes);
    if (wres) {
        if (a.residual) return launch_variant<EPI_RESIDUAL, true>(s, P, (int)grid);
        if (a.gelu) return launch_variant<EPI_GELU, true>(s, P, (int)grid);
        return launch_variant<EPI_PLAIN, true>(s, P, (int)grid);
    }
    if (a.residual) return launch_variant<EPI_RESIDUAL, false>(s, P, (int)grid);
    if (a.gelu) return launch_variant<EPI_GELU, false>(s, P, (int)grid);
    return launch_variant<EPI_PLAIN, false>(s, P, (int)grid);
}

}  // namespace ivit
