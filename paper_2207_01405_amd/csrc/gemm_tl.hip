// Dense layers with long rows (K of some thousand bytes, e.g. the second MLP layer of the 768-wide model; I-ViT,
// arXiv 2207.01405, Sec. 3.2, Eq. 7-10; residual add of Eq. 1-2; ShiftGELU of Sec. 3.4, Algorithm 2): neither operand
// fits registers or LDS, so both stream through LDS in steps of 128 bytes of K.
//
// A workgroup of four wavefronts (one per SIMD) computes tiles of 256 tokens x 128 channels, one after the other; a
// wavefront owns 128 tokens x 64 channels of the tile (4 x 2 MFMA tiles of 32 x 32, 128 accumulator registers), so a
// k-step reads six 1 KB fragments for eight MFMAs.  (With 64 x 64 per wavefront every MFMA would need 1 KB from LDS;
// and the rate at which a compute unit fills LDS from global memory, about 40 bytes per cycle when whole 128-byte
// lines are requested and half of that with 64-byte pieces, asks for at least this tile area per byte loaded and for
// stages that are a whole line wide.)  Three stages of [256 + 128 rows][128 bytes] are filled by LDS-direct loads two
// and a half stages ahead, also across tile boundaries; rows are stored without padding, the 16-byte pieces of a
// row permuted by an XOR with bits of the row number so that the fragment reads spread over the banks (which piece a
// lane fetches is free with LDS-direct loads, only where it lands is fixed).  One barrier per stage.  The epilogue is
// that of gemm_rs.hip: tokens are the "A" operand, so a lane holds one channel and 16 tokens of an MFMA tile, the
// requantisation constants of its channels sit in registers, and results (and the residual) pass through
// wavefront-private LDS with the transposing LDS read so that global memory sees 16-byte pieces of rows.  That staging
// lives in the buffer of the tile's last stage, whose refill waits until the epilogue is over.
#include "regst_common.hpp"
#include <algorithm>

namespace ivit {

namespace {

using namespace regst;

constexpr int TM = 256, TN = 128, BK = 128, NS = 3;             // tile, bytes of K per stage, stages in LDS
constexpr int KSTEPS = BK / 32;                                 // MFMA k-steps per stage
constexpr int TL_NW = 4;

struct TlParams {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N; int K;
    int tiles_m, tiles_n;
    int rnd;
};

struct TlLayout {
    static constexpr int STG = (TM + TN) * BK;                     // bytes of a stage
    static constexpr int DPW = (TM + TN) * (BK / 16) / 64 / TL_NW;  // load instructions per wavefront and stage
    static constexpr int XI = TM * (BK / 16) / 64 / TL_NW;          // ... of which the first XI fetch activations
    static constexpr int OT = 32 * 2 * OP;                         // output staging tile of a wavefront (two channel tiles)
    static constexpr int RP = 64 + 16, RS16 = RP / 16;             // residual staging: pitch of a token row, 16-byte slots in it
    static constexpr int RNI = (32 * RS16 + 63) / 64;
    static constexpr int RT = RNI * 1024;
    static constexpr int EW = OT + 2 * RT;                         // epilogue staging of a wavefront (inside a stage buffer)
    static constexpr int LUT = NS * STG;
    static constexpr int TOTAL = LUT + 256;
    static_assert(DPW * 64 * TL_NW * 16 == STG && XI * 64 * TL_NW * 16 == TM * BK, "whole load instructions");
    static_assert(DPW >= 8 && KSTEPS == 4 && (NS - 1) * DPW <= 63, "load schedule, wait counts");
    static_assert(TL_NW * EW <= STG && TOTAL + 1024 <= 160 * 1024, "LDS");
};

template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

template <int EPI>
__global__ __launch_bounds__(256) void gemm_tl_kernel(TlParams P) {
    using LY = TlLayout;
    constexpr int STG = LY::STG, DPW = LY::DPW, XI = LY::XI, OT = LY::OT, RP = LY::RP, RS16 = LY::RS16, RNI = LY::RNI, RT = LY::RT;
    constexpr int NW = TL_NW;

    extern __shared__ __align__(1024) int8_t lds[];
    int8_t* gelu_lut = lds + LY::LUT;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wv >> 1, wn = wv & 1;                       // which 128 tokens, which 64 channels of the tile
    const int lj = lane & 31, lg = lane >> 5;
    const int N = P.N, K = P.K;
    const int64_t M = P.M;
    const int S = K / BK;                                      // stages per tile

    // workgroups of one XCD (block id modulo 8) get consecutive logical ids; consecutive tiles share their tokens
    const int G = gridDim.x, xcd = blockIdx.x % NXCD;
    const int L = xcd * (G / NXCD) + min(xcd, G % NXCD) + blockIdx.x / NXCD;
    const int ntiles = P.tiles_m * P.tiles_n;
    if (L >= ntiles) return;                                   // (the same for all wavefronts of a workgroup)
    const int my_tiles = (ntiles - L + G - 1) / G;
    const int total_stages = my_tiles * S;

    if (EPI == EPI_GELU && tid < 256) {
        const int32_t I = (int32_t)(int8_t)tid;
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c, P.rnd);
    }

    // ---- the loads of a stage.  Load instruction n = 4 i + wavefront fills LDS rows 8 n .. 8 n + 7, eight lanes a row:
    // lane l lands in physical piece l % 8 of row 32 i + r, r = 8 wavefront + l / 8, and fetches the piece
    // (l % 8) ^ ((r / 2) % 8) of that row for it.  Rows 0 .. 255 are tokens: row 32 g + r holds token
    // 32 g + token_of_row(r) of the tile; rows 256 .. 383 are channels.
    const uint32_t lds0 = lds_offset(lds) + wv * 1024;
    const int ld_r = 8 * wv + (lane >> 3);
    const int ld_tok = token_of_row(ld_r), ld_col = 16 * ((lane & 7) ^ ((ld_r >> 1) & 7));
    uint32_t w_off[DPW - XI];
#pragma unroll
    for (int i = 0; i < DPW - XI; ++i) w_off[i] = (uint32_t)((32 * i + ld_r) * K + ld_col);
    // the stage being requested: tile, stage inside it, scalar bases, per-lane offsets of the token rows
    int iss_tile = L, iss_s = 0, issued = 0;
    uint32_t x_off[XI];
    const int8_t* iss_x = nullptr; const int8_t* iss_w = nullptr;
    auto issue_setup = [&]() __attribute__((always_inline)) {  // a new tile on the request side
        const int tm = iss_tile / P.tiles_n, tn = iss_tile % P.tiles_n;
        const int64_t m0 = (int64_t)tm * TM;
        const int last = (int)min64(M - m0, TM) - 1;           // rows past the matrix repeat its last row; never stored
        iss_x = uniform_ptr(P.x + m0 * K);
        iss_w = uniform_ptr(P.w + (int64_t)tn * TN * K);
#pragma unroll
        for (int i = 0; i < XI; ++i) x_off[i] = (uint32_t)(min(32 * i + ld_tok, last) * K + ld_col);
    };
    auto issue_one = [&](int i, int buf) __attribute__((always_inline)) {   // load instruction i of the stage being requested
        const uint32_t dst = lds0 + buf * STG + i * (NW * 1024);
        if (i < XI) dma16(iss_x, x_off[i], dst); else dma16(iss_w, w_off[i - XI], dst);
    };
    auto issue_done = [&]() __attribute__((always_inline)) {       // on to the next stage
        ++issued; iss_x += BK; iss_w += BK;
        if (++iss_s == S) { iss_s = 0; iss_tile += G; if (issued < total_stages) issue_setup(); }
    };
    issue_setup();
#pragma unroll 1
    for (int g = 0; g < NS && g < total_stages; ++g) {
#pragma unroll
        for (int i = 0; i < DPW; ++i) issue_one(i, g);
        issue_done();
    }

    // ---- fragment reads: piece 2 kk + lg of row R, at its permuted place
    int sw[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) sw[kk] = 16 * ((2 * kk + lg) ^ ((lj >> 1) & 7));
    const int a_row0 = (wm * 128 + lj) * BK, b_row0 = (TM + wn * 64 + lj) * BK;
    v4i fa[KSTEPS][4], fb[KSTEPS][2];                           // [k-step of a stage][MFMA tile]; fetched two k-steps ahead
    auto read_frags = [&](int buf, int kk) __attribute__((always_inline)) {
        const int8_t* st = lds + buf * STG;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) fa[kk][mt] = *reinterpret_cast<const v4i*>(st + a_row0 + mt * 32 * BK + sw[kk]);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) fb[kk][nt] = *reinterpret_cast<const v4i*>(st + b_row0 + nt * 32 * BK + sw[kk]);
    };

    // ---- epilogue state (as in gemm_rs.hip with two channel tiles per wavefront)
    int rs_row[RNI], rs_colo[RNI];
#pragma unroll
    for (int i = 0; i < RNI; ++i) {
        const int s = 64 * i + lane;
        rs_row[i] = min(s / RS16, 31);
        rs_colo[i] = wn * 64 + 16 * min(s % RS16, 3);
    }
    const int rr_base = ((lane >> 5) * 16 + ((lane & 15) >> 1)) * RP + 16 * ((lane >> 4) & 1) + 8 * (lane & 1);
    int st_src[2];
    uint32_t st_dst[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int B = lane >> 4, o_src = lane & 1, b = (lane & 15) >> 1, o_dst = (lane >> 3) & 1, j = lane & 7;
        const int hs = 8 * s + 2 * B + o_src, hd = 8 * s + 2 * B + o_dst;
        st_src[s] = (16 * (hs % 4) + b) * OP + 8 * (hs / 4);
        st_dst[s] = (uint32_t)((8 * (hd / 4) + j) * N + 16 * (hd % 4));
    }
    const int32_t rb = P.res_rq.b, rc = P.res_rq.c, rh = P.rnd << ((P.res_rq.c - 1) & 31);
    int64_t wlim = 127;
    int sh24 = 24;
    bool res_24 = true;
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
        res_24 = res_ok;
    }

    v16i acc[4][2];
    __syncthreads();                                            // the ShiftGELU table
    // the first stage
    {
        if (total_stages >= 3) wait_vm<2 * DPW>(); else if (total_stages == 2) wait_vm<DPW>(); else wait_vm0();
        __syncthreads();
        read_frags(0, 0);
        read_frags(0, 1);
    }

    int g = 0, cur = 0;                                         // stage being multiplied (counted over all tiles), its buffer
#pragma unroll 1
    for (int t = L; t < ntiles; t += G) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = v16i{};
        int held = 0;
#pragma unroll 1
        for (int s = 0; s < S; ++s, ++g) {
            // ---- first half of the stage: fetch the fragments of its second half, multiply
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                read_frags(cur, kk + 2);
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[kk][mt], fb[kk][nt], acc[mt][nt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- second half: the next stage has to be there (loads complete in order: all but those of the one stage
            // that may have been requested after it), and once every wavefront is here nobody reads this stage's buffer
            // any more (all its fragments are in registers: the barrier waits for the LDS reads too)
            if (issued - (g + 2) >= 1) wait_vm<DPW>(); else wait_vm0();
            __syncthreads();
            const int nxt = cur + 1 == NS ? 0 : cur + 1;
            const bool more = g + 1 < total_stages;
            // stage g + NS goes into the buffer of stage g; after the last stage of a tile the epilogue borrows that
            // buffer first
            const bool req = issued < total_stages && s + 1 < S;
#pragma unroll
            for (int kk = 2; kk < 4; ++kk) {
                if (more) read_frags(nxt, kk - 2);
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[kk][mt], fb[kk][nt], acc[mt][nt], 0, 0, 0);
                    if (req) {
#pragma unroll
                        for (int i = 0; i < DPW; ++i)
                            if (i * 8 / DPW == (kk - 2) * 4 + mt) issue_one(i, cur);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (req) issue_done();
            held = cur;
            cur = nxt;
        }

        // ---- epilogue of tile t: this wavefront's 4 x 2 MFMA tiles, one group of 32 tokens at a time
        const int tm = t / P.tiles_n, tn = t % P.tiles_n;
        const int n0w = tn * TN + wn * 64;
        const int64_t row_w = (int64_t)tm * TM + wm * 128;      // first token of the wavefront's part
        int8_t* out_w = lds + held * STG + wv * LY::EW;         // staging: the buffer of the tile's last stage
        int8_t* res_w = out_w + OT;
        const uint32_t res_off = lds_offset(res_w);
        // requantisation constants of the lane's two channels (24-bit form, derivation in gemm_rs.hip)
        int32_t c_lo[2], c_hi[2], c_mb[2], c_ad[2], pb[2], pc[2], pbias[2];
        bool chan_24 = res_24;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int ch = n0w + 32 * cb + lj;
            pb[cb] = P.rq_b[ch]; pc[cb] = P.rq_c[ch]; pbias[cb] = P.bias ? P.bias[ch] : 0;
        }
        // the residual tiles of the first two token groups, while the constants are worked out
        auto res_span_issue = [&](int mt, int half) __attribute__((always_inline)) {
            const int64_t r0 = row_w + 32 * mt;
            const int rows = (int)max64(min64(M - r0, 32), 0);
            const int8_t* base = uniform_ptr(rows > 0 ? P.residual + r0 * N : P.residual + (M - 1) * N);
            const int last = __builtin_amdgcn_readfirstlane(max(rows, 1) - 1);
#pragma unroll
            for (int i = 0; i < RNI; ++i)
                dma16(base, (uint32_t)(__mul24(min(rs_row[i], last), N) + n0w - wn * 64 + rs_colo[i]), res_off + half * RT + i * 1024);
        };
        if (EPI == EPI_RESIDUAL) { res_span_issue(0, 0); res_span_issue(1, 1); }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            int32_t lo = 0, hi = 0, mb = 0, ad = 0;
            bool ok = chan_24 && pc[cb] >= 1 && pc[cb] <= sh24 && pb[cb] >= 1 && pb[cb] < (1 << ((pc[cb] - 1) & 31));
            if (ok) {
                const int64_t half = (int64_t)P.rnd << (pc[cb] - 1), two_c = (int64_t)1 << pc[cb];
                const int64_t Lp = (int64_t)((uint32_t)(wlim * two_c - half + pb[cb] - 1) / (uint32_t)pb[cb]);
                const int64_t Ln = -(int64_t)((uint32_t)((wlim - 1) * two_c + 1 + half + pb[cb] - 1) / (uint32_t)pb[cb]);
                const int64_t l = Ln - pbias[cb], h = Lp - pbias[cb];
                ok = l >= -(1 << 23) && h < (1 << 23);
                lo = (int32_t)l; hi = (int32_t)h; mb = pb[cb] << (sh24 - pc[cb]);
                ad = (int32_t)(uint32_t)((uint64_t)((int64_t)pbias[cb] * pb[cb] + half) << (sh24 - pc[cb]));
            }
            chan_24 = chan_24 && ok;
            c_lo[cb] = lo; c_hi[cb] = hi; c_mb[cb] = mb; c_ad[cb] = ad;
        }
        // (nothing in the epilogue is shared between wavefronts: each decides for itself)
        const bool fast24 = __builtin_amdgcn_ballot_w64(chan_24) == ~0ull;
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");  // the last MFMAs have written the accumulators (asm readers below)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            v2i rw[2][2] = {};
            if (EPI == EPI_RESIDUAL) {
                // its residual tile has landed: requested two token groups earlier, and what was requested after it is
                // the next group's residual tile and the stores of the groups in between
                if (mt == 0) wait_vm<RNI>(); else if (mt == 1) wait_vm<RNI + 2>(); else if (mt == 2) wait_vm<RNI + 4>(); else wait_vm<4>();
                const int8_t* tr = res_w + (mt & 1) * RT + rr_base;
#pragma unroll
                for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        rw[cb][h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(tr + 8 * h * RP + 32 * cb));
            }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                v4i ow;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t o[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int32_t a = acc[mt][cb][4 * d + r];
                        if (fast24) {
                            const int32_t m = med3(a, c_lo[cb], c_hi[cb]);
                            if (EPI == EPI_RESIDUAL) {
                                const int32_t t1 = (__mul24(m, c_mb[cb]) + c_ad[cb]) >> 23;
                                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[cb][d >> 1][d & 1] >> (8 * r));
                                const int32_t t2 = (__mul24(res, rb) + rh) >> rc;
                                o[r] = (uint32_t)clamp8(t1 + t2) & 0xffu;
                            } else {
                                o[r] = (uint32_t)(__mul24(m, c_mb[cb]) + c_ad[cb]) >> 24;
                                if (EPI == EPI_GELU) o[r] = (uint32_t)(uint8_t)gelu_lut[o[r]];
                            }
                        } else {
                            int64_t r64 = rnd_shift64(a + pbias[cb], pb[cb], pc[cb], P.rnd);
                            if (EPI == EPI_RESIDUAL) {
                                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[cb][d >> 1][d & 1] >> (8 * r));
                                r64 += rnd_shift64(res, P.res_rq.b, P.res_rq.c, P.rnd);
                            }
                            int32_t v = clamp8_64(r64);
                            if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                            o[r] = (uint32_t)v & 0xffu;
                        }
                    }
                    ow[d] = (int)(o[0] | (o[1] << 8) | (o[2] << 16) | (o[3] << 24));
                }
                *reinterpret_cast<v4i*>(out_w + (32 * cb + lj) * OP + 16 * lg) = ow;
            }
            if (EPI == EPI_RESIDUAL && mt + 2 < 4) {            // (its half has been read: the values are in use above)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                res_span_issue(mt + 2, mt & 1);
            }
            const int64_t r0 = row_w + 32 * mt;
            const int rows = __builtin_amdgcn_readfirstlane((int)max64(min64(M - r0, 32), 0));
            const __amdgpu_buffer_rsrc_t y_buf =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uniform_ptr(P.y + r0 * N + n0w)), 0, rows * N, 0x00020000);
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const v2i a = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src[s2]));
                const v2i b = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src[s2] + 8 * OP));
                __builtin_amdgcn_raw_buffer_store_b128(v4i{a[0], a[1], b[0], b[1]}, y_buf, (int)st_dst[s2], 0, 0);
            }
        }
        // the held-back stage, once no wavefront uses the staging any more
        if (issued < total_stages) {
            __syncthreads();
#pragma unroll
            for (int i = 0; i < DPW; ++i) issue_one(i, held);
            issue_done();
        }
    }
    wait_vm0();
}

template <int EPI>
hipError_t launch_tl(hipStream_t s, const TlParams& P, int grid) {
    constexpr size_t lds_bytes = TlLayout::TOTAL;
    hipLaunchKernelGGL((gemm_tl_kernel<EPI>), dim3(grid), dim3(256), lds_bytes, s, P);
    return hipGetLastError();
}

}  // namespace

// Shapes this kernel takes: K a multiple of 128 and at least three stages long, N a multiple of 128, dense rows;
// offsets inside a tile are 32-bit.
bool linear_tl_takes(const LinearArgs& a) {
    if (a.K < NS * BK || (a.K % BK) != 0 || (a.N % TN) != 0) return false;
    if ((int64_t)TM * a.K > 0x7fffffffLL || (int64_t)TN * a.K > 0x7fffffffLL || (int64_t)32 * a.N > 0x7fffffffLL) return false;
    if ((a.M + TM - 1) / TM * (a.N / TN) > 0x7fffffffLL) return false;
    return (a.ldx == 0 || a.ldx == a.K) && a.M >= 1;
}

hipError_t launch_linear_tl(hipStream_t s, const LinearArgs& a) {
    TlParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.K = a.K; P.rnd = a.floor_shift ? 0 : 1;
    P.tiles_m = (int)((a.M + TM - 1) / TM); P.tiles_n = a.N / TN;
    const int grid = (int)std::min<int64_t>((int64_t)P.tiles_m * P.tiles_n, num_cus());
    if (a.residual) return launch_tl<EPI_RESIDUAL>(s, P, grid);
    if (a.gelu) return launch_tl<EPI_GELU>(s, P, grid);
    return launch_tl<EPI_PLAIN>(s, P, grid);
}

}  // namespace ivit
