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
// wavefront-private LDS with the transposing LDS read so that global memory sees 16-byte pieces of rows.
//
// With one wavefront per SIMD nothing else runs while a wavefront works through its epilogue, about a third of a tile's
// time at K = 3072.  So the finished accumulators move to a second register set (the accumulators of the tile being
// multiplied live in AGPRs) and their epilogue rides along with the next tile's first eighteen stages, half a result
// between two pairs of MFMAs; the residual values arrive one MFMA tile at a time through a 1 KB slot per wavefront,
// requested two stages ahead.  Tiles with fewer than eighteen stages, the last tile of a workgroup and parameters
// outside the 24-bit form take the epilogue alone, between two tiles.  Measured on 50432 x 768 x 3072 (one session):
// tiled kernel of gemm_i8.hip 212 us, this kernel with 64-byte stages 186 us, with 128-byte stages 162 us, with the
// epilogue riding along 150 us; without its loads 130 us, without loads and fragment reads 109 us: the one
// instruction stream per SIMD is what bounds it.
#include "regst_common.hpp"
#include <algorithm>
#include <type_traits>
#include <utility>

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
    static constexpr int OPT = 32;                                 // output staging of a wavefront: [64 channels][32 tokens]
    static constexpr int OT = 64 * OPT;
    static constexpr int RT = 32 * 32;                             // residual staging of a wavefront: [32 tokens][32 channels]
    static constexpr int LUT = NS * STG, OUT = LUT + 256, RES = OUT + TL_NW * OT;
    static constexpr int TOTAL = RES + TL_NW * RT;
    static_assert(DPW * 64 * TL_NW * 16 == STG && XI * 64 * TL_NW * 16 == TM * BK, "whole load instructions");
    static_assert(DPW >= 8 && KSTEPS == 4 && 2 * DPW + 2 <= 63, "load schedule, wait counts");
    static_assert(TOTAL + 1024 <= 160 * 1024, "LDS");
};

template <int N, class F> __device__ __forceinline__ void static_for(F&& f) {
    [&]<int... I>(std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>()), ...); }(std::make_integer_sequence<int, N>());
}
template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

template <int EPI>
__global__ __launch_bounds__(256) void gemm_tl_kernel(TlParams P) {
    using LY = TlLayout;
    constexpr int STG = LY::STG, DPW = LY::DPW, XI = LY::XI;
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
    // on to the next stage; after the last one the request side stays where it is, and the loads that the remaining
    // stages still issue (every stage issues its twelve, which keeps the wait counts fixed) fetch that stage again,
    // into a buffer nobody reads any more
    auto issue_done = [&]() __attribute__((always_inline)) {
        if (++issued < total_stages) {
            iss_x += BK; iss_w += BK;
            if (++iss_s == S) { iss_s = 0; iss_tile += G; issue_setup(); }
        }
    };
    issue_setup();
#pragma unroll 1
    for (int g = 0; g < NS; ++g) {                              // (a tile has three stages at least)
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

    // ---- epilogue state.  The epilogue of a tile runs while the next tile is multiplied: its accumulators move to a
    // second set of registers (prev), and the 16 half-units of work (a unit is one MFMA tile of 32 tokens x 32 channels;
    // eight per wavefront) are spread over the k-steps of 16 stages, two results a k-step.
    int8_t* out_w = lds + LY::OUT + wv * LY::OT;               // [64 channels][32 tokens] of one token group
    int8_t* res_w = lds + LY::RES + wv * LY::RT;               // [32 tokens][32 channels] of one unit
    const uint32_t res_off = lds_offset(res_w);
    const int rr_base = ((lane >> 5) * 16 + ((lane & 15) >> 1)) * 32 + 16 * ((lane >> 4) & 1) + 8 * (lane & 1);
    int st_src[2];
    uint32_t st_dst[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int B = lane >> 4, o_src = lane & 1, b = (lane & 15) >> 1, o_dst = (lane >> 3) & 1, j = lane & 7;
        const int hs = 8 * s + 2 * B + o_src, hd = 8 * s + 2 * B + o_dst;
        st_src[s] = (16 * (hs % 4) + b) * LY::OPT + 8 * (hs / 4);
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
    // of the tile whose results wait in prev
    int64_t p_row = 0;                                          // first token of the wavefront's part
    int p_n0 = 0;                                               // first channel
    int32_t c_lo[2], c_hi[2], c_mb[2], c_ad[2], pb[2], pc[2], pbias[2];
    bool fast24 = false;
    v2i rw[2] = {};                                             // the unit's residual values, as the accumulators lie
    v4i ow = {};                                                // its results, four tokens a register

    v16i acc[4][2], prev[4][2];

    // the residual values of unit u = 2 mt + cb: one load instruction, two lanes a token
    auto res_issue = [&](int u) __attribute__((always_inline)) {
        const int64_t r0 = p_row + 32 * (u >> 1);
        const int rows = (int)max64(min64(M - r0, 32), 0);
        const int8_t* base = uniform_ptr(rows > 0 ? P.residual + r0 * N : P.residual + (M - 1) * N);
        const int last = __builtin_amdgcn_readfirstlane(max(rows, 1) - 1);
        dma16(base, (uint32_t)(__mul24(min(lane >> 1, last), N) + p_n0 + 32 * (u & 1) + 16 * (lane & 1)), res_off);
    };
    auto res_read = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
            rw[h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(res_w + rr_base + 8 * h * 32));
    };
    // constants of the tile in prev: requantisation in the 24-bit form (derivation in gemm_rs.hip) where every channel of
    // the wavefront admits it
    auto epi_begin = [&]() __attribute__((always_inline)) {
        bool chan_24 = res_24;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int ch = p_n0 + 32 * cb + lj;
            pb[cb] = P.rq_b[ch]; pc[cb] = P.rq_c[ch]; pbias[cb] = P.bias ? P.bias[ch] : 0;
        }
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
        fast24 = __builtin_amdgcn_ballot_w64(chan_24) == ~0ull;
    };
    // results 4 d + r0 and 4 d + r0 + 1 of unit (mt, cb), 24-bit form
    auto epi_pair = [&](auto mtc, auto cbc, auto dc, auto r0c) __attribute__((always_inline)) {
        constexpr int mt = decltype(mtc)::value, cb = decltype(cbc)::value, d = decltype(dc)::value, r0 = decltype(r0c)::value;
#pragma unroll
        for (int r = r0; r < r0 + 2; ++r) {
            const int32_t m = med3(prev[mt][cb][4 * d + r], c_lo[cb], c_hi[cb]);
            uint32_t o;
            if (EPI == EPI_RESIDUAL) {
                const int32_t t1 = (__mul24(m, c_mb[cb]) + c_ad[cb]) >> 23;
                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[d >> 1][d & 1] >> (8 * r));
                const int32_t t2 = (__mul24(res, rb) + rh) >> rc;
                o = (uint32_t)clamp8(t1 + t2) & 0xffu;
            } else {
                o = (uint32_t)(__mul24(m, c_mb[cb]) + c_ad[cb]) >> 24;
                if (EPI == EPI_GELU) o = (uint32_t)(uint8_t)gelu_lut[o];
            }
            if (r == 0) ow[d] = (int)o; else ow[d] |= (int)(o << (8 * r));
        }
    };
    // the same in 64-bit arithmetic, a whole unit
    auto epi_unit_slow = [&](auto mtc, auto cbc) __attribute__((always_inline)) {
        constexpr int mt = decltype(mtc)::value, cb = decltype(cbc)::value;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int64_t r64 = rnd_shift64(prev[mt][cb][4 * d + r] + pbias[cb], pb[cb], pc[cb], P.rnd);
                if (EPI == EPI_RESIDUAL) {
                    const int32_t res = (int32_t)(int8_t)((uint32_t)rw[d >> 1][d & 1] >> (8 * r));
                    r64 += rnd_shift64(res, P.res_rq.b, P.res_rq.c, P.rnd);
                }
                int32_t v = clamp8_64(r64);
                if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
                o[r] = (uint32_t)v & 0xffu;
            }
            ow[d] = (int)(o[0] | (o[1] << 8) | (o[2] << 16) | (o[3] << 24));
        }
    };
    // a finished unit goes to the staging tile; with the second unit of a token group the group goes to global memory
    auto epi_put = [&](auto mtc, auto cbc) __attribute__((always_inline)) {
        constexpr int mt = decltype(mtc)::value, cb = decltype(cbc)::value;
        *reinterpret_cast<v4i*>(out_w + (32 * cb + lj) * LY::OPT + 16 * lg) = ow;
        if (cb == 1) {
            const int64_t r0 = p_row + 32 * mt;
            const int rows = __builtin_amdgcn_readfirstlane((int)max64(min64(M - r0, 32), 0));
            const __amdgpu_buffer_rsrc_t y_buf =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uniform_ptr(P.y + r0 * N + p_n0)), 0, rows * N, 0x00020000);
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const v2i a = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src[s2]));
                const v2i b = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src[s2] + 8 * LY::OPT));
                __builtin_amdgcn_raw_buffer_store_b128(v4i{a[0], a[1], b[0], b[1]}, y_buf, (int)st_dst[s2], 0, 0);
            }
        }
    };
    // the whole epilogue of the tile in prev, nothing else going on (short rows, the last tile, or 64-bit arithmetic)
    auto epi_alone = [&]() __attribute__((always_inline)) {
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");  // (the last MFMAs have written their results)
        static_for<8>([&](auto uc) __attribute__((always_inline)) {
            constexpr int u = decltype(uc)::value;
            const std::integral_constant<int, u / 2> mtc; const std::integral_constant<int, u % 2> cbc;
            if (EPI == EPI_RESIDUAL) {
                if (u > 0) res_issue(u);                        // (unit 0 was requested when the tile ended)
                wait_vm0();
                res_read();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // before the next unit's values overwrite the slot
            }
            if (fast24) {
                static_for<8>([&](auto qc) __attribute__((always_inline)) {
                    constexpr int q = decltype(qc)::value;
                    epi_pair(mtc, cbc, std::integral_constant<int, q / 2>(), std::integral_constant<int, 2 * (q % 2)>());
                });
            } else {
                epi_unit_slow(mtc, cbc);
            }
            epi_put(mtc, cbc);
        });
    };

    __syncthreads();                                            // the ShiftGELU table
    // the first stage
    {
        wait_vm<2 * DPW>();
        __syncthreads();
        read_frags(0, 0);
        read_frags(0, 1);
    }

    int cur = 0;                                                // buffer of the stage being multiplied
    constexpr bool RES = EPI == EPI_RESIDUAL;
    // One stage.  U = -1: nothing else; U = 0 .. 15: half-unit U of the epilogue of the tile in prev rides along (unit
    // U / 2, results 8 (U % 2) .. + 7 of a lane).  Other vector memory instructions of the epilogue, all before the
    // stage's own loads: with the first half of unit u the request for the residual values of unit u + 1; and after
    // the second half of a token group's second unit two stores (epi_put, called by the tile loop).
    int32_t tq = 0, oq[3] = {};                                 // a result half done; the results waiting for the fourth of their register
    auto stage = [&](auto uc) __attribute__((always_inline)) {
        constexpr int U = decltype(uc)::value;
        constexpr bool EP = U >= 0;
        constexpr int unit = EP ? U / 2 : 0, ph = EP ? U % 2 : 0, emt = unit / 2, cb = unit % 2;
        auto extras = [](int u) constexpr {
            if (u < 0) return 0;
            return u % 2 == 0 ? (RES && u / 2 < 7 ? 1 : 0) : ((u / 2) % 2 == 1 ? 2 : 0);
        };
        const int nxt = cur + 1 == NS ? 0 : cur + 1;
        if (EP && ph == 0 && RES) {
            // requested two stages ago, before the loads of those stages and the stores of the stage between
            wait_vm<2 * DPW + extras(U - 1)>();
            res_read();
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk == 2) {
                // the next stage has to be there (loads complete in order; younger than the loads of stage g + 1 are the
                // stores after the stage before last, the request of the last stage, its loads, the stores after it, the
                // request of this stage), and once every wavefront is here nobody reads this stage's buffer any more (all
                // its fragments are in registers: the barrier waits for the LDS reads too)
                wait_vm<DPW + (U >= 2 && U % 2 == 1 ? extras(U - 2) : 0) + (U >= 1 ? extras(U - 1) : 0) + extras(U)>();
                __syncthreads();
            }
            read_frags(kk < 2 ? cur : nxt, (kk + 2) % 4);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[kk][mt], fb[kk][nt], acc[mt][nt], 0, 0, 0);
                if (kk >= 2) {                                  // stage g + NS goes into the buffer of stage g
#pragma unroll
                    for (int i = 0; i < DPW; ++i)
                        if (i * 8 / DPW == (kk - 2) * 4 + mt) issue_one(i, cur);
                }
                if (EP) {
                    // half a result per pair of MFMAs, each half ending in a statement that keeps it in its place; the
                    // four results of a register are put together by two byte permutes
                    const int v = 2 * kk + (mt >> 1), d = 2 * ph + (v >> 2), r = v & 3;     // (constants once the loops are unrolled)
                    if ((mt & 1) == 0) {
                        const int32_t m = med3(prev[emt][cb][4 * d + r], c_lo[cb], c_hi[cb]);
                        if (RES) tq = (__mul24(m, c_mb[cb]) + c_ad[cb]) >> 23;
                        else tq = __mul24(m, c_mb[cb]) + c_ad[cb];                          // result in the top byte
                        if (EPI == EPI_GELU) tq = (int32_t)(uint8_t)gelu_lut[(uint32_t)tq >> 24];   // result in the low byte
                        asm volatile("" : "+v"(tq));
                    } else {
                        int32_t o = tq;
                        if (RES) {
                            const int32_t res = (int32_t)(int8_t)((uint32_t)rw[d >> 1][d & 1] >> (8 * r));
                            const int32_t t2 = (__mul24(res, rb) + rh) >> rc;
                            o = clamp8(tq + t2);                                            // result in the low byte
                        }
                        if (r == 3) {
                            constexpr bool low = EPI != EPI_PLAIN;
                            const uint32_t p01 = __builtin_amdgcn_perm((uint32_t)oq[1], (uint32_t)oq[0], low ? 0x0c0c0400u : 0x0c0c0703u);
                            const uint32_t p23 = __builtin_amdgcn_perm((uint32_t)o, (uint32_t)oq[2], low ? 0x04000c0cu : 0x07030c0cu);
                            o = (int32_t)(p01 | p23);
                            asm volatile("" : "+v"(o));
                            ow[d] = o;
                        } else {
                            asm volatile("" : "+v"(o));
                            oq[r] = o;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (EP && kk == 0 && ph == 0 && RES && unit < 7) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // this unit's values are in registers
                res_issue(unit + 1);
            }
        }
        issue_done();
        cur = nxt;
    };

    bool have_prev = false;
#pragma unroll 1
    for (int it = 0; it <= my_tiles; ++it) {
        const bool tile = it < my_tiles;
        bool ride = false;                                      // the epilogue rides along with this tile's stages
        if (have_prev) {
            epi_begin();
            ride = tile && fast24 && S >= 18;
            if (!ride) epi_alone();
        }
        if (!tile) break;
        const int t = L + it * G;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = v16i{};
        int s = 0;
        if (ride) {
            stage(std::integral_constant<int, -1>());
            stage(std::integral_constant<int, -1>());
            static_for<16>([&](auto uc) __attribute__((always_inline)) {
                stage(uc);
                if (decltype(uc)::value % 2 == 1) epi_put(std::integral_constant<int, decltype(uc)::value / 4>(),
                                                          std::integral_constant<int, (decltype(uc)::value / 2) % 2>());
            });
            s = 18;
        }
#pragma unroll 1
        for (; s < S; ++s) stage(std::integral_constant<int, -1>());

        // the tile's results wait in prev for their epilogue; its first residual values are on their way
        const int tm = t / P.tiles_n, tn = t % P.tiles_n;
        p_row = (int64_t)tm * TM + wm * 128;
        p_n0 = tn * TN + wn * 64;
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) prev[mt][nt] = acc[mt][nt];
        if (RES) res_issue(0);
        have_prev = true;
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
    if ((int64_t)TM * a.K > 0x7fffffffLL || (int64_t)TN * a.K > 0x7fffffffLL || a.N >= (1 << 23)) return false;   // (N is a 24-bit factor)
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
