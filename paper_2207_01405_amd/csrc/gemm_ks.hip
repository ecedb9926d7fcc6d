// Dense layers with K = 1536 (the second MLP layer of the 384-wide models; I-ViT, arXiv 2207.01405, Sec. 3.2,
// Eq. 7-10; residual add of Eq. 1-2; ShiftGELU of Sec. 3.4, Algorithm 2): weights in registers, K split over pairs of
// wavefronts.
//
// A row of K = 1536 bytes is too long for a wavefront to keep the weights of two channel tiles in registers, and with
// one tile every 1 KB fragment of activations read from LDS would feed a single MFMA, which the LDS cannot sustain.
// So the four wavefronts of a workgroup (one per SIMD) form two pairs; a pair owns two tiles of 32 output channels, and
// each of its wavefronts keeps HALF of K of both tiles in accumulation registers (2 x 32 channels x 768 bytes).  Both
// read their half of the 32-token tile's activations from LDS (a fragment feeds two MFMAs) and end with partial sums of
// both channel tiles; each then hands the partial sums of one tile to its partner through LDS and finishes the other:
// after the exchange a wavefront owns 32 tokens x 32 channels, one channel per lane, requantisation constants in four
// registers, exactly as in the kernel for short rows (gemm_rs.hip), whose load, store and epilogue forms are reused.
// The activations of a tile (48 KB) pass through two LDS buffers, filled by LDS-direct loads one tile ahead.  There
// are two sets of accumulators: while tile t is multiplied, the sums of tile t - 1 are exchanged, requantised and
// stored between the MFMAs.  Two barriers per tile: one for the exchange, one before the buffer of the tile just read
// is filled again.  What bounds it is data movement inside the compute unit: per tile 96 KB of fragment reads, 48 KB
// of loads landing and 32 KB of exchange pass through the LDS in the 1536 cycles the MFMAs of the tile take, and every
// workgroup first brings 192 KB of weights through the load path (about 43 bytes per cycle and compute unit, measured).
#include "regst_common.hpp"
#include <algorithm>

namespace ivit {

namespace {

using namespace regst;

constexpr int KK = 1536, KHALF = 768, KS = KHALF / 32;         // K, the bytes of it a wavefront multiplies, its k-steps per tile

struct KsParams {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N;
    int slabs, q;                            // channel slabs (four tiles of 32 channels), workgroups per slab
    int stages;                              // token tiles of 32
    int rnd;                                 // 1: round to nearest, 0: floor (every requantisation of the epilogue)
};

template <int EPI>
struct KsLayout {
    static constexpr int NW = 4, NT = 64 * NW;
    static constexpr int P16 = KK / 16 + 1, PITCH = 16 * P16;      // activation row in LDS: K bytes + one 16-byte pad piece
    static constexpr int NWI = (32 * P16 + 63) / 64;               // load instructions (64 lanes x 16 bytes) per tile
    static constexpr int NI = (NWI + NW - 1) / NW;                 // ... per wavefront at most
    static constexpr int XT = NWI * 1024;                          // bytes of a stage buffer
    static constexpr int XB = 4096;                                // exchange slot of a wavefront: 16 registers x 64 lanes
    static constexpr int OT = 32 * OP;                             // output staging tile of a wavefront
    static constexpr int RP = 32 + 16, RS16 = RP / 16;             // residual staging: pitch of a token row, 16-byte slots in it
    static constexpr int RNI = (32 * RS16 + 63) / 64;
    static constexpr int RT = RNI * 1024;
    // stage buffer 1, the exchange slots, the output and residual staging and the ShiftGELU table share their memory with
    // the weight chunks of the prologue; stage buffer 0 lies beyond, so that the first tile can be requested at the start
    static constexpr int XS1 = 0, EXC = XT, OUT = EXC + NW * XB, RES = OUT + NW * OT;
    static constexpr int LUT = RES + (EPI == EPI_RESIDUAL ? NW * 2 * RT : 0);
    static constexpr int MAIN = LUT + 256;
    static constexpr int CK = 192;                                 // bytes of K per weight chunk of the prologue
    static constexpr int CNI = (32 * (CK / 16 + 1) + 63) / 64;     // load instructions per chunk (one wavefront's 32 rows)
    static constexpr int CBUF = CNI * 1024;                        // a chunk buffer
    static constexpr int STAGING = NW * 2 * CBUF;                  // two per wavefront
    static constexpr int XS0 = MAIN > STAGING ? MAIN : STAGING;
    static constexpr int TOTAL = XS0 + XT;
    __host__ __device__ static constexpr int stage_offset(int b) { return b == 0 ? XS0 : XS1; }
    static_assert(KHALF % CK == 0 && CK % 32 == 0, "half a row must be a whole number of weight chunks");
    static_assert(TOTAL + 1024 <= 160 * 1024, "LDS");
};

template <int EPI>
__global__ __launch_bounds__(256) void gemm_ks_kernel(KsParams P) {
    using LY = KsLayout<EPI>;
    constexpr int NW = LY::NW, PITCH = LY::PITCH, P16 = LY::P16, NWI = LY::NWI, NI = LY::NI, OT = LY::OT;
    constexpr int RP = LY::RP, RS16 = LY::RS16, RNI = LY::RNI, RT = LY::RT, XB = LY::XB;
    constexpr int RG = 3;                                      // ring of A fragments: RG - 1 k-steps of prefetch distance (4 and 6: no faster)
    constexpr int SYNC = KS - RG;                              // k-step of the barrier after which the tile's buffer is filled again
    constexpr int XSTEP = 2;                                   // k-step of the barrier of the exchange
    constexpr int NPS = 3, NA = NPS * RG;                      // loads of a tile requested in k-steps SYNC .. KS - 1 (NPS per step); the rest
    constexpr int NPN = 2;                                     // in the first k-steps of the next tile (NPN per step)
    static_assert(KS % RG == 0 && NPS * (KS - SYNC) == NA && NA + NPN * XSTEP >= NI, "the requests of a tile fit their k-steps");
    static_assert(KS - SYNC >= RNI, "the residual requests fit the k-steps after the barrier");

    extern __shared__ __align__(1024) int8_t lds[];
    int8_t* gelu_lut = lds + LY::LUT;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = wv >> 1, kh = wv & 1;                       // pair, and which half of K this wavefront multiplies
    const int lj = lane & 31, lg = lane >> 5;
    const int N = P.N;
    const int64_t M = P.M;
    const int Nt = N >> 5;

    // workgroups of one XCD (block id modulo 8) get consecutive logical ids, so the slabs that share a token tile,
    // and therefore read the same activations, sit on the same L2
    const int G = gridDim.x, xcd = blockIdx.x % NXCD;
    const int L = xcd * (G / NXCD) + min(xcd, G % NXCD) + blockIdx.x / NXCD;
    const int slab = L % P.slabs, wi = L / P.slabs;
    // the pair's tiles are slab * 4 + 2 cg and + 1; this wavefront finishes ("owns") the one numbered like its half of K
    // and hands over the other.  Local tile 0 is the own one, local tile 1 the other, for both wavefronts of a pair.
    const int tile_own = slab * 4 + 2 * cg + kh;
    const int n0w = tile_own * 32;
    const int ntile = wi < P.stages ? (P.stages - wi + P.q - 1) / P.q : 0;     // token tiles of this workgroup; tile k is wi + k q
    if (ntile == 0) return;                                    // (the same for all wavefronts of a workgroup)

    // ---- requantisation parameters of this lane's channel: requested first, used after the weights are in place
    int32_t pb, pc, pbias;
    {
        const int ch = min(tile_own, Nt - 1) * 32 + lj;        // channel tiles past the last one repeat it; never stored
        pb = P.rq_b[ch]; pc = P.rq_c[ch]; pbias = P.bias ? P.bias[ch] : 0;
    }

    // ---- activation loads (as in gemm_rs.hip): load instruction n = i NW + wavefront of a tile covers slots 64 n ..
    // 64 n + 63; slot s is piece s % P16 of LDS row s / P16, and LDS row r holds token token_of_row(r) of the tile
    const uint32_t xs_off = lds_offset(lds) + wv * 1024;
    int ld_row[NI], ld_col[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int s = 64 * (i * NW + wv) + lane;
        ld_row[i] = token_of_row(min(s / P16, 31));
        ld_col[i] = 16 * min(s % P16, KK / 16 - 1);
    }
    const int row_step = P.q * 32;                             // rows between two tiles of this workgroup
    struct Cursor {                                            // a tile some steps ahead
        const int8_t* p;                                       // its first row (never dereferenced when rows <= 0)
        int rows;                                              // rows of the matrix from there on (<= 0: past the end)
    };
    auto cursor = [&](const int8_t* base, int64_t row_bytes, int ahead) __attribute__((always_inline)) -> Cursor {
        const int64_t row0 = ((int64_t)wi + (int64_t)ahead * P.q) * 32;
        return Cursor{base + row0 * row_bytes, (int)max64(M - row0, -(1 << 30))};
    };
    const int64_t x_step = (int64_t)row_step * KK, n_step = (int64_t)row_step * N;
    auto advance = [&](Cursor& c, int64_t step_bytes) __attribute__((always_inline)) { c.p += step_bytes; c.rows -= row_step; };
    const int8_t* x_last = P.x + (M - 1) * KK;                 // a tile past the matrix reads its last row instead
    struct Span { const int8_t* base; int last; };             // where a tile starts, and its last row that exists
    auto span_of = [&](const Cursor& c, const int8_t* fallback) __attribute__((always_inline)) -> Span {
        return Span{uniform_ptr(c.rows > 0 ? c.p : fallback), __builtin_amdgcn_readfirstlane(min(max(c.rows, 1), 32) - 1)};
    };
    auto issue_act_one = [&](const Span& sp, uint32_t dst, int i) __attribute__((always_inline)) {
        if (i >= NI) return;
        if ((i + 1) * NW > NWI && i * NW + wv >= NWI) return;  // the tile ends inside the last round of instructions
        dma16(sp.base, (uint32_t)(__mul24(min(ld_row[i], sp.last), KK) + ld_col[i]), dst + i * (NW * 1024));
    };
    // the first tile is requested before anything else: it lands while the weights are brought in
    {
        const Span s0 = span_of(cursor(P.x, KK, 0), x_last);
#pragma unroll
        for (int i = 0; i < NI; ++i) issue_act_one(s0, xs_off + LY::stage_offset(0), i);
    }

    // ---- weights.  Lane (lj, lg) needs, for local tile cbl and k-step ks, bytes 32 ks + 16 lg .. + 15 of this wavefront's
    // half of the row of channel lj of that tile: read like that from global memory, every load instruction would touch
    // 32 rows.  Instead each wavefront brings ITS rows through a piece of LDS of its own, in chunks of [32 channels][192
    // bytes of K] fetched as whole row pieces by LDS-direct loads, two chunks in flight, and picks its fragments out of
    // them.  Nothing is shared between wavefronts here, so the only waits are those for the wavefront's own loads.
    v4i W[2][KS];
    {
        constexpr int CK = LY::CK, CP16 = CK / 16 + 1, CPITCH = 16 * CP16, CNI = LY::CNI, CBUF = LY::CBUF;
        constexpr int NCHUNK = 2 * (KHALF / CK), KP = KHALF / CK;
        int8_t* wst = lds + wv * 2 * CBUF;                      // this wavefront's two chunk buffers
        const uint32_t wst_off = lds_offset(wst);
        auto issue_chunk = [&](int c) __attribute__((always_inline)) {
            const int cbl = c / KP, kp = c % KP;
            const int tile = slab * 4 + 2 * cg + (cbl == 0 ? kh : 1 - kh);
            const int ch0 = min(tile, Nt - 1) * 32;
#pragma unroll
            for (int i = 0; i < CNI; ++i) {                     // (slots past the chunk repeat its last row into the slack)
                const int s = 64 * i + lane;
                const int row = min(s / CP16, 31), piece = min(s % CP16, CK / 16 - 1);
                dma16(uniform_ptr(P.w), (uint32_t)((ch0 + row) * KK + kh * KHALF + kp * CK + 16 * piece), wst_off + (c & 1) * CBUF + i * 1024);
            }
        };
        issue_chunk(0);
        issue_chunk(1);
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) {
            // loads complete in order: all but the CNI of the following chunk
            if (c + 1 < NCHUNK) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(CNI) : "memory"); else wait_vm0();
            const int cbl = c / KP, kp = c % KP;
            const int8_t* src = wst + (c & 1) * CBUF + lj * CPITCH + 16 * lg;
#pragma unroll
            for (int s = 0; s < CK / 32; ++s) {
                W[cbl][kp * (CK / 32) + s] = *reinterpret_cast<const v4i*>(src + 32 * s);
                // (read only by MFMAs, which take this operand from the accumulation registers just as well)
                asm volatile("" : "+a"(W[cbl][kp * (CK / 32) + s]));
            }
            // (the statements above have used what they read: the buffer can be filled again)
            if (c + 2 < NCHUNK) issue_chunk(c + 2);
        }
        __syncthreads();                                        // everyone is done with the chunk buffers: the memory they share with the main loop is free
    }

    // ---- residual tile of a wavefront: [32 tokens][RP] bytes, slot s = 64 i + lane = piece s % RS16 of token s / RS16
    int8_t* out_w = lds + LY::OUT + wv * OT;
    int8_t* res_w = lds + LY::RES + wv * 2 * RT;
    int8_t* exc_own = lds + LY::EXC + wv * XB;                  // where this wavefront leaves the sums it hands over
    const int8_t* exc_partner = lds + LY::EXC + (wv ^ 1) * XB;
    const uint32_t res_off = lds_offset(res_w);
    int rs_col[RNI], rs_row[RNI];
    if (EPI == EPI_RESIDUAL) {
#pragma unroll
        for (int i = 0; i < RNI; ++i) {
            const int s = 64 * i + lane;
            rs_row[i] = min(s / RS16, 31);
            rs_col[i] = min(n0w + 16 * min(s % RS16, 1), N - 16);
        }
    }
    const int8_t* res_last = P.residual ? P.residual + (M - 1) * N : nullptr;     // a tile past the matrix reads its last row
    auto issue_res_one = [&](const Span& sp, uint32_t dst, int i) __attribute__((always_inline)) {
        dma16(sp.base, (uint32_t)(__mul24(min(rs_row[i], sp.last), N) + rs_col[i]), dst + i * 1024);
    };
    // transposing read of the residual tile (see gemm_rs.hip): lane L = 16 B + j gets channel (16 B + j) % 32, tokens
    // 16 (B / 2) + 8 h + 0..7
    const int rr_base = ((lane >> 5) * 16 + ((lane & 15) >> 1)) * RP + 16 * ((lane >> 4) & 1) + 8 * (lane & 1);
    auto read_res = [&](int half, v2i (&rw)[2]) __attribute__((always_inline)) {
        const int8_t* t = res_w + half * RT + rr_base;
#pragma unroll
        for (int h = 0; h < 2; ++h)
            rw[h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(t + 8 * h * RP));
    };

    {
        const Span s1 = span_of(cursor(P.x, KK, 1), x_last);
#pragma unroll
        for (int i = 0; i < NI; ++i) issue_act_one(s1, xs_off + LY::stage_offset(1), i);
        if (EPI == EPI_RESIDUAL) {
            Cursor r0 = cursor(P.residual, N, 0);
            const Span rs0 = span_of(r0, res_last);
#pragma unroll
            for (int i = 0; i < RNI; ++i) issue_res_one(rs0, res_off, i);
        }
    }

    // ---- requantisation constants of the lane's channel (24-bit form, derivation in gemm_rs.hip): the sum is limited to
    // [lo, hi], then one 24-bit multiply-add leaves the int8 result in the top byte (residual layers: one bit lower, the
    // residual term by a second multiply-add).  A workgroup with a channel outside the conditions of that form takes the
    // general 64-bit form for all of its channels.
    int32_t c_lo = 0, c_hi = 0, c_mb = 0, c_ad = 0;
    bool chan_24 = true;
    int64_t wlim = 127;
    int sh24 = 24;
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
    {
        bool ok = chan_24 && pc >= 1 && pc <= sh24 && pb >= 1 && pb < (1 << ((pc - 1) & 31));
        if (ok) {
            const int64_t half = (int64_t)P.rnd << (pc - 1), two_c = (int64_t)1 << pc;
            const int64_t Lp = (int64_t)((uint32_t)(wlim * two_c - half + pb - 1) / (uint32_t)pb);
            const int64_t Ln = -(int64_t)((uint32_t)((wlim - 1) * two_c + 1 + half + pb - 1) / (uint32_t)pb);
            const int64_t l = Ln - pbias, h = Lp - pbias;
            ok = l >= -(1 << 23) && h < (1 << 23);
            c_lo = (int32_t)l; c_hi = (int32_t)h; c_mb = pb << (sh24 - pc);
            c_ad = (int32_t)(uint32_t)((uint64_t)((int64_t)pbias * pb + half) << (sh24 - pc));
        }
        chan_24 = chan_24 && ok;
    }
    if (EPI == EPI_GELU && tid < 256) {
        const int32_t I = (int32_t)(int8_t)tid;
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c, P.rnd);
    }
    const bool fast24 = __syncthreads_and(chan_24) != 0;
    if (!fast24) { c_lo = pb; c_hi = pc; c_mb = pbias; c_ad = 0; }     // the general form keeps the raw parameters instead

    // ---- output (as in gemm_rs.hip with one channel tile): a lane's 16 results are one 16-byte write into row lj of the
    // staging tile; the one store instruction of a tile covers its eight half-blocks of 8 tokens x 16 channels
    int st_src;
    uint32_t st_dst;
    {
        const int B = lane >> 4, o_src = lane & 1, b = (lane & 15) >> 1, o_dst = (lane >> 3) & 1, j = lane & 7;
        const int hs = 2 * B + o_src, hd = 2 * B + o_dst;
        st_src = (16 * (hs % 2) + b) * OP + 8 * (hs / 2);
        st_dst = n0w + 16 * (hd % 2) < N ? (uint32_t)((8 * (hd / 2) + j) * N + 16 * (hd % 2)) : 0x80000000u;
    }
    auto tile_buffer = [&](const Cursor& c) __attribute__((always_inline)) {
        int8_t* base = const_cast<int8_t*>(uniform_ptr(c.p + n0w));
        const int rows = __builtin_amdgcn_readfirstlane(min(max(c.rows, 0), 32));
        return __builtin_amdgcn_make_buffer_rsrc(base, 0, rows * N, 0x00020000);
    };

    const int32_t rb = P.res_rq.b, rc = P.res_rq.c, rh = P.rnd << ((P.res_rq.c - 1) & 31);
    // one epilogue unit: the four outputs e = 4 d .. 4 d + 3 of the own channel tile -> one packed word
    auto unit_fast = [&](const v16i& a, int d, const v2i (&rw)[2]) __attribute__((always_inline)) -> int {
        uint32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t m = med3(a[4 * d + r], c_lo, c_hi);
            if (EPI == EPI_RESIDUAL) {
                const int32_t t1 = (__mul24(m, c_mb) + c_ad) >> 23;
                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[d >> 1][d & 1] >> (8 * r));
                const int32_t t2 = (__mul24(res, rb) + rh) >> rc;
                o[r] = (uint32_t)clamp8(t1 + t2);
            } else {
                o[r] = (uint32_t)(__mul24(m, c_mb) + c_ad);                       // result in the top byte
                if (EPI == EPI_GELU) o[r] = (uint32_t)gelu_lut[o[r] >> 24];        // result in the low byte
            }
        }
        const bool low = EPI != EPI_PLAIN;
        const uint32_t p01 = __builtin_amdgcn_perm(o[1], o[0], low ? 0x0c0c0400u : 0x0c0c0703u);
        const uint32_t p23 = __builtin_amdgcn_perm(o[3], o[2], low ? 0x04000c0cu : 0x07030c0cu);
        return (int)(p01 | p23);
    };
    auto unit_general = [&](const v16i& a, int d, const v2i (&rw)[2]) __attribute__((always_inline)) -> int {
        uint32_t o[4];
        const int32_t b = c_lo, c = c_hi, bias = c_mb;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int64_t r64 = rnd_shift64(a[4 * d + r] + bias, b, c, P.rnd);
            if (EPI == EPI_RESIDUAL) {
                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[d >> 1][d & 1] >> (8 * r));
                r64 += rnd_shift64(res, P.res_rq.b, P.res_rq.c, P.rnd);
            }
            int32_t v = clamp8_64(r64);
            if (EPI == EPI_GELU) v = gelu_lut[(uint8_t)v];
            o[r] = (uint32_t)v;
        }
        const uint32_t p01 = __builtin_amdgcn_perm(o[1], o[0], 0x0c0c0400u);
        const uint32_t p23 = __builtin_amdgcn_perm(o[3], o[2], 0x04000c0cu);
        return (int)(p01 | p23);
    };
    // the sums handed over: register e of lane l at word 64 e + l of the slot (whole 16-byte pieces per lane and quad)
    auto hand_over = [&](const v16i& a) __attribute__((always_inline)) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
            *reinterpret_cast<v4i*>(exc_own + qd * 1024 + lane * 16) = v4i{a[4 * qd], a[4 * qd + 1], a[4 * qd + 2], a[4 * qd + 3]};
    };
    auto take_over = [&](v4i (&in)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) in[qd] = *reinterpret_cast<const v4i*>(exc_partner + qd * 1024 + lane * 16);
    };

    // this lane's A fragment of k-step ks of the tile in the stage buffer at offset b: + 32 ks
    const int a_base = lj * PITCH + kh * KHALF + 16 * lg;
    v4i af[RG];
    {
        const int8_t* xa = lds + LY::stage_offset(0) + a_base;
#pragma unroll
        for (int i = 0; i < RG - 1; ++i) af[i] = *reinterpret_cast<const v4i*>(xa + 32 * i);
    }

    v16i accA[2], accB[2];
    v2i rw[2] = {};
    Cursor c_req, c_res, c_out, c_prev;                         // tile being requested, residual tile being requested, tile k, tile k - 1
    Span q_pend = {nullptr, 0};                                 // the tile whose request was begun in the previous tile
    uint32_t q_pend_dst = 0;

    // Token tile k in the stage buffer at offset b0 (the other one, b1, holds tile k + 1 or is being filled with it):
    // multiply into `cur`; when `ep`, `prev` holds the partial sums of tile k - 1, which are exchanged, completed,
    // requantised and stored between the MFMAs.  Residual tile j is in half j % 2 of the residual staging (`hp`: that of
    // tile k - 1, and of tile k + 1, which is requested after the barrier).
    auto tile_step = [&]<bool ep, bool fast>(int b0, int b1, int hp, v16i (&cur)[2], v16i (&prev)[2]) __attribute__((always_inline)) {
        v4i ow, in[4];
        v2i sa = {}, sb = {};
        const int8_t* xa = lds + b0 + a_base;
        const int8_t* xb = lds + b1 + a_base;
        const auto sc = [](int v) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(v); };
        const Span q_span = span_of(c_req, x_last);
        const uint32_t q_dst = (uint32_t)sc(xs_off + b0);
        const Span r_span = EPI == EPI_RESIDUAL ? span_of(c_res, res_last) : Span{nullptr, 0};
        const uint32_t r_dst = (uint32_t)sc(res_off + hp * RT);
        const __amdgpu_buffer_rsrc_t y_buf = tile_buffer(c_prev);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ep && ks == XSTEP) __syncthreads();             // the sums handed over in k-step 0 are in LDS
            // fragment ks + RG - 1: of the next tile once this one runs out (valid since the barrier of this tile)
            if (ks + RG - 1 < KS) af[(ks + RG - 1) % RG] = *reinterpret_cast<const v4i*>(xa + 32 * (ks + RG - 1));
            else af[(ks + RG - 1) % RG] = *reinterpret_cast<const v4i*>(xb + 32 * (ks + RG - 1 - KS));
            if (ks == SYNC) {
                // the read above was the last one of this tile's buffer: once every wavefront has got its data (the barrier
                // waits for the LDS reads of the wavefront too) the buffer can be filled again; the other buffer has landed
                static_assert(SYNC + RG - 1 == KS - 1, "the last fragment of the tile is read right before the barrier");
                wait_vm0();
                __syncthreads();
            }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                if (ks == 0) {
                    const v16i zero = {};
                    cur[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks % RG], W[cb][ks], zero, 0, 0, 0);
                } else {
                    cur[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks % RG], W[cb][ks], cur[cb], 0, 0, 0);
                }
            }
            if (ep) {
                if (ks == 0) hand_over(prev[1]);
                if (ks == XSTEP) { take_over(in); if (EPI == EPI_RESIDUAL) read_res(hp, rw); }
                if (ks == XSTEP + 1) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) prev[0][e] += in[e >> 2][e & 3];
                }
                if (ks >= XSTEP + 2 && ks < XSTEP + 10 && ((ks - XSTEP) & 1) == 0) {          // four units, every other k-step
                    const int d = (ks - XSTEP - 2) >> 1;
                    ow[d] = fast ? unit_fast(prev[0], d, rw) : unit_general(prev[0], d, rw);
                    if (d == 3) *reinterpret_cast<v4i*>(out_w + lj * OP + 16 * lg) = ow;
                }
                if (ks == XSTEP + 10) {
                    sa = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src));
                    sb = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src + 8 * OP));
                }
                if (ks == XSTEP + 11) __builtin_amdgcn_raw_buffer_store_b128(v4i{sa[0], sa[1], sb[0], sb[1]}, y_buf, (int)st_dst, 0, 0);
            }
            if (ks < XSTEP && q_pend.base) {                    // the rest of the request begun in the previous tile
#pragma unroll
                for (int n = 0; n < NPN; ++n) issue_act_one(q_pend, q_pend_dst, NA + NPN * ks + n);
            }
            if (ks >= SYNC) {
                const int j = ks - SYNC;
#pragma unroll
                for (int n = 0; n < NPS; ++n) issue_act_one(q_span, q_dst, NPS * j + n);
                if (EPI == EPI_RESIDUAL && j < RNI) issue_res_one(r_span, r_dst, j);       // past the last tile: a repeat, never used
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        q_pend = q_span; q_pend_dst = q_dst;
        c_prev = c_out;
        advance(c_out, n_step);
        advance(c_req, x_step);
        advance(c_res, n_step);
    };

    // the results of the last tile
    auto drain = [&]<bool fast>(v16i (&last)[2], int hp) __attribute__((always_inline)) {
        v4i ow, in[4];
        hand_over(last[1]);
        wait_vm0();                                             // (the residual tile of the last tile has landed)
        __syncthreads();
        take_over(in);
        if (EPI == EPI_RESIDUAL) read_res(hp, rw);
#pragma unroll
        for (int e = 0; e < 16; ++e) last[0][e] += in[e >> 2][e & 3];
#pragma unroll
        for (int d = 0; d < 4; ++d) ow[d] = fast ? unit_fast(last[0], d, rw) : unit_general(last[0], d, rw);
        *reinterpret_cast<v4i*>(out_w + lj * OP + 16 * lg) = ow;
        const __amdgpu_buffer_rsrc_t y_buf = tile_buffer(c_prev);
        const v2i sa = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src));
        const v2i sb = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src + 8 * OP));
        __builtin_amdgcn_raw_buffer_store_b128(v4i{sa[0], sa[1], sb[0], sb[1]}, y_buf, (int)st_dst, 0, 0);
    };
    auto run = [&]<bool fast>() __attribute__((always_inline)) {
        c_req = cursor(P.x, KK, 2);
        c_res = cursor(P.residual, N, 1);
        c_out = cursor(P.y, N, 0);
        c_prev = c_out;
        constexpr int B0 = LY::stage_offset(0), B1 = LY::stage_offset(1);
        tile_step.template operator()<false, fast>(B0, B1, 1, accA, accB);       // tile 0; residual tile 1 goes to half 1
        for (int k = 1; k < ntile; k += 2) {
            tile_step.template operator()<true, fast>(B1, B0, 0, accB, accA);   // tile k odd: epilogue of tile k - 1 (half 0), request of tile k + 1 (half 0)
            if (k + 1 < ntile) tile_step.template operator()<true, fast>(B0, B1, 1, accA, accB);
        }
        if (ntile & 1) drain.template operator()<fast>(accA, 0); else drain.template operator()<fast>(accB, 1);
    };
    if (fast24) run.template operator()<true>(); else run.template operator()<false>();
    wait_vm0();            // LDS-direct loads still in flight (repeats of the last tile) must land before the LDS is released
}

template <int EPI>
hipError_t launch_ks(hipStream_t s, const KsParams& P, int grid) {
    constexpr size_t lds_bytes = KsLayout<EPI>::TOTAL;
    hipLaunchKernelGGL((gemm_ks_kernel<EPI>), dim3(grid), dim3(256), lds_bytes, s, P);
    return hipGetLastError();
}

}  // namespace

// Shapes this kernel takes: K = 1536, N a multiple of 32, dense rows, at most 2^30 of them; offsets inside the weight
// matrix and inside a token tile are 32-bit.
bool linear_ks_takes(const LinearArgs& a) {
    if (a.K != KK) return false;
    if ((int64_t)a.N * a.K > 0x7fffffffLL) return false;
    if (a.M > (1 << 30)) return false;
    return (a.N & 31) == 0 && (a.ldx == 0 || a.ldx == a.K) && a.M >= 1;
}

hipError_t launch_linear_ks(hipStream_t s, const LinearArgs& a) {
    KsParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.rnd = a.floor_shift ? 0 : 1;
    const int nt = a.N / 32;
    P.slabs = (nt + 3) / 4;
    P.stages = (int)((a.M + 31) / 32);
    P.q = std::max(1, std::min(P.stages, num_cus() / P.slabs));
    const int grid = P.q * P.slabs;
    if (a.residual) return launch_ks<EPI_RESIDUAL>(s, P, grid);
    if (a.gelu) return launch_ks<EPI_GELU>(s, P, grid);
    return launch_ks<EPI_PLAIN>(s, P, grid);
}

}  // namespace ivit
