// Dense layers with K of a few hundred bytes (I-ViT, arXiv 2207.01405, Sec. 3.2, Eq. 7-10; residual add of Eq. 1-2;
// ShiftGELU of Sec. 3.4, Algorithm 2): the weights stay in REGISTERS for the whole kernel.
//
// A workgroup has GR groups of four wavefronts (one wavefront of each group per SIMD).  Wavefront w of a group owns
// NCB tiles of 32 output channels and keeps their weights (all of K) in accumulation registers as the MFMA "B"
// operand, so the matrix cores read no weights from LDS; the groups hold the same channels and work on different
// token tiles.  The workgroup walks over stages of GR tiles of 32 tokens: the activations of a stage are fetched
// straight from global memory into LDS (LDS-direct loads, no register pass) two stages ahead, and every wavefront
// reads its group's tile from there as the "A" operand, one 1 KB fragment per NCB MFMAs.  The accumulator of a lane
// is then ONE channel and 16 tokens, so the four requantisation constants of a channel live in four registers for the
// whole kernel: the epilogue reads no tables.
//   K = 768: the weights leave room for one wavefront per SIMD (GR = 1).  It has two sets of accumulators; while
// token tile t is multiplied, the results of tile t - 1 are requantised between the MFMAs (an issued MFMA executes in
// the background, and nothing else could fill the gaps).
//   K = 384 and K = 192: two wavefronts per SIMD (GR = 2) with one set of accumulators each; a tile is requantised
// right after its multiply while the other wavefront of the SIMD multiplies.
// Everything else a tile needs (one barrier, the loads of a later tile, the stores of an earlier one) is spread over
// the k-steps, one piece per step.  What bounds the kernel is the rate at which a SIMD issues instructions of any kind
// (about one per 4.4 cycles, measured), so the tile loop is written to need few of them: tile bookkeeping in 32-bit
// scalars, one address computation per load, stores through a buffer descriptor whose bounds check replaces lane masks.
// The int8 results (16 tokens of a channel per lane) are turned into token rows through wavefront-private LDS with
// the transposing LDS read of gfx950 (ds_read_b64_tr_b8) and leave as 16-byte pieces of contiguous row segments; the
// residual operand comes in by the mirror image of that path.
#include "regst_common.hpp"
#include <algorithm>

namespace ivit {

namespace {

using namespace regst;

struct RsParams {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N; int64_t ldx;
    int slabs, q;                            // channel slabs (4 NCB tiles each), workgroups per slab
    int stages;                              // stages of GR token tiles of 32
    int rnd;                                 // 1: round to nearest, 0: floor (every requantisation of the epilogue)
};

template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

template <int KS, int NCB, int EPI, int GR>
struct RsLayout {
    static constexpr int NW = 4 * GR, NT = 64 * NW;               // wavefronts, threads
    static constexpr int K = 32 * KS;
    static constexpr int P16 = 2 * KS + 1, PITCH = 16 * P16;       // activation row in LDS: K bytes + one 16-byte pad piece
    static constexpr int NWI = (32 * GR * P16 + 63) / 64;          // load instructions (64 lanes x 16 bytes) per stage
    static constexpr int NI = (NWI + NW - 1) / NW;                 // ... per wavefront at most
    static constexpr int XT = NWI * 1024;                          // bytes of a stage
    static constexpr int OT = 32 * NCB * OP;                       // output staging tile of a wavefront
    static constexpr int RP = 32 * NCB + 16, RS16 = RP / 16;       // residual staging: pitch of a token row, 16-byte slots in it
    static constexpr int RNI = (32 * RS16 + 63) / 64;              // residual load instructions per lane and tile
    static constexpr int RT = RNI * 1024;
    // stage buffers 1 and 2, the output and residual staging and the ShiftGELU table share their memory with the weight
    // chunks of the prologue; stage buffer 0 lies beyond both, so that the first stage can be requested at the very start
    static constexpr int XS1 = 0, OUT = 2 * XT, RES = OUT + NW * OT;
    static constexpr int LUT = RES + (EPI == EPI_RESIDUAL ? NW * 2 * RT : 0);
    static constexpr int MAIN = LUT + 256;
    static constexpr int CK = K < WCK ? K : WCK;                   // bytes of K per weight chunk of the prologue
    static constexpr int CPITCH = CK + 16;                         // its row pitch in LDS
    static constexpr int CWI = 4 * 32 * (CPITCH / 16) / 64;        // load instructions per chunk: [4 wavefronts][32 channels][CPITCH]
    static constexpr int NCHUNK = NCB * (K / CK);                  // weight chunks of the prologue
    static constexpr int WNI = (CWI + NW - 1) / NW;                // load instructions per wavefront and chunk
    static constexpr int WCHUNK = WNI * NW * 1024;                 // LDS bytes of a chunk (whole rounds of all wavefronts)
    static constexpr int STAGING = (NCHUNK > 1 ? 2 : 1) * WCHUNK;  // the chunks pass through the same memory, before the main loop
    static constexpr int XS0 = MAIN > STAGING ? MAIN : STAGING;
    static constexpr int TOTAL = XS0 + XT;
    __host__ __device__ static constexpr int stage_offset(int b) { return b == 0 ? XS0 : XS1 + (b - 1) * XT; }
    static_assert(K % CK == 0 && (4 * 32 * (CPITCH / 16)) % 64 == 0, "K must be a whole number of weight chunks");
    static_assert(TOTAL + 1024 <= 160 * 1024, "LDS");
};

template <int EPI, int KS, int NCB, int GR>
__global__ __launch_bounds__(256 * GR) void gemm_rs_kernel(RsParams P) {
    using LY = RsLayout<KS, NCB, EPI, GR>;
    constexpr int NW = LY::NW, NT = LY::NT;
    constexpr int K = LY::K, PITCH = LY::PITCH, P16 = LY::P16, NWI = LY::NWI, NI = LY::NI, OT = LY::OT;
    constexpr int RP = LY::RP, RS16 = LY::RS16, RNI = LY::RNI, RT = LY::RT, WNI = LY::WNI, WCHUNK = LY::WCHUNK;
    constexpr int RG = (KS % 3 == 0) ? 3 : 4;                  // ring of A fragments: RG - 1 k-steps of prefetch distance
    constexpr int NU = 4 * NCB;                                // epilogue units (4 outputs each) per token tile and lane
    constexpr int SYNC = KS / 2;                               // k-step of the barrier
    static_assert(KS % RG == 0, "ring must align with the tile");
    static_assert(SYNC >= 2 && SYNC <= KS - RG, "the first fragments of the next tile are read after the barrier");
    static_assert(KS - SYNC >= NI && (EPI != EPI_RESIDUAL || KS - SYNC >= RNI) && KS - SYNC >= NCB + 1, "the work after the barrier is spread over its k-steps");

    extern __shared__ __align__(1024) int8_t lds[];
    int8_t* Xs = lds;                                          // stage buffer b at LY::stage_offset(b), XT bytes each
    int8_t* Out = lds + LY::OUT;                               // [waves][OT]
    int8_t* Res = lds + LY::RES;                               // [waves][2][RT]   (residual layers only)
    int8_t* gelu_lut = lds + LY::LUT;                          // [256]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: what depends on it stays scalar
    const int wq = wv & 3, grp = wv >> 2;                      // owner of channels (SIMD), group
    const int lj = lane & 31, lg = lane >> 5;
    const int N = P.N;
    const int64_t M = P.M;
    const int Nt = N >> 5;

    // workgroups of one XCD (block id modulo 8) get consecutive logical ids, so the slabs that share a token tile,
    // and therefore read the same activations, sit on the same L2
    const int G = gridDim.x, xcd = blockIdx.x % NXCD;
    const int L = xcd * (G / NXCD) + min(xcd, G % NXCD) + blockIdx.x / NXCD;
    const int slab = L % P.slabs, wi = L / P.slabs;
    const int tile0 = (slab * 4 + wq) * NCB;                   // first channel tile of this wavefront
    const int n0w = tile0 * 32;                                // its first channel
    const int ntile = wi < P.stages ? (P.stages - wi + P.q - 1) / P.q : 0;      // stages of this workgroup; stage k is wi + k q
    if (ntile == 0) return;                                    // (the same for all wavefronts of a workgroup)

    // ---- requantisation parameters of this lane's channels: requested first, used after the weights are in place
    int32_t pb[NCB], pc[NCB], pbias[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        const int ch = min(tile0 + cb, Nt - 1) * 32 + lj;      // channel tiles past the last one repeat it; never stored
        pb[cb] = P.rq_b[ch]; pc[cb] = P.rq_c[ch]; pbias[cb] = P.bias ? P.bias[ch] : 0;
    }

    // ---- activation loads: load instruction n (64 lanes x 16 bytes, n = i NW + wavefront) of a stage covers slots
    // 64 n .. 64 n + 63; slot s is piece s % P16 of LDS row s / P16, and LDS row r holds token token_of_row(r % 32) of
    // tile r / 32 of the stage, so that the lanes of an MFMA "A" read sit in consecutive LDS rows (the pad piece repeats
    // the last one; slots past the last row repeat it and land in the slack of the stage).  The address of a piece is
    // a scalar base (the stage) plus a 32-bit offset per lane, computed once; only a ragged last stage, whose missing
    // rows repeat the last row of the matrix, computes offsets of its own.  What a stage or tile needs beyond that
    // (its base pointer, how many of its rows exist) is scalar state that moves on by a fixed step per tile.
    constexpr int SR = 32 * GR;                                // rows of a stage
    const uint32_t xs_off = lds_offset(Xs) + wv * 1024;
    const int ldx = (int)P.ldx;                                // (K: far below 2^24, the offsets inside a stage are 24-bit products)
    int ld_row[NI], ld_col[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int s = 64 * (i * NW + wv) + lane;
        const int r = min(s / P16, SR - 1);
        ld_row[i] = 32 * (r >> 5) + token_of_row(r & 31);
        ld_col[i] = 16 * min(s % P16, 2 * KS - 1);
    }
    const int row_step = P.q * SR;                             // rows between two stages of this workgroup
    struct Cursor {                                            // a stage (or this group's tile of it) some steps ahead
        const int8_t* p;                                       // its first row (never dereferenced when rows <= 0)
        int rows;                                              // rows of the matrix from there on (<= 0: past the end)
    };
    auto cursor = [&](const int8_t* base, int64_t row_bytes, int ahead, int row_in_stage) __attribute__((always_inline)) -> Cursor {
        const int64_t row0 = ((int64_t)wi + (int64_t)ahead * P.q) * SR + row_in_stage;
        return Cursor{base + row0 * row_bytes, (int)max64(M - row0, -(1 << 30))};
    };
    const int64_t x_step = (int64_t)row_step * P.ldx, n_step = (int64_t)row_step * N;
    auto advance = [&](Cursor& c, int64_t step_bytes) __attribute__((always_inline)) { c.p += step_bytes; c.rows -= row_step; };
    const int8_t* x_last = P.x + (M - 1) * P.ldx;              // a stage past the matrix reads its last row instead
    // What a load instruction needs of its stage: where it starts and which is its last row that exists (the rows
    // after it repeat it) -- two scalars; every lane limits its row and forms its offset from them (two instructions).
    struct Span { const int8_t* base; int last; };
    auto span_of = [&](const Cursor& c, const int8_t* fallback, int rows_max) __attribute__((always_inline)) -> Span {
        return Span{uniform_ptr(c.rows > 0 ? c.p : fallback), __builtin_amdgcn_readfirstlane(min(max(c.rows, 1), rows_max) - 1)};
    };
    auto issue_act_one = [&](const Span& sp, uint32_t dst, int i) __attribute__((always_inline)) {
        if ((i + 1) * NW > NWI && i * NW + wv >= NWI) return;  // the stage ends inside the last round of instructions
        dma16(sp.base, (uint32_t)(__mul24(min(ld_row[i], sp.last), ldx) + ld_col[i]), dst + i * (NW * 1024));
    };

    // the first stage is requested before anything else: it lands while the weights are brought in
    {
        const Span s0 = span_of(cursor(P.x, P.ldx, 0, 0), x_last, SR);
#pragma unroll
        for (int i = 0; i < NI; ++i) issue_act_one(s0, xs_off + LY::stage_offset(0), i);
    }

    // ---- weights.  Lane (lj, lg) needs, for channel tile cb and k-step ks, bytes 32 ks + 16 lg .. + 15 of the row of
    // channel 32 cb + lj: read like that from global memory, every load instruction would touch 32 rows.  Instead the
    // workgroup brings them through LDS in chunks of [4 wavefronts][32 channels][384 bytes of K] with LDS-direct loads
    // of whole rows (two chunks in flight), and every wavefront picks its fragments out of its part of the chunk.
    v4i W[NCB][KS];
    {
        constexpr int NCHUNK = LY::NCHUNK, CK = LY::CK, CPITCH = LY::CPITCH, KH = K / CK, W16 = CPITCH / 16;
        const uint32_t stg = lds_offset(lds);
        auto issue_chunk = [&](int c) __attribute__((always_inline)) {
            const int cb = c / KH, kh = c % KH;
#pragma unroll
            for (int i = 0; i < WNI; ++i) {                     // (instructions past the chunk repeat its last row into the slack)
                const int s = 64 * (i * NW + wv) + lane;
                const int row = min(s / W16, 4 * 32 - 1), piece = min(s % W16, CK / 16 - 1);
                const int ch = min((slab * 4 + (row >> 5)) * NCB + cb, Nt - 1) * 32 + (row & 31);
                dma16(uniform_ptr(P.w), (uint32_t)(ch * K + kh * CK + 16 * piece), stg + (c & 1) * WCHUNK + (i * NW + wv) * 1024);
            }
        };
        issue_chunk(0);
        if (NCHUNK > 1) issue_chunk(1);
#pragma unroll
        for (int c = 0; c < NCHUNK; ++c) {
            // loads complete in order: all but the WNI of the following chunk
            if (c + 1 < NCHUNK) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(WNI) : "memory"); else wait_vm0();
            __syncthreads();
            const int cb = c / KH, kh = c % KH;
            const int8_t* src = lds + (c & 1) * WCHUNK + (wq * 32 + lj) * CPITCH + 16 * lg;
#pragma unroll
            for (int s = 0; s < CK / 32; ++s) {
                W[cb][kh * (CK / 32) + s] = *reinterpret_cast<const v4i*>(src + 32 * s);
                // the weights are only ever read by MFMAs, which take this operand from the accumulation registers just
                // as well: pinning them there leaves the ordinary vector registers to the accumulators and the epilogue
                asm volatile("" : "+a"(W[cb][kh * (CK / 32) + s]));
            }
            __syncthreads();                                    // everyone has read the chunk: its memory is free again
            if (c + 2 < NCHUNK) issue_chunk(c + 2);
        }
    }

    // ---- residual tile of a wavefront: [32 tokens][RP] bytes, slot s = 64 i + lane = piece s % RS16 of token s / RS16
    int8_t* out_w = Out + wv * OT;
    int8_t* res_w = Res + wv * 2 * RT;
    static_assert(NT >= 256, "the ShiftGELU table is filled by threads 0 .. 255");
    const uint32_t res_off = lds_offset(res_w);
    int rs_col[RNI], rs_row[RNI];
    if (EPI == EPI_RESIDUAL) {
#pragma unroll
        for (int i = 0; i < RNI; ++i) {
            const int s = 64 * i + lane;
            rs_row[i] = min(s / RS16, 31);
            rs_col[i] = min(n0w + 16 * min(s % RS16, 2 * NCB - 1), N - 16);
        }
    }
    const int8_t* res_last = P.residual ? P.residual + (M - 1) * N : nullptr;     // a tile past the matrix reads its last row
    auto issue_res_one = [&](const Span& sp, uint32_t dst, int i) __attribute__((always_inline)) {
        dma16(sp.base, (uint32_t)(__mul24(min(rs_row[i], sp.last), N) + rs_col[i]), dst + i * 1024);
    };
    // transposing read of the residual tile: in every block of 16 lanes the even lanes name eight 8-byte rows and lanes
    // 0-7 receive their columns, the odd lanes name eight more and lanes 8-15 receive theirs.  Lane L = 16 B + j is to
    // get channel (16 B + j) % 32 of tile cb, tokens 16 (B / 2) + 8 h + 0..7: source lane 16 B + 2 b + o names token
    // 16 (B / 2) + 8 h + b, channels 16 (B % 2) + 8 o + 0..7.
    const int rr_base = ((lane >> 5) * 16 + ((lane & 15) >> 1)) * RP + 16 * ((lane >> 4) & 1) + 8 * (lane & 1);
    auto read_res = [&](int par, v2i (&rw)[NCB][2]) __attribute__((always_inline)) {
        const int8_t* t = res_w + par * RT + rr_base;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                rw[cb][h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(t + 8 * h * RP + 32 * cb));
    };

    {
        const Span s1 = span_of(cursor(P.x, P.ldx, 1, 0), x_last, SR);
#pragma unroll
        for (int i = 0; i < NI; ++i) issue_act_one(s1, xs_off + LY::stage_offset(1), i);
        if (EPI == EPI_RESIDUAL) {
            const Span r0 = span_of(cursor(P.residual, N, 0, 32 * grp), res_last, 32);
#pragma unroll
            for (int i = 0; i < RNI; ++i) issue_res_one(r0, res_off, i);
        }
    }

    // ---- requantisation constants (while the first activations are on their way).  With v = dot + bias the int8 result
    // clamp8((v b + h) >> c), h the rounding addend (2^(c-1), or 0 for the bare shift of Eq. 10), is the same for all
    // v >= Lp (127) and all v <= Ln (-127), Lp / Ln being the first v that reach +-127; so the dot product is limited to
    // [Ln - bias, Lp - bias] first (one median of three), after
    // which T = v b + h lies in (-128 2^c, 128 2^c), T 2^(24-c) fits 32 bits and its top byte is the result: one
    // 24-bit multiply-add by b 2^(24-c), the addend (modulo 2^32) carrying bias and rounding.  Needs c <= 24,
    // b < 2^(c-1) and bounds within 24 bits.  Residual layers: the first term only has to be exact within
    // +-(127 + R2), R2 the largest magnitude of the residual term (<= 128 required), because beyond that the clamped
    // sum is +-127 whatever is added; it then needs nine bits and is kept one bit lower.  A workgroup with a channel
    // outside these conditions takes the general 64-bit form for all of its channels.
    int32_t c_lo[NCB], c_hi[NCB], c_mb[NCB], c_ad[NCB];
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
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        int32_t lo = 0, hi = 0, mb = 0, ad = 0;
        bool ok = chan_24 && pc[cb] >= 1 && pc[cb] <= sh24 && pb[cb] >= 1 && pb[cb] < (1 << ((pc[cb] - 1) & 31));
        if (ok) {
            const int64_t half = (int64_t)P.rnd << (pc[cb] - 1), two_c = (int64_t)1 << pc[cb];
            // (both numerators are below 256 * 2^24 = 2^32: unsigned 32-bit divisions, a fraction of the cost of 64-bit ones)
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
    if (EPI == EPI_GELU && tid < 256) {
        const int32_t I = (int32_t)(int8_t)tid;
        gelu_lut[tid] = (int8_t)requant64(shiftgelu_raw(I, P.gelu_p), P.gelu_rq.b, P.gelu_rq.c, P.rnd);
    }
    // (no wait for the loads just requested: stage 0 landed before the first weight chunk was read, loads completing in
    // order; stage 1 and the residual tile are first read after the barrier inside tile 0, which waits for them)
    const bool fast24 = __syncthreads_and(chan_24) != 0;
    if (!fast24) {                                              // the general form keeps the raw parameters instead
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) { c_lo[cb] = pb[cb]; c_hi[cb] = pc[cb]; c_mb[cb] = pbias[cb]; c_ad[cb] = 0; }
    }

    // ---- output: a lane's 16 results of channel tile cb (tokens 16 lg .. 16 lg + 15 of channel lj) are one 16-byte
    // write into row 32 cb + lj of the staging tile; store instruction s then covers eight half-blocks of 8 tokens x 16
    // channels, half-block 8 s + 2 B + o = 2 NCB tb + cg being tokens 8 tb .. + 7, channels 16 cg .. + 15: lane
    // L = 16 B + 8 o + j receives token 8 tb + j (two transposing reads: channels 16 cg + 0..7, + 8..15) and stores 16
    // bytes of a row of y.
    int st_src[NCB];
    uint32_t st_dst[NCB];
#pragma unroll
    for (int s = 0; s < NCB; ++s) {
        const int B = lane >> 4, o_src = lane & 1, b = (lane & 15) >> 1, o_dst = (lane >> 3) & 1, j = lane & 7;
        const int hs = 8 * s + 2 * B + o_src, hd = 8 * s + 2 * B + o_dst;
        st_src[s] = (16 * (hs % (2 * NCB)) + b) * OP + 8 * (hs / (2 * NCB));
        // where this lane's piece goes, relative to the tile's first row at the wavefront's first channel; pieces of
        // channel tiles past the last one get an offset no buffer reaches
        st_dst[s] = n0w + 16 * (hd % (2 * NCB)) < N ? (uint32_t)((8 * (hd / (2 * NCB)) + j) * N + 16 * (hd % (2 * NCB))) : 0x80000000u;
    }
    auto store_read = [&](int s, v2i& a, v2i& b) __attribute__((always_inline)) {
        a = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src[s]));
        b = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(out_w + st_src[s] + 8 * OP));
    };
    // The rows of a tile that exist, from the wavefront's first channel on, as a buffer: a store past its end (a row
    // that does not exist, a channel tile past the last one) is dropped by the hardware, so no lane is masked by hand.
    auto tile_buffer = [&](const Cursor& c) __attribute__((always_inline)) {
        int8_t* base = const_cast<int8_t*>(uniform_ptr(c.p + n0w));
        const int rows = __builtin_amdgcn_readfirstlane(min(max(c.rows, 0), 32));
        return __builtin_amdgcn_make_buffer_rsrc(base, 0, rows * N, 0x00020000);
    };
    auto store_write = [&](__amdgpu_buffer_rsrc_t buf, int s, const v2i& a, const v2i& b) __attribute__((always_inline)) {
        __builtin_amdgcn_raw_buffer_store_b128(v4i{a[0], a[1], b[0], b[1]}, buf, (int)st_dst[s], 0, 0);
    };

    const int32_t rb = P.res_rq.b, rc = P.res_rq.c, rh = P.rnd << ((P.res_rq.c - 1) & 31);

    // one epilogue unit: the four outputs e = 4 d .. 4 d + 3 of channel tile cb -> one packed word
    auto unit_fast = [&](const v16i& a, int cb, int d, const v2i (&rw)[NCB][2]) __attribute__((always_inline)) -> int {
        uint32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int32_t m = med3(a[4 * d + r], c_lo[cb], c_hi[cb]);
            if (EPI == EPI_RESIDUAL) {
                const int32_t t1 = (__mul24(m, c_mb[cb]) + c_ad[cb]) >> 23;
                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[cb][d >> 1][d & 1] >> (8 * r));
                const int32_t t2 = (__mul24(res, rb) + rh) >> rc;
                o[r] = (uint32_t)clamp8(t1 + t2);
            } else {
                o[r] = (uint32_t)(__mul24(m, c_mb[cb]) + c_ad[cb]);              // result in the top byte
                if (EPI == EPI_GELU) o[r] = (uint32_t)gelu_lut[o[r] >> 24];        // result in the low byte
            }
        }
        const bool low = EPI != EPI_PLAIN;
        const uint32_t p01 = __builtin_amdgcn_perm(o[1], o[0], low ? 0x0c0c0400u : 0x0c0c0703u);
        const uint32_t p23 = __builtin_amdgcn_perm(o[3], o[2], low ? 0x04000c0cu : 0x07030c0cu);
        return (int)(p01 | p23);
    };
    auto unit_general = [&](const v16i& a, int cb, int d, const v2i (&rw)[NCB][2]) __attribute__((always_inline)) -> int {
        uint32_t o[4];
        const int32_t b = c_lo[cb], c = c_hi[cb], bias = c_mb[cb];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int64_t r64 = rnd_shift64(a[4 * d + r] + bias, b, c, P.rnd);
            if (EPI == EPI_RESIDUAL) {
                const int32_t res = (int32_t)(int8_t)((uint32_t)rw[cb][d >> 1][d & 1] >> (8 * r));
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
    auto put_out = [&](int cb, const v4i& w4) __attribute__((always_inline)) {
        *reinterpret_cast<v4i*>(out_w + (32 * cb + lj) * OP + 16 * lg) = w4;
    };

    // The stage of token tile k is stage buffer k % 3.  One barrier per tile, before the first fragments of tile k + 1 are
    // read: wait for this wavefront's loads (all requested most of a tile earlier), barrier (now every wavefront's
    // loads of stage k + 1 have landed and nobody reads stage k - 1 any more); in the k-steps after it, one piece per
    // step: the stores of tile k - 1, the requests of stage k + 2 (into the buffer of k - 1) and of residual tile k + 1.
    const int a_base = (32 * grp + lj) * PITCH + 16 * lg;       // this lane's A fragment of k-step ks: + 32 ks
    v4i af[RG];
    {
        const int8_t* xa = Xs + LY::stage_offset(0) + a_base;
#pragma unroll
        for (int i = 0; i < RG - 1; ++i) af[i] = *reinterpret_cast<const v4i*>(xa + 32 * i);
    }

    v16i accA[NCB], accB[NCB];
    v2i rw[NCB][2] = {};
    Cursor c_req, c_res, c_out, c_prev;                         // stage being requested, residual tile being requested, tile k, tile k - 1
    int par = 0;                                                // residual tile k is in half `par` of the residual staging
    bool stored = false;                                        // the tile step before this one has issued stores

    // Token tile k in the stage buffer at offset b0 (the one at b1 holds stage k + 1, the one at b2 is free for stage
    // k + 2): multiply into `cur`.  With one wavefront per SIMD (GR == 1) there are two sets of accumulators and, when
    // `ep`, `prev` (tile k - 1) is requantised between the MFMAs, in the k-steps before the barrier, and stored after it.
    // With two wavefronts per SIMD (GR == 2) there is a single set: tile k is requantised right after its multiply
    // (the other wavefront of the SIMD multiplies meanwhile), and `ep` only says whether tile k - 1 is there to be
    // stored.  (Measured alternatives that gained nothing and are not kept: two sets with two wavefronts per SIMD,
    // which just fits 128 registers; holding the two wavefronts of a SIMD half a tile apart through the barrier.)
    constexpr bool TWO_SETS = GR == 1;
    auto tile_step = [&]<bool ep, bool fast>(int b0, int b1, int b2, v16i (&cur)[NCB], const v16i (&prev)[NCB]) __attribute__((always_inline)) {
        v4i ow[NCB];
        v2i sa = {}, sb = {};
        if (EPI == EPI_RESIDUAL && ep && TWO_SETS) read_res(par ^ 1, rw);
        constexpr int FIRST = SYNC;                            // k-step of the first piece of the work that follows the barrier
        const int8_t* xa = Xs + b0 + a_base;
        const int8_t* xb = Xs + b1 + a_base;
        // this tile's scalars, pinned in scalar registers (recomputing them at every use would cost more instructions
        // than the loads and stores themselves)
        const auto sc = [](int v) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(v); };
        const Span q_span = span_of(c_req, x_last, SR);
        const uint32_t q_dst = (uint32_t)sc(xs_off + b2);
        const Span r_span = EPI == EPI_RESIDUAL ? span_of(c_res, res_last, 32) : Span{nullptr, 0};
        const uint32_t r_dst = (uint32_t)sc(res_off + (par ^ 1) * RT);
        const __amdgpu_buffer_rsrc_t y_buf = tile_buffer(c_prev);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks == SYNC) {
                // this wavefront's loads have landed; the stores of the tile before, requested after them, may still be
                // on their way (memory operations complete in the order of their requests)
                if (stored) wait_vm<NCB>(); else wait_vm0();
                __syncthreads();
            }
            // fragment ks + RG - 1: of the next tile once this one runs out (valid since the barrier of this tile)
            if (ks + RG - 1 < KS) af[(ks + RG - 1) % RG] = *reinterpret_cast<const v4i*>(xa + 32 * (ks + RG - 1));
            else af[(ks + RG - 1) % RG] = *reinterpret_cast<const v4i*>(xb + 32 * (ks + RG - 1 - KS));
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                if (ks == 0) {
                    const v16i zero = {};
                    cur[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks % RG], W[cb][ks], zero, 0, 0, 0);
                } else {
                    cur[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks % RG], W[cb][ks], cur[cb], 0, 0, 0);
                }
            }
            // epilogue units of the previous tile, spread over k-steps 1 .. SYNC - 1 (not in step 0: the asm statements
            // that read the accumulators get no hazard wait states from the compiler, and the last MFMA of the previous
            // tile has only just been issued there)
            if (TWO_SETS && ep && ks >= 1 && ks < SYNC) {
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    if (1 + u * (SYNC - 1) / NU != ks) continue;
                    const int cb = u >> 2, d = u & 3;
                    ow[cb][d] = fast ? unit_fast(prev[cb], cb, d, rw) : unit_general(prev[cb], cb, d, rw);
                    if (d == 3) put_out(cb, ow[cb]);
                }
            }
            if (ks >= FIRST) {
                // loads first, stores last: a wait for the loads then leaves the stores out
                const int j = ks - FIRST;
                constexpr int S0 = KS - FIRST - NCB - 1;        // step of the first store's LDS read
                static_assert(S0 >= 0 && S0 + 1 >= NI - 1 && (EPI != EPI_RESIDUAL || S0 + 1 >= RNI - 1), "stores follow the loads");
                if (j < NI) issue_act_one(q_span, q_dst, j);
                if (EPI == EPI_RESIDUAL && j < RNI) issue_res_one(r_span, r_dst, j);     // past the last tile: a repeat, never used
                if (ep && j >= S0 + 1 && j <= S0 + NCB) store_write(y_buf, j - S0 - 1, sa, sb);
                if (ep && j >= S0 && j < S0 + NCB) store_read(j - S0, sa, sb);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (!TWO_SETS) {
            if (EPI == EPI_RESIDUAL) read_res(par, rw);         // residual tile k landed before barrier k
            asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");      // the last MFMAs have written the accumulators
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int cb = u >> 2, d = u & 3;
                ow[cb][d] = fast ? unit_fast(cur[cb], cb, d, rw) : unit_general(cur[cb], cb, d, rw);
                if (d == 3) put_out(cb, ow[cb]);
            }
        }
        // on to tile k + 1
        stored = ep;
        c_prev = c_out;
        advance(c_out, n_step);
        advance(c_req, x_step);
        advance(c_res, n_step);
        par ^= 1;
    };

    // the results of the last tile (tile ntile - 1 went into accA when ntile is odd)
    auto drain = [&]<bool fast>(const v16i (&last)[NCB]) __attribute__((always_inline)) {
        if (TWO_SETS) {
            v4i ow[NCB];
            if (EPI == EPI_RESIDUAL) { wait_vm0(); read_res(par ^ 1, rw); }
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");      // the last MFMAs have written the accumulators
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int cb = u >> 2, d = u & 3;
                ow[cb][d] = fast ? unit_fast(last[cb], cb, d, rw) : unit_general(last[cb], cb, d, rw);
                if (d == 3) put_out(cb, ow[cb]);
            }
        }
        const __amdgpu_buffer_rsrc_t y_buf = tile_buffer(c_prev);
#pragma unroll
        for (int s = 0; s < NCB; ++s) {
            v2i a, b;
            store_read(s, a, b);
            store_write(y_buf, s, a, b);
        }
    };
    auto start = [&](int ahead) __attribute__((always_inline)) {
        c_req = cursor(P.x, P.ldx, ahead, 0);
        c_res = cursor(P.residual, N, 1, 32 * grp);
        c_out = cursor(P.y, N, 0, 32 * grp);
        c_prev = c_out;
        par = 0;
    };
    auto run_one_set = [&]<bool fast>() __attribute__((always_inline)) {
        start(2);
        tile_step.template operator()<false, fast>(LY::stage_offset(0), LY::stage_offset(1), LY::stage_offset(2), accA, accA);
        int b0 = LY::stage_offset(1), b1 = LY::stage_offset(2), b2 = LY::stage_offset(0);
        for (int k = 1; k < ntile; ++k) {
            tile_step.template operator()<true, fast>(b0, b1, b2, accA, accA);
            const int t = b0; b0 = b1; b1 = b2; b2 = t;
        }
        drain.template operator()<fast>(accA);
    };
    auto run = [&]<bool fast>() __attribute__((always_inline)) {
        if (!TWO_SETS) {
            run_one_set.template operator()<fast>();
            return;
        }
        start(2);
        tile_step.template operator()<false, fast>(LY::stage_offset(0), LY::stage_offset(1), LY::stage_offset(2), accA, accB);
        int b0 = LY::stage_offset(1), b1 = LY::stage_offset(2), b2 = LY::stage_offset(0);
        for (int k = 1; k < ntile; k += 2) {
            tile_step.template operator()<true, fast>(b0, b1, b2, accB, accA);
            { const int t = b0; b0 = b1; b1 = b2; b2 = t; }
            if (k + 1 < ntile) {
                tile_step.template operator()<true, fast>(b0, b1, b2, accA, accB);
                const int t = b0; b0 = b1; b1 = b2; b2 = t;
            }
        }
        if (ntile & 1) drain.template operator()<fast>(accA); else drain.template operator()<fast>(accB);
    };
    if (fast24) run.template operator()<true>(); else run.template operator()<false>();
    wait_vm0();            // LDS-direct loads still in flight (repeats of the last stage) must land before the LDS is released
}

template <int EPI, int KS, int NCB, int GR>
hipError_t launch_rs(hipStream_t s, const RsParams& P, int grid) {
    constexpr size_t lds_bytes = RsLayout<KS, NCB, EPI, GR>::TOTAL;
    hipLaunchKernelGGL((gemm_rs_kernel<EPI, KS, NCB, GR>), dim3(grid), dim3(256 * GR), lds_bytes, s, P);
    return hipGetLastError();
}

template <int KS, int NCB, int GR>
hipError_t launch_rs_epi(hipStream_t s, RsParams& P, const LinearArgs& a) {
    const int nt = a.N / 32;
    P.slabs = (nt + 4 * NCB - 1) / (4 * NCB);
    P.stages = (int)((a.M + 32 * GR - 1) / (32 * GR));
    P.q = std::max(1, std::min(P.stages, num_cus() / P.slabs));
    const int grid = P.q * P.slabs;
    if (KS < 12 && a.residual) return hipErrorInvalidValue;     // (refused by linear_rs_takes)
    if constexpr (KS >= 12) {                                   // (rows of 192 bytes: the tile's k-steps do not hold a residual layer's loads)
        if (a.residual) return launch_rs<EPI_RESIDUAL, KS, NCB, GR>(s, P, grid);
    }
    if (a.gelu) return launch_rs<EPI_GELU, KS, NCB, GR>(s, P, grid);
    return launch_rs<EPI_PLAIN, KS, NCB, GR>(s, P, grid);
}

}  // namespace

// Shapes this kernel takes: K = 384 or 768, or 192 without a residual (the weights of a wavefront must fit its
// registers, and the k-steps are unrolled), N a multiple of 32, dense rows, at most 2^30 of them; offsets inside the weight matrix and inside a token
// tile are 32-bit.
bool linear_rs_takes(const LinearArgs& a) {
    if (a.K != 384 && a.K != 768 && !(a.K == 192 && !a.residual)) return false;
    if ((int64_t)a.N * a.K > 0x7fffffffLL) return false;
    if (a.M > (1 << 30)) return false;                         // row counts are kept in 32 bits
    return (a.N & 31) == 0 && (a.ldx == 0 || a.ldx == a.K) && a.M >= 1;
}

hipError_t launch_linear_rs(hipStream_t s, const LinearArgs& a) {
    RsParams P;
    P.x = a.x; P.w = a.w; P.bias = a.bias; P.rq_b = a.rq_b; P.rq_c = a.rq_c;
    P.residual = a.residual; P.res_rq = a.res_rq; P.gelu_p = a.gelu_p; P.gelu_rq = a.gelu_rq;
    P.y = a.y; P.M = a.M; P.N = a.N; P.ldx = a.K; P.rnd = a.floor_shift ? 0 : 1;
    // K = 384: 64 channels per wavefront leave room for two wavefronts per SIMD; K = 768: one
    if (a.K == 192) return launch_rs_epi<6, 2, 2>(s, P, a);
    if (a.K == 384) return launch_rs_epi<12, 2, 2>(s, P, a);
    return launch_rs_epi<24, 2, 1>(s, P, a);
}

}  // namespace ivit
