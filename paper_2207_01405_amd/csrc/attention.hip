// Fused integer multi-head attention for gfx950 (I-ViT, arXiv 2207.01405: Eq. 3-4 with the dyadic
// pipeline of Sec. 3.2 and Shiftmax of Sec. 3.3 / Algorithm 1):
//   A = requant(Q K^T) [+ relative-position bias];  P = Shiftmax(rows of A);  O = requant(P V).
//
// One workgroup (4 wavefronts) handles one (image-or-window, head) at a time: K and V live in LDS, both
// row by row as they come from memory, and each wavefront takes 16 query tokens at a time.  Scores are produced by
// v_mfma_i32_16x16x64_i8 (d = 64) or 16x16x32 (d = 32) in the orientation keys x queries, so that a lane
// holds, for ONE query, four keys of every 16-key tile: the whole score row of a query sits in the
// registers of four lanes.  Max and sum need an in-lane pass plus two cross-lane steps; ShiftExp is a
// table lookup on Delta = max - value (at most 510); the packed int8 probabilities are already laid out as
// the MFMA "B" operand (contraction index = key) of O^T = V^T P^T, so scores and probabilities never
// leave registers.  The "A" operand of that product, V^T, is read from the rows of V with the transposing
// LDS read of gfx950 (ds_read_b64_tr_b8): the lanes of a 16-lane block name eight key rows each for the even and
// the odd lanes, so the key order the register layout asks for and the choice of features are a matter of which
// addresses the lanes name, and V needs no rearranging when it is written.  One exchange between neighbouring
// lane blocks then gives every lane d/4 consecutive features of its query: one 16-byte (d = 64) store.
//
// The kernel is bound by the vector ALU (about a dozen integer operations per score element against
// 2 d multiply-accumulates on the matrix core), so the per-element path is kept minimal: debug taps, the
// bias and the 64-bit requantisation are compiled in only when asked for (template flags), and masking
// of padded keys is done only for key tiles that are not completely valid.
#include <algorithm>

#include "ivit_kernels.hpp"

namespace ivit {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int ATT_WAVES = 4, ATT_THREADS = 64 * ATT_WAVES;   // wavefronts per workgroup

typedef int v2i_att __attribute__((ext_vector_type(2)));

// Constants of the 24-bit requantisation of one per-tensor dyadic pair (no bias): the accumulator is limited to
// [lo, hi], the first values that give -127 / +127, after which (v b + 2^(c-1)) 2^(24-c) fits 32 bits with the int8
// result in its top byte.  Valid for c <= 24, b < 2^(c-1) and bounds inside 24 bits (narrow_of() decides).
struct Narrow { int32_t lo, hi, mb, ad; };

// FAST: 0 general 64-bit requantisation, 1 pairs that fit 32 bits, 2 the 24-bit form above (and the 24-bit IntDiv).
template <int FAST>
__device__ __forceinline__ int32_t requant8(int32_t v, Dyadic d, Narrow n, int32_t rnd) {
    if (FAST == 2) {
        // The median of three as the one instruction, by hand because the compiler cannot know lo <= hi.  The compiler
        // does not see what an asm statement reads and puts no wait states between it and the producer of v: v must
        // have been written long before (here: MFMA results of a whole tile sweep), never by the instruction just
        // before (a dot product feeding this directly was seen to read a stale register).
        int32_t m;
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(m) : "v"(v), "v"(n.lo), "v"(n.hi));
        return (__mul24(m, n.mb) + n.ad) >> 24;
    }
    return FAST ? clamp8(rnd_shift_fit32(v, d.b, d.c, rnd)) : requant64(v, d.b, d.c, rnd);
}

// Four values at once: the four medians first, then the four multiply-adds, so that no instruction reads the result of
// the asm statement right before it (the compiler, not knowing what the statement is, would put a wait state there).
template <int FAST>
__device__ __forceinline__ void requant8x4(int32_t (&v)[4], Dyadic d, Narrow n, int32_t rnd) {
    if (FAST == 2) {
        int32_t m[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) asm("v_med3_i32 %0, %1, %2, %3" : "=v"(m[r]) : "v"(v[r]), "v"(n.lo), "v"(n.hi));
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (__mul24(m[r], n.mb) + n.ad) >> 24;
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = requant8<FAST>(v[r], d, n, rnd);
    }
}

// FAST: both dyadic pairs are rescales by at most 1 with c <= 31 (32-bit requantisation) and the row sum always
// exceeds 2^(k_out-1), so that IntDiv is one multiply-high by the pre-shifted reciprocal.
// TFIX: 0, or the token count known at compile time (49, the 7 x 7 windows; 197, the 14 x 14 patches with a class token):
// every test of a key or query against T then folds, and the absent keys of the last key tile cost nothing.
template <int D, int NKT, bool TAPS, bool BIAS, bool MASK, int FAST, int TFIX = 0>
__global__ __launch_bounds__(ATT_THREADS, 3) void attention_kernel(const int8_t* __restrict__ qkv,
                                                        const int8_t* __restrict__ rel_bias,
                                                        const int8_t* __restrict__ mask, int n_mask,
                                                        const int32_t* __restrict__ tok_index, int n_win,
                                                        int8_t* __restrict__ o, int n_items, int split, int T_arg, int C, int H,
                                                        Dyadic qk, ShiftParams sm, Dyadic pv, Narrow nqk, Narrow npv, int rnd,
                                                        int8_t* __restrict__ tap_s, int8_t* __restrict__ tap_p) {
    const int T = TFIX ? TFIX : T_arg;
    constexpr int KROW = D + 16;                  // K row pitch (bytes)
    constexpr int NKC = (NKT + 3) / 4;            // 64-key chunks of the P V contraction
    constexpr int VP = D == 64 ? 72 : 40;         // V row pitch (bytes): the transposing reads below meet no bank twice
    constexpr int ND = D / 16;                    // 16-feature tiles of the output
    constexpr int DCH = D / 16;                   // 16-byte chunks per K / V row
    __shared__ __align__(16) int8_t Ks[NKT * 16 * KROW];
    __shared__ __align__(16) int8_t Vs[NKC * 64 * VP];
    // table of ShiftExp(-delta): int8 scores give delta <= 254; with a bias and the mask the exact range is wider,
    // and beyond the table the value is 0 whenever it can occur (see the mask comment below)
    constexpr int NLUT = MASK ? 1024 : (BIAS ? 512 : 256);
    __shared__ uint32_t lut[NLUT];                // (whole words: the value comes out of the read ready to use)

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int li = lane & 15, lg = lane >> 4;
    // (the ShiftExp table is filled inside the first item, once its loads of K, V and Q are on their way)
    // keys beyond the 16-key tiles but inside the last 64-key chunk multiply probabilities that are zero;
    // clear their rows once so that no uninitialised LDS is ever read
    for (int i = NKT * 16 * VP / 4 + tid; i < NKC * 64 * VP / 4; i += ATT_THREADS) reinterpret_cast<uint32_t*>(Vs)[i] = 0u;

    const int sh = sm.m_bits - (sm.k_out - 1);
    const uint32_t top = (1u << (sm.k_out - 1)) - 1u;
    const int nqt = (T + 15) >> 4;
    const int nfull = T >> 4;                      // key tiles whose 16 keys all exist

    // workgroups of one XCD (block id modulo 8) take consecutive items: the heads of an image share 128-byte lines of
    // qkv (two 64-byte head slices per line), which then meet in one L2
    const int G = gridDim.x, xcd = blockIdx.x % 8;
    const int first = xcd * (G / 8) + min(xcd, G % 8) + blockIdx.x / 8;
    // Rows of qkv / o.  Without a table token t of window b is row b T + t.  With one (BIAS instances only) the rows
    // come from the index table of the window's position inside its image; an entry outside the image is clamped,
    // never followed.  The table entries this thread needs for an item (its K / V pieces and its first query tile) are
    // fetched one item ahead, so that the loads of K, V and Q never wait for an index.
    constexpr int NPC = (NKT * 16 * DCH + ATT_THREADS - 1) / ATT_THREADS;     // 16-byte pieces per thread and operand
    const int tpi = n_win * T;                     // tokens per image
    const bool gather = BIAS && tok_index != nullptr;
    int kvrow[NPC], qrow0 = 0, kvnext[NPC], qnext = 0;
    auto fetch_rows = [&](int work, int (&kv)[NPC], int& qr) {
        const int item = work / split, b = item / H;
        const int32_t* tr = tok_index + (b % n_win) * T;
        const int r0 = (b / n_win) * tpi;
#pragma unroll
        for (int it = 0; it < NPC; ++it) {
            const int key = min((tid + ATT_THREADS * it) / DCH, T - 1);
            kv[it] = r0 + (int)min((uint32_t)tr[key], (uint32_t)(tpi - 1));
        }
        qr = r0 + (int)min((uint32_t)tr[min((work % split + split * ((wv + item) % ATT_WAVES)) * 16 + li, T - 1)], (uint32_t)(tpi - 1));
    };
    // a work item is one (window, head) or, with split > 1, every split-th query tile of it: when there are too few
    // (window, head) pairs to give every workgroup slot of the device one, each pair is shared by `split` workgroups
    // (K and V are staged by each of them; they are small)
    const int n_work = n_items * split;
    if (BIAS) { if (gather && first < n_work) fetch_rows(first, kvrow, qrow0); }

    for (int work = first; work < n_work; work += G) {
        const int item = work / split, part = work % split;
        // this wavefront's first query tile.  The tiles rarely divide evenly among the wavefronts (13 tiles of 197
        // tokens: one wavefront gets four, the others three); which wavefront starts moves on with the item, so that
        // the workgroups that share a compute unit do not all give the extra tile to the same SIMD.
        const int qt0 = part + split * ((wv + item) % ATT_WAVES);
        const int b = item / H, h = item % H;
        const int8_t* base = qkv + h * D;
        const int32_t* trow = gather ? tok_index + (b % n_win) * T : nullptr;
        const int64_t row0 = gather ? (int64_t)(b / n_win) * tpi : (int64_t)b * T;
        auto row_of = [&](int t) -> int64_t {      // any token of this window (t < T)
            if (BIAS) { if (trow) return row0 + (int)min((uint32_t)trow[t], (uint32_t)(tpi - 1)); }
            return row0 + t;
        };
        auto q_row = [&](int qt) -> int64_t {      // row of this lane's query of tile qt
            if (BIAS) { if (gather && qt == qt0) return qrow0; }
            return row_of(min(qt * 16 + li, T - 1));
        };
        __syncthreads();                           // table ready / previous item's readers done
        // the query fragment of a tile is requested one tile ahead, the first one together with K and V
        auto load_q64 = [&](int qt) { return *reinterpret_cast<const v4i*>(base + q_row(qt) * 3 * C + 16 * lg); };
        auto load_q32 = [&](int qt) { return *reinterpret_cast<const long*>(base + q_row(qt) * 3 * C + 8 * lg); };
        v4i qn64 = {0, 0, 0, 0};
        long qn32 = 0;
        if (D == 64) qn64 = load_q64(qt0); else qn32 = load_q32(qt0);
        // all of this thread's K and V pieces are requested before the first one is used: one memory latency per item
        v4i kreg[NPC], vreg[NPC];
#pragma unroll
        for (int it = 0; it < NPC; ++it) {
            const int c = tid + ATT_THREADS * it;
            const int key = min(c / DCH, T - 1), part = c % DCH;
            int64_t row = row0 + key;
            if (BIAS) { if (gather) row = kvrow[it]; }
            const int8_t* kv_row = base + row * 3 * C + 16 * part;
            kreg[it] = *reinterpret_cast<const v4i*>(kv_row + C);
            vreg[it] = *reinterpret_cast<const v4i*>(kv_row + 2 * C);
        }
        if (work == first) {                       // the table, while the first loads are in flight (visible after the barrier below)
            for (int i = tid; i < NLUT; i += ATT_THREADS) lut[i] = shiftexp(-i, sm.i0, sm.n_shift);
        }
        const int64_t orow0 = q_row(qt0);          // output row of the first query tile (before the indices move on)
        if (BIAS) {
            if (gather && work + G < n_work) {
                fetch_rows(work + G, kvnext, qnext);
#pragma unroll
                for (int it = 0; it < NPC; ++it) kvrow[it] = kvnext[it];
                qrow0 = qnext;
            }
        }
#pragma unroll
        for (int it = 0; it < NPC; ++it) {
            const int c = tid + ATT_THREADS * it;
            if (c >= NKT * 16 * DCH) break;
            const int key = c / DCH, part = c % DCH;
            const v4i kv = key < T ? kreg[it] : v4i{0, 0, 0, 0};
            const v4i vv = key < T ? vreg[it] : v4i{0, 0, 0, 0};
            *reinterpret_cast<v4i*>(&Ks[key * KROW + 16 * part]) = kv;
            v2i_att* vdst = reinterpret_cast<v2i_att*>(&Vs[key * VP + 16 * part]);      // (rows are 8-byte aligned)
            vdst[0] = v2i_att{vv[0], vv[1]};
            vdst[1] = v2i_att{vv[2], vv[3]};
        }
        __syncthreads();

        for (int qt = qt0; qt < nqt; qt += split * ATT_WAVES) {
            const int q = qt * 16 + li;            // this lane's query token
            const int qc = min(q, T - 1);
            int32_t sc[NKT][4];
            // ---- scores: S^T tile t = K_t (16 keys x D) . Q^T (D x 16 queries)
            if (D == 64) {
                const v4i qf = qn64;
                qn64 = load_q64(qt + split * ATT_WAVES);
#pragma unroll
                for (int t = 0; t < NKT; ++t) {
                    const v4i kf = *reinterpret_cast<const v4i*>(&Ks[(16 * t + li) * KROW + 16 * lg]);
                    const v4i r = __builtin_amdgcn_mfma_i32_16x16x64_i8(kf, qf, v4i{0, 0, 0, 0}, 0, 0, 0);
                    sc[t][0] = r[0]; sc[t][1] = r[1]; sc[t][2] = r[2]; sc[t][3] = r[3];
                    if ((t & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // at most four K fragments in flight
                }
            } else {
                const long qf = qn32;
                qn32 = load_q32(qt + split * ATT_WAVES);
#pragma unroll
                for (int t = 0; t < NKT; ++t) {
                    const long kf = *reinterpret_cast<const long*>(&Ks[(16 * t + li) * KROW + 8 * lg]);
                    const v4i r = __builtin_amdgcn_mfma_i32_16x16x32_i8(kf, qf, v4i{0, 0, 0, 0}, 0, 0, 0);
                    sc[t][0] = r[0]; sc[t][1] = r[1]; sc[t][2] = r[2]; sc[t][3] = r[3];
                    if ((t & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
            }
            // requant8 reads the MFMA results through an asm statement, which gets no hazard wait states from the
            // compiler: the last MFMA above (8 passes: 10 wait states) is given its time by hand
            if (FAST == 2) {
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_nop 7");
                asm volatile("s_nop 3");
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- requantise, add the bias, row maximum.  Lane (li, lg) holds keys 16 t + 4 lg + r.
            const int64_t tap_row = ((int64_t)item * T + qc) * T;
            // BIAS: a relative-position bias and / or the shifted-window mask.  A masked key gets -100 I_0 (the -100
            // the windowed models add, at the integer scale of the logits).  All of this is exact int32 arithmetic;
            // only the table is finite: an unmasked key is at most 508 below the row maximum, and for a masked key
            // ShiftExp(-delta) is 0 for every delta >= 1024 it can reach (delta >= 100 I_0 - 508, and a non-zero
            // value needs delta < 23 I_0), so entries past the table read as 0.
            const int8_t* brow = (BIAS && rel_bias) ? rel_bias + ((int64_t)h * T + qc) * T : nullptr;
            const int8_t* mrow = MASK ? mask + ((int64_t)(b % n_mask) * T + qc) * T : nullptr;
            const int32_t mask_add = -100 * sm.i0;
            int32_t mx = INT32_MIN;
#pragma unroll
            for (int t = 0; t < NKT; ++t) {
                if (t < nfull) {                   // uniform: every key of the tile exists
                    // the lane's four keys are four consecutive bytes of the bias and the mask row: one (unaligned)
                    // dword each instead of four byte loads
                    uint32_t bw = 0, mw = 0;
                    if (BIAS) { if (!MASK || brow) __builtin_memcpy(&bw, brow + 16 * t + 4 * lg, 4); }
                    if (MASK) __builtin_memcpy(&mw, mrow + 16 * t + 4 * lg, 4);
                    requant8x4<FAST>(sc[t], qk, nqk, rnd);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int key = 16 * t + 4 * lg + r;
                        int32_t a = sc[t][r];
                        if (TAPS) { if (tap_s && q < T) tap_s[tap_row + key] = (int8_t)a; }
                        if (BIAS) a += (int32_t)(int8_t)(bw >> (8 * r));
                        if (MASK) { if ((mw >> (8 * r)) & 0xffu) a += mask_add; }
                        sc[t][r] = a;
                    }
                    mx = max(mx, max(sc[t][0], sc[t][1]));       // two three-operand maxima per tile
                    mx = max(mx, max(sc[t][2], sc[t][3]));
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int key = 16 * t + 4 * lg + r;
                        int32_t a = requant8<FAST>(sc[t][r], qk, nqk, rnd);
                        if (key < T) {
                            if (TAPS) { if (tap_s && q < T) tap_s[tap_row + key] = (int8_t)a; }
                            if (BIAS) { if (!MASK || brow) a += brow[key]; }
                            if (MASK) { if (mrow[key]) a += mask_add; }
                            mx = max(mx, a);
                        }
                        sc[t][r] = a;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);     // keep the 64-bit temporaries of one tile at a time
            }
            mx = rows_allreduce(mx, [](int32_t a, int32_t b) { return max(a, b); });
            // ---- ShiftExp by table, row sum.  The byte offset 4 (max - a) of the table entry is one 24-bit multiply-add.
            int32_t sum = 0;
            const int32_t mx4 = 4 * mx;
            const char* lut_b = reinterpret_cast<const char*>(lut);
#pragma unroll
            for (int t = 0; t < NKT; ++t) {
                if (t < nfull) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int32_t e;
                        if (MASK) {
                            const int32_t delta = mx - sc[t][r];
                            e = delta < NLUT ? (int32_t)lut[min(delta, NLUT - 1)] : 0;
                        } else {
                            e = (int32_t)*reinterpret_cast<const uint32_t*>(lut_b + (__mul24(sc[t][r], -4) + mx4));
                        }
                        sc[t][r] = e;
                        sum += e;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int key = 16 * t + 4 * lg + r;
                        int32_t e;
                        if (MASK) {
                            const int32_t delta = key < T ? mx - sc[t][r] : NLUT;
                            e = delta < NLUT ? (int32_t)lut[min(delta, NLUT - 1)] : 0;
                        } else {
                            e = key < T ? (int32_t)lut[mx - sc[t][r]] : 0;
                        }
                        sc[t][r] = e;
                        sum += e;
                    }
                }
                if (t & 1) __builtin_amdgcn_sched_barrier(0);
            }
            sum = rows_allreduce(sum, [](int32_t a, int32_t b) { return a + b; });
            // ---- IntDiv and packing: the four keys of tile t become one word of the "B" operand
            const uint32_t inv = (1u << sm.m_bits) / (uint32_t)sum;
            const uint32_t inv_hi = FAST ? inv << (32 - sh) : 0u;      // FAST: inv < 2^sh, 1 <= sh <= 31
            uint32_t pk[NKC * 4];
#pragma unroll
            for (int t = 0; t < NKC * 4; ++t) pk[t] = 0u;
#pragma unroll
            for (int t = 0; t < NKT; ++t) {
                if (FAST == 2 && !TAPS) {
                    // M - (k_out - 1) = 24 here: inv < 2^24 and the ShiftExp values are below 2^16, so inv * e (at most
                    // 2^31) is one 24-bit multiply and the quotient is its top byte
                    uint32_t pr[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) pr[r] = mul_u24(inv, (uint32_t)sc[t][r]);
                    pk[t] = __builtin_amdgcn_perm(pr[1], pr[0], 0x0c0c0703u) | __builtin_amdgcn_perm(pr[3], pr[2], 0x07030c0cu);
                    continue;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (TAPS) {
                        const uint32_t p = FAST ? min(__umulhi(inv_hi, (uint32_t)sc[t][r]), top)
                                                : min((inv * (uint32_t)sc[t][r]) >> sh, top);
                        const int key = 16 * t + 4 * lg + r;
                        if (tap_p && q < T && key < T) tap_p[tap_row + key] = (int8_t)p;
                        pk[t] |= p << (8 * r);
                    } else {
                        // IntDiv gives at most 2^(k_out-1), which fits a byte: clamp the four of a word together below
                        const uint32_t p = FAST ? __umulhi(inv_hi, (uint32_t)sc[t][r]) : (inv * (uint32_t)sc[t][r]) >> sh;
                        pk[t] |= p << (8 * r);
                    }
                }
            }
            if (!TAPS) {
#pragma unroll
                for (int t = 0; t < NKT; ++t) pk[t] -= (pk[t] >> (sm.k_out - 1)) & 0x01010101u;   // bytewise min(p, 2^(k_out-1) - 1)
            }
            // ---- O^T = V^T P^T : "A" = V^T rows (features), "B" = packed probabilities (keys x queries).
            // Contraction position 16 lg + 4 j + r of chunk c is key 64 c + 16 j + 4 lg + r (the layout of pk).  A
            // transposing read hands lane i of a 16-lane block byte i' of the 8-byte row named by lane 2 i' (i < 8)
            // or 2 i' + 1 (i >= 8): the even lanes name keys j = 2 hh + (b >> 2), r = b & 3 (b = half the lane number)
            // at features 8 n .. 8 n + 7, the odd lanes the same keys at features D/2 + 8 n .., so that row i of
            // output tile n is feature 8 n + i (i < 8) or D/2 + 8 n + i - 8.
            const int8_t* vbase = Vs + (4 * lg + 16 * ((li >> 1) >> 2) + ((li >> 1) & 3)) * VP + ((li & 1) ? D / 2 : 0);
            v4i oacc[ND];
#pragma unroll
            for (int n = 0; n < ND; ++n) oacc[n] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int c = 0; c < NKC; ++c) {
                const v4i pf = {(int)pk[4 * c], (int)pk[4 * c + 1], (int)pk[4 * c + 2], (int)pk[4 * c + 3]};
#pragma unroll
                for (int n = 0; n < ND; ++n) {
                    typedef v2i_att __attribute__((address_space(3))) * lds_v2i;
                    const v2i_att v0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(vbase + (64 * c) * VP + 8 * n));
                    const v2i_att v1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(vbase + (64 * c + 32) * VP + 8 * n));
                    const v4i vf = {v0[0], v0[1], v1[0], v1[1]};
                    oacc[n] = __builtin_amdgcn_mfma_i32_16x16x64_i8(vf, pf, oacc[n], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- requantise and store: lane block lg holds rows 4 lg + r of every tile n, i.e. features
            // (lg >= 2 ? D/2 : 0) + 8 n + 4 (lg & 1) + r of query q; exchanging tile n + ND/2 of the even blocks with tile
            // n of the odd ones leaves block lg with the D/4 consecutive features lg (D/4) ..
            if (FAST == 2) {                       // as above: asm readers of fresh MFMA results
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_nop 7");
                asm volatile("s_nop 3");
                __builtin_amdgcn_sched_barrier(0);
            }
            uint32_t ow[ND];
#pragma unroll
            for (int n = 0; n < ND; ++n) {
                uint32_t w = 0;
                int32_t ov[4] = {oacc[n][0], oacc[n][1], oacc[n][2], oacc[n][3]};
                requant8x4<FAST>(ov, pv, npv, rnd);
#pragma unroll
                for (int r = 0; r < 4; ++r) w |= ((uint32_t)ov[r] & 0xffu) << (8 * r);
                ow[n] = w;
            }
#pragma unroll
            for (int n = 0; n < ND / 2; ++n) {
                // (odd blocks of the first operand <-> even blocks of the second)
                const auto sw = __builtin_amdgcn_permlane16_swap(ow[n], ow[n + ND / 2], false, false);
                ow[n] = sw[0]; ow[n + ND / 2] = sw[1];
            }
            if (q < T) {
                int8_t* op = o + (qt == qt0 ? orow0 : row_of(q)) * C + h * D + lg * (D / 4);
                if (D == 64) *reinterpret_cast<uint4*>(op) = make_uint4(ow[0], ow[2], ow[1], ow[3]);
                else *reinterpret_cast<uint2*>(op) = make_uint2(ow[0], ow[1 % ND]);
            }
        }
    }
}

// The 24-bit constants of a pair, or false when the pair needs the wider forms.
// (rnd = 1: the rounding addend h is 2^(c-1); rnd = 0: the bare shift of Eq. 10, h = 0)
static bool narrow_of(Dyadic d, int rnd, Narrow& n) {
    if (d.c < 1 || d.c > 24 || d.b < 1 || d.b >= (1 << (d.c - 1))) return false;
    const int64_t half = (int64_t)rnd << (d.c - 1), two_c = (int64_t)1 << d.c;
    const int64_t hi = (127 * two_c - half + d.b - 1) / d.b;             // first v with (v b + h) >> c >= 127
    const int64_t lo = -((126 * two_c + 1 + half + d.b - 1) / d.b);      // last v with (v b + h) >> c <= -127
    if (lo < -(1 << 23) || hi >= (1 << 23)) return false;
    n.lo = (int32_t)lo; n.hi = (int32_t)hi; n.mb = d.b << (24 - d.c); n.ad = (int32_t)(half << (24 - d.c));
    return true;
}

template <int D, int NKT>
static void launch_flags(hipStream_t s, const AttentionArgs& a, int grid, int split, bool taps, bool bias, bool fast) {
    const int n_items = a.B * a.H;
    Narrow nqk{}, npv{};
    // the 24-bit forms: both requantisations, and IntDiv with its quotient in the top byte of a 24-bit product
    const int rnd = a.floor_shift ? 0 : 1;
    const bool narrow = narrow_of(a.qk_rq, rnd, nqk) && narrow_of(a.pv_rq, rnd, npv) && a.sm.m_bits - (a.sm.k_out - 1) == 24;
#define IVIT_ATT(TAPS_, BIAS_, MASK_, FAST_, TFIX_)                                                                         \
    hipLaunchKernelGGL((attention_kernel<D, NKT, TAPS_, BIAS_, MASK_, FAST_, TFIX_>), dim3(grid), dim3(ATT_THREADS), 0, s,     \
                       a.qkv, a.rel_bias, a.mask, a.n_mask, a.tok_index, a.n_win, a.o, n_items, split, a.T, a.C, a.H, a.qk_rq, \
                       a.sm, a.pv_rq, nqk, npv, rnd, a.tap_scores, a.tap_probs)
    // the production paths are <no taps, fast>, with the 24-bit requantisation when both pairs allow it; everything else
    // shares one fully general instantiation per bias / mask combination (a mask is always compiled with the bias code,
    // which tests the bias pointer)
    const bool masked = a.mask != nullptr;
    constexpr int T49 = (D == 32 && NKT == 4) ? 49 : 0;                        // the windowed models' shape
    constexpr int T197 = (D == 64 && NKT == 13) ? 197 : 0;                     // 14 x 14 patches and a class token
    if (T197 && a.T == 197 && !taps && fast && !bias) {
        if (narrow) IVIT_ATT(false, false, false, 2, T197); else IVIT_ATT(false, false, false, 1, T197);
    } else if (T49 && a.T == 49 && !taps && fast && bias) {
        if (masked) { if (narrow) IVIT_ATT(false, true, true, 2, T49); else IVIT_ATT(false, true, true, 1, T49); }
        else { if (narrow) IVIT_ATT(false, true, false, 2, T49); else IVIT_ATT(false, true, false, 1, T49); }
    } else if (!taps && fast) {
        if (masked) { if (narrow) IVIT_ATT(false, true, true, 2, 0); else IVIT_ATT(false, true, true, 1, 0); }
        else if (bias) { if (narrow) IVIT_ATT(false, true, false, 2, 0); else IVIT_ATT(false, true, false, 1, 0); }
        else { if (narrow) IVIT_ATT(false, false, false, 2, 0); else IVIT_ATT(false, false, false, 1, 0); }
    } else {
        if (masked) IVIT_ATT(true, true, true, 0, 0);
        else if (bias) IVIT_ATT(true, true, false, 0, 0);
        else IVIT_ATT(true, false, false, 0, 0);
    }
#undef IVIT_ATT
}

template <int D>
static hipError_t launch_d(hipStream_t s, const AttentionArgs& a, int grid, int split, int nkt, bool taps, bool bias, bool fast) {
    if (nkt <= 4) launch_flags<D, 4>(s, a, grid, split, taps, bias, fast);
    else if (nkt <= 8) launch_flags<D, 8>(s, a, grid, split, taps, bias, fast);
    else if (nkt <= 13) launch_flags<D, 13>(s, a, grid, split, taps, bias, fast);
    else launch_flags<D, 16>(s, a, grid, split, taps, bias, fast);
    return hipGetLastError();
}

static bool fits32_host(Dyadic d) { return d.c >= 1 && d.c <= 31 && d.b >= 1 && (uint32_t)d.b <= (1u << d.c); }

hipError_t launch_attention(hipStream_t s, const AttentionArgs& a) {
    const int64_t n_items = (int64_t)a.B * a.H;
    if (n_items == 0) return hipSuccess;
    const int nkt = (a.T + 15) / 16;
    // With fewer (window, head) pairs than compute units, several workgroups share a pair (each takes every split-th
    // query tile) so that the device is filled: about two workgroups per CU, down to one tile per wavefront.  With
    // more pairs than that sharing only adds staging work (measured: 768 pairs, 30 us unshared, 33 us shared by two).
    const int split = (int)std::max<int64_t>(1, std::min<int64_t>(2 * (int64_t)num_cus() / n_items, (nkt + ATT_WAVES - 1) / ATT_WAVES));
    // workgroups per CU: windows of at most 64 tokens need little LDS and few registers, and their short items are
    // bound by latency, so many more workgroups are kept in flight (8192 windows x 3 heads: 86 us with 4, 72 us with 16)
    // (up to 16 per CU, as long as each still loops over about four items, which keeps the rounds even)
    const int64_t n_work = n_items * split, cus = num_cus();
    const int64_t wgs = nkt <= 4 ? std::max<int64_t>(4 * cus, std::min<int64_t>(16 * cus, n_work / 4)) : 4 * cus;
    const int grid = (int)std::min<int64_t>(n_work, wgs);
    const int d = a.C / a.H;
    const int sh = a.sm.m_bits - (a.sm.k_out - 1);
    const bool fast = fits32_host(a.qk_rq) && fits32_host(a.pv_rq) && sh >= 1 &&
                      ((int64_t)a.sm.i0 << a.sm.n_shift) > ((int64_t)1 << (a.sm.k_out - 1));
    const bool taps = a.tap_scores || a.tap_probs;
    const int64_t R = (int64_t)a.B * a.T;
    TraceScope trace(s, KIND_ATTENTION, 4 * n_items * a.T * a.T * d, 4 * R * a.C + (a.rel_bias ? (int64_t)a.H * a.T * a.T : 0));
    const bool bias = a.rel_bias != nullptr || a.mask != nullptr || a.tok_index != nullptr;
    return d == 64 ? launch_d<64>(s, a, grid, split, nkt, taps, bias, fast) : launch_d<32>(s, a, grid, split, nkt, taps, bias, fast);
}

}  // namespace ivit
