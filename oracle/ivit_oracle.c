/*
 * I-ViT integer-only encoder forward: CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, obviously
 * correct statement of what the hot path computes.  It exists so that the GPU
 * library can be compared with it bit for bit; nothing in the product path may
 * call it, and it shares no code, header, table or constant with the HIP
 * sources.  Every intermediate is int64; there is no blocking, fusion or
 * reordering beyond what the paper's equations and algorithms state.
 *
 * Sources (I-ViT, arXiv 2207.01405): Sec. 3.1 Eq. 1-6 (block structure,
 * symmetric quantisation), Sec. 3.2 Eq. 7-10 (dyadic pipeline), Sec. 3.3
 * Eq. 11-16 + Algorithm 1 (Shiftmax), Sec. 3.4 Eq. 17-18 + Algorithm 2
 * (ShiftGELU), Sec. 3.5 Eq. 19-20 (I-LayerNorm).
 *
 * Where the paper is silent the reading taken is stated at the function.
 * Functions whose reading is a choice, not fixed by the paper (rounding mode of
 * the requantisation, I-LayerNorm's integer affine step, the residual add) are
 * pinned by the tests only against the mathematics of that reading.
 *
 * Conventions: ">>" on a signed value is an arithmetic shift (floor division
 * by a power of two; gcc guarantees this for signed operands); fdiv() is floor
 * division.  Tensors are row-major.  All pointers are host pointers.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t i0, n_shift, m_bits, k_out; } orc_shift_params;
typedef struct { int32_t b, c; } orc_dyadic;

/* ---------------------------------------------------------------- primitives */

static int64_t fdiv(int64_t a, int64_t b) {          /* floor(a / b), b != 0 */
    int64_t q = a / b, r = a % b;
    if (r != 0 && ((r < 0) != (b < 0))) q -= 1;
    return q;
}

/* Rounded right shift: floor(v / 2^c + 1/2), c >= 1.  Eq. 8 rounds the
 * rescaled accumulator and Eq. 10 realises the rescale as multiply + shift;
 * the reading taken is round-half-up done by adding 2^(c-1) before the shift. */
int64_t orc_rnd_shift(int64_t v, int32_t c) {
    return (v + ((int64_t)1 << (c - 1))) >> c;
}

/* Symmetric k-bit clamp (Eq. 6: symmetric uniform quantisation): [-(2^(k-1)-1), 2^(k-1)-1]. */
int64_t orc_clamp_k(int64_t v, int32_t k) {
    int64_t m = ((int64_t)1 << (k - 1)) - 1;
    return v < -m ? -m : (v > m ? m : v);
}

/* Dyadic requantisation to int8 (Eq. 8-10): clamp_8(round(b * v / 2^c)). */
int64_t orc_requant(int64_t v, int32_t b, int32_t c) {
    return orc_clamp_k(orc_rnd_shift((int64_t)b * v, c), 8);
}

/* The other reading of Eq. 10, kept as a selectable mode: the equation is printed as a bare shift,
 * I_out = (I_in * b) >> c, which is floor(b v / 2^c) with no rounding term.  floor_shift != 0 takes that; 0 is the
 * rounded form above.  Used by the *_mode entry points of the Dense layer and of attention. */
static int64_t shift_mode(int64_t v, int32_t c, int32_t floor_shift) {
    return floor_shift ? (v >> c) : orc_rnd_shift(v, c);
}
static int64_t requant_mode(int64_t v, int32_t b, int32_t c, int32_t floor_shift) {
    return orc_clamp_k(shift_mode((int64_t)b * v, c, floor_shift), 8);
}

/* ShiftExp (Algorithm 1; Eq. 13-15) for I <= 0, with I_0 = round(1/S) given by
 * the caller and N the left pre-shift of the algorithm's footnote.  Returns
 * I_exp with S/2^N * I_exp ~ exp(S*I).  The printed "I_b << (N-q)" is read as
 * (I_b << N) >> q, which is the same value when q <= N and the floor of the
 * shifted value when q > N (a negative shift count has no other meaning). */
int64_t orc_shiftexp(int64_t I, int32_t i0, int32_t n_shift) {
    int64_t Ip = I + (I >> 1) - (I >> 4);            /* I * (1.0111)_b ~ I * log2(e) */
    int64_t q  = fdiv(Ip, -(int64_t)i0);             /* integer part, >= 0            */
    int64_t r  = -(Ip - q * (-(int64_t)i0));         /* decimal part, in [0, I_0)     */
    int64_t Ib = ((-r) >> 1) + i0;                   /* 2^x ~ x/2 + 1 on (-1, 0]      */
    if (q > 62) return 0;
    return (Ib << n_shift) >> q;
}

/* IntDiv (Eq. 16): (floor(2^M / I2) * I1) >> (M - (k-1)), I2 > 0. */
int64_t orc_intdiv(int64_t i1, int64_t i2, int32_t k_out, int32_t m_bits) {
    int64_t inv = fdiv((int64_t)1 << m_bits, i2);
    return (inv * i1) >> (m_bits - (k_out - 1));
}

static int32_t bitlen(int64_t v) { int32_t n = 0; while (v > 0) { n++; v >>= 1; } return n; }

/* Integer square root by the fixed-count iteration of Eq. 20:
 * I_0 = 2^floor(bit(v)/2), I_{i+1} = (I_i + floor(v / I_i)) >> 1, exactly ten
 * iterations, the tenth iterate returned.  v = 0 returns 0 (the iteration
 * would divide by zero; the paper does not treat the case). */
int64_t orc_isqrt10(int64_t v) {
    if (v <= 0) return 0;
    int64_t x = (int64_t)1 << (bitlen(v) / 2);
    for (int it = 0; it < 10; ++it) {
        if (x == 0) return 0;
        x = (x + fdiv(v, x)) >> 1;
    }
    return x;
}

/* ----------------------------------------------------------------- operators */

/* ShiftGELU on one element (Algorithm 2; Eq. 17-18).  The algorithm's
 * max(I_p) is read elementwise as max(I_p, 0): Eq. 18 is an identity for any
 * I_max, and this is the smallest shift that makes both ShiftExp arguments
 * non-positive.  Returns I_in * I_div (scale S_in / 2^(k_out-1)). */
int64_t orc_shiftgelu_raw1(int64_t I, orc_shift_params p) {
    int64_t Ip = I + (I >> 1) + (I >> 3) + (I >> 4);                 /* I * (1.1011)_b ~ 1.702 I */
    int64_t mx = Ip > 0 ? Ip : 0;
    int64_t e1 = orc_shiftexp(Ip - mx, p.i0, p.n_shift);
    int64_t e2 = orc_shiftexp(-mx, p.i0, p.n_shift);
    int64_t dv = orc_intdiv(e1, e1 + e2, p.k_out, p.m_bits);
    return I * dv;
}

void orc_shiftgelu_raw(const int8_t* x, int32_t* g, int64_t n, orc_shift_params p) {
    for (int64_t i = 0; i < n; ++i) g[i] = (int32_t)orc_shiftgelu_raw1(x[i], p);
}

/* ShiftGELU with the maximum of Algorithm 2 taken over each row of the tensor (the other reading of the
 * algorithm's max(I_p), which names no axis): m = max(0, max_j I_p[j]) (the floor at 0 keeps the argument of
 * ShiftExp(-m) non-positive), I_exp = ShiftExp(I_p - m), I_exp' = ShiftExp(-m), I_div = IntDiv(I_exp,
 * I_exp + I_exp'), result I * I_div requantised to int8.  Far below a large row maximum both ShiftExp values
 * shift out to 0; there I_div is taken as 0 (the paper does not treat the case).  Needs a wide ShiftExp
 * (I_0 << N up to 2^30) to be usable. */
void orc_shiftgelu_rowmax(const int8_t* x, int8_t* y, int64_t rows, int32_t cols, orc_shift_params p, orc_dyadic out_rq) {
    for (int64_t r = 0; r < rows; ++r) {
        const int8_t* xr = x + r * (int64_t)cols;
        int64_t m = 0;
        for (int32_t j = 0; j < cols; ++j) {
            int64_t I = xr[j], Ip = I + (I >> 1) + (I >> 3) + (I >> 4);
            if (Ip > m) m = Ip;
        }
        int64_t e2 = orc_shiftexp(-m, p.i0, p.n_shift);
        for (int32_t j = 0; j < cols; ++j) {
            int64_t I = xr[j], Ip = I + (I >> 1) + (I >> 3) + (I >> 4);
            int64_t e1 = orc_shiftexp(Ip - m, p.i0, p.n_shift);
            int64_t dv = (e1 + e2 > 0) ? orc_intdiv(e1, e1 + e2, p.k_out, p.m_bits) : 0;
            y[r * (int64_t)cols + j] = (int8_t)orc_requant(I * dv, out_rq.b, out_rq.c);
        }
    }
}

/* ShiftGELU followed by the dyadic requantisation of its int16-range result to int8. */
void orc_shiftgelu(const int8_t* x, int8_t* y, int64_t n, orc_shift_params p, orc_dyadic out_rq) {
    for (int64_t i = 0; i < n; ++i)
        y[i] = (int8_t)orc_requant(orc_shiftgelu_raw1(x[i], p), out_rq.b, out_rq.c);
}

/* Shiftmax over each row (Algorithm 1).  x is [rows, ld] with `cols` used per
 * row, y is [rows, cols] dense.  An optional int8 bias (relative-position bias
 * of windowed attention, [H, T, cols]) is added to row r from
 * bias[(r / T) % H][r % T][:] before the maximum is subtracted.  The result is
 * limited to 2^(k_out-1)-1 so that it is a signed k_out-bit value (Eq. 16 can
 * reach 2^(k_out-1) exactly when one element carries the whole row). */
/* The additive mask of shifted-window attention: where mask_row[j] != 0 the logit gets -100 (in real units, the
 * value the windowed models add), i.e. -100 * I_0 at the integer scale, before the maximum is taken.  ShiftExp of
 * such a value is 0 unless I_0 is tiny, so masked keys drop out of the row; nothing else is special-cased. */
#define ORC_MASK_LOGIT 100

static void shiftmax_row(const int8_t* xr, const int8_t* br, const int8_t* mr, int8_t* yr, int32_t cols,
                         orc_shift_params p, int64_t* e) {
    int64_t top = ((int64_t)1 << (p.k_out - 1)) - 1;
    int64_t mx = INT64_MIN;
    for (int32_t j = 0; j < cols; ++j) {
        e[j] = (int64_t)xr[j] + (br ? br[j] : 0) - ((mr && mr[j]) ? (int64_t)ORC_MASK_LOGIT * p.i0 : 0);
        if (e[j] > mx) mx = e[j];
    }
    int64_t sum = 0;
    for (int32_t j = 0; j < cols; ++j) { e[j] = orc_shiftexp(e[j] - mx, p.i0, p.n_shift); sum += e[j]; }
    for (int32_t j = 0; j < cols; ++j) {
        int64_t o = orc_intdiv(e[j], sum, p.k_out, p.m_bits);
        yr[j] = (int8_t)(o > top ? top : o);
    }
}

void orc_shiftmax(const int8_t* x, const int8_t* bias, int32_t H, int32_t T, int8_t* y,
                  int64_t rows, int32_t cols, int32_t ld, orc_shift_params p) {
    int64_t* e = (int64_t*)malloc(sizeof(int64_t) * (size_t)(cols > 0 ? cols : 1));
    for (int64_t r = 0; r < rows; ++r) {
        const int8_t* br = bias ? bias + (((r / T) % H) * (int64_t)T + (r % T)) * cols : NULL;
        shiftmax_row(x + r * (int64_t)ld, br, NULL, y + r * (int64_t)cols, cols, p, e);
    }
    free(e);
}

/* I-LayerNorm over each row of x [rows, C] (Eq. 19-20).  Integer mean (rounded
 * to nearest), population variance (floored), standard deviation by
 * orc_isqrt10 (at least 1), then the normalisation as an integer division in
 * the manner of Eq. 16 with f_bits in the role of M: f = floor(2^F / std),
 * n_i = (x_i - mean) * f, followed by the integer affine step
 * y_i = n_i * gamma_q[i] + beta_q[i] and a rounded shift by c_shift to int8
 * (gamma_q and beta_q carry the output scale, folded in by the host). */
void orc_ilayernorm(const int8_t* x, const int32_t* gamma_q, const int32_t* beta_q, int8_t* y,
                    int64_t rows, int32_t C, int32_t f_bits, int32_t c_shift) {
    for (int64_t r = 0; r < rows; ++r) {
        const int8_t* xr = x + r * (int64_t)C;
        int64_t s = 0;
        for (int32_t i = 0; i < C; ++i) s += xr[i];
        int64_t mean = fdiv(s + C / 2, C);
        int64_t ss = 0;
        for (int32_t i = 0; i < C; ++i) { int64_t d = xr[i] - mean; ss += d * d; }
        int64_t var = fdiv(ss, C);
        int64_t sd = orc_isqrt10(var);
        if (sd < 1) sd = 1;
        int64_t f = fdiv((int64_t)1 << f_bits, sd);
        for (int32_t i = 0; i < C; ++i) {
            int64_t n = (xr[i] - mean) * f;
            int64_t v = n * gamma_q[i] + beta_q[i];
            y[r * (int64_t)C + i] = (int8_t)orc_clamp_k(orc_rnd_shift(v, c_shift), 8);
        }
    }
}

/* Dense / MatMul with the dyadic pipeline (Eq. 7-10): x [M,K] int8, w [N,K]
 * int8 (one row per output channel), acc_j = sum_k x_k w_jk + bias_j in exact
 * integers, y_j = requant(acc_j; b_j, c_j) per output channel.
 *  - residual != NULL: the residual stream [M,N] is requantised on its own to
 *    the output scale and added before the clamp (Eq. 1-2):
 *    y = clamp_8(rnd_shift(b_j acc_j, c_j) + rnd_shift(b_r res, c_r)).
 *  - gelu != NULL: the int8 result goes through ShiftGELU and the dyadic
 *    requantisation of its output (Eq. 5: GELU sits between the two MLP layers). */
void orc_linear_requant_mode(const int8_t* x, const int8_t* w, const int32_t* bias,
                             const int32_t* rq_b, const int32_t* rq_c,
                             const int8_t* residual, orc_dyadic res_rq,
                             const orc_shift_params* gelu, orc_dyadic gelu_rq,
                             int8_t* y, int64_t M, int32_t N, int32_t K, int32_t floor_shift) {
    for (int64_t m = 0; m < M; ++m) {
        const int8_t* xr = x + m * (int64_t)K;
        for (int32_t j = 0; j < N; ++j) {
            const int8_t* wr = w + (int64_t)j * K;
            int64_t acc = bias ? bias[j] : 0;
            for (int32_t k = 0; k < K; ++k) acc += (int64_t)xr[k] * wr[k];
            int64_t v;
            if (residual) {
                v = shift_mode((int64_t)rq_b[j] * acc, rq_c[j], floor_shift)
                  + shift_mode((int64_t)res_rq.b * residual[m * (int64_t)N + j], res_rq.c, floor_shift);
                v = orc_clamp_k(v, 8);
            } else {
                v = requant_mode(acc, rq_b[j], rq_c[j], floor_shift);
            }
            if (gelu) v = requant_mode(orc_shiftgelu_raw1(v, *gelu), gelu_rq.b, gelu_rq.c, floor_shift);
            y[m * (int64_t)N + j] = (int8_t)v;
        }
    }
}

void orc_linear_requant(const int8_t* x, const int8_t* w, const int32_t* bias,
                        const int32_t* rq_b, const int32_t* rq_c,
                        const int8_t* residual, orc_dyadic res_rq,
                        const orc_shift_params* gelu, orc_dyadic gelu_rq,
                        int8_t* y, int64_t M, int32_t N, int32_t K) {
    orc_linear_requant_mode(x, w, bias, rq_b, rq_c, residual, res_rq, gelu, gelu_rq, y, M, N, K, 0);
}

/* ------------------------------------------------------ attention and blocks */

typedef struct { int32_t B, T, C, H, F; } orc_dims;

typedef struct {
    const int32_t *ln1_gamma, *ln1_beta; int32_t ln1_f_bits, ln1_c_shift;
    const int8_t* w_qkv; const int32_t *bias_qkv, *qkv_rq_b, *qkv_rq_c;
    orc_dyadic qk_rq; const int8_t* rel_bias; orc_shift_params softmax; orc_dyadic pv_rq;
    const int8_t* w_proj; const int32_t *bias_proj, *proj_rq_b, *proj_rq_c; orc_dyadic res1_rq;
    const int32_t *ln2_gamma, *ln2_beta; int32_t ln2_f_bits, ln2_c_shift;
    const int8_t* w_fc1; const int32_t *bias_fc1, *fc1_rq_b, *fc1_rq_c;
    orc_shift_params gelu; orc_dyadic gelu_rq;
    const int8_t* w_fc2; const int32_t *bias_fc2, *fc2_rq_b, *fc2_rq_c; orc_dyadic res2_rq;
    const int8_t* attn_mask; int32_t n_mask;          /* [n_mask, T, T], NULL: none (shifted-window attention) */
} orc_block_params;

/* Optional taps: every intermediate int tensor of a block (any may be NULL). */
typedef struct { int8_t *u, *qkv, *scores, *probs, *o, *xhat, *v, *h; } orc_taps;

/* Multi-head attention on the packed qkv tensor [B*T, 3C] (Eq. 3-4): columns
 * [0,C) are Q, [C,2C) K, [2C,3C) V, head h owning columns h*d..(h+1)*d of each.
 * Per image and head: A = requant(Q K^T; qk_rq) (the 1/sqrt(d) of Eq. 4 is part
 * of the dyadic pair, by the homogeneity argument of Sec. 3.1), an optional
 * int8 relative-position bias [H,T,T] is added, P = Shiftmax(rows of A),
 * O = requant(P V; pv_rq), heads concatenated into o [B*T, C]. */
void orc_attention_mode(const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask, int8_t* o,
                        orc_dims d, orc_dyadic qk_rq, orc_shift_params sm, orc_dyadic pv_rq,
                        int8_t* tap_scores, int8_t* tap_probs, int32_t floor_shift) {
    int32_t T = d.T, C = d.C, H = d.H, hd = d.C / d.H;
    int8_t* a = (int8_t*)malloc((size_t)T * T);
    int8_t* p = (int8_t*)malloc((size_t)T * T);
    int64_t* erow = (int64_t*)malloc(sizeof(int64_t) * (size_t)T);
    for (int32_t b = 0; b < d.B; ++b)
        for (int32_t h = 0; h < H; ++h) {
            const int8_t* base = qkv + (int64_t)b * T * 3 * C + h * hd;
            for (int32_t i = 0; i < T; ++i)
                for (int32_t j = 0; j < T; ++j) {
                    int64_t acc = 0;
                    for (int32_t k = 0; k < hd; ++k)
                        acc += (int64_t)base[(int64_t)i * 3 * C + k] * base[(int64_t)j * 3 * C + C + k];
                    a[i * T + j] = (int8_t)requant_mode(acc, qk_rq.b, qk_rq.c, floor_shift);
                }
            /* window b uses mask[b % n_mask] ([T, T], shared by the heads): the windows of an image are consecutive */
            for (int32_t i = 0; i < T; ++i)
                shiftmax_row(a + i * T, rel_bias ? rel_bias + ((int64_t)h * T + i) * T : NULL,
                             mask ? mask + ((int64_t)(b % n_mask) * T + i) * T : NULL, p + i * T, T, sm, erow);
            for (int32_t i = 0; i < T; ++i)
                for (int32_t k = 0; k < hd; ++k) {
                    int64_t acc = 0;
                    for (int32_t j = 0; j < T; ++j)
                        acc += (int64_t)p[i * T + j] * base[(int64_t)j * 3 * C + 2 * C + k];
                    o[((int64_t)b * T + i) * C + h * hd + k] = (int8_t)requant_mode(acc, pv_rq.b, pv_rq.c, floor_shift);
                }
            int64_t off = ((int64_t)b * H + h) * T * T;
            if (tap_scores) memcpy(tap_scores + off, a, (size_t)T * T);
            if (tap_probs) memcpy(tap_probs + off, p, (size_t)T * T);
        }
    free(a); free(p); free(erow);
}

void orc_attention_masked(const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask, int8_t* o,
                          orc_dims d, orc_dyadic qk_rq, orc_shift_params sm, orc_dyadic pv_rq,
                          int8_t* tap_scores, int8_t* tap_probs) {
    orc_attention_mode(qkv, rel_bias, mask, n_mask, o, d, qk_rq, sm, pv_rq, tap_scores, tap_probs, 0);
}

void orc_attention(const int8_t* qkv, const int8_t* rel_bias, int8_t* o,
                   orc_dims d, orc_dyadic qk_rq, orc_shift_params sm, orc_dyadic pv_rq,
                   int8_t* tap_scores, int8_t* tap_probs) {
    orc_attention_masked(qkv, rel_bias, NULL, 1, o, d, qk_rq, sm, pv_rq, tap_scores, tap_probs);
}

/* One encoder block (Eq. 1-2): Xhat = MSA(LN(X)) + X ; Y = MLP(LN(Xhat)) + Xhat. */
void orc_encoder_block(const int8_t* x, int8_t* y, const orc_block_params* p, orc_dims d, const orc_taps* taps) {
    int64_t R = (int64_t)d.B * d.T;
    int32_t C = d.C, F = d.F;
    orc_dyadic none = {0, 0};
    int8_t* u    = (int8_t*)malloc((size_t)R * C);
    int8_t* qkv  = (int8_t*)malloc((size_t)R * 3 * C);
    int8_t* o    = (int8_t*)malloc((size_t)R * C);
    int8_t* xhat = (int8_t*)malloc((size_t)R * C);
    int8_t* v    = (int8_t*)malloc((size_t)R * C);
    int8_t* h    = (int8_t*)malloc((size_t)R * F);
    orc_ilayernorm(x, p->ln1_gamma, p->ln1_beta, u, R, C, p->ln1_f_bits, p->ln1_c_shift);
    orc_linear_requant(u, p->w_qkv, p->bias_qkv, p->qkv_rq_b, p->qkv_rq_c, NULL, none, NULL, none, qkv, R, 3 * C, C);
    orc_attention_masked(qkv, p->rel_bias, p->attn_mask, p->attn_mask ? p->n_mask : 1, o, d, p->qk_rq, p->softmax, p->pv_rq,
                         taps ? taps->scores : NULL, taps ? taps->probs : NULL);
    orc_linear_requant(o, p->w_proj, p->bias_proj, p->proj_rq_b, p->proj_rq_c, x, p->res1_rq, NULL, none, xhat, R, C, C);
    orc_ilayernorm(xhat, p->ln2_gamma, p->ln2_beta, v, R, C, p->ln2_f_bits, p->ln2_c_shift);
    orc_linear_requant(v, p->w_fc1, p->bias_fc1, p->fc1_rq_b, p->fc1_rq_c, NULL, none, &p->gelu, p->gelu_rq, h, R, F, C);
    orc_linear_requant(h, p->w_fc2, p->bias_fc2, p->fc2_rq_b, p->fc2_rq_c, xhat, p->res2_rq, NULL, none, y, R, C, F);
    if (taps) {
        if (taps->u)    memcpy(taps->u, u, (size_t)R * C);
        if (taps->qkv)  memcpy(taps->qkv, qkv, (size_t)R * 3 * C);
        if (taps->o)    memcpy(taps->o, o, (size_t)R * C);
        if (taps->xhat) memcpy(taps->xhat, xhat, (size_t)R * C);
        if (taps->v)    memcpy(taps->v, v, (size_t)R * C);
        if (taps->h)    memcpy(taps->h, h, (size_t)R * F);
    }
    free(u); free(qkv); free(o); free(xhat); free(v); free(h);
}

/* Stack of blocks, with an optional final I-LayerNorm (gamma == NULL: none). */
void orc_forward(const int8_t* x, int8_t* y, const orc_block_params* blocks, int32_t n_blocks,
                 const int32_t* fin_gamma, const int32_t* fin_beta, int32_t fin_f_bits, int32_t fin_c_shift,
                 orc_dims d) {
    int64_t n = (int64_t)d.B * d.T * d.C;
    int8_t* a = (int8_t*)malloc((size_t)n);
    int8_t* b = (int8_t*)malloc((size_t)n);
    memcpy(a, x, (size_t)n);
    for (int32_t l = 0; l < n_blocks; ++l) {
        orc_encoder_block(a, b, &blocks[l], d, NULL);
        int8_t* t = a; a = b; b = t;
    }
    if (fin_gamma) orc_ilayernorm(a, fin_gamma, fin_beta, y, (int64_t)d.B * d.T, d.C, fin_f_bits, fin_c_shift);
    else memcpy(y, a, (size_t)n);
    free(a); free(b);
}

/* ------------------------------------------- array forms of the primitives */
/* Plain loops over the scalar functions above, so that tests can sweep large
 * ranges without a Python call per element. */
void orc_requant_vec(const int64_t* v, int64_t* out, int64_t n, int32_t b, int32_t c) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_requant(v[i], b, c);
}
void orc_rnd_shift_vec(const int64_t* v, int64_t* out, int64_t n, int32_t c) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_rnd_shift(v[i], c);
}
void orc_isqrt10_vec(const int64_t* v, int64_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_isqrt10(v[i]);
}
void orc_shiftexp_vec(const int64_t* v, int64_t* out, int64_t n, int32_t i0, int32_t n_shift) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_shiftexp(v[i], i0, n_shift);
}
