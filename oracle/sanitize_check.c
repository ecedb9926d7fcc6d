/* TEST INFRASTRUCTURE ONLY.  Builds the oracle together with this driver under AddressSanitizer and
 * UndefinedBehaviorSanitizer (signed overflow and out-of-range shifts are errors there) and runs it on inputs chosen
 * to reach the largest intermediates the ABI allows: saturated int8 operands with K = 3072, 31-bit multipliers with
 * shifts up to 46, one-hot rows for I-LayerNorm, dominant and flat rows for Shiftmax.  The oracle's claim that int64
 * never overflows and that every shift count is in range is checked by running, not by reading.
 *
 *   gcc -O1 -g -std=c11 -fsanitize=address,undefined -fno-sanitize-recover=all oracle/sanitize_check.c -o check && ./check
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ivit_oracle.c"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33); }
static int8_t rnd8(int mode) {          /* 0: uniform, 1: saturated +-127, 2: all +127 */
    if (mode == 2) return 127;
    if (mode == 1) return (rnd() & 1) ? 127 : -127;
    return (int8_t)((int)(rnd() % 255) - 127);
}
static int8_t* buf8(size_t n, int mode) { int8_t* p = malloc(n ? n : 1); for (size_t i = 0; i < n; ++i) p[i] = rnd8(mode); return p; }
static int32_t* buf32(size_t n, int32_t lo, int32_t hi) {
    int32_t* p = malloc(4 * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = lo + (int32_t)(rnd() % (uint32_t)(hi - lo + 1));
    return p;
}
static uint64_t checksum(const int8_t* p, size_t n) { uint64_t h = 1469598103934665603ull; for (size_t i = 0; i < n; ++i) h = (h ^ (uint8_t)p[i]) * 1099511628211ull; return h; }

static void dense_extremes(void) {
    const int M = 5, N = 7, K = 3072;
    for (int mode = 0; mode < 3; ++mode) {
        int8_t *x = buf8((size_t)M * K, mode), *w = buf8((size_t)N * K, mode), *res = buf8((size_t)M * N, mode), *y = malloc(M * N);
        int32_t *bias = buf32(N, -(1 << 20), 1 << 20);
        int32_t *b = buf32(N, 1, 0x7fffffff), *c = buf32(N, 1, 46);
        orc_dyadic rr = {0x7fffffff, 46};
        orc_linear_requant(x, w, bias, b, c, res, rr, NULL, rr, y, M, N, K);
        orc_shift_params g = {32, 10, 31, 8};
        orc_linear_requant(x, w, bias, b, c, NULL, rr, &g, rr, y, M, N, K);
        printf("dense mode %d: %016llx\n", mode, (unsigned long long)checksum(y, (size_t)M * N));
        free(x); free(w); free(res); free(y); free(bias); free(b); free(c);
    }
}

static void rowwise_extremes(void) {
    const int C = 1024, rows = 6;
    int8_t* x = calloc((size_t)rows * C, 1); int8_t* y = malloc((size_t)rows * C);
    for (int i = 0; i < C; ++i) { x[0 * C + i] = 127; x[1 * C + i] = -128; x[2 * C + i] = (i & 1) ? 127 : -128; x[4 * C + i] = (int8_t)(i % 255 - 127); }
    x[3 * C + 5] = 127; x[5 * C + 1023] = -128;
    int32_t *gamma = buf32(C, -511, 511), *beta = buf32(C, -(1 << 24), 1 << 24);
    orc_ilayernorm(x, gamma, beta, y, rows, C, 16, 19);
    printf("ilayernorm: %016llx\n", (unsigned long long)checksum(y, (size_t)rows * C));
    const int i0s[] = {1, 4, 32, 64, 255, 65535};
    for (int k = 0; k < 6; ++k) {
        int n = 0; while ((i0s[k] << (n + 1)) <= 65535) ++n;
        orc_shift_params p = {i0s[k], n, 31, 8};
        orc_shiftmax(x, NULL, 1, 1, y, rows, C, C, p);
        int8_t* bias = buf8((size_t)2 * 3 * C, 1);
        orc_shiftmax(x, bias, 2, 3, y, rows, C, C, p);
        orc_dyadic rq = {0x7fffffff, 40};
        orc_shiftgelu(x, y, (int64_t)rows * C, p, rq);
        printf("shift ops i0=%d: %016llx\n", i0s[k], (unsigned long long)checksum(y, (size_t)rows * C));
        free(bias);
    }
    for (int64_t v = 0; v < 70000; ++v) (void)orc_isqrt10(v);
    (void)orc_isqrt10(((int64_t)1 << 62) - 1);
    free(x); free(y); free(gamma); free(beta);
}

static void block_saturated(void) {
    orc_dims d = {2, 17, 64, 2, 128};
    const int R = d.B * d.T, C = d.C, F = d.F;
    orc_block_params p; memset(&p, 0, sizeof p);
    p.ln1_gamma = buf32(C, 200, 300); p.ln1_beta = buf32(C, -(1 << 22), 1 << 22); p.ln1_f_bits = 16; p.ln1_c_shift = 19;
    p.ln2_gamma = buf32(C, 200, 300); p.ln2_beta = buf32(C, -(1 << 22), 1 << 22); p.ln2_f_bits = 16; p.ln2_c_shift = 19;
    p.w_qkv = buf8((size_t)3 * C * C, 1); p.bias_qkv = buf32(3 * C, -1000, 1000); p.qkv_rq_b = buf32(3 * C, 1 << 14, (1 << 15) - 1); p.qkv_rq_c = buf32(3 * C, 16, 20);
    p.qk_rq = (orc_dyadic){30000, 20}; p.pv_rq = (orc_dyadic){30000, 18};
    p.rel_bias = buf8((size_t)d.H * d.T * d.T, 1);
    p.softmax = (orc_shift_params){32, 10, 31, 8}; p.gelu = (orc_shift_params){8, 12, 31, 8};
    p.w_proj = buf8((size_t)C * C, 1); p.bias_proj = buf32(C, -1000, 1000); p.proj_rq_b = buf32(C, 1 << 14, (1 << 15) - 1); p.proj_rq_c = buf32(C, 16, 20);
    p.res1_rq = (orc_dyadic){32767, 15}; p.res2_rq = (orc_dyadic){32767, 15};
    p.w_fc1 = buf8((size_t)F * C, 1); p.bias_fc1 = buf32(F, -1000, 1000); p.fc1_rq_b = buf32(F, 1 << 14, (1 << 15) - 1); p.fc1_rq_c = buf32(F, 16, 20);
    p.gelu_rq = (orc_dyadic){30000, 20};
    p.w_fc2 = buf8((size_t)C * F, 1); p.bias_fc2 = buf32(C, -1000, 1000); p.fc2_rq_b = buf32(C, 1 << 14, (1 << 15) - 1); p.fc2_rq_c = buf32(C, 16, 20);
    int8_t *x = buf8((size_t)R * C, 1), *y = malloc((size_t)R * C);
    orc_taps t = {malloc((size_t)R * C), malloc((size_t)R * 3 * C), malloc((size_t)d.B * d.H * d.T * d.T), malloc((size_t)d.B * d.H * d.T * d.T),
                  malloc((size_t)R * C), malloc((size_t)R * C), malloc((size_t)R * C), malloc((size_t)R * F)};
    orc_encoder_block(x, y, &p, d, &t);
    orc_block_params two[2] = {p, p};
    orc_forward(x, y, two, 2, p.ln1_gamma, p.ln1_beta, 16, 19, d);
    printf("block + forward: %016llx\n", (unsigned long long)checksum(y, (size_t)R * C));
    free(x); free(y); free(t.u); free(t.qkv); free(t.scores); free(t.probs); free(t.o); free(t.xhat); free(t.v); free(t.h);
    free((void*)p.ln1_gamma); free((void*)p.ln1_beta); free((void*)p.ln2_gamma); free((void*)p.ln2_beta);
    free((void*)p.w_qkv); free((void*)p.bias_qkv); free((void*)p.qkv_rq_b); free((void*)p.qkv_rq_c); free((void*)p.rel_bias);
    free((void*)p.w_proj); free((void*)p.bias_proj); free((void*)p.proj_rq_b); free((void*)p.proj_rq_c);
    free((void*)p.w_fc1); free((void*)p.bias_fc1); free((void*)p.fc1_rq_b); free((void*)p.fc1_rq_c);
    free((void*)p.w_fc2); free((void*)p.bias_fc2); free((void*)p.fc2_rq_b); free((void*)p.fc2_rq_c);
}

int main(void) {
    dense_extremes();
    rowwise_extremes();
    block_saturated();
    printf("sanitize_check: ok\n");
    return 0;
}
