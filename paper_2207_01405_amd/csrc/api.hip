// C-ABI layer of libivit.so: argument validation (host only, before any launch), the launch sequence of
// one encoder block (I-ViT, arXiv 2207.01405, Eq. 1-5) and of the block stack.  See include/ivit.h.
#include "../../include/ivit.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "ivit_kernels.hpp"

namespace {

using ivit::Dyadic;
using ivit::ShiftParams;

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int check_dyadic(ivit_dyadic d) { return (d.b >= 1 && d.c >= 1 && d.c <= 46) ? IVIT_OK : IVIT_ERR_PARAM; }

inline int check_shift(const ivit_shift_params& p) {
    if (p.i0 < 1 || p.n_shift < 0 || p.n_shift > 16) return IVIT_ERR_PARAM;
    if (((int64_t)p.i0 << p.n_shift) > 65535) return IVIT_ERR_PARAM;
    if (p.k_out < 2 || p.k_out > 8) return IVIT_ERR_PARAM;
    if (p.m_bits < p.k_out - 1 || p.m_bits > 31) return IVIT_ERR_PARAM;
    return IVIT_OK;
}

inline int check_ln(int32_t C, int32_t f_bits, int32_t c_shift) {
    if (C < 4 || C > 2048 || (C & 3)) return IVIT_ERR_SHAPE;
    if (f_bits < 1 || f_bits > 20 || c_shift < 1 || c_shift > 31) return IVIT_ERR_PARAM;
    return IVIT_OK;
}

inline ShiftParams sp(const ivit_shift_params& p) { return ShiftParams{p.i0, p.n_shift, p.m_bits, p.k_out}; }
inline Dyadic dy(ivit_dyadic d) { return Dyadic{d.b, d.c}; }
thread_local int last_hip_error = 0;      // hipError_t behind the calling thread's last IVIT_ERR_HIP
inline int hip_status(hipError_t e) {
    if (e == hipSuccess) return IVIT_OK;
    last_hip_error = (int)e;
    return IVIT_ERR_HIP;
}

int check_dims(const ivit_dims* d) {
    if (!d) return IVIT_ERR_NULL;
    if (d->B < 0 || d->T < 1 || d->T > 256 || d->C < 16 || d->H < 1 || d->F < 16) return IVIT_ERR_SHAPE;
    if (d->C % d->H != 0) return IVIT_ERR_SHAPE;
    const int hd = d->C / d->H;
    if (hd != 32 && hd != 64) return IVIT_ERR_SHAPE;
    if ((d->C & 15) || (d->F & 15) || d->C > 1024 || d->F > 65536) return IVIT_ERR_SHAPE;
    if ((int64_t)d->B * d->T > 0x7fffffffLL) return IVIT_ERR_SHAPE;
    return IVIT_OK;
}

// A token-index table needs the relative-position bias (the gathering kernels are the windowed ones) and a
// window count that divides the number of windows.
int check_tok_index(const int32_t* tok_index, int32_t n_win, const int8_t* rel_bias, const ivit_dims* d) {
    if (!tok_index) return IVIT_OK;
    if (!rel_bias) return IVIT_ERR_NULL;
    if (n_win < 1 || d->B % n_win != 0 || (int64_t)n_win * d->T > 0x7fffffffLL) return IVIT_ERR_SHAPE;
    if (!aligned(tok_index, 4)) return IVIT_ERR_ALIGN;
    return IVIT_OK;
}

inline size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Workspace { int8_t *act0, *act1, *u, *qkv, *o, *xhat, *h; };

size_t carve(const ivit_dims* d, void* base, Workspace* w) {
    const size_t R = (size_t)d->B * d->T, C = d->C, F = d->F;
    size_t off = 0;
    auto take = [&](size_t n) { size_t o = off; off += up256(n); return base ? static_cast<int8_t*>(base) + o : nullptr; };
    int8_t* a0 = take(R * C); int8_t* a1 = take(R * C); int8_t* u = take(R * C); int8_t* qkv = take(R * 3 * C);
    int8_t* o = take(R * C); int8_t* xh = take(R * C); int8_t* h = take(R * F);
    if (w) *w = Workspace{a0, a1, u, qkv, o, xh, h};
    return off;
}

int check_block(const ivit_block_params* p, const ivit_dims* d) {
    if (!p) return IVIT_ERR_NULL;
    if (!p->ln1_gamma || !p->ln1_beta || !p->w_qkv || !p->qkv_rq_b || !p->qkv_rq_c || !p->w_proj || !p->proj_rq_b ||
        !p->proj_rq_c || !p->ln2_gamma || !p->ln2_beta || !p->w_fc1 || !p->fc1_rq_b || !p->fc1_rq_c || !p->w_fc2 ||
        !p->fc2_rq_b || !p->fc2_rq_c)
        return IVIT_ERR_NULL;
    int st;
    if ((st = check_ln(d->C, p->ln1_f_bits, p->ln1_c_shift)) != IVIT_OK) return st;
    if ((st = check_ln(d->C, p->ln2_f_bits, p->ln2_c_shift)) != IVIT_OK) return st;
    if ((st = check_dyadic(p->qk_rq)) != IVIT_OK || (st = check_dyadic(p->pv_rq)) != IVIT_OK ||
        (st = check_dyadic(p->res1_rq)) != IVIT_OK || (st = check_dyadic(p->res2_rq)) != IVIT_OK ||
        (st = check_dyadic(p->gelu_rq)) != IVIT_OK)
        return st;
    if ((st = check_shift(p->softmax)) != IVIT_OK || (st = check_shift(p->gelu)) != IVIT_OK) return st;
    if (p->attn_mask && p->n_mask < 1) return IVIT_ERR_SHAPE;
    if ((st = check_tok_index(p->tok_index, p->n_win, p->rel_bias, d)) != IVIT_OK) return st;
    if (!aligned(p->w_qkv, 16) || !aligned(p->w_proj, 16) || !aligned(p->w_fc1, 16) || !aligned(p->w_fc2, 16))
        return IVIT_ERR_ALIGN;
    const void* i32s[] = {p->ln1_gamma, p->ln1_beta, p->bias_qkv, p->qkv_rq_b, p->qkv_rq_c, p->bias_proj, p->proj_rq_b,
                          p->proj_rq_c, p->ln2_gamma, p->ln2_beta, p->bias_fc1, p->fc1_rq_b, p->fc1_rq_c, p->bias_fc2,
                          p->fc2_rq_b, p->fc2_rq_c};
    for (const void* q : i32s)
        if (!aligned(q, 4)) return IVIT_ERR_ALIGN;
    return IVIT_OK;
}

// Launch sequence of one block on buffers of the carved workspace.  Arguments already validated.
hipError_t run_block(hipStream_t s, const int8_t* x, int8_t* y, const ivit_block_params* p, const ivit_dims* d,
                     const Workspace& w, const ivit_debug_taps* taps) {
    const int64_t R = (int64_t)d->B * d->T;
    const int C = d->C, F = d->F;
    if (R == 0) return hipSuccess;
    hipError_t e;
    auto tap = [&](int8_t* dst, const int8_t* src, size_t n) -> hipError_t {
        return dst ? hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToDevice, s) : hipSuccess;
    };
    // u = LN1(x)
    if ((e = ivit::launch_ilayernorm(s, x, p->ln1_gamma, p->ln1_beta, w.u, R, C, p->ln1_f_bits, p->ln1_c_shift))) return e;
    if (taps && (e = tap(taps->u, w.u, (size_t)R * C))) return e;
    // qkv = Dense(u)
    ivit::LinearArgs la{};
    la.x = w.u; la.w = p->w_qkv; la.bias = p->bias_qkv; la.rq_b = p->qkv_rq_b; la.rq_c = p->qkv_rq_c;
    la.residual = nullptr; la.gelu = false; la.y = w.qkv; la.M = R; la.N = 3 * C; la.K = C;
    if ((e = ivit::launch_linear(s, la))) return e;
    if (taps && (e = tap(taps->qkv, w.qkv, (size_t)R * 3 * C))) return e;
    // o = attention(qkv)
    ivit::AttentionArgs aa{};
    aa.qkv = w.qkv; aa.rel_bias = p->rel_bias; aa.o = w.o; aa.B = d->B; aa.T = d->T; aa.C = C; aa.H = d->H;
    aa.mask = p->attn_mask; aa.n_mask = p->attn_mask ? p->n_mask : 1;
    aa.tok_index = p->tok_index; aa.n_win = p->tok_index ? p->n_win : 1;
    aa.qk_rq = dy(p->qk_rq); aa.sm = sp(p->softmax); aa.pv_rq = dy(p->pv_rq);
    aa.tap_scores = taps ? taps->scores : nullptr; aa.tap_probs = taps ? taps->probs : nullptr;
    if ((e = ivit::launch_attention(s, aa))) return e;
    if (taps && (e = tap(taps->o, w.o, (size_t)R * C))) return e;
    // xhat = Dense(o) + x
    la = ivit::LinearArgs{};
    la.x = w.o; la.w = p->w_proj; la.bias = p->bias_proj; la.rq_b = p->proj_rq_b; la.rq_c = p->proj_rq_c;
    la.residual = x; la.res_rq = dy(p->res1_rq); la.gelu = false; la.y = w.xhat; la.M = R; la.N = C; la.K = C;
    if ((e = ivit::launch_linear(s, la))) return e;
    if (taps && (e = tap(taps->xhat, w.xhat, (size_t)R * C))) return e;
    // v = LN2(xhat)   (reuses the u buffer)
    if ((e = ivit::launch_ilayernorm(s, w.xhat, p->ln2_gamma, p->ln2_beta, w.u, R, C, p->ln2_f_bits, p->ln2_c_shift))) return e;
    if (taps && (e = tap(taps->v, w.u, (size_t)R * C))) return e;
    // h = ShiftGELU(Dense(v))
    la = ivit::LinearArgs{};
    la.x = w.u; la.w = p->w_fc1; la.bias = p->bias_fc1; la.rq_b = p->fc1_rq_b; la.rq_c = p->fc1_rq_c;
    la.residual = nullptr; la.gelu = true; la.gelu_p = sp(p->gelu); la.gelu_rq = dy(p->gelu_rq);
    la.y = w.h; la.M = R; la.N = F; la.K = C;
    if ((e = ivit::launch_linear(s, la))) return e;
    if (taps && (e = tap(taps->h, w.h, (size_t)R * F))) return e;
    // y = Dense(h) + xhat
    la = ivit::LinearArgs{};
    la.x = w.h; la.w = p->w_fc2; la.bias = p->bias_fc2; la.rq_b = p->fc2_rq_b; la.rq_c = p->fc2_rq_c;
    la.residual = w.xhat; la.res_rq = dy(p->res2_rq); la.gelu = false; la.y = y; la.M = R; la.N = C; la.K = F;
    return ivit::launch_linear(s, la);
}

// Scratch of ivit_encoder_block_static: one array per GPU, allocated by the loader with the code object and held
// until the process ends.  In host code the name below is only a handle for hipGetSymbolAddress; the address the
// kernels get is looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[IVIT_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void* scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return IVIT_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return IVIT_ERR_HIP;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return IVIT_OK;
}

}  // namespace

extern "C" {

#ifndef IVIT_BUILD_ID
#define IVIT_BUILD_ID "unknown"
#endif
const char* ivit_build_id(void) { return IVIT_BUILD_ID; }

const char* ivit_strerror(int status) {
    switch (status) {
        case IVIT_OK: return "ok";
        case IVIT_ERR_NULL: return "a required pointer is NULL";
        case IVIT_ERR_SHAPE: return "unsupported shape";
        case IVIT_ERR_PARAM: return "integer parameter out of range";
        case IVIT_ERR_ALIGN: return "pointer not aligned as required";
        case IVIT_ERR_WORKSPACE: return "workspace missing or too small";
        case IVIT_ERR_HIP: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

int ivit_last_hip_error(void) { return last_hip_error; }

int ivit_linear_requant(void* stream, const int8_t* x, const int8_t* w, const int32_t* bias, const int32_t* rq_b,
                        const int32_t* rq_c, const int8_t* residual, ivit_dyadic res_rq, const ivit_shift_params* gelu,
                        ivit_dyadic gelu_rq, int8_t* y, int64_t M, int32_t N, int32_t K) {
    return ivit_linear_requant_ex(stream, x, w, bias, rq_b, rq_c, residual, res_rq, gelu, gelu_rq, y, M, N, K, nullptr);
}

int ivit_linear_requant_ex(void* stream, const int8_t* x, const int8_t* w, const int32_t* bias, const int32_t* rq_b,
                           const int32_t* rq_c, const int8_t* residual, ivit_dyadic res_rq, const ivit_shift_params* gelu,
                           ivit_dyadic gelu_rq, int8_t* y, int64_t M, int32_t N, int32_t K, const ivit_linear_options* opt) {
    if (opt && (opt->kernel < IVIT_KERNEL_AUTO || opt->kernel > IVIT_KERNEL_BIG_TILES)) return IVIT_ERR_PARAM;
    if (opt && opt->rounding != IVIT_ROUND_NEAREST && opt->rounding != IVIT_ROUND_FLOOR) return IVIT_ERR_PARAM;
    if (M < 0 || N < 1 || K < 16 || K > 65536 || (K & 15)) return IVIT_ERR_SHAPE;
    if (M > 0 && (!x || !y)) return IVIT_ERR_NULL;             // an empty tensor may have no storage
    if (!w || !rq_b || !rq_c) return IVIT_ERR_NULL;
    if ((M + 127) / 128 * (int64_t)((N + 127) / 128) > 0x7fffffffLL) return IVIT_ERR_SHAPE;
    if (residual && gelu) return IVIT_ERR_PARAM;
    int st;
    if (residual && (st = check_dyadic(res_rq)) != IVIT_OK) return st;
    if (gelu && ((st = check_shift(*gelu)) != IVIT_OK || (st = check_dyadic(gelu_rq)) != IVIT_OK)) return st;
    if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16) || (residual && !aligned(residual, 16))) return IVIT_ERR_ALIGN;
    if (!aligned(rq_b, 4) || !aligned(rq_c, 4) || (bias && !aligned(bias, 4))) return IVIT_ERR_ALIGN;
    ivit::LinearArgs a{};
    a.x = x; a.w = w; a.bias = bias; a.rq_b = rq_b; a.rq_c = rq_c; a.residual = residual;
    a.res_rq = residual ? dy(res_rq) : Dyadic{1, 1};
    a.gelu = gelu != nullptr;
    if (gelu) { a.gelu_p = sp(*gelu); a.gelu_rq = dy(gelu_rq); }
    a.y = y; a.M = M; a.N = N; a.K = K;
    a.kernel = opt ? opt->kernel : ivit::LINEAR_AUTO;
    a.floor_shift = opt && opt->rounding == IVIT_ROUND_FLOOR;
    if (a.kernel == ivit::LINEAR_REG_STATIONARY && M > 0 && !ivit::linear_rs_takes(a) && !ivit::linear_ks_takes(a)) return IVIT_ERR_SHAPE;
    if (a.kernel == ivit::LINEAR_BIG_TILES && M > 0 && !ivit::linear_tl_takes(a)) return IVIT_ERR_SHAPE;
    return hip_status(ivit::launch_linear(static_cast<hipStream_t>(stream), a));
}

int ivit_shiftmax(void* stream, const int8_t* x, const int8_t* bias, int32_t H, int32_t T, int8_t* y, int64_t rows,
                  int32_t cols, int32_t ld, ivit_shift_params p) {
    if (rows < 0 || cols < 1 || cols > 1024 || ld < cols) return IVIT_ERR_SHAPE;
    if (rows > 0 && (!x || !y)) return IVIT_ERR_NULL;
    if (bias && (H < 1 || T < 1)) return IVIT_ERR_SHAPE;
    int st = check_shift(p);
    if (st != IVIT_OK) return st;
    return hip_status(ivit::launch_shiftmax(static_cast<hipStream_t>(stream), x, bias, bias ? H : 1, bias ? T : 1, y,
                                            rows, cols, ld, sp(p)));
}

int ivit_shiftgelu(void* stream, const int8_t* x, int8_t* y, int64_t n, ivit_shift_params p, ivit_dyadic out_rq) {
    if (n < 0) return IVIT_ERR_SHAPE;
    if (n > 0 && (!x || !y)) return IVIT_ERR_NULL;
    int st;
    if ((st = check_shift(p)) != IVIT_OK || (st = check_dyadic(out_rq)) != IVIT_OK) return st;
    return hip_status(ivit::launch_shiftgelu(static_cast<hipStream_t>(stream), x, y, nullptr, n, sp(p), dy(out_rq)));
}

int ivit_shiftgelu_rowmax(void* stream, const int8_t* x, int8_t* y, int64_t rows, int32_t cols, ivit_shift_params p,
                          ivit_dyadic out_rq) {
    if (rows < 0 || cols < 4 || cols > 4096 || (cols & 3)) return IVIT_ERR_SHAPE;
    if (rows > 0 && (!x || !y)) return IVIT_ERR_NULL;
    // the wide form of the shift parameters: ShiftExp values up to 2^30, reciprocal of IntDiv up to 2^46
    if (p.i0 < 1 || p.n_shift < 0 || p.n_shift > 30 || ((int64_t)p.i0 << p.n_shift) > ((int64_t)1 << 30)) return IVIT_ERR_PARAM;
    if (p.k_out < 2 || p.k_out > 8 || p.m_bits < p.k_out - 1 || p.m_bits > 46) return IVIT_ERR_PARAM;
    int st = check_dyadic(out_rq);
    if (st != IVIT_OK) return st;
    if (!aligned(x, 4) || !aligned(y, 4)) return IVIT_ERR_ALIGN;
    return hip_status(ivit::launch_shiftgelu_rowmax(static_cast<hipStream_t>(stream), x, y, rows, cols, sp(p), dy(out_rq)));
}

int ivit_shiftgelu_raw(void* stream, const int8_t* x, int16_t* y16, int64_t n, ivit_shift_params p) {
    if (n < 0) return IVIT_ERR_SHAPE;
    if (n > 0 && (!x || !y16)) return IVIT_ERR_NULL;
    int st = check_shift(p);
    if (st != IVIT_OK) return st;
    if (!aligned(y16, 2)) return IVIT_ERR_ALIGN;
    return hip_status(ivit::launch_shiftgelu(static_cast<hipStream_t>(stream), x, nullptr, y16, n, sp(p), Dyadic{1, 1}));
}

int ivit_ilayernorm(void* stream, const int8_t* x, const int32_t* gamma_q, const int32_t* beta_q, int8_t* y,
                    int64_t rows, int32_t C, int32_t f_bits, int32_t c_shift) {
    if (rows < 0) return IVIT_ERR_SHAPE;
    if (!gamma_q || !beta_q || (rows > 0 && (!x || !y))) return IVIT_ERR_NULL;
    int st = check_ln(C, f_bits, c_shift);
    if (st != IVIT_OK) return st;
    if (!aligned(x, 4) || !aligned(y, 4) || !aligned(gamma_q, 4) || !aligned(beta_q, 4)) return IVIT_ERR_ALIGN;
    return hip_status(ivit::launch_ilayernorm(static_cast<hipStream_t>(stream), x, gamma_q, beta_q, y, rows, C, f_bits, c_shift));
}

size_t ivit_workspace_bytes(const ivit_dims* d) {
    if (check_dims(d) != IVIT_OK) return 0;
    return carve(d, nullptr, nullptr) + 256;      // never 0 for valid dimensions, even with B == 0
}

int ivit_attention(void* stream, const int8_t* qkv, const int8_t* rel_bias, int8_t* o, const ivit_dims* d,
                   ivit_dyadic qk_rq, ivit_shift_params softmax, ivit_dyadic pv_rq, int8_t* tap_scores,
                   int8_t* tap_probs) {
    return ivit_attention_masked(stream, qkv, rel_bias, nullptr, 1, o, d, qk_rq, softmax, pv_rq, tap_scores, tap_probs);
}

int ivit_attention_masked(void* stream, const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask,
                          int8_t* o, const ivit_dims* d, ivit_dyadic qk_rq, ivit_shift_params softmax,
                          ivit_dyadic pv_rq, int8_t* tap_scores, int8_t* tap_probs) {
    return ivit_window_attention(stream, qkv, rel_bias, mask, n_mask, nullptr, 1, o, d, qk_rq, softmax, pv_rq, tap_scores,
                                 tap_probs);
}

int ivit_window_attention(void* stream, const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask,
                          const int32_t* tok_index, int32_t n_win, int8_t* o, const ivit_dims* d, ivit_dyadic qk_rq,
                          ivit_shift_params softmax, ivit_dyadic pv_rq, int8_t* tap_scores, int8_t* tap_probs) {
    return ivit_window_attention_ex(stream, qkv, rel_bias, mask, n_mask, tok_index, n_win, o, d, qk_rq, softmax, pv_rq,
                                    tap_scores, tap_probs, nullptr);
}

int ivit_window_attention_ex(void* stream, const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask,
                             const int32_t* tok_index, int32_t n_win, int8_t* o, const ivit_dims* d, ivit_dyadic qk_rq,
                             ivit_shift_params softmax, ivit_dyadic pv_rq, int8_t* tap_scores, int8_t* tap_probs,
                             const ivit_attention_options* opt) {
    if (!d) return IVIT_ERR_NULL;
    if (opt && opt->rounding != IVIT_ROUND_NEAREST && opt->rounding != IVIT_ROUND_FLOOR) return IVIT_ERR_PARAM;
    if (mask && n_mask < 1) return IVIT_ERR_SHAPE;
    int st;
    if ((st = check_dims(d)) != IVIT_OK) return st;
    if ((st = check_tok_index(tok_index, n_win, rel_bias, d)) != IVIT_OK) return st;
    if (d->B > 0 && (!qkv || !o)) return IVIT_ERR_NULL;
    if ((st = check_dyadic(qk_rq)) != IVIT_OK || (st = check_dyadic(pv_rq)) != IVIT_OK ||
        (st = check_shift(softmax)) != IVIT_OK)
        return st;
    if (!aligned(qkv, 16) || !aligned(o, 16)) return IVIT_ERR_ALIGN;
    ivit::AttentionArgs a{};
    a.qkv = qkv; a.rel_bias = rel_bias; a.o = o; a.B = d->B; a.T = d->T; a.C = d->C; a.H = d->H;
    a.mask = mask; a.n_mask = mask ? n_mask : 1;
    a.tok_index = tok_index; a.n_win = tok_index ? n_win : 1;
    a.qk_rq = dy(qk_rq); a.sm = sp(softmax); a.pv_rq = dy(pv_rq); a.tap_scores = tap_scores; a.tap_probs = tap_probs;
    a.floor_shift = opt && opt->rounding == IVIT_ROUND_FLOOR;
    return hip_status(ivit::launch_attention(static_cast<hipStream_t>(stream), a));
}

int ivit_encoder_block(void* stream, const int8_t* x, int8_t* y, const ivit_block_params* p, const ivit_dims* d,
                       void* workspace, size_t workspace_bytes, const ivit_debug_taps* taps) {
    if (!p || !d) return IVIT_ERR_NULL;
    int st;
    if ((st = check_dims(d)) != IVIT_OK) return st;
    if (d->B > 0 && (!x || !y)) return IVIT_ERR_NULL;
    if ((st = check_block(p, d)) != IVIT_OK) return st;
    if (!workspace || workspace_bytes < ivit_workspace_bytes(d)) return IVIT_ERR_WORKSPACE;
    if (!aligned(workspace, 256) || !aligned(x, 16) || !aligned(y, 16)) return IVIT_ERR_ALIGN;
    Workspace w;
    carve(d, workspace, &w);
    return hip_status(run_block(static_cast<hipStream_t>(stream), x, y, p, d, w, taps));
}

int ivit_encoder_block_static(void* stream, const int8_t* x, int8_t* y, const ivit_block_params* p, const ivit_dims* d,
                              const ivit_debug_taps* taps) {
    if (!p || !d) return IVIT_ERR_NULL;
    int st;
    if ((st = check_dims(d)) != IVIT_OK) return st;
    if (d->B > 0 && (!x || !y)) return IVIT_ERR_NULL;
    if ((st = check_block(p, d)) != IVIT_OK) return st;
    if (carve(d, nullptr, nullptr) > (size_t)IVIT_STATIC_SCRATCH_BYTES) return IVIT_ERR_WORKSPACE;
    if (!aligned(x, 16) || !aligned(y, 16)) return IVIT_ERR_ALIGN;
    void* base = nullptr;
    if ((st = static_scratch(&base)) != IVIT_OK) return st;
    // every buffer carved from the scratch is written in full by the launch that produces it before anything reads
    // it, so what an earlier call left there never shows and nothing has to be cleared
    Workspace w;
    carve(d, base, &w);
    return hip_status(run_block(static_cast<hipStream_t>(stream), x, y, p, d, w, taps));
}

int ivit_forward(void* stream, const int8_t* x, int8_t* y, const ivit_block_params* blocks, int32_t n_blocks,
                 const ivit_final_ln* final_ln, const ivit_dims* d, void* workspace, size_t workspace_bytes) {
    if (!d || (n_blocks > 0 && !blocks)) return IVIT_ERR_NULL;
    if (n_blocks < 0) return IVIT_ERR_SHAPE;
    int st;
    if ((st = check_dims(d)) != IVIT_OK) return st;
    if (d->B > 0 && (!x || !y)) return IVIT_ERR_NULL;
    for (int l = 0; l < n_blocks; ++l)
        if ((st = check_block(&blocks[l], d)) != IVIT_OK) return st;
    if (final_ln) {
        if (!final_ln->gamma || !final_ln->beta) return IVIT_ERR_NULL;
        if ((st = check_ln(d->C, final_ln->f_bits, final_ln->c_shift)) != IVIT_OK) return st;
        if (!aligned(final_ln->gamma, 4) || !aligned(final_ln->beta, 4)) return IVIT_ERR_ALIGN;
    }
    if (!workspace || workspace_bytes < ivit_workspace_bytes(d)) return IVIT_ERR_WORKSPACE;
    if (!aligned(workspace, 256) || !aligned(x, 16) || !aligned(y, 16)) return IVIT_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace w;
    carve(d, workspace, &w);
    const size_t n = (size_t)d->B * d->T * d->C;
    if (n == 0) return IVIT_OK;
    // block l reads cur and writes into the other ping-pong buffer; the last producer writes y directly
    const int8_t* cur = x;
    for (int l = 0; l < n_blocks; ++l) {
        const bool last = (l == n_blocks - 1) && !final_ln;
        int8_t* dst = last ? y : (cur == w.act0 ? w.act1 : w.act0);
        hipError_t e = run_block(s, cur, dst, &blocks[l], d, w, nullptr);
        if (e != hipSuccess) return IVIT_ERR_HIP;
        cur = dst;
    }
    if (final_ln)
        return hip_status(ivit::launch_ilayernorm(s, cur, final_ln->gamma, final_ln->beta, y, (int64_t)d->B * d->T, d->C,
                                                  final_ln->f_bits, final_ln->c_shift));
    if (n_blocks == 0) return hip_status(hipMemcpyAsync(y, x, n, hipMemcpyDeviceToDevice, s));
    return IVIT_OK;
}

int ivit_embed_tokens(void* stream, const int8_t* patch_tok, const int8_t* cls, const int8_t* pos,
                      ivit_dyadic tok_rq, ivit_dyadic pos_rq, int8_t* tokens, int32_t B, int32_t P, int32_t C) {
    if (B < 0 || P < 0 || C < 16 || (C & 15)) return IVIT_ERR_SHAPE;
    if (B > 0 && (!cls || !pos || !tokens || (P > 0 && !patch_tok))) return IVIT_ERR_NULL;
    int st;
    if ((st = check_dyadic(tok_rq)) != IVIT_OK || (st = check_dyadic(pos_rq)) != IVIT_OK) return st;
    if (!aligned(patch_tok, 16) || !aligned(cls, 16) || !aligned(pos, 16) || !aligned(tokens, 16)) return IVIT_ERR_ALIGN;
    return hip_status(ivit::launch_embed_tokens(static_cast<hipStream_t>(stream), patch_tok, cls, pos, dy(tok_rq),
                                                dy(pos_rq), tokens, B, P, C));
}

int ivit_classifier_head(void* stream, const int8_t* tokens, int32_t T, const int8_t* w, const int32_t* bias,
                         const int32_t* rq_b, const int32_t* rq_c, int8_t* logits, int32_t B, int32_t N, int32_t C) {
    if (B < 0 || T < 1 || N < 1 || C < 16 || C > 65536 || (C & 15)) return IVIT_ERR_SHAPE;
    if (B > 0 && (!tokens || !logits)) return IVIT_ERR_NULL;
    if (!w || !rq_b || !rq_c) return IVIT_ERR_NULL;
    if (!aligned(tokens, 16) || !aligned(w, 16) || !aligned(logits, 16)) return IVIT_ERR_ALIGN;
    if (!aligned(rq_b, 4) || !aligned(rq_c, 4) || (bias && !aligned(bias, 4))) return IVIT_ERR_ALIGN;
    ivit::LinearArgs a{};
    a.x = tokens; a.w = w; a.bias = bias; a.rq_b = rq_b; a.rq_c = rq_c; a.residual = nullptr;
    a.res_rq = Dyadic{1, 1}; a.gelu = false;
    a.y = logits; a.M = B; a.N = N; a.K = C; a.ldx = (int64_t)T * C;
    return hip_status(ivit::launch_linear(static_cast<hipStream_t>(stream), a));
}

size_t ivit_image_workspace_bytes(const ivit_dims* d) {
    if (!d || check_dims(d) != IVIT_OK) return 0;
    const size_t act = ((size_t)d->B * d->T * d->C + 255) / 256 * 256;
    return ivit_workspace_bytes(d) + 3 * act;
}

int ivit_forward_image(void* stream, const int8_t* patches, int8_t* logits, const ivit_image_params* ip,
                       const ivit_block_params* blocks, int32_t n_blocks, const ivit_final_ln* final_ln,
                       const ivit_dims* d, void* workspace, size_t workspace_bytes) {
    // everything that can be checked on the host is checked before the first launch: a failed call launches nothing
    if (!ip || !d || !final_ln || (n_blocks > 0 && !blocks)) return IVIT_ERR_NULL;
    if (n_blocks < 0) return IVIT_ERR_SHAPE;
    int st;
    if ((st = check_dims(d)) != IVIT_OK) return st;
    if (ip->patch_dim < 16 || ip->patch_dim > 65536 || (ip->patch_dim & 15) || ip->n_classes < 1) return IVIT_ERR_SHAPE;
    if (d->B > 0 && (!patches || !logits)) return IVIT_ERR_NULL;
    if (!ip->w_patch || !ip->patch_rq_b || !ip->patch_rq_c || !ip->w_head || !ip->head_rq_b || !ip->head_rq_c) return IVIT_ERR_NULL;
    if (d->B > 0 && (!ip->cls || !ip->pos)) return IVIT_ERR_NULL;
    if ((st = check_dyadic(ip->tok_rq)) != IVIT_OK || (st = check_dyadic(ip->pos_rq)) != IVIT_OK) return st;
    for (int l = 0; l < n_blocks; ++l)
        if ((st = check_block(&blocks[l], d)) != IVIT_OK) return st;
    if (!final_ln->gamma || !final_ln->beta) return IVIT_ERR_NULL;
    if ((st = check_ln(d->C, final_ln->f_bits, final_ln->c_shift)) != IVIT_OK) return st;
    if (!workspace || workspace_bytes < ivit_image_workspace_bytes(d)) return IVIT_ERR_WORKSPACE;
    if (!aligned(workspace, 256) || !aligned(patches, 16) || !aligned(logits, 16) || !aligned(ip->w_patch, 16) ||
        !aligned(ip->cls, 16) || !aligned(ip->pos, 16) || !aligned(ip->w_head, 16))
        return IVIT_ERR_ALIGN;
    const void* i32s[] = {ip->bias_patch, ip->patch_rq_b, ip->patch_rq_c, ip->bias_head, ip->head_rq_b, ip->head_rq_c,
                          final_ln->gamma, final_ln->beta};
    for (const void* q : i32s)
        if (!aligned(q, 4)) return IVIT_ERR_ALIGN;
    const size_t act = ((size_t)d->B * d->T * d->C + 255) / 256 * 256;
    int8_t* base = static_cast<int8_t*>(workspace);
    int8_t* patch_tok = base;
    int8_t* tok_in = base + act;
    int8_t* tok_out = base + 2 * act;
    void* inner = base + 3 * act;
    const int P = d->T - 1;
    if (P > 0 && (st = ivit_linear_requant(stream, patches, ip->w_patch, ip->bias_patch, ip->patch_rq_b, ip->patch_rq_c, nullptr,
                                           ivit_dyadic{1, 1}, nullptr, ivit_dyadic{1, 1}, patch_tok, (int64_t)d->B * P, d->C,
                                           ip->patch_dim)) != IVIT_OK)
        return st;
    if ((st = ivit_embed_tokens(stream, patch_tok, ip->cls, ip->pos, ip->tok_rq, ip->pos_rq, tok_in, d->B, P, d->C)) != IVIT_OK) return st;
    if ((st = ivit_forward(stream, tok_in, tok_out, blocks, n_blocks, final_ln, d, inner, workspace_bytes - 3 * act)) != IVIT_OK) return st;
    return ivit_classifier_head(stream, tok_out, d->T, ip->w_head, ip->bias_head, ip->head_rq_b, ip->head_rq_c, logits,
                                d->B, ip->n_classes, d->C);
}

int ivit_patch_merge_gather(void* stream, const int8_t* x, int8_t* y, int32_t B, int32_t g, int32_t C) {
    if (B < 0 || g < 2 || (g & 1) || g > 4096 || C < 16 || (C & 15) || C > 65536) return IVIT_ERR_SHAPE;
    if (B > 0 && (!x || !y)) return IVIT_ERR_NULL;
    if (!aligned(x, 16) || !aligned(y, 16)) return IVIT_ERR_ALIGN;
    return hip_status(ivit::launch_patch_merge_gather(static_cast<hipStream_t>(stream), x, y, B, g, C));
}

int ivit_mean_pool(void* stream, const int8_t* x, int8_t* y, int32_t B, int32_t T, int32_t C, ivit_dyadic rq) {
    if (B < 0 || T < 1 || T > (1 << 24) || C < 4 || (C & 3)) return IVIT_ERR_SHAPE;    // |sum| <= 127 T fits int32
    if (B > 0 && (!x || !y)) return IVIT_ERR_NULL;
    int st = check_dyadic(rq);
    if (st != IVIT_OK) return st;
    if (!aligned(x, 4) || !aligned(y, 4)) return IVIT_ERR_ALIGN;
    return hip_status(ivit::launch_mean_pool(static_cast<hipStream_t>(stream), x, y, B, T, C, dy(rq)));
}

}  // extern "C"

// ---- hierarchical windowed model: embedding, stages of blocks with patch merging between them, pooling, head ------
namespace {

struct SwinPlan {
    ivit_dims dims[4];       // per stage: B = windows, T = window^2, C, H, F
    int grid[4];             // tokens per image side in each stage
    size_t act, inner, pooled, total;
};

int check_final_ln(const ivit_final_ln& l, int C) {
    if (!l.gamma || !l.beta) return IVIT_ERR_NULL;
    int st = check_ln(C, l.f_bits, l.c_shift);
    if (st != IVIT_OK) return st;
    return (aligned(l.gamma, 4) && aligned(l.beta, 4)) ? IVIT_OK : IVIT_ERR_ALIGN;
}

// Validates everything that can be validated on the host and sizes the workspace.
int plan_swin(const ivit_swin_params* p, int32_t B, SwinPlan* plan) {
    if (!p) return IVIT_ERR_NULL;
    if (B < 0 || p->n_stages < 1 || p->n_stages > 4 || p->window < 1 || p->window > 16 || p->grid < p->window ||
        p->grid > 4096 || p->patch_dim < 16 || (p->patch_dim & 15) || p->n_classes < 1)
        return IVIT_ERR_SHAPE;
    if (!p->w_patch || !p->patch_rq_b || !p->patch_rq_c || !p->w_head || !p->head_rq_b || !p->head_rq_c) return IVIT_ERR_NULL;
    int st;
    int g = p->grid;
    size_t act = 0, inner = 0;
    for (int s = 0; s < p->n_stages; ++s) {
        const ivit_swin_stage& sg = p->stages[s];
        if (s > 0) {
            if (g & 1) return IVIT_ERR_SHAPE;
            g >>= 1;
            if (sg.C != 2 * p->stages[s - 1].C) return IVIT_ERR_SHAPE;
            if (!sg.w_merge || !sg.merge_rq_b || !sg.merge_rq_c) return IVIT_ERR_NULL;
            if ((st = check_final_ln(sg.merge_ln, 2 * sg.C)) != IVIT_OK) return st;       // over 4 C of the previous stage
            if (!aligned(sg.w_merge, 16) || !aligned(sg.merge_rq_b, 4) || !aligned(sg.merge_rq_c, 4)) return IVIT_ERR_ALIGN;
        }
        if (g % p->window != 0 || sg.n_blocks < 0 || (sg.n_blocks > 0 && !sg.blocks)) return IVIT_ERR_SHAPE;
        const int64_t n_win = (int64_t)(g / p->window) * (g / p->window);
        if ((int64_t)B * n_win > 0x7fffffffLL) return IVIT_ERR_SHAPE;
        ivit_dims d{(int32_t)(B * n_win), p->window * p->window, sg.C, sg.H, sg.F};
        if (sg.H < 1 || (st = check_dims(&d)) != IVIT_OK) return st;
        for (int l = 0; l < sg.n_blocks; ++l) {
            const ivit_block_params& bp = sg.blocks[l];
            if ((st = check_block(&bp, &d)) != IVIT_OK) return st;
            // with more than one window per image the tokens (kept in image order) must be gathered into windows
            if (n_win > 1 && (!bp.tok_index || bp.n_win != n_win)) return bp.tok_index ? IVIT_ERR_SHAPE : IVIT_ERR_NULL;
            if (bp.tok_index && bp.n_win != n_win) return IVIT_ERR_SHAPE;
            if (bp.attn_mask && bp.n_mask != n_win) return IVIT_ERR_SHAPE;
        }
        plan->dims[s] = d;
        plan->grid[s] = g;
        act = std::max(act, up256((size_t)B * g * g * sg.C));
        inner = std::max(inner, ivit_workspace_bytes(&d));
    }
    if ((st = check_final_ln(p->embed_ln, p->stages[0].C)) != IVIT_OK) return st;
    if ((st = check_final_ln(p->final_ln, p->stages[p->n_stages - 1].C)) != IVIT_OK) return st;
    if ((st = check_dyadic(p->pool_rq)) != IVIT_OK) return st;
    if (!aligned(p->w_patch, 16) || !aligned(p->w_head, 16)) return IVIT_ERR_ALIGN;
    plan->act = act;
    plan->inner = inner;
    plan->pooled = up256((size_t)B * p->stages[p->n_stages - 1].C);
    plan->total = 4 * act + plan->pooled + inner;
    return IVIT_OK;
}

}  // namespace

extern "C" {

size_t ivit_swin_workspace_bytes(const ivit_swin_params* p, int32_t B) {
    SwinPlan plan;
    return plan_swin(p, B, &plan) == IVIT_OK ? plan.total : 0;
}

int ivit_forward_swin(void* stream, const int8_t* patches, int8_t* logits, const ivit_swin_params* p, int32_t B,
                      void* workspace, size_t workspace_bytes) {
    SwinPlan plan;
    int st = plan_swin(p, B, &plan);
    if (st != IVIT_OK) return st;
    if (B > 0 && (!patches || !logits)) return IVIT_ERR_NULL;
    if (!workspace || workspace_bytes < plan.total) return IVIT_ERR_WORKSPACE;
    if (!aligned(workspace, 256) || !aligned(patches, 16) || !aligned(logits, 16)) return IVIT_ERR_ALIGN;
    if (B == 0) return IVIT_OK;
    int8_t* base = static_cast<int8_t*>(workspace);
    int8_t* buf[2] = {base, base + plan.act};
    int8_t* cat = base + 2 * plan.act;
    int8_t* catn = base + 3 * plan.act;
    int8_t* pooled = base + 4 * plan.act;
    void* inner = pooled + plan.pooled;
    const ivit_dyadic one{1, 1};
    // embedding: patch Dense, then I-LayerNorm
    const int g0 = p->grid, C0 = p->stages[0].C;
    const int64_t R0 = (int64_t)B * g0 * g0;
    if ((st = ivit_linear_requant(stream, patches, p->w_patch, p->bias_patch, p->patch_rq_b, p->patch_rq_c, nullptr, one,
                                  nullptr, one, buf[0], R0, C0, p->patch_dim)) != IVIT_OK) return st;
    if ((st = ivit_ilayernorm(stream, buf[0], p->embed_ln.gamma, p->embed_ln.beta, buf[1], R0, C0, p->embed_ln.f_bits,
                              p->embed_ln.c_shift)) != IVIT_OK) return st;
    int cur = 1;
    for (int s = 0; s < p->n_stages; ++s) {
        const ivit_swin_stage& sg = p->stages[s];
        const int g = plan.grid[s];
        const int64_t R = (int64_t)B * g * g;
        if (s > 0) {     // patch merging: 2 x 2 concatenation, I-LayerNorm over 4 C_prev = 2 C, Dense to C without bias
            const int Cp = p->stages[s - 1].C;
            if ((st = ivit_patch_merge_gather(stream, buf[cur], cat, B, 2 * g, Cp)) != IVIT_OK) return st;
            if ((st = ivit_ilayernorm(stream, cat, sg.merge_ln.gamma, sg.merge_ln.beta, catn, R, 4 * Cp, sg.merge_ln.f_bits,
                                      sg.merge_ln.c_shift)) != IVIT_OK) return st;
            if ((st = ivit_linear_requant(stream, catn, sg.w_merge, nullptr, sg.merge_rq_b, sg.merge_rq_c, nullptr, one,
                                          nullptr, one, buf[cur ^ 1], R, sg.C, 4 * Cp)) != IVIT_OK) return st;
            cur ^= 1;
        }
        if (sg.n_blocks > 0) {
            if ((st = ivit_forward(stream, buf[cur], buf[cur ^ 1], sg.blocks, sg.n_blocks, nullptr, &plan.dims[s], inner,
                                   plan.inner)) != IVIT_OK) return st;
            cur ^= 1;
        }
    }
    const int sl = p->n_stages - 1, gl = plan.grid[sl], Cl = p->stages[sl].C;
    if ((st = ivit_ilayernorm(stream, buf[cur], p->final_ln.gamma, p->final_ln.beta, buf[cur ^ 1], (int64_t)B * gl * gl, Cl,
                              p->final_ln.f_bits, p->final_ln.c_shift)) != IVIT_OK) return st;
    if ((st = ivit_mean_pool(stream, buf[cur ^ 1], pooled, B, gl * gl, Cl, p->pool_rq)) != IVIT_OK) return st;
    return ivit_linear_requant(stream, pooled, p->w_head, p->bias_head, p->head_rq_b, p->head_rq_c, nullptr, one, nullptr,
                               one, logits, B, p->n_classes, Cl);
}

}  // extern "C"
