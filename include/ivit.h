/*
 * ivit.h - C ABI of the MI355X (gfx950) integer-only ViT encoder library.
 *
 * The library computes the integer-only forward pass of a Vision-Transformer
 * encoder as described in "I-ViT: Integer-only Quantization for Efficient
 * Vision Transformer Inference" (arXiv 2207.01405): int8 x int8 -> int32
 * Dense / MatMul with dyadic requantisation (Sec. 3.2), Shiftmax (Sec. 3.3,
 * Algorithm 1), ShiftGELU (Sec. 3.4, Algorithm 2) and I-LayerNorm (Sec. 3.5).
 *
 * General rules
 *  - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *    never allocates or frees device memory.  Scratch space for the block /
 *    forward calls is a caller-supplied workspace (one exception, stated there:
 *    ivit_encoder_block_static uses a fixed array inside the library's device image).
 *  - Parameter structs (ivit_shift_params, ivit_dyadic, ivit_dims,
 *    ivit_block_params, ivit_final_ln, ivit_debug_taps) are HOST structs read
 *    before the launch; pointers inside them are device pointers.
 *  - `stream` is a hipStream_t (NULL = the default stream).  Work is enqueued
 *    on it and the call returns without synchronising.
 *  - Tensors are row-major and dense unless a leading dimension is given.
 *    Weights are [N_out, K] with K contiguous.  Per-channel parameters are
 *    int32 [N_out] device arrays.
 *  - A tensor with no elements (M, rows, n or B equal to 0) may be passed as NULL.
 *  - Every function returns IVIT_OK (0) or a negative ivit_status.  Arguments
 *    are validated before anything is launched; a failed call launches nothing.
 *    Nothing throws or aborts.  Input and output may not alias unless stated.
 *  - Integer semantics: ">>" is an arithmetic shift (floor); round(v, c) =
 *    (v + 2^(c-1)) >> c; clamp8(v) = min(max(v, -127), 127);
 *    requant(v; b, c) = clamp8(round(b * v, c)) with the product in 64 bits.
 *  - The library reads no environment variables.  After an IVIT_ERR_HIP, ivit_last_hip_error() gives the
 *    hipError_t behind the calling thread's most recent one.
 *  - Values in device parameter arrays cannot be checked on the host: rq_b must
 *    hold 1 <= b < 2^31 and rq_c must hold 1 <= c <= 46; other values give
 *    unspecified results (never a fault).
 */
#ifndef IVIT_H
#define IVIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    IVIT_OK = 0,
    IVIT_ERR_NULL = -1,       /* a required pointer is NULL                                  */
    IVIT_ERR_SHAPE = -2,      /* a dimension is negative, zero where not allowed, too large,
                                 or not a multiple the kernels need                          */
    IVIT_ERR_PARAM = -3,      /* an integer parameter is outside its stated range            */
    IVIT_ERR_ALIGN = -4,      /* a pointer is not aligned as stated                          */
    IVIT_ERR_WORKSPACE = -5,  /* workspace is NULL or smaller than ivit_workspace_bytes()    */
    IVIT_ERR_HIP = -6         /* the HIP runtime reported an error at launch                 */
} ivit_status;

/* Parameters of ShiftExp / IntDiv (Algorithm 1, Eq. 13-16):
 *   i0      I_0 = round(1 / S_in), the integer image of 1.0 at the input scale, >= 1
 *   n_shift N, the left pre-shift of ShiftExp (Algorithm 1, footnote); i0 << n_shift <= 65535
 *   m_bits  M of IntDiv (Eq. 16), k_out - 1 <= m_bits <= 31
 *   k_out   output bit width of IntDiv, 2..8 (output scale 1 / 2^(k_out-1)) */
typedef struct { int32_t i0, n_shift, m_bits, k_out; } ivit_shift_params;

/* A per-tensor dyadic number b / 2^c (Eq. 9): 1 <= b < 2^31, 1 <= c <= 46. */
typedef struct { int32_t b, c; } ivit_dyadic;

/* Shape of an encoder: B images (or attention windows), T tokens each, width C,
 * H heads (C = H * d, d in {32, 64}), MLP width F.  Rows R = B * T. */
typedef struct { int32_t B, T, C, H, F; } ivit_dims;

/* Everything one encoder block needs (Eq. 1-5).  Pointers are device pointers. */
typedef struct {
    const int32_t *ln1_gamma, *ln1_beta;  int32_t ln1_f_bits, ln1_c_shift;   /* I-LayerNorm before MSA   */
    const int8_t  *w_qkv;                                                    /* [3C, C]: Q rows, K rows, V rows */
    const int32_t *bias_qkv /*nullable*/, *qkv_rq_b, *qkv_rq_c;              /* [3C]                     */
    ivit_dyadic    qk_rq;                 /* rescale of Q K^T to int8 scores; carries 1/sqrt(d) (Eq. 4)  */
    const int8_t  *rel_bias;              /* nullable, [H, T, T]: added to the int8 scores (windowed attention) */
    ivit_shift_params softmax;            /* Shiftmax on the score rows                                  */
    ivit_dyadic    pv_rq;                 /* rescale of P V to int8                                      */
    const int8_t  *w_proj;  const int32_t *bias_proj /*nullable*/, *proj_rq_b, *proj_rq_c;   /* [C, C], [C] */
    ivit_dyadic    res1_rq;               /* rescale of the residual X before the first add (Eq. 1)      */
    const int32_t *ln2_gamma, *ln2_beta;  int32_t ln2_f_bits, ln2_c_shift;   /* I-LayerNorm before MLP   */
    const int8_t  *w_fc1;   const int32_t *bias_fc1 /*nullable*/, *fc1_rq_b, *fc1_rq_c;      /* [F, C], [F] */
    ivit_shift_params gelu;  ivit_dyadic gelu_rq;                            /* ShiftGELU and its int8 rescale */
    const int8_t  *w_fc2;   const int32_t *bias_fc2 /*nullable*/, *fc2_rq_b, *fc2_rq_c;      /* [C, F], [C] */
    ivit_dyadic    res2_rq;               /* rescale of the residual Xhat before the second add (Eq. 2)  */
    const int8_t  *attn_mask;             /* nullable, [n_mask, T, T]: mask of shifted-window attention, see
                                             ivit_attention_masked                                       */
    int32_t        n_mask;                /* window b uses attn_mask[b % n_mask]; ignored without a mask  */
    const int32_t *tok_index;             /* nullable, [n_win, T]: the tokens stay in image order and attention
                                             gathers its windows through this table, see ivit_window_attention */
    int32_t        n_win;                 /* windows per image; ignored without a table                   */
} ivit_block_params;

/* Optional device buffers that receive every intermediate int8 tensor of a block
 * (any member may be NULL): u = LN1(x) [R,C]; qkv [R,3C]; scores = requantised Q K^T
 * before the bias [B,H,T,T]; probs = Shiftmax output [B,H,T,T]; o = attention output
 * [R,C]; xhat [R,C]; v = LN2(xhat) [R,C]; h = MLP hidden after ShiftGELU [R,F]. */
typedef struct { int8_t *u, *qkv, *scores, *probs, *o, *xhat, *v, *h; } ivit_debug_taps;

/* Final I-LayerNorm after the last block (optional in ivit_forward). */
typedef struct { const int32_t *gamma, *beta; int32_t f_bits, c_shift; } ivit_final_ln;

/* Text for a status code (static storage, never NULL). */
const char* ivit_strerror(int status);

/* Identifier of the sources this library was built from: a digest over the kernel sources and this header, set by
 * the build script ("unknown" when built by other means).  Host memory, static; never NULL.  The Python binding
 * compares it with the sources next to it and refuses a library built from other ones. */
const char* ivit_build_id(void);

/* Dense / MatMul with the dyadic pipeline (Sec. 3.2, Eq. 7-10), optionally fused
 * with the residual add of Eq. 1-2 or with ShiftGELU (Eq. 5, Algorithm 2).
 *   acc[m][j] = sum_k x[m][k] * w[j][k] + bias[j]                      (exact, int32)
 *   y[m][j]   = requant(acc; rq_b[j], rq_c[j])                                        plain
 *   y[m][j]   = clamp8(round(rq_b[j]*acc, rq_c[j]) + round(res_rq.b*residual[m][j], res_rq.c))  residual != NULL
 *   y[m][j]   = requant(ShiftGELU(requant(acc; ...); *gelu); gelu_rq)                 gelu != NULL
 * x [M,K] int8, w [N,K] int8, bias [N] int32 or NULL, rq_b / rq_c [N] int32,
 * residual [M,N] int8 or NULL, y [M,N] int8.  residual and gelu exclude each other.
 * Requirements: M >= 0 (M == 0 is a no-op), N >= 1, 16 <= K <= 65536, K % 16 == 0;
 * x, w, y, residual 16-byte aligned, int32 arrays 4-byte aligned.
 * res_rq / gelu_rq are ignored when the matching pointer is NULL.
 * Errors: NULL, SHAPE, PARAM (dyadic or shift parameters out of range, both fusions at once), ALIGN, HIP. */
int ivit_linear_requant(void* stream, const int8_t* x, const int8_t* w, const int32_t* bias,
                        const int32_t* rq_b, const int32_t* rq_c,
                        const int8_t* residual, ivit_dyadic res_rq,
                        const ivit_shift_params* gelu, ivit_dyadic gelu_rq,
                        int8_t* y, int64_t M, int32_t N, int32_t K);

/* ivit_linear_requant with options (opt == NULL: exactly ivit_linear_requant).
 *   kernel  which Dense kernel runs; results are identical for every choice (Sec. 3.2 fixes the arithmetic, not
 *           the schedule), so this is a switch for tests and measurements:
 *           IVIT_KERNEL_AUTO            chosen from the shape;
 *           IVIT_KERNEL_MANY_ROWS       never the kernel written for few rows;
 *           IVIT_KERNEL_REG_STATIONARY  the kernels that keep the weights in registers; they take K = 384, 768 or
 *                                       1536 (and K = 192 for layers without a residual) with N % 32 == 0 only,
 *                                       other shapes give IVIT_ERR_SHAPE.
 *           IVIT_KERNEL_BIG_TILES       the kernel that streams both operands through LDS in 256 x 128 tiles; it
 *                                       takes K % 128 == 0, K >= 384, N % 128 == 0 only (else IVIT_ERR_SHAPE).
 *   rounding  how every dyadic requantisation of the layer (Sec. 3.2, Eq. 8-10: the output's, the residual's, the
 *           one after ShiftGELU) turns b v / 2^c into an integer:
 *           IVIT_ROUND_NEAREST          (b v + 2^(c-1)) >> c, the rounding Eq. 8 asks for carried into Eq. 10 (what
 *                                       every entry point without options does);
 *           IVIT_ROUND_FLOOR            (b v) >> c, Eq. 10 exactly as printed, a bare arithmetic shift.
 * Errors: as ivit_linear_requant; PARAM for an unknown option value. */
enum { IVIT_KERNEL_AUTO = 0, IVIT_KERNEL_MANY_ROWS = 1, IVIT_KERNEL_REG_STATIONARY = 2, IVIT_KERNEL_BIG_TILES = 3 };
enum { IVIT_ROUND_NEAREST = 0, IVIT_ROUND_FLOOR = 1 };
typedef struct { int32_t kernel; int32_t rounding; } ivit_linear_options;
int ivit_linear_requant_ex(void* stream, const int8_t* x, const int8_t* w, const int32_t* bias,
                           const int32_t* rq_b, const int32_t* rq_c,
                           const int8_t* residual, ivit_dyadic res_rq,
                           const ivit_shift_params* gelu, ivit_dyadic gelu_rq,
                           int8_t* y, int64_t M, int32_t N, int32_t K, const ivit_linear_options* opt);

/* The hipError_t (as an int) behind the most recent IVIT_ERR_HIP returned to the calling thread; 0 if there was none. */
int ivit_last_hip_error(void);

/* Shiftmax (Sec. 3.3, Algorithm 1) on each row: subtract the row maximum, ShiftExp,
 * IntDiv by the row sum, limit to 2^(k_out-1) - 1.
 * x [rows, ld] int8 (the first `cols` entries of each row are used, ld >= cols),
 * y [rows, cols] int8 dense.  bias (nullable) is an int8 table [H, T, cols] added to the
 * input before the maximum is taken; row r uses bias[(r / T) % H][r % T][:] (rows ordered
 * image-or-window major, then head, then query token).  With bias == NULL, H and T are ignored.
 * Requirements: rows >= 0, 1 <= cols <= 1024; with bias: H >= 1, T >= 1.
 * Errors: NULL, SHAPE, PARAM (shift parameters), HIP. */
int ivit_shiftmax(void* stream, const int8_t* x, const int8_t* bias, int32_t H, int32_t T,
                  int8_t* y, int64_t rows, int32_t cols, int32_t ld, ivit_shift_params p);

/* ShiftGELU (Sec. 3.4, Algorithm 2) elementwise, the maximum of the algorithm read per
 * element as max(I_p, 0), followed by the dyadic rescale of I_in * I_div to int8.
 * x, y [n] int8 (y may alias x).  n >= 0.  Errors: NULL, SHAPE, PARAM, HIP. */
int ivit_shiftgelu(void* stream, const int8_t* x, int8_t* y, int64_t n,
                   ivit_shift_params p, ivit_dyadic out_rq);

/* Same, but returns the raw product I_in * I_div (|value| <= 127 * 2^(k_out-1)) as int16,
 * i.e. the tensor before its rescale to int8.  y16 [n] int16, 2-byte aligned. */
int ivit_shiftgelu_raw(void* stream, const int8_t* x, int16_t* y16, int64_t n, ivit_shift_params p);

/* ShiftGELU with the other reading of Algorithm 2's max(I_p), which names no axis: the maximum over each row,
 * m = max(0, max_j I_p[row][j]); I_exp = ShiftExp(I_p - m), I_exp' = ShiftExp(-m), I_div = IntDiv(I_exp, I_exp + I_exp')
 * (0 where both ShiftExp values have shifted out to 0), y = requant(I * I_div; out_rq).  Far from a large row maximum
 * this form loses the value altogether unless ShiftExp is wide, so here the shift parameters may be wide:
 * i0 << n_shift <= 2^30 and k_out - 1 <= m_bits <= 46 (the reciprocal of IntDiv is formed in 64 bits).
 * x, y int8 [rows, cols] dense, 4-byte aligned (y may alias x); rows >= 0, 4 <= cols <= 4096, cols % 4 == 0.
 * Errors: NULL, SHAPE, PARAM, ALIGN, HIP. */
int ivit_shiftgelu_rowmax(void* stream, const int8_t* x, int8_t* y, int64_t rows, int32_t cols, ivit_shift_params p,
                          ivit_dyadic out_rq);

/* I-LayerNorm (Sec. 3.5, Eq. 19-20) on each row of x [rows, C]:
 *   mean = floor((sum x + floor(C/2)) / C);  var = floor(sum (x - mean)^2 / C);
 *   std  = max(1, tenth iterate of I <- (I + floor(var / I)) >> 1 from I = 2^floor(bitlen(var)/2));
 *   f = floor(2^f_bits / std);  y = clamp8(round((x - mean) * f * gamma_q[i] + beta_q[i], c_shift)).
 * gamma_q, beta_q [C] int32 carry the output scale (folded by the host).
 * Requirements: rows >= 0, 4 <= C <= 2048, C % 4 == 0, 1 <= f_bits <= 20, 1 <= c_shift <= 31,
 * x and y 4-byte aligned; |gamma_q| < 2^15 and |(x - mean) * f * gamma_q + beta_q| < 2^31 - 2^(c_shift-1)
 * (a precondition on device data: the two products are taken with 24-bit factors; outside it the values are
 * unspecified, nothing faults; ivit_ilayernorm_limits gives parameter bounds that satisfy it for every row).
 * Errors: NULL, SHAPE, PARAM, ALIGN, HIP. */
int ivit_ilayernorm(void* stream, const int8_t* x, const int32_t* gamma_q, const int32_t* beta_q,
                    int8_t* y, int64_t rows, int32_t C, int32_t f_bits, int32_t c_shift);

/* Host helper for the precondition of ivit_ilayernorm: bounds on the device parameters under which its 32-bit
 * arithmetic is exact for EVERY possible row (Sec. 3.5 normalises by an integer standard deviation, so
 * |x - mean| * f never exceeds 2 sqrt(C) 2^f_bits).  With |gamma_q| <= *gamma_max and |beta_q| <= *beta_max
 * (2^30, one less at c_shift = 31) no row can overflow; parameters beyond these bounds may still be fine for the rows
 * actually seen (the bound is reached only by rows that are constant but for a few spikes).  *gamma_max == 0 means that no gamma is safe for all rows.
 * Errors: SHAPE, PARAM (as ivit_ilayernorm), NULL. */
int ivit_ilayernorm_limits(int32_t C, int32_t f_bits, int32_t c_shift, int32_t* gamma_max, int32_t* beta_max);

/* Bytes of workspace ivit_encoder_block / ivit_forward need for these dimensions
 * (0 if the dimensions are invalid). */
size_t ivit_workspace_bytes(const ivit_dims* d);

/* One encoder block (Eq. 1-2): xhat = MSA(LN(x)) + x;  y = MLP(LN(xhat)) + xhat, every
 * step integer-only.  x, y [B*T, C] int8 (y must not alias x).  The packed qkv tensor is
 * [B*T, 3C] with columns [0,C) = Q, [C,2C) = K, [2C,3C) = V and head h owning columns
 * h*d .. (h+1)*d of each third.  taps may be NULL.
 * Requirements: B >= 0, 1 <= T <= 256, C = H*d with d in {32, 64}, C % 16 == 0, F % 16 == 0,
 * C, F <= 65536 (C <= 1024 for the LayerNorm); workspace 256-byte aligned.
 * Errors: NULL, SHAPE, PARAM, ALIGN, WORKSPACE, HIP. */
int ivit_encoder_block(void* stream, const int8_t* x, int8_t* y, const ivit_block_params* p,
                       const ivit_dims* d, void* workspace, size_t workspace_bytes,
                       const ivit_debug_taps* taps);

/* ivit_encoder_block for callers that cannot allocate device memory (code under HIP graph capture, serving loops
 * that must not call hipMalloc, harnesses that forbid it): same arguments, checks and results, but the intermediate
 * tensors live in a scratch array of IVIT_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy
 * per GPU, held until the process ends) instead of a caller's workspace.  The call itself allocates and frees
 * nothing.  Dimensions whose intermediates do not fit (roughly B * T * (9 C + F) bytes) give IVIT_ERR_WORKSPACE.
 * All calls on one GPU share that GPU's array: calls that may run at the same time (different streams, different
 * threads) race on it and must be serialised by the caller; calls on one stream are ordered and safe.  Nothing in
 * the array has to survive between calls.  The device of `stream` must be the current device.
 * Errors: NULL, SHAPE, PARAM, ALIGN, WORKSPACE (too large for the scratch), HIP. */
#define IVIT_STATIC_SCRATCH_BYTES (32u << 20)
int ivit_encoder_block_static(void* stream, const int8_t* x, int8_t* y, const ivit_block_params* p,
                              const ivit_dims* d, const ivit_debug_taps* taps);

/* n_blocks encoder blocks in sequence (n_blocks >= 0), then the optional final
 * I-LayerNorm.  `blocks` is a host array.  x, y [B*T, C] int8 (y must not alias x). */
int ivit_forward(void* stream, const int8_t* x, int8_t* y, const ivit_block_params* blocks, int32_t n_blocks,
                 const ivit_final_ln* final_ln, const ivit_dims* d, void* workspace, size_t workspace_bytes);

/* Fused multi-head attention on a packed qkv tensor [B*T, 3C] (Eq. 3-4), the step of the
 * block between the QKV Dense and the projection:
 *   A = requant(Q K^T; qk_rq) [+ rel_bias];  P = Shiftmax(rows of A);  O = requant(P V; pv_rq),
 * heads concatenated into o [B*T, C].  tap_scores / tap_probs (nullable) receive A before the
 * bias and P, each [B,H,T,T] int8.  Requirements as for ivit_encoder_block; qkv and o 16-byte aligned.
 * Errors: NULL, SHAPE, PARAM, ALIGN, HIP. */
int ivit_attention(void* stream, const int8_t* qkv, const int8_t* rel_bias, int8_t* o, const ivit_dims* d,
                   ivit_dyadic qk_rq, ivit_shift_params softmax, ivit_dyadic pv_rq,
                   int8_t* tap_scores, int8_t* tap_probs);

/* The same with the additive mask of shifted-window attention (the windowed models of Table 1 add -100 to the
 * logits of token pairs that the cyclic shift brought together): where mask[b % n_mask][i][j] != 0 the score
 * of query i and key j of window b gets -100 * I_0 (that is -100 at the integer scale of the logits, I_0 being
 * softmax.i0) after the rescale and the bias and before the row maximum; ShiftExp of such a value is 0 unless
 * I_0 is tiny, so those keys drop out of the row.  mask int8 [n_mask, T, T], shared by the heads, nullable
 * (then n_mask is ignored); the windows of an image are consecutive values of b.  Errors as ivit_attention,
 * SHAPE if a mask is given with n_mask < 1. */
int ivit_attention_masked(void* stream, const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask,
                          int8_t* o, const ivit_dims* d, ivit_dyadic qk_rq, ivit_shift_params softmax,
                          ivit_dyadic pv_rq, int8_t* tap_scores, int8_t* tap_probs);

/* Windowed attention on tokens that stay in image order (the windowed models of Table 1: every step of a block but
 * attention acts on single tokens, so the cyclic shift and the window partition of those models reduce to WHICH
 * rows attention reads and writes).  d->B counts windows, n_win of them per image, d->T tokens per window; image
 * m owns rows [m * n_win * T, (m + 1) * n_win * T) of qkv and o, and token t of its window w is row
 * m * n_win * T + tok_index[w * T + t].  tok_index int32 [n_win, T] (device) should be a permutation of
 * 0 .. n_win * T - 1; entries outside that range are clamped into it (never a fault), and repeated entries make
 * windows overwrite each other's output rows.  With tok_index == NULL this is ivit_attention_masked.  The taps
 * stay window-major [B, H, T, T].  A table requires rel_bias (NULL), n_win >= 1 dividing d->B (SHAPE). */
int ivit_window_attention(void* stream, const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask,
                          const int32_t* tok_index, int32_t n_win, int8_t* o, const ivit_dims* d, ivit_dyadic qk_rq,
                          ivit_shift_params softmax, ivit_dyadic pv_rq, int8_t* tap_scores, int8_t* tap_probs);

/* ivit_window_attention with options (opt == NULL: exactly ivit_window_attention).
 *   rounding  IVIT_ROUND_NEAREST or IVIT_ROUND_FLOOR, as in ivit_linear_options, for the two dyadic requantisations
 *             of the layer (Sec. 3.2, Eq. 8-10 applied to Eq. 3-4): the scores Q K^T before Shiftmax and the output
 *             P V.  Shiftmax itself (Algorithm 1) has no rounding step and is the same in both modes.
 * Errors: as ivit_window_attention; PARAM for an unknown option value. */
typedef struct { int32_t rounding; } ivit_attention_options;
int ivit_window_attention_ex(void* stream, const int8_t* qkv, const int8_t* rel_bias, const int8_t* mask, int32_t n_mask,
                             const int32_t* tok_index, int32_t n_win, int8_t* o, const ivit_dims* d, ivit_dyadic qk_rq,
                             ivit_shift_params softmax, ivit_dyadic pv_rq, int8_t* tap_scores, int8_t* tap_probs,
                             const ivit_attention_options* opt);

/* Per-launch timing for benchmarks.  Between ivit_trace_begin and ivit_trace_end every kernel launch the
 * library makes (from any entry point, on any stream) is bracketed by two HIP events recorded on the stream
 * of the launch.  ivit_trace_end waits for the recorded events, then fills the HOST arrays (each nullable,
 * `capacity` entries) with, per launch in launch order: elapsed milliseconds, kind (1 I-LayerNorm, 2 Dense,
 * 3 Dense + residual, 4 Dense + ShiftGELU, 5 attention, 6 Shiftmax, 7 ShiftGELU, 8 token assembly, 9 patch-merging
 * gather, 10 mean pooling), algorithmic integer
 * operations (2 per int8 multiply-accumulate; 0 for row-wise kernels) and algorithmic HBM bytes (each
 * operand read once, each result written once); *count receives the number of launches seen.
 * One trace at a time per process, not thread-safe; launches beyond max_launches make ivit_trace_end
 * return IVIT_ERR_HIP.  Events are host objects: no device memory is allocated.
 * Errors: SHAPE (max_launches < 1), PARAM (begin while active / end while inactive), HIP. */
int ivit_trace_begin(int32_t max_launches);
int ivit_trace_end(float* ms, int32_t* kind, int64_t* ops, int64_t* bytes, int32_t capacity, int32_t* count);

/* ---- Embedding layer and classifier head around the encoder (Sec. 3.1; Sec. 3.2 states that the embedding
 * layer's Conv follows the same dyadic pipeline as Dense).  A 16 x 16 stride-16 Conv on an image is a Dense
 * layer on flattened patches; cutting the image into patches is a permutation and is left to the caller. ------ */

/* Token assembly: for image b, tokens[b, 0, :] comes from the class token, tokens[b, 1 + p, :] from
 * patch_tok[b, p, :] (the output of the patch Dense, ivit_linear_requant); each is rescaled by tok_rq and the
 * position embedding pos[t, :] rescaled by pos_rq is added (the two-scale addition rule of the residuals):
 *   tokens = clamp8(round(src * b_t, c_t) + round(pos * b_p, c_p)).
 * patch_tok int8 [B * P, C], cls int8 [C], pos int8 [P + 1, C], tokens int8 [B * (P + 1), C]; all 16-byte
 * aligned; C % 16 == 0, P >= 0, B >= 0.  Errors: NULL, SHAPE, PARAM (dyadic pairs), ALIGN, HIP. */
int ivit_embed_tokens(void* stream, const int8_t* patch_tok, const int8_t* cls, const int8_t* pos,
                      ivit_dyadic tok_rq, ivit_dyadic pos_rq, int8_t* tokens, int32_t B, int32_t P, int32_t C);

/* Classifier head: logits[b, :] = requant(tokens[b * T, :] . w^T + bias; rq_b, rq_c), a Dense layer on the class
 * token (row 0) of every image.  tokens int8 [B * T, C], w int8 [N, C], bias int32 [N] (nullable), rq int32 [N],
 * logits int8 [B, N]; C % 16 == 0; tokens, w, logits 16-byte aligned.  Errors as ivit_linear_requant. */
int ivit_classifier_head(void* stream, const int8_t* tokens, int32_t T, const int8_t* w, const int32_t* bias,
                         const int32_t* rq_b, const int32_t* rq_c, int8_t* logits, int32_t B, int32_t N, int32_t C);

/* Parameters of the embedding layer and the head (host struct, device pointers). */
typedef struct {
    const int8_t* w_patch;        /* [C, patch_dim]                                                 */
    const int32_t* bias_patch;    /* [C], nullable                                                  */
    const int32_t* patch_rq_b;    /* [C]                                                            */
    const int32_t* patch_rq_c;    /* [C]                                                            */
    int32_t patch_dim;            /* bytes of a flattened patch, multiple of 16                     */
    const int8_t* cls;            /* [C]                                                            */
    const int8_t* pos;            /* [T, C]                                                         */
    ivit_dyadic tok_rq, pos_rq;
    const int8_t* w_head;         /* [n_classes, C]                                                 */
    const int32_t* bias_head;     /* [n_classes], nullable                                          */
    const int32_t* head_rq_b;     /* [n_classes]                                                    */
    const int32_t* head_rq_c;     /* [n_classes]                                                    */
    int32_t n_classes;
} ivit_image_params;

/* Workspace of ivit_forward_image: that of ivit_forward plus the patch tokens and two token buffers. */
size_t ivit_image_workspace_bytes(const ivit_dims* d);

/* Patches in, logits out: patch Dense, token assembly, the block stack, the final I-LayerNorm (required here) and
 * the head.  patches int8 [B * (T - 1), patch_dim], logits int8 [B, n_classes]; d->T counts the class token.
 * Errors: those of the parts; WORKSPACE if smaller than ivit_image_workspace_bytes(d). */
int ivit_forward_image(void* stream, const int8_t* patches, int8_t* logits, const ivit_image_params* ip,
                       const ivit_block_params* blocks, int32_t n_blocks, const ivit_final_ln* final_ln,
                       const ivit_dims* d, void* workspace, size_t workspace_bytes);

/* ---- Hierarchical windowed models (the Swin rows of Table 1).  The paper names the models and gives no equations for
 * their structure; what is implemented is the published Swin Transformer layout with every operator replaced by the
 * integer one of Sec. 3: tokens of an image stay in raster order [B, g, g, C]; a block attends inside window x window
 * windows of the image shifted cyclically by -shift (ivit_window_attention with the tables below); between stages
 * patch merging halves the grid and doubles the width; the head reads the average of the final tokens. ------------- */

/* Concatenation step of patch merging: y[b, i, j, :] = x[b, 2i, 2j, :] | x[b, 2i+1, 2j, :] | x[b, 2i, 2j+1, :] |
 * x[b, 2i+1, 2j+1, :].  x int8 [B, g, g, C], y int8 [B, g/2, g/2, 4C], both 16-byte aligned; g even, C % 16 == 0.
 * (I-LayerNorm over 4C and a Dense layer without bias follow: ivit_ilayernorm, ivit_linear_requant.)
 * Errors: NULL, SHAPE, ALIGN, HIP. */
int ivit_patch_merge_gather(void* stream, const int8_t* x, int8_t* y, int32_t B, int32_t g, int32_t C);

/* Average pooling as a dyadic rescale of the token sum (the factor 1 / T is part of b / 2^c, Sec. 3.2):
 * y[b, c] = requant(sum_t x[b, t, c]; rq).  x int8 [B, T, C], y int8 [B, C], 4-byte aligned; C % 4 == 0, T <= 2^24.
 * Errors: NULL, SHAPE, PARAM, ALIGN, HIP. */
int ivit_mean_pool(void* stream, const int8_t* x, int8_t* y, int32_t B, int32_t T, int32_t C, ivit_dyadic rq);

/* Host helpers (HOST pointers, nothing is launched).  Token-index table [n_win, T] and mask [n_win, T, T] of
 * (shifted-)window attention on a g x g raster grid, n_win = (g / window)^2, T = window^2: the image is shifted by
 * -shift along both axes and cut into windows in raster order; index[w][t] is the raster position in the unshifted
 * image of token t of window w; mask[w][i][j] = 1 where tokens i and j of window w come from parts of the image
 * that the shift brought together (all 0 for shift == 0).  g % window == 0, 0 <= shift < window.
 * Errors: NULL, SHAPE, PARAM. */
int ivit_swin_window_index(int32_t g, int32_t window, int32_t shift, int32_t* index);
int ivit_swin_shift_mask(int32_t g, int32_t window, int32_t shift, int8_t* mask);

/* One stage: n_blocks blocks of width C (H heads, MLP width F); every stage but the first starts with patch merging
 * (I-LayerNorm merge_ln over 4 C_prev = 2 C channels, Dense w_merge [C, 4 C_prev] without bias).  Blocks of a
 * stage with more than one window per image must carry tok_index / n_win (and attn_mask / n_mask when shifted). */
typedef struct {
    int32_t C, H, F, n_blocks;
    const ivit_block_params* blocks;      /* host array [n_blocks]                                   */
    ivit_final_ln merge_ln;               /* unused (zero) in the first stage                        */
    const int8_t* w_merge;                /* [C, 4 C_prev]                                           */
    const int32_t *merge_rq_b, *merge_rq_c;   /* [C]                                                 */
} ivit_swin_stage;

typedef struct {
    int32_t grid, window;                 /* tokens per image side after the embedding; per window side (<= 16)  */
    int32_t n_stages;                     /* 1..4; stage s works on a grid of grid / 2^s                        */
    int32_t patch_dim, n_classes;
    const int8_t* w_patch;  const int32_t *bias_patch /*nullable*/, *patch_rq_b, *patch_rq_c;   /* [C0, patch_dim] */
    ivit_final_ln embed_ln;               /* I-LayerNorm after the patch Dense                                   */
    ivit_swin_stage stages[4];
    ivit_final_ln final_ln;
    ivit_dyadic pool_rq;
    const int8_t* w_head;   const int32_t *bias_head /*nullable*/, *head_rq_b, *head_rq_c;      /* [n_classes, C_last] */
} ivit_swin_params;

/* Workspace of ivit_forward_swin for B images (0 if the parameters are invalid). */
size_t ivit_swin_workspace_bytes(const ivit_swin_params* p, int32_t B);

/* Patches in, logits out.  patches int8 [B * grid^2, patch_dim] in raster order, logits int8 [B, n_classes], both
 * 16-byte aligned; workspace 256-byte aligned.  Everything the host can check is checked before the first launch.
 * Errors: those of the parts; SHAPE also for a grid the windows or the merging do not divide, a stage whose width is
 * not twice the previous one, or tables whose window count differs from the stage's; NULL for a multi-window stage
 * without tok_index. */
int ivit_forward_swin(void* stream, const int8_t* patches, int8_t* logits, const ivit_swin_params* p, int32_t B,
                      void* workspace, size_t workspace_bytes);

/* ---- Host helpers: the floating-point side of a quantised model -> the integers this library takes. --------
 * Pure host code on HOST pointers; nothing is launched.  They realise Sec. 3.1 Eq. 6 (symmetric uniform
 * quantisation), the dyadic number of Sec. 3.2 and the I_0 of Algorithm 1, with the readings the kernels use
 * (symmetric integer range, round to nearest with ties away from zero on the host). */

/* Measurement helper (no part of the method): launches, on `stream`, a kernel that does nothing but issue
 * v_mfma_i32_32x32x32_i8 (one wavefront per SIMD on every compute unit, 16 `iters` MFMAs each), with constant operands
 * or, if random_operands != 0, pseudo-random ones.  *int8_ops receives the integer operations the launch performs
 * (2 per multiply-accumulate); the caller times the launch with events on the same stream and so gets the rate the
 * matrix cores sustain, the practical ceiling the Dense kernels (Sec. 3.2) are compared with besides the vendor peak.
 * After completion the first 8 bytes of scratch hold the shader clock cycles the loop took on one wavefront (int64).
 * scratch: device memory, 256-byte aligned, at least 256 + 1024 * (number of compute units) bytes.
 * Errors: NULL, PARAM (iters outside 1 .. 2^24), WORKSPACE, ALIGN, HIP. */
int ivit_probe_mfma_rate(void* stream, int32_t random_operands, int32_t iters, void* scratch, size_t scratch_bytes,
                         int64_t* int8_ops);

/* q[i] = clamp(round(r[i] / S), -(2^(k-1) - 1), 2^(k-1) - 1) with S = m / (2^(k-1) - 1) (Eq. 6 with the
 * symmetric range); *scale (nullable) receives S.  n >= 0, m > 0 and finite, 2 <= k <= 8.  NaN inputs give 0.
 * Errors: NULL, SHAPE (n < 0), PARAM (m, k). */
int ivit_quantize_symmetric(const float* r, int64_t n, float m, int32_t k, int8_t* q, float* scale);

/* b / 2^c ~ x with 2^(bits-1) <= b < 2^bits where the shift allows it (Sec. 3.2): c = bits - 1 - floor(log2 x),
 * b = round(x 2^c); c is limited to [1, 46], b to [1, 2^31 - 1].  |b / 2^c - x| <= 2^-(c+1) unless a limit is
 * hit.  x > 0 and finite, 2 <= bits <= 31.  Errors: NULL, PARAM (x, bits, or x so large that c < 1 would be needed
 * with b beyond 2^31 - 1). */
int ivit_dyadic_from_float(double x, int32_t bits, ivit_dyadic* out);

/* ShiftExp / IntDiv parameters for an input scale S (Algorithm 1): i0 = round(1 / S) (at least 1),
 * n_shift = width - bitlen(i0) so that ShiftExp values stay below 2^width (width <= 16), m_bits and k_out as
 * given.  Errors: NULL, PARAM (S <= 0 or not finite, width outside [2, 16], i0 needing more than `width` bits,
 * k_out outside [2, 8], m_bits outside [k_out - 1, 31]). */
int ivit_shift_params_from_scale(double s, int32_t width, int32_t m_bits, int32_t k_out, ivit_shift_params* out);

#ifdef __cplusplus
}
#endif
#endif /* IVIT_H */
