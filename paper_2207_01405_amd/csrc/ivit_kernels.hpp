// Host-side launchers of the gfx950 kernels (internal to libivit.so; the public surface is include/ivit.h).
// Each launcher assumes arguments already validated by the C-ABI layer and returns a hipError_t.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ivit_device.hpp"

namespace ivit {

hipError_t launch_ilayernorm(hipStream_t s, const int8_t* x, const int32_t* gamma_q, const int32_t* beta_q,
                             int8_t* y, int64_t rows, int C, int f_bits, int c_shift);

hipError_t launch_shiftmax(hipStream_t s, const int8_t* x, const int8_t* bias, int H, int T, int8_t* y,
                           int64_t rows, int cols, int ld, ShiftParams p);

hipError_t launch_shiftgelu(hipStream_t s, const int8_t* x, int8_t* y8, int16_t* y16, int64_t n,
                            ShiftParams p, Dyadic out_rq);

hipError_t launch_shiftgelu_rowmax(hipStream_t s, const int8_t* x, int8_t* y, int64_t rows, int cols, ShiftParams p,
                                   Dyadic rq);

struct LinearArgs {
    const int8_t* x; const int8_t* w; const int32_t* bias; const int32_t* rq_b; const int32_t* rq_c;
    const int8_t* residual; Dyadic res_rq;
    bool gelu; ShiftParams gelu_p; Dyadic gelu_rq;
    int8_t* y; int64_t M; int N; int K;
    int64_t ldx;                         // bytes between rows of x; 0 means K (dense rows)
    int kernel;                          // 0: chosen from the shape; otherwise one of LinearKernel, forced (tests, measurements)
    int floor_shift;                     // 0: requantisations round to nearest (Eq. 8 through Eq. 10); 1: bare shift of Eq. 10 (floor)
};
enum LinearKernel { LINEAR_AUTO = 0, LINEAR_MANY_ROWS = 1, LINEAR_REG_STATIONARY = 2, LINEAR_BIG_TILES = 3 };
hipError_t launch_linear(hipStream_t s, const LinearArgs& a);
// Register-stationary kernel (gemm_rs.hip): whether it takes this shape at all, and its launch.
bool linear_rs_takes(const LinearArgs& a);
hipError_t launch_linear_rs(hipStream_t s, const LinearArgs& a);
// The same with K = 1536 split over pairs of wavefronts (gemm_ks.hip).
bool linear_ks_takes(const LinearArgs& a);
hipError_t launch_linear_ks(hipStream_t s, const LinearArgs& a);
// Long rows, both operands streamed through LDS in 256 x 128 tiles (gemm_tl.hip).
bool linear_tl_takes(const LinearArgs& a);
hipError_t launch_linear_tl(hipStream_t s, const LinearArgs& a);
hipError_t launch_embed_tokens(hipStream_t s, const int8_t* patch_tok, const int8_t* cls, const int8_t* pos, Dyadic tok_rq,
                               Dyadic pos_rq, int8_t* tokens, int B, int P, int C);

hipError_t launch_patch_merge_gather(hipStream_t s, const int8_t* x, int8_t* y, int B, int g, int C);
hipError_t launch_mean_pool(hipStream_t s, const int8_t* x, int8_t* y, int B, int T, int C, Dyadic rq);

struct AttentionArgs {
    const int8_t* qkv; const int8_t* rel_bias; int8_t* o;
    const int8_t* mask; int n_mask;      // shifted-window mask [n_mask, T, T] or nullptr
    const int32_t* tok_index; int n_win; // rows of the tokens of the n_win windows of an image [n_win, T], or nullptr
    int B, T, C, H;
    Dyadic qk_rq; ShiftParams sm; Dyadic pv_rq;
    int8_t* tap_scores; int8_t* tap_probs;
    int floor_shift;                     // as LinearArgs::floor_shift, for both requantisations (scores, output)
};
hipError_t launch_attention(hipStream_t s, const AttentionArgs& a);

// Number of compute units of the current device (cached); used to size persistent grids.
int num_cus();

// Kinds of launches reported by the trace (ivit_trace_end); values are part of the C ABI.
enum LaunchKind { KIND_ILAYERNORM = 1, KIND_GEMM = 2, KIND_GEMM_RESIDUAL = 3, KIND_GEMM_GELU = 4,
                  KIND_ATTENTION = 5, KIND_SHIFTMAX = 6, KIND_SHIFTGELU = 7, KIND_EMBED = 8, KIND_PATCH_MERGE = 9, KIND_MEAN_POOL = 10 };

// Brackets one kernel launch with two HIP events on its stream while a trace is active; otherwise a no-op.
// ops = algorithmic integer operations (2 per int8 multiply-accumulate), bytes = algorithmic HBM bytes.
class TraceScope {
public:
    TraceScope(hipStream_t s, int kind, int64_t ops, int64_t bytes);
    ~TraceScope();
    TraceScope(const TraceScope&) = delete;
    TraceScope& operator=(const TraceScope&) = delete;
private:
    hipStream_t stream_;
    int slot_;
};

}  // namespace ivit
