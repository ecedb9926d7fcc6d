// Measurement helper: the rate at which this part issues v_mfma_i32_32x32x32_i8 when nothing else is going on.
// The int8 peak that the Dense layers of I-ViT (arXiv 2207.01405, Sec. 3.2) are priced against is a vendor figure at
// the nominal clock; what the matrix cores sustain depends on the operands (switching activity moves the clock), so
// the benchmark measures it next to the kernels: one wavefront per SIMD, four independent accumulators, no memory
// traffic inside the loop.  With constant operands every MFMA multiplies the same registers; with random operands
// each accumulator has its own pseudo-random A and B registers.
#include "../../include/ivit.h"
#include "ivit_kernels.hpp"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int PROBE_THREADS = 256;          // one wavefront per SIMD
constexpr int PROBE_MFMA_PER_ITER = 16;

template <bool RANDOM>
__global__ __launch_bounds__(PROBE_THREADS) void mfma_rate_kernel(int iters, int64_t* cycles, int32_t* sink) {
    const int tid = threadIdx.x;
    v4i a[4], b[4];
    uint32_t h = 0x9e3779b9u * (uint32_t)(blockIdx.x * PROBE_THREADS + tid + 1);
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 4; ++i) {
            h = h * 1664525u + 1013904223u;              // a linear congruential step: any spread of bytes will do
            a[j][i] = RANDOM ? (int)h : 0x01010101;
            h = h * 1664525u + 1013904223u;
            b[j][i] = RANDOM ? (int)h : 0x01010101;
        }
    v16i acc[4] = {};
    const int64_t t0 = clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < PROBE_MFMA_PER_ITER / 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[j], b[j], acc[j], 0, 0, 0);
    }
    const int64_t t1 = clock64();
    int s = 0;
    for (int j = 0; j < 4; ++j)
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    sink[blockIdx.x * PROBE_THREADS + tid] = s;
    if (tid == 0 && blockIdx.x == 0) *cycles = t1 - t0;
}

}  // namespace

extern "C" int ivit_probe_mfma_rate(void* stream, int32_t random_operands, int32_t iters, void* scratch, size_t scratch_bytes,
                                    int64_t* int8_ops) {
    if (!scratch || !int8_ops) return IVIT_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return IVIT_ERR_PARAM;
    const int cus = ivit::num_cus();
    const size_t need = 256 + (size_t)cus * PROBE_THREADS * sizeof(int32_t);
    if (scratch_bytes < need) return IVIT_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(scratch) & 255) return IVIT_ERR_ALIGN;
    int64_t* cycles = static_cast<int64_t*>(scratch);
    int32_t* sink = reinterpret_cast<int32_t*>(static_cast<char*>(scratch) + 256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (random_operands) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(cus), dim3(PROBE_THREADS), 0, s, iters, cycles, sink);
    else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(cus), dim3(PROBE_THREADS), 0, s, iters, cycles, sink);
    if (hipGetLastError() != hipSuccess) return IVIT_ERR_HIP;
    // 2 operations per multiply-accumulate, 32 x 32 x 32 of them per MFMA, one MFMA per wavefront
    *int8_ops = (int64_t)cus * (PROBE_THREADS / 64) * (int64_t)iters * PROBE_MFMA_PER_ITER * (2LL * 32 * 32 * 32);
    return IVIT_OK;
}
