// Pieces shared by the Dense kernels built on LDS-direct loads (gemm_rs.hip, gemm_ks.hip, gemm_tl.hip): those
// loads, scalar pointers, the median of three, the token order of the MFMA "A" operand.
#pragma once
#include "ivit_kernels.hpp"

namespace ivit {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace regst {

enum Epilogue { EPI_PLAIN = 0, EPI_RESIDUAL = 1, EPI_GELU = 2 };
constexpr int NXCD = 8;
constexpr int OP = 48;                       // pitch (bytes) of a channel row of the output staging tile: 32 tokens + padding
constexpr int WCK = 384;                     // bytes of K per weight chunk of the prologue
constexpr int WPITCH = WCK + 16;             // its row pitch in LDS
constexpr int WWI = 4 * 32 * (WPITCH / 16) / 64;    // load instructions (64 lanes x 16 bytes) per chunk: [4 wavefronts][32 channels][WPITCH]

__device__ __forceinline__ uint32_t lds_offset(const int8_t* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) int8_t*)p;
}
__device__ __forceinline__ const int8_t* uniform_ptr(const int8_t* p) {          // a pointer every lane agrees on -> scalar registers
    const uint64_t v = (uint64_t)p;
    // (the builtin returns a signed int: each half goes through uint32_t so that nothing is sign-extended into the other)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (const int8_t*)(((uint64_t)hi << 32) | (uint64_t)lo);
}

// 16 bytes per lane from global memory straight into LDS: lane l's piece, read at base + off, lands at lds + 16 l
// (base and lds are the same for all lanes).  Written as asm statements so that the compiler does not make every
// later LDS read wait for all such loads; the waits are placed by hand (s_waitcnt vmcnt) where the data is first read.
__device__ __forceinline__ void dma16(const int8_t* base, uint32_t off, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 : : "s"(__builtin_amdgcn_readfirstlane(lds_wave_base)), "v"(off), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ int32_t med3(int32_t v, int32_t lo, int32_t hi) {
    int32_t m;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(m) : "v"(v), "v"(lo), "v"(hi));
    return m;
}

// Token of the tile that sits in row i of the MFMA "A" operand.  Accumulator register e = 4 q + r of lane group g is
// row 8 q + 4 g + r of the product; with this assignment it is token 16 g + e: a lane holds 16 consecutive tokens.
__device__ __forceinline__ int token_of_row(int i) { return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3); }

}  // namespace regst
}  // namespace ivit
