// Device-side pieces shared by the matrix-core kernels (contractions and attention): the vector types of the
// MFMA operands, the raw-buffer constants, the LDS-only barrier, the tanh-form GELU and the LDS swizzle key.
#pragma once

#include "common.h"

namespace sd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;              // one MFMA operand of a lane
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;              // a lane's share of a 32 x 32 tile
typedef __attribute__((__vector_size__(4 * sizeof(unsigned int)))) unsigned int u32x4;    // one 16-byte piece

constexpr int kBufFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family resource word 3)
// Offset of accesses that must not happen.  Only the VGPR offset is range-checked (the scalar offset is
// not), so everything that decides validity goes into the VGPR offset; buffers are < 2 GiB (checked on
// the host), and 2 GiB plus any in-matrix offset cannot wrap around 2^32.
constexpr uint32_t kOutOfRange = 0x80000000u;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global load in flight,
// which would cut a prefetch that runs ahead of the barrier down to what one compute phase can hide; a stage
// hand-over needs the LDS writes and reads alone.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ inline float gelu_fast(float x) {
    // tanh form: 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u))
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return x * __builtin_amdgcn_rcpf(1.f + __expf(-2.f * u));    // 1 ulp reciprocal: the result is rounded to bf16 anyway
}

// 16-byte piece c of a 128-byte tile row r is stored at piece c ^ key(r).  A fragment read touches 16-byte pieces of
// 32 consecutive rows at one logical piece index; rows are 128 bytes apart, so rows of equal parity share
// their banks and the key must separate them: any 16 consecutive rows get 16 distinct (parity, key) pairs.
__device__ inline int swizzle_key(int row) { return (row & 7) ^ ((row >> 3) & 1); }

}  // namespace sd
