// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): the counter-based generator behind every random
// draw of Algorithm 1 (reveal decisions, token samples, acceptance uniforms r).
// counter = (position, step, sequence, stream); key = the 64-bit seed.  Usable on the device and on the
// host (the host only replays the drafter's reveal schedule, to leave out steps that reveal nothing).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

struct Philox4 { uint32_t x, y, z, w; };

__host__ __device__ inline uint32_t mulhi32(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32); }

__host__ __device__ inline Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t seed) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = mulhi32(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = mulhi32(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{c0, c1, c2, c3};
}

// 24-bit integer numerator m of the uniform u = m * 2^-24 in [0, 1).
__host__ __device__ inline uint32_t uniform_bits(uint32_t word) { return word >> 8; }
__device__ inline float uniform_f32(uint32_t word) { return (float)(word >> 8) * 5.9604644775390625e-8f; }
__device__ inline double uniform_f64(uint32_t word) { return (double)(word >> 8) * 5.9604644775390625e-8; }

// Is slot k of sequence b revealed at reverse step `step` of the drafter (given that it is still masked)?
// Probability 1/step (Algorithm 1's sampling loop with the masked-diffusion drafter): u < 1/step with
// u = m 2^-24, decided exactly in integers as m * step < 2^24.  stream: Philox counter word 3 of the drafter's draws.
__host__ __device__ inline bool reveal_now(int k, int step, int b, uint32_t stream, uint64_t seed) {
    if (step == 1) return true;
    const Philox4 r = philox4x32_10((uint32_t)k, (uint32_t)step, (uint32_t)b, stream, seed);
    return (uint64_t)uniform_bits(r.x) * (uint64_t)step < (1ull << 24);
}

}  // namespace sd
