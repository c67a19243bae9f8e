// Device-side pieces shared by the matrix-core kernels (contractions and attention): the vector types of the
// MFMA operands, the raw-buffer constants, the LDS-only barrier, the tanh-form GELU, the LDS swizzle key, the
// description of a folded normalisation and the epilogue of the kernels with workgroup-shared tiles.
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

// Workgroup -> tile for the contractions.  Workgroups are handed to the 8 XCDs round-robin by linear id and every XCD has
// its own L2, so the tiles that share the larger operand are given to one XCD, back to back: the tile list, ordered by
// that operand's tile index first (row tile when x is the larger operand, column tile when W is), is cut into eight
// consecutive pieces of equal length, piece i for XCD i.  A tile of the larger operand then reaches one L2 (two where a
// cut falls inside it) and every XCD has the same number of workgroups to within one -- dealing out whole row or column
// tiles leaves XCDs with 3 against 2 of them (17 row tiles) or 5 against 4 (33).
// x_stationary: 0 -- W is the larger operand (column tile first); 1 -- x is (row tile first); 2 -- x is larger but W is
// not small beside it: the columns form two groups, the list is group 0 row tile by row tile, then group 1, so an XCD
// pulls half of W and a quarter of x into its L2 instead of all of W and an eighth of x.
// The grid is xcd_grid() workgroups; false: a padding workgroup.
__device__ inline bool xcd_tile(int tiles_m, int tiles_n, int x_stationary, int& tm, int& tn) {
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int total = tiles_m * tiles_n;
    int lin = xcd * total / 8 + local;
    if (lin >= (xcd + 1) * total / 8) return false;
    if (x_stationary == 0) { tn = lin / tiles_m; tm = lin - tn * tiles_m; return true; }
    int c0 = 0, w = tiles_n;
    if (x_stationary == 2) {
        w = tiles_n / 2;
        if (lin >= tiles_m * w) { lin -= tiles_m * w; c0 = w; w = tiles_n - w; }
    }
    tm = lin / w;
    tn = c0 + lin - tm * w;
    return true;
}
// How to order the tiles of an m x n x k contraction (see xcd_tile): two column groups when both operands are of a size
// (x fetched by two groups of XCDs and W by four costs less than x once and W eight times iff x < 4 W).
inline int xcd_order(int64_t m, int64_t n, int tiles_n) { return m > n ? (tiles_n >= 2 && m < 4 * n ? 2 : 1) : 0; }
inline int xcd_grid(int tiles_m, int tiles_n) { return 8 * ((tiles_m * tiles_n + 7) / 8); }

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

// Normalisation folded around the contraction (no normalised copy of the residual stream h, no separate
// normalisation kernel).  For y = W norm(h) + bias:
//   LayerNorm (NF = 1):  y_n = rstd_m (sum_k h_mk g_k W_nk - mu_m u_n) + v_n,  u = W g,  v = W beta + bias
//   RMSNorm   (NF = 2):  y_n = rstd_m  sum_k h_mk g_k W_nk + bias_n
// The A operand x = bf16(h g) and the row sums of h are prepared by whoever produced h: the residual
// epilogue EPI_RESID_NORM of the previous contraction (below) or the row kernel that follows the
// embedding.  The row sums arrive as `parts` partial pairs (sum h, sum h^2) per row, added here in a
// fixed order; u and v are precomputed per layer.
struct FoldIn {
    const float* stats;  // [M][parts][2]
    const float* u;      // W g, [N] (LayerNorm only)
    int parts;
    float eps;
};
// EPI_RESID_NORM: y (fp32, the residual stream) += acc + bias as EPI_RESID, and for the normalisation that
// follows: xg[m][n] = bf16(y[m][n] gain[n]) and, per row and per 32-column tile, (sum y, sum y^2) over the
// tile's columns -> stats[m][n / 32][2].
struct FoldOut {
    const float* gain;   // [N]
    bf16_t* xg;          // [M][N]
    float* stats;        // [M][ceil(N / 32)][2]
};

// Epilogue of the kernels whose four waves share a workgroup tile (gemm_tile.hip, gemm_pipe.hip).  Wave (wm, wn) holds
// TM x TN accumulator tiles of 32 x 32 (accumulator e of a tile: row 8 (e / 4) + 4 half + e % 4, column lane & 31) of a
// tile with BM rows at (m_base, n_base).  scratch: LDS that is free once every wave has left the K loop -- rstd and
// -rstd mu of the BM rows, then one padded 32 x 32 tile per wave for the row sums of EPI_RESID_NORM.  fs1, fs2 (NF > 0):
// the sums of h and h^2 of row m_base + 64 t + (thread >> 2), complete in every thread.  bvs, uvs, gvns: bias, W gain and
// the next normalisation's gain at this lane's columns.  No barrier after the first two.
template <int EPI, int NF, int TM, int TN, int BM>
__device__ inline void shared_tile_epilogue(const floatx16 (&acc)[TM][TN], float* scratch, const float* fs1, const float* fs2,
                                            const float (&bvs)[TN], const float (&uvs)[TN], const float (&gvns)[TN], int wave,
                                            int wm, int wn, int m_base, int n_base, void* Y, int M, int N, int K, int ldy,
                                            const FoldIn& nf, const FoldOut& fo) {
    const int lane = threadIdx.x & 63, r = lane & 31, half = lane >> 5;
    float* const ab = scratch;                                            // [BM][2]
    float* const rowsum = ab + BM * 2 + wave * (32 * 33);
    if constexpr (NF > 0 || EPI == EPI_RESID_NORM) __syncthreads();
    if constexpr (NF > 0) {
        if ((threadIdx.x & 3) == 0) {
#pragma unroll
            for (int t = 0; t < BM / 64; ++t) {
                const float mu = NF == 1 ? fs1[t] / (float)K : 0.f;
                const float var = fmaxf(fs2[t] / (float)K - mu * mu, 0.f);
                const float rstd = rsqrtf(var + nf.eps);
                ab[(64 * t + (threadIdx.x >> 2)) * 2 + 0] = rstd;
                ab[(64 * t + (threadIdx.x >> 2)) * 2 + 1] = -rstd * mu;
            }
        }
        __syncthreads();
    }

    constexpr bool kResid = EPI == EPI_RESID || EPI == EPI_RESID_NORM;
    constexpr uint32_t kOutBytes = (EPI == EPI_STORE || EPI == EPI_GELU) ? 2u : 4u;
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(Y, 0, (uint32_t)M * (uint32_t)ldy * kOutBytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rxg = __builtin_amdgcn_make_buffer_rsrc(fo.xg, 0, (EPI == EPI_RESID_NORM) ? (uint32_t)M * (uint32_t)N * 2u : 0u, kBufFlags);
    const int wm_base = m_base + wm * 32 * TM;
    const int parts_out = (N + 31) / 32;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col0 = n_base + wn * 32 * TN + 32 * j;
        const uint32_t n = (uint32_t)(col0 + r);
        const uint32_t yoff = n < (uint32_t)N ? ((uint32_t)(wm_base + 4 * half) * (uint32_t)ldy + n) * kOutBytes : kOutOfRange;
        const uint32_t xgoff = n < (uint32_t)N ? ((uint32_t)(wm_base + 4 * half) * (uint32_t)N + n) * 2u : kOutOfRange;
        const float bv = bvs[j], uv = uvs[j], gvn = gvns[j];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int lr = 32 * i + 8 * (e >> 2) + (e & 3);          // row within the wave's part, minus 4 * half
                const uint32_t so = (uint32_t)lr * (uint32_t)ldy * kOutBytes;
                float v = acc[i][j][e];
                if constexpr (NF > 0) {
                    const int row = wm * 32 * TM + lr + 4 * half;
                    v = fmaf(ab[row * 2 + 0], v, ab[row * 2 + 1] * uv);
                }
                v += bv;
                if constexpr (EPI == EPI_GELU) v = gelu_fast(v);
                if constexpr (kResid) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ry, yoff + so, 0, 0));
                if constexpr (kOutBytes == 2)
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v)), ry, yoff + so, 0, 0);
                else
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), ry, yoff + so, 0, 0);
                if constexpr (EPI == EPI_RESID_NORM) {
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v * gvn)), rxg,
                                                          xgoff + (uint32_t)lr * (uint32_t)N * 2u, 0, 0);
                    rowsum[(8 * (e >> 2) + 4 * half + (e & 3)) * 33 + r] = v;       // columns >= N hold 0
                }
            }
            if constexpr (EPI == EPI_RESID_NORM) {
                // Row sums of this 32 x 32 tile, columns ascending (LDS operations of one wave execute in order).
                const int row = wm_base + 32 * i + lane;
                if (lane < 32 && row < M && col0 < N) {
                    float t1 = 0.f, t2 = 0.f;
#pragma unroll
                    for (int cc = 0; cc < 32; ++cc) {
                        const float x = rowsum[lane * 33 + cc];
                        t1 += x;
                        t2 = fmaf(x, x, t2);
                    }
                    float* so_ = fo.stats + ((size_t)row * parts_out + col0 / 32) * 2;
                    so_[0] = t1;
                    so_[1] = t2;
                }
            }
        }
    }
}

}  // namespace sd
