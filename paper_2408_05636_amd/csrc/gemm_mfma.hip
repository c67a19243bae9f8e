// bf16 contraction y = epilogue(x W^T + bias) on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation), for the QKV / projection / MLP / LM-head layers.
//
// Both operands are K-contiguous (x: [M, K], W: [N, K]).  A wave owns MT x NT tiles of 32 x 32
// outputs and walks K in chunks of 64.  Per chunk and 32-row operand tile it issues four 16-byte
// loads per lane with 8 consecutive lanes on one 128-byte line (fully coalesced: a scattered
// "one row per lane" pattern is bound by the texture-address unit, not by bandwidth), parks them
// in registers PD chunks ahead, then passes them through a wave-private, XOR-swizzled LDS tile to
// reach the MFMA operand layout (lane l supplies 8 consecutive k of row l & 31).  The LDS tile is
// private to the wave, so the K loop has no workgroup barrier and waves of a workgroup drift
// freely; bank conflicts are avoided by storing 16-byte piece c of row r at piece c ^ (r & 7).
//
// A workgroup is WM x WN x KS waves (KS = waves that split the K range of one tile and reduce
// through LDS in a fixed order: deterministic results, no atomics).
#include "common.h"

namespace sd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned int)))) unsigned int u32x4;   // one 16-byte piece
constexpr int kBufFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family resource word 3)
// Offset of accesses that must not happen.  Only the VGPR offset is range-checked (the scalar offset is
// not), so everything that decides validity goes into the VGPR offset; buffers are < 2 GiB (checked on
// the host), and 2 GiB plus any in-matrix offset cannot wrap around 2^32.
constexpr uint32_t kOutOfRange = 0x80000000u;

__device__ inline float gelu_fast(float x) {
    // tanh form: 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u))
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return x / (1.f + __expf(-2.f * u));
}

template <int MT, int NT, int WM, int WN, int KS, int PD, int EPI>
__global__ __launch_bounds__(256) void k_linear_mfma(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W,
                                                     const float* __restrict__ bias, void* Y, int M,
                                                     int N, int K, int ldy, int tiles_m, int tiles_n) {
    static_assert(WM * WN * KS == 4, "four waves per workgroup");
    // The wave index is uniform across the wave; telling the compiler so keeps everything derived from it
    // (tile bases, K offsets) in scalar registers -- a scalar buffer offset it believes divergent costs a
    // serialising loop around every load.
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    const int wm = wave % WM, wn = (wave / WM) % WN, wk = wave / (WM * WN);
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.
    // Column tile tn lives on XCD tn % 8 with all its row tiles, launched back to back: a panel of W is
    // then fetched into exactly one L2 instead of being pulled through the fabric by several of them.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tn = xcd + 8 * (local / tiles_m), tm = local % tiles_m;
    if (tn >= tiles_n) return;                          // padding workgroup of an XCD with fewer column tiles
    const int m_base = (tm * WM + wm) * 32 * MT;
    const int n_base = (tn * WN + wn) * 32 * NT;

    constexpr int TILES = MT + NT;                       // 32-row operand tiles of this wave: x tiles, then W tiles
    __shared__ u32x4 stage_all[4][TILES * 256];          // 4 KB per tile and wave
    u32x4* stage = stage_all[wave];

    // All global traffic goes through buffer resources: the per-lane byte offset stays in one VGPR,
    // the K advance is a scalar offset (no address arithmetic in the loop), and out-of-range rows
    // need neither clamping nor branches -- loads beyond the matrix return 0, stores are dropped.
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(X), 0, (uint32_t)M * (uint32_t)K * 2u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W), 0, (uint32_t)N * (uint32_t)K * 2u, kBufFlags);
    // Load geometry: instruction i of a tile covers rows 8i .. 8i+7, lane -> (row 8i + lrow, 16-byte piece pc).
    const int lrow = lane >> 3, pc = lane & 7;
    uint32_t goff[TILES][4];                             // byte offsets of this lane's pieces at k = 0
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t row = t < MT ? (uint32_t)(m_base + 32 * t + 8 * i + lrow) : (uint32_t)(n_base + 32 * (t - MT) + 8 * i + lrow);
            const uint32_t lim = t < MT ? (uint32_t)M : (uint32_t)N;
            goff[t][i] = row < lim ? (row * (uint32_t)K + 8u * pc) * 2u : kOutOfRange;
        }
    const int wslot = lrow * 8 + (pc ^ lrow);            // swizzled slot of this lane's piece within an 8-row group

    floatx16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // What the epilogue will need from memory (bias, and the residual stream for the accumulate
    // epilogue) is requested now, so that these round trips overlap the K loop instead of following it.
    constexpr bool kPrefetchResid = MT * NT <= 2;
    constexpr uint32_t kOutBytes = (EPI == EPI_STORE || EPI == EPI_GELU) ? 2u : 4u;
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(Y, 0, (uint32_t)M * (uint32_t)ldy * kOutBytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (uint32_t)N * 4u : 0u, kBufFlags);
    // Output element (row m_base + 32 i + 8 (e/4) + 4 half + e%4, column n_base + 32 j + r): the lane part of
    // the byte offset; the (i, e) part is wave-uniform and goes into the scalar offset of each access.
    uint32_t yoff[NT];
    float bv[NT];
    floatx16 yres[kPrefetchResid ? MT : 1][kPrefetchResid ? NT : 1];
    if (wk == 0) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t n = (uint32_t)(n_base + 32 * j + r);
            yoff[j] = n < (uint32_t)N ? ((uint32_t)(m_base + 4 * half) * (uint32_t)ldy + n) * kOutBytes : kOutOfRange;
            bv[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, n * 4u, 0, 0));
        }
        if constexpr (kPrefetchResid && EPI == EPI_RESID) {
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        yres[i][j][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                            ry, yoff[j] + (uint32_t)(32 * i + 8 * (e >> 2) + (e & 3)) * (uint32_t)ldy * 4u, 0, 0));
        }
    }

    // K loop.  Two software pipelines: global -> registers runs PD chunks ahead (hides L2 / HBM
    // latency), registers -> LDS -> operand fragments runs one chunk ahead of the MFMAs (hides the LDS
    // round trip).  This wave's chunks are wk, wk + KS, ...; local chunk i is global chunk wk + i*KS.
    // The steady-state loop has no conditional loads (the compiler's wait counts would otherwise
    // degrade to "wait for everything"); the last full group and the remainder are peeled.
    static_assert(PD % 2 == 0, "fragment double buffering assumes an even pipeline depth");
    const int n_chunks = K / 64;
    const int n_mine = n_chunks > wk ? (n_chunks - wk + KS - 1) / KS : 0;
    if (n_mine > 0) {
        u32x4 g[PD][TILES][4];
        bf16x8 f[2][TILES][4];
#define SD_GLOAD(P, LOCAL)                                                                               \
    {                                                                                                    \
        const uint32_t koff_ = (uint32_t)(wk + (LOCAL) * KS) * 128u;                                     \
        _Pragma("unroll") for (int t = 0; t < TILES; ++t) _Pragma("unroll") for (int i = 0; i < 4; ++i)  \
            g[P][t][i] = __builtin_amdgcn_raw_buffer_load_b128(t < MT ? rx : rw, goff[t][i], koff_, 0);  \
    }
// LDS operations of one wave execute in order: the fragment reads see the writes before them, and
// the writes of the next chunk cannot overtake the reads of this one.
#define SD_STAGE_TO_FRAG(P, FB)                                                                          \
    {                                                                                                    \
        _Pragma("unroll") for (int t = 0; t < TILES; ++t) _Pragma("unroll") for (int i = 0; i < 4; ++i)  \
            stage[t * 256 + i * 64 + wslot] = g[P][t][i];                                                \
        _Pragma("unroll") for (int t = 0; t < TILES; ++t) _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) \
            f[FB][t][s4] = __builtin_bit_cast(bf16x8, stage[t * 256 + r * 8 + ((2 * s4 + half) ^ (r & 7))]); \
    }
#define SD_MMA(FB)                                                                                       \
    {                                                                                                    \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) _Pragma("unroll") for (int i = 0; i < MT; ++i)  \
            _Pragma("unroll") for (int j = 0; j < NT; ++j)                                               \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[FB][i][s4], f[FB][MT + j][s4], acc[i][j], 0, 0, 0); \
    }
        const int full = n_mine / PD, rem = n_mine % PD;
#pragma unroll
        for (int p = 0; p < PD; ++p) SD_GLOAD(p, min(p, n_mine - 1))
        SD_STAGE_TO_FRAG(0, 0)
        for (int it = 0; it + 1 < full; ++it) {
#pragma unroll
            for (int p = 0; p < PD; ++p) {
                SD_GLOAD(p, (it + 1) * PD + p)           // stage p was consumed one step ago
                SD_STAGE_TO_FRAG((p + 1) % PD, (p + 1) & 1)
                SD_MMA(p & 1)
            }
        }
        if (full > 0) {
#pragma unroll
            for (int p = 0; p < PD; ++p) {
                if (p < rem) SD_GLOAD(p, full * PD + p)
                if (p < PD - 1 || rem > 0) SD_STAGE_TO_FRAG((p + 1) % PD, (p + 1) & 1)
                SD_MMA(p & 1)
            }
        }
#pragma unroll
        for (int p = 0; p < PD; ++p)
            if (p < rem) {
                if (p + 1 < rem) SD_STAGE_TO_FRAG((p + 1) % PD, (p + 1) & 1)
                SD_MMA(p & 1)
            }
#undef SD_GLOAD
#undef SD_STAGE_TO_FRAG
#undef SD_MMA
    }

    if constexpr (KS > 1) {           // fixed-order reduction over the K-splitting waves
        static_assert(sizeof(stage_all) >= (KS - 1) * MT * NT * 16 * 64 * sizeof(float), "reduction buffer aliases the staging tiles");
        float (*red)[MT * NT * 16][64] = reinterpret_cast<float (*)[MT * NT * 16][64]>(&stage_all[0][0]);
        __syncthreads();               // every wave has finished with its staging tile
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) red[wk - 1][(i * NT + j) * 16 + e][lane] = acc[i][j][e];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int k = 0; k < KS - 1; ++k)
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] += red[k][(i * NT + j) * 16 + e][lane];
    }

    // Epilogue.  Accumulator e of a 32 x 32 tile: row m = 8*(e/4) + 4*half + e%4, column n = lane & 31,
    // so each store instruction writes runs of 32 consecutive columns.  No branches: rows >= M fall
    // behind the end of the buffer, columns >= N carry the out-of-range offset, and the hardware drops both.
    // (The epilogue kind is a template parameter: with a run-time switch the compiler puts a full
    // memory wait in front of every store and the 16 stores of a tile serialise.)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const uint32_t so = (uint32_t)(32 * i + 8 * (e >> 2) + (e & 3)) * (uint32_t)ldy * kOutBytes;
                float v = acc[i][j][e] + bv[j];
                if constexpr (EPI == EPI_GELU) v = gelu_fast(v);
                if constexpr (EPI == EPI_RESID) {
                    if constexpr (kPrefetchResid) v += yres[i][j][e];
                    else v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ry, yoff[j] + so, 0, 0));
                }
                if constexpr (kOutBytes == 2)
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v)), ry, yoff[j] + so, 0, 0);
                else
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), ry, yoff[j] + so, 0, 0);
            }
}

template <int MT, int NT, int WM, int WN, int KS, int PD>
static hipError_t launch_variant(const void* x, const void* w, const float* bias, void* y, int m, int n, int k,
                                 int ldy, int epi, hipStream_t st) {
    const int tiles_n = (n + 32 * NT * WN - 1) / (32 * NT * WN), tiles_m = (m + 32 * MT * WM - 1) / (32 * MT * WM);
    const int grid = 8 * ((tiles_n + 7) / 8) * tiles_m;       // every XCD gets the id range of the fullest one
    const bf16_t* xb = (const bf16_t*)x;
    const bf16_t* wb = (const bf16_t*)w;
    switch (epi) {
        case EPI_STORE: k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI_STORE><<<grid, 256, 0, st>>>(xb, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n); break;
        case EPI_GELU: k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI_GELU><<<grid, 256, 0, st>>>(xb, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n); break;
        case EPI_RESID: k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI_RESID><<<grid, 256, 0, st>>>(xb, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n); break;
        default: k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI_F32><<<grid, 256, 0, st>>>(xb, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n); break;
    }
    return hipGetLastError();
}

bool linear_mfma_supported(int dtype, int m, int n, int k, int ldy) {
    const int64_t lim = (int64_t)1 << 31;       // every operand is addressed through a < 2 GiB buffer resource
    return dtype == SD_DTYPE_BF16 && k % 64 == 0 && m > 0 && n > 0 && (int64_t)m * k * 2 < lim && (int64_t)n * k * 2 < lim &&
           ((int64_t)m + 64) * ldy * 4 < lim;
}

static int g_variant_override = -1;
void linear_mfma_set_variant(int v) { g_variant_override = v; }

#define SD_VARIANT(ID, MT, NT, WM, WN, KS, PD)                                                      \
    case ID:                                                                                        \
        if (kernel_name) *kernel_name = "k_linear_mfma<" #MT "," #NT "," #WM "," #WN "," #KS "," #PD ">"; \
        return launch_variant<MT, NT, WM, WN, KS, PD>(x, w, bias, y, m, n, k, ldy, epi, st);

hipError_t launch_linear_mfma(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epi, hipStream_t st, const char** kernel_name) {
    const long tiles64 = (long)((n + 63) / 64) * ((m + 63) / 64);
    int v;
    if (g_variant_override >= 0) v = g_variant_override;
    else if (m <= 32 || tiles64 < 160) v = 0;   // few tiles: smallest tile, K split over the four waves
    else if (tiles64 < 4096) v = 5;
    else v = 3;
    switch (v) {
        SD_VARIANT(0, 1, 1, 1, 1, 4, 2)     // 32 x 32 tile, four waves split K
        SD_VARIANT(1, 1, 1, 1, 1, 4, 4)     // the same with a deeper global pipeline (long K)
        SD_VARIANT(2, 1, 1, 2, 2, 1, 4)     // 64 x 64 tile, one 32 x 32 quadrant per wave
        SD_VARIANT(3, 2, 2, 2, 2, 1, 2)     // 128 x 128 tile, one 64 x 64 quadrant per wave
        SD_VARIANT(4, 1, 1, 1, 2, 2, 2)     // 32 x 64 tile, two column halves x two K halves
        SD_VARIANT(5, 1, 1, 2, 2, 1, 2)     // as 2 with a shallower global pipeline (more waves per SIMD)
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sd
