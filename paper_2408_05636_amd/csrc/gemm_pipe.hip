// bf16 contraction y = epilogue(x W^T + bias) for a few hundred rows and more, with the operand tiles
// sent from global memory straight into LDS (buffer_load ... lds of gfx950: 16 bytes per lane, no register
// staging, no LDS store instruction) through a ring of NS stages.  The shared-tile kernel (gemm_tile.hip) passes
// its tiles through two register sets (64 VGPRs, a store instruction per 16 bytes, two chunks of prefetch at
// most); here the tiles cost no registers and no instruction slots beyond the request, and a stage can hold
// several chunks, so a few-hundred-row contraction spends fewer of its cycles outside the MFMAs.  (Depth itself
// is not what pays: with two or three chunks in flight the pace is set by the LDS traffic of the tile, and 4, 6
// or 8 stages run alike.)
//
// A workgroup of four waves (WMV x WNV) owns a BM x BN tile, wave (wm, wn) a (32 TM) x (32 TN) part of it.
// K is walked in chunks of 64, KC chunks per stage.  A chunk of a stage holds the x tile (BM rows of 128 bytes)
// and the W tile (BN rows); piece c (16 bytes) of row r sits at piece c ^ key(r), the same XOR swizzle as in the
// shared-tile kernel.  One load instruction fills 8 consecutive rows: lane l lands at piece l & 7 of row l >> 3 of
// those eight (the hardware places lane l at base + 16 l), so the swizzle is applied by choosing which piece of
// global memory lane l asks for.  Rows beyond M or N carry an out-of-range offset and arrive as zeros.
//
// The loads are written in assembly: the compiler then neither knows about them nor waits for them, and the loop
// waits by hand -- "all but the newest (NS - 2) stages have landed" before the barrier that hands the oldest
// stage to the matrix cores.  Operand reads and MFMAs stay ordinary code with compiler-managed waits.
//   step c:  wait for stage c; barrier (everybody has stage c, everybody is done with stage c - 1);
//            request stage c + NS - 1 into the memory stage c - 1 used; multiply stage c.
// The last NS - 1 steps request nothing and wait for one stage less each.
#include <string>

#include "mfma_common.hip.h"

namespace sd {

// 64 x 16 bytes from a raw buffer (descriptor in scalar registers) to LDS bytes lds_addr + 16 lane.  The LDS base
// travels in M0; an LDS-bound load needs one wait state after M0 is written (the compiler would insert it for
// its own code, not inside an asm block).
__device__ inline void dma16(u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
// At most N of this wave's loads still in flight, then the workgroup barrier.
template <int N>
__device__ inline void wait_loads_and_barrier() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" :: "n"(N) : "memory");
}
__device__ inline u32x4 raw_descriptor(const void* p, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    u32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
    d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    d[2] = __builtin_amdgcn_readfirstlane(bytes);
    d[3] = (uint32_t)kBufFlags;
    return d;
}

template <int EPI, int WMV, int WNV, int TM, int TN, int NS, int KC, int NF>
__global__ __launch_bounds__(256) void k_linear_pipe(const void* __restrict__ Xv, const bf16_t* __restrict__ W,
                                                     const float* __restrict__ bias, void* Y, int M, int N, int K,
                                                     int ldy, int tiles_m, int tiles_n, int x_stationary,
                                                     FoldIn nf, FoldOut fo) {
    static_assert(WMV * WNV == 4, "four waves");
    constexpr int BM = 32 * TM * WMV, BN = 32 * TN * WNV;
    static_assert(BM % 64 == 0, "the row-sum gather works on 64 rows at a time");
    constexpr int LX = BM / 32, LW = BN / 32, L = (LX + LW) * KC;   // loads per wave and stage
    static_assert((NS - 2) * L <= 63, "too many loads in flight for the wait counter");
    constexpr int kChunkVecs = (BM + BN) * 8;                   // one chunk of both tiles, u32x4 units
    constexpr int kStageVecs = kChunkVecs * KC;                 // a stage holds KC consecutive chunks
    constexpr uint32_t kStageBytes = kStageVecs * 16u;
    extern __shared__ u32x4 smem[];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    const int wm = wave % WMV, wn = wave / WMV;
    int tn, tm;                 // XCD-aware tile order: the larger operand's tiles stay in one L2
    if (!xcd_tile(tiles_m, tiles_n, x_stationary, tm, tn)) return;
    const int m_base = tm * BM, n_base = tn * BN;

    const u32x4 dx = raw_descriptor(Xv, (uint32_t)M * (uint32_t)K * 2u);
    const u32x4 dw = raw_descriptor(W, (uint32_t)N * (uint32_t)K * 2u);

    // Load i of a wave fills tile rows 32 i + 8 wave .. + 7; lane l brings the piece that belongs at piece l & 7 of
    // row 32 i + 8 wave + (l >> 3), whose key is (l >> 3) ^ (wave & 1) for every i.
    const int lrow = lane >> 3;
    const int piece = (lane & 7) ^ (lrow ^ (wave & 1));
    uint32_t xoff[LX], woff[LW];
#pragma unroll
    for (int i = 0; i < LX; ++i) {
        const uint32_t row = (uint32_t)(m_base + 32 * i + 8 * wave + lrow);
        xoff[i] = row < (uint32_t)M ? (row * (uint32_t)K + 8u * piece) * 2u : kOutOfRange;
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const uint32_t row = (uint32_t)(n_base + 32 * i + 8 * wave + lrow);
        woff[i] = row < (uint32_t)N ? (row * (uint32_t)K + 8u * piece) * 2u : kOutOfRange;
    }
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem) + (uint32_t)wave * 1024u;
#define SD_PIPE_REQUEST(STAGE, GROUP)                                                               \
    _Pragma("unroll") for (int kc = 0; kc < KC; ++kc) {                                             \
        const uint32_t sb_ = lds0 + (uint32_t)(STAGE) * kStageBytes + (uint32_t)(kc * kChunkVecs * 16); \
        const uint32_t so_ = (uint32_t)((GROUP) * KC + kc) * 128u;                                  \
        _Pragma("unroll") for (int i = 0; i < LX; ++i) dma16(dx, xoff[i], so_, sb_ + (uint32_t)i * 4096u); \
        _Pragma("unroll") for (int i = 0; i < LW; ++i) dma16(dw, woff[i], so_, sb_ + (uint32_t)(BM * 128 + i * 4096)); \
    }

    // operand fragments: offsets (u32x4 units inside a stage) of this lane's piece for k step s4
    int offa[TM][4], offb[TN][4];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = wm * 32 * TM + 32 * i + r;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) offa[i][s4] = row * 8 + ((2 * s4 + half) ^ swizzle_key(row));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int row = wn * 32 * TN + 32 * j + r;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) offb[j][s4] = BM * 8 + row * 8 + ((2 * s4 + half) ^ swizzle_key(row));
    }
    bf16x8 fa[2][TM], fb[2][TN];
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

// Operand fragments are double-buffered by hand: the LDS reads of k step s4 + 1 are in flight while the
// matrix cores work on step s4.
#define SD_PIPE_FRAGS(SP, FB, S4)                                                                   \
    {                                                                                               \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[FB][i] = __builtin_bit_cast(bf16x8, (SP)[offa[i][S4]]); \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[FB][j] = __builtin_bit_cast(bf16x8, (SP)[offb[j][S4]]); \
    }
#define SD_PIPE_COMPUTE(STAGE)                                                                      \
    {                                                                                               \
        const u32x4* sp_ = smem + (STAGE) * kStageVecs;                                             \
        SD_PIPE_FRAGS(sp_, 0, 0)                                                                    \
        _Pragma("unroll") for (int q = 0; q < 4 * KC; ++q) {        /* k steps of 16 over the KC chunks of the stage */ \
            if (q + 1 < 4 * KC) SD_PIPE_FRAGS(sp_ + ((q + 1) >> 2) * kChunkVecs, (q + 1) & 1, (q + 1) & 3) \
            __builtin_amdgcn_sched_barrier(0);     /* keep the reads of the next step ahead of these MFMAs */ \
            _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j) \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[q & 1][i], fb[q & 1][j], acc[i][j], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }                                                                                           \
    }

    // Row sums of a folded normalisation: thread t adds the partial pairs p = (t & 3), (t & 3) + 4, ... of row
    // 64 g + (t >> 2); the four threads of a row are combined by two lane exchanges.  The first eight pairs of a
    // thread (all of them up to K = 1024) are requested here, ahead of the tile loads, and added up after the
    // loop, so that nothing waits for them; longer rows add their remaining pairs right away.
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    constexpr int NG = NF > 0 ? BM / 64 : 1;
    f32x2 sv[NG][8];
    float b1[NG][4] = {}, b2[NG][4] = {};
    if constexpr (NF > 0) {
#pragma unroll
        for (int t = 0; t < NG; ++t) {
            const int row = min(m_base + 64 * t + (int)(threadIdx.x >> 2), M - 1);     // rows past M repeat the last one (never stored)
            const f32x2* sp = reinterpret_cast<const f32x2*>(nf.stats) + (size_t)row * nf.parts;
            const int p0 = threadIdx.x & 3;
#pragma unroll
            for (int u = 0; u < 8; ++u) sv[t][u] = sp[min(p0 + 4 * u, nf.parts - 1)];
            for (int p = p0 + 32; p < nf.parts; p += 32) {
                f32x2 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = sp[min(p + 4 * u, nf.parts - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool have = p + 4 * u < nf.parts;
                    b1[t][u & 3] += have ? v[u][0] : 0.f;
                    b2[t][u & 3] += have ? v[u][1] : 0.f;
                }
            }
        }
    }

    // Per-column operands of the epilogue, requested ahead of everything else: their round trip is over long
    // before the loop ends (and, being older than every tile load, they never delay the waits of the loop).
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(nf.u), 0, (NF == 1) ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rgn = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(fo.gain), 0, (EPI == EPI_RESID_NORM) ? (uint32_t)N * 4u : 0u, kBufFlags);
    float bvs[TN], uvs[TN], gvns[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const uint32_t n = (uint32_t)(n_base + wn * 32 * TN + 32 * j + r);
        bvs[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, n * 4u, 0, 0));
        uvs[j] = NF == 1 ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ru, n * 4u, 0, 0)) : 0.f;
        gvns[j] = EPI == EPI_RESID_NORM ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rgn, n * 4u, 0, 0)) : 0.f;
    }

    const int n_chunks = K / (64 * KC);          // groups of KC chunks: >= NS - 1, K a multiple of 64 KC (checked by the launcher)
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) SD_PIPE_REQUEST(s, s)

    int c = 0, stage = 0, fill = NS - 1;        // stage of chunk c; stage that chunk c + NS - 1 goes to
    for (; c + NS - 1 < n_chunks; ++c) {
        wait_loads_and_barrier<(NS - 2) * L>();
        SD_PIPE_REQUEST(fill, c + NS - 1)
        SD_PIPE_COMPUTE(stage)
        stage = stage + 1 == NS ? 0 : stage + 1;
        fill = fill + 1 == NS ? 0 : fill + 1;
    }
    // the last NS - 1 chunks: nothing left to request, one stage less in flight each time
#define SD_PIPE_TAIL(T)                                                                             \
    if constexpr ((T) < NS - 1) {                                                                   \
        wait_loads_and_barrier<(NS - 2 - (T)) * L * ((T) < NS - 1)>();                              \
        SD_PIPE_COMPUTE(stage)                                                                      \
        stage = stage + 1 == NS ? 0 : stage + 1;                                                    \
    }
    SD_PIPE_TAIL(0) SD_PIPE_TAIL(1) SD_PIPE_TAIL(2) SD_PIPE_TAIL(3) SD_PIPE_TAIL(4) SD_PIPE_TAIL(5) SD_PIPE_TAIL(6)
    static_assert(NS - 1 <= 7, "extend the tail");
#undef SD_PIPE_TAIL
#undef SD_PIPE_REQUEST
#undef SD_PIPE_FRAGS
#undef SD_PIPE_COMPUTE

    // Epilogue (shared with the register-staged tile kernel); its LDS scratch is the ring, free once every wave has
    // left the loop.  The row sums of a folded normalisation are completed first.
    float fs1[NG], fs2[NG];
    if constexpr (NF > 0) {
#pragma unroll
        for (int t = 0; t < NG; ++t) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool have = (int)(threadIdx.x & 3) + 4 * u < nf.parts;
                b1[t][u & 3] += have ? sv[t][u][0] : 0.f;
                b2[t][u & 3] += have ? sv[t][u][1] : 0.f;
            }
            fs1[t] = (b1[t][0] + b1[t][1]) + (b1[t][2] + b1[t][3]);
            fs2[t] = (b2[t][0] + b2[t][1]) + (b2[t][2] + b2[t][3]);
            fs1[t] += __shfl_xor(fs1[t], 1, 64); fs2[t] += __shfl_xor(fs2[t], 1, 64);
            fs1[t] += __shfl_xor(fs1[t], 2, 64); fs2[t] += __shfl_xor(fs2[t], 2, 64);
        }
    }
    shared_tile_epilogue<EPI, NF, TM, TN, BM>(acc, reinterpret_cast<float*>(smem), fs1, fs2, bvs, uvs, gvns, wave, wm, wn, m_base,
                                              n_base, Y, M, N, K, ldy, nf, fo);
}

// Tile shapes: id -> (waves WMV x WNV, wave part TM x TN of 32 x 32 tiles, stages, chunks per stage)
//   0:  64 x  64, 4 stages of 1 chunk (64 KB)     1:  64 x 128, 4 x 1 (96 KB)
//   2: 128 x 128, 4 x 1 (128 KB)                  3: 256 x 128, 3 x 1 (144 KB)
//   4:  64 x  64, 3 stages of 2 chunks (96 KB)    5:  64 x 128, 3 x 2 (144 KB)   -- K a multiple of 128
// Two chunks per stage halve what a step costs besides its MFMAs (the wait and barrier, the burst of load
// requests, the first operand read that nothing hides): with 4 MFMAs per wave and chunk (64 x 64) that is most of it.
constexpr int kPipeShapeCount = 6;
struct PipeShape { int wmv, wnv, tm, tn, ns, kc, bm, bn; };
static const PipeShape kPipeShapes[kPipeShapeCount] = {{2, 2, 1, 1, 4, 1, 64, 64}, {1, 4, 2, 1, 4, 1, 64, 128}, {2, 2, 2, 2, 4, 1, 128, 128},
                                                       {2, 2, 4, 2, 3, 1, 256, 128}, {2, 2, 1, 1, 3, 2, 64, 64}, {1, 4, 2, 1, 3, 2, 64, 128}};

static std::string g_pipe_names[kPipeShapeCount][5][3];
static const char* pipe_name(int shape, int epi, int nfk) {      // the template arguments, as a profiler prints them
    std::string& s = g_pipe_names[shape][epi][nfk];
    if (s.empty()) {
        const PipeShape& p = kPipeShapes[shape];
        s = "k_linear_pipe<" + std::to_string(epi) + "," + std::to_string(p.wmv) + "," + std::to_string(p.wnv) + "," +
            std::to_string(p.tm) + "," + std::to_string(p.tn) + "," + std::to_string(p.ns) + "," + std::to_string(p.kc) + "," + std::to_string(nfk) + ">";
    }
    return s.c_str();
}

template <int EPI, int WMV, int WNV, int TM, int TN, int NS, int KC, int NF>
static hipError_t launch_pipe_kernel(int grid, hipStream_t st, const void* x, const bf16_t* wb, const float* bias, void* y,
                                     int m, int n, int k, int ldy, int tiles_m, int tiles_n, int xs, const FoldIn& fi,
                                     const FoldOut& fo) {
    constexpr int kLds = NS * KC * (32 * TM * WMV + 32 * TN * WNV) * 128;
    static_assert(kLds >= (32 * TM * WMV * 2 + 4 * 32 * 33) * 4, "epilogue scratch fits in the stages");
    static bool raised = false;                   // more than the default 64 KB of LDS: allowed once per kernel
    if (!raised) {
        const hipError_t e = hipFuncSetAttribute((const void*)k_linear_pipe<EPI, WMV, WNV, TM, TN, NS, KC, NF>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    launch_kernel(k_linear_pipe<EPI, WMV, WNV, TM, TN, NS, KC, NF>, dim3(grid), dim3(256), kLds, st, x, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n, xs, fi, fo);
    return hipGetLastError();
}

template <int WMV, int WNV, int TM, int TN, int NS, int KC>
static hipError_t launch_pipe(const void* x, const bf16_t* wb, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epi, const NormIn& ni, const NormOut& no, hipStream_t st) {
    constexpr int BM = 32 * TM * WMV, BN = 32 * TN * WNV;
    if (k % (64 * KC) != 0 || k / (64 * KC) < NS - 1) return hipErrorNotSupported;
    const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
    const int xs = xcd_order(m, n, tiles_n);
    const int grid = xcd_grid(tiles_m, tiles_n);
    const FoldIn fi{ni.stats, ni.u, ni.parts, ni.eps};
    const FoldOut fo{no.gain, static_cast<bf16_t*>(no.xg), no.stats};
#define SD_GO(EPI, NF) return launch_pipe_kernel<EPI, WMV, WNV, TM, TN, NS, KC, NF>(grid, st, x, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n, xs, fi, fo)
    if (ni.kind == 0) {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 0);
            case EPI_GELU: SD_GO(EPI_GELU, 0);
            case EPI_RESID: if (no.gain) SD_GO(EPI_RESID_NORM, 0); else SD_GO(EPI_RESID, 0);
            default: SD_GO(EPI_F32, 0);
        }
    } else if (ni.kind == 1) {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 1);
            case EPI_GELU: SD_GO(EPI_GELU, 1);
            case EPI_F32: SD_GO(EPI_F32, 1);
            default: return hipErrorInvalidValue;
        }
    } else {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 2);
            case EPI_GELU: SD_GO(EPI_GELU, 2);
            case EPI_F32: SD_GO(EPI_F32, 2);
            default: return hipErrorInvalidValue;
        }
    }
#undef SD_GO
}

// Tile shape for a contraction, -1: leave it to the other kernels.  The ring pays off for a few hundred to a couple of
// thousand rows (the drafter's layers at batch 1, the batched target pass).  Every shape moves its operands from L2 to
// the CU at about the same 24 bytes per clock and CU (deeper rings, more chunks per stage or requesting all operand
// fragments of a stage at once change nothing), so what counts is bytes per CU: measured with the balanced XCD order,
// K = 768 (1600 alike), a round of 64 x 64 tiles costs about 2.5 us and a round of 128 x 128 tiles about 5.4 us on top
// of 3.6 us per launch; 64 x 64 workgroups share a CU two at a time (64 KB of LDS), 128 x 128 ones have it alone.  So:
// the small tile while the 256 CUs hold all of them about twice, the large one after that; 64 x 128 tiles (one wave per
// 32 columns) win nowhere.  When the small tiles fit the chip once, two chunks per stage (fewer waits and barriers) are
// a little faster still -- 1056 x 768 x 3072 with the residual epilogue: 16.4 us against 20.0 for the wave-private quadrants.
int linear_pipe_shape(int m, int n, int k) {
    if (m < 192 || m > 2048 || k / 64 < 5) return -1;
    const long t64 = (long)((m + 63) / 64) * ((n + 63) / 64), t128 = (long)((m + 127) / 128) * ((n + 127) / 128);
    // narrow outputs: below about a thousand rows the wave-private quadrants with their K split inside the workgroup are
    // faster (272 x 768 x 3072: 7.0 us against 12.5)
    if (n < 2048) return (m >= 800 && n >= 512) ? (t64 <= 256 && k % 128 == 0 ? 4 : 0) : -1;
    const double cost64 = 2.5 * (t64 <= 256 ? 1.0 : t64 / 256.0), cost128 = 5.4 * (double)((t128 + 255) / 256);
    if (cost128 < cost64) return 2;
    return t64 <= 256 && k % 128 == 0 ? 4 : 0;
}

// x bf16 [m, k], w bf16 [n, k]; same shape limits as the few-row kernel (linear_mfma_supported); ni / no as there.
// shape: index into the table above.  hipErrorNotSupported: K shorter than the ring.
hipError_t launch_linear_pipe(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epi, const NormIn& ni, const NormOut& no, int shape, hipStream_t st,
                              const char** kernel_name) {
    if (epi < 0 || epi > 3 || shape < 0 || shape >= kPipeShapeCount) return hipErrorInvalidValue;
    if (kernel_name) *kernel_name = pipe_name(shape, no.gain ? (int)EPI_RESID_NORM : epi, ni.kind);
    const bf16_t* wb = static_cast<const bf16_t*>(w);
    switch (shape) {
        case 0: return launch_pipe<2, 2, 1, 1, 4, 1>(x, wb, bias, y, m, n, k, ldy, epi, ni, no, st);
        case 1: return launch_pipe<1, 4, 2, 1, 4, 1>(x, wb, bias, y, m, n, k, ldy, epi, ni, no, st);
        case 2: return launch_pipe<2, 2, 2, 2, 4, 1>(x, wb, bias, y, m, n, k, ldy, epi, ni, no, st);
        case 3: return launch_pipe<2, 2, 4, 2, 3, 1>(x, wb, bias, y, m, n, k, ldy, epi, ni, no, st);
        case 4: return launch_pipe<2, 2, 1, 1, 3, 2>(x, wb, bias, y, m, n, k, ldy, epi, ni, no, st);
        default: return launch_pipe<1, 4, 2, 1, 3, 2>(x, wb, bias, y, m, n, k, ldy, epi, ni, no, st);
    }
}

}  // namespace sd
