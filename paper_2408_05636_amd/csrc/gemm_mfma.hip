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
// freely; bank conflicts are avoided by an XOR swizzle of the 16-byte pieces of a row.
//
// A workgroup is WM x WN x KS waves (KS = waves that split the K range of one tile and reduce
// through LDS in a fixed order: deterministic results).
//
// Few-row contractions (the target's gamma + 1 query rows) have too few output tiles to pull the
// weights at HBM speed, so the K range can also be split over gridDim.y workgroups: each writes its
// fp32 partial tile to a workspace and takes a ticket; whichever workgroup draws the last ticket adds
// the partials in split order 0, 1, ... (its own included, read back from memory, so the result does
// not depend on which one was last) and runs the epilogue.  Nobody waits for anybody.
#include <algorithm>
#include <string>

#include "mfma_common.hip.h"

namespace sd {

// K split across workgroups: gsplit = gridDim.y ranges; part holds gsplit records per output tile,
// ticket one counter per output tile (zero before the launch, zero again after it).
struct SplitArgs {
    float* part;
    unsigned int* ticket;
    int gsplit;
    int x_stationary;   // workgroup -> tile mapping, see the kernel
    void* y1;           // NormOut::y1, y2, c1, c2, ld12: where the output columns from c1 on go (NULL: to Y)
    void* y2;
    int c1, c2, ld12;
    const float* rope_cs;   // NormOut::rope_cs, rope_cols, rope_dh (EPI_STORE_ROPE)
    int rope_cols, rope_dh;
};

template <int MT, int NT, int WM, int WN, int KS, int PD, int EPI, int NF, int WNT>
__global__ __launch_bounds__(256, (MT * NT == 1 ? 3 : 1)) void k_linear_mfma(const void* __restrict__ Xv, const bf16_t* __restrict__ W,
                                                     const float* __restrict__ bias, void* Y, int M,
                                                     int N, int K, int ldy, int tiles_m, int tiles_n, FoldIn nf,
                                                     FoldOut fo, SplitArgs sk) {
    const bf16_t* X = static_cast<const bf16_t*>(Xv);
    static_assert(WM * WN * KS == 4, "four waves per workgroup");
    // The wave index is uniform across the wave; telling the compiler so keeps everything derived from it
    // (tile bases, K offsets) in scalar registers -- a scalar buffer offset it believes divergent costs a
    // serialising loop around every load.
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    const int wm = wave % WM, wn = (wave / WM) % WN, wk = wave / (WM * WN);
    // Tile of this workgroup (XCD-aware order, see xcd_tile): with the weights larger (few rows) a panel of W is
    // fetched into one L2 instead of being pulled through the fabric by several of them; with x larger (many rows) x
    // is streamed from HBM once while W, which then fits an L2, is re-read from there.
    int tn, tm;
    if (!xcd_tile(tiles_m, tiles_n, sk.x_stationary, tm, tn)) return;
    const int m_base = (tm * WM + wm) * 32 * MT;
    const int n_base = (tn * WN + wn) * 32 * NT;
    // EPI_STORE_ROPE (one column tile per wave): a tile inside the rotated columns does not take 32 consecutive W rows but
    // 16 pairs (i, i + dh / 2) of one head -- tile-local column q is W row / output column cm0 + (q & 15) + (q >> 4) * cm_half --
    // so that both elements of a pair sit in one wave, 16 lanes apart, and the epilogue can rotate them.
    int cm0 = n_base, cm_half = 16;
    bool rotated = false;
    if constexpr (EPI == EPI_STORE_ROPE) {
        rotated = n_base < sk.rope_cols;
        if (rotated) {
            const int tph = sk.rope_dh / 32, tl = n_base / 32;
            cm0 = (tl / tph) * sk.rope_dh + 16 * (tl % tph);
            cm_half = sk.rope_dh / 2;
        }
    }
#define SD_COLMAP(Q) (cm0 + ((Q) & 15) + ((Q) >> 4) * cm_half)

    constexpr int TILES = MT + NT;                       // 32-row operand tiles of this wave: x tiles, then W tiles
    __shared__ u32x4 stage_all[4][TILES * 256];          // 4 KB per tile and wave
    u32x4* stage = stage_all[wave];

    // All global traffic goes through buffer resources: the per-lane byte offset stays in one VGPR,
    // the K advance is a scalar offset (no address arithmetic in the loop), and out-of-range rows
    // need neither clamping nor branches -- loads beyond the matrix return 0, stores are dropped.
    constexpr uint32_t kXBytes = 2u;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(X), 0, (uint32_t)M * (uint32_t)K * kXBytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W), 0, (uint32_t)N * (uint32_t)K * 2u, kBufFlags);
    // Load geometry: instruction i of a tile covers rows 8i .. 8i+7, lane -> (row 8i + lrow, 16-byte piece pc).
    const int lrow = lane >> 3, pc = lane & 7;
    uint32_t goff[TILES][4];                             // byte offsets of this lane's pieces at k = 0
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t row = t < MT ? (uint32_t)(m_base + 32 * t + 8 * i + lrow)
                                        : (EPI == EPI_STORE_ROPE ? (uint32_t)SD_COLMAP(8 * i + lrow) : (uint32_t)(n_base + 32 * (t - MT) + 8 * i + lrow));
            const uint32_t lim = t < MT ? (uint32_t)M : (uint32_t)N;
            goff[t][i] = row < lim ? (row * (uint32_t)K + 8u * pc) * (t < MT ? kXBytes : 2u) : kOutOfRange;
        }
    // Swizzled slot of this lane's piece within the 8-row group i (row 8 i + lrow): piece c of row r sits at
    // piece c ^ key(r), key(r) = (r & 7) ^ ((r >> 3) & 1).  A fragment read covers 32 rows at one logical piece;
    // rows are 128 bytes apart, so rows of equal parity share banks and the key must separate any 16 of them.
    const int wslot2[2] = {lrow * 8 + (pc ^ lrow), lrow * 8 + (pc ^ lrow ^ 1)};
    const int rkey = (r & 7) ^ ((r >> 3) & 1);

    floatx16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // K loop.  Two software pipelines: global -> registers runs PD chunks ahead (hides L2 / HBM
    // latency), registers -> LDS -> operand fragments runs one chunk ahead of the MFMAs (hides the LDS
    // round trip).
    // The steady-state loop has no conditional loads (the compiler's wait counts would otherwise
    // degrade to "wait for everything"); the last full group and the remainder are peeled.
    static_assert(PD % 2 == 0, "fragment double buffering assumes an even pipeline depth");
    const int n_chunks = K / 64;
    // chunks [c0, c1) belong to this workgroup (all of them unless K is split over gridDim.y)
    const int c0 = (int)((long)blockIdx.y * n_chunks / sk.gsplit), c1 = (int)((long)(blockIdx.y + 1) * n_chunks / sk.gsplit);
    // The KS waves take contiguous shares [lo, hi) of them: measured on this part, four waves that each stream
    // their own stretch of a row pull 25-40 % more bytes per second from HBM than four waves that interleave
    // 128-byte pieces of the same stretch.
    const int lo = c0 + (int)((long)(c1 - c0) * wk / KS), hi = c0 + (int)((long)(c1 - c0) * (wk + 1) / KS);
    const int n_mine = hi - lo;
    // WNT: weights that only one workgroup reads (a single row tile) are fetched with the non-temporal hint
    // (+5-10 % streaming rate, and they do not push x out of L2); with several row tiles the later ones
    // find the panel in L2 and the hint would throw that away.
    constexpr int kAuxW = WNT ? 2 : 0;
    // The first PD chunks of both operands are requested before anything else that needs a round trip (epilogue
    // operands, the row sums of a folded normalisation): those waits would otherwise sit in front of the loop.
    u32x4 g[PD][TILES][4];
#define SD_GLOAD(P, LOCAL)                                                                               \
    {                                                                                                    \
        const uint32_t koff_ = (uint32_t)(lo + (LOCAL)) * 128u;                                          \
        _Pragma("unroll") for (int t = 0; t < TILES; ++t) _Pragma("unroll") for (int i = 0; i < 4; ++i)  \
            g[P][t][i] = t < MT ? __builtin_amdgcn_raw_buffer_load_b128(rx, goff[t][i], koff_, 0)        \
                                : __builtin_amdgcn_raw_buffer_load_b128(rw, goff[t][i], koff_, kAuxW);   \
    }
    if (n_mine > 0) {
#pragma unroll
        for (int p = 0; p < PD; ++p) SD_GLOAD(p, min(p, n_mine - 1))
    }
    __builtin_amdgcn_sched_barrier(0);

    // What the epilogue will need from memory (bias, and the residual stream for the accumulate
    // epilogue) is requested now, so that these round trips overlap the K loop instead of following it.
    constexpr bool kResid = EPI == EPI_RESID || EPI == EPI_RESID_NORM;
    constexpr bool kPrefetchResid = MT * NT <= 2;
    constexpr uint32_t kOutBytes = (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_STORE_ROPE) ? 2u : 4u;
    // Where this wave's columns go: normally Y; with a column split (plain store, one column tile per wave; the split
    // points are multiples of 32, so a tile lies on one side) the tiles from c1 / c2 on go to y1 / y2.
    void* Yo = Y;
    int ldo = ldy, ncol0 = 0;
    if constexpr ((EPI == EPI_STORE || EPI == EPI_STORE_ROPE) && NT == 1) {
        if (sk.y1 != nullptr && n_base >= sk.c1) {
            const bool second = n_base >= sk.c2;
            Yo = second ? sk.y2 : sk.y1;
            ldo = sk.ld12;
            ncol0 = second ? sk.c2 : sk.c1;
        }
    }
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(Yo, 0, (uint32_t)M * (uint32_t)ldo * kOutBytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (uint32_t)N * 4u : 0u, kBufFlags);
    // Output element (row m_base + 32 i + 8 (e/4) + 4 half + e%4, column n_base + 32 j + r): the lane part of
    // the byte offset; the (i, e) part is wave-uniform and goes into the scalar offset of each access.
    uint32_t yoff[NT];
    float bv[NT], uv[NT], gv[NT];
    const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(nf.u), 0, (NF == 1) ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rgn = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(fo.gain), 0, (EPI == EPI_RESID_NORM) ? (uint32_t)N * 4u : 0u, kBufFlags);
    floatx16 yres[kPrefetchResid ? MT : 1][kPrefetchResid ? NT : 1];
    if (wk == 0) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t n = EPI == EPI_STORE_ROPE ? (uint32_t)SD_COLMAP(r) : (uint32_t)(n_base + 32 * j + r);
            yoff[j] = n < (uint32_t)N ? ((uint32_t)(m_base + 4 * half) * (uint32_t)ldo + (n - (uint32_t)ncol0)) * kOutBytes : kOutOfRange;
            bv[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, n * 4u, 0, 0));
            uv[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ru, n * 4u, 0, 0));
            gv[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rgn, n * 4u, 0, 0));
        }
        if constexpr (kPrefetchResid && kResid) {
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        yres[i][j][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                            ry, yoff[j] + (uint32_t)(32 * i + 8 * (e >> 2) + (e & 3)) * (uint32_t)ldo * 4u, 0, 0));
        }
    }

    // Row sums of the folded normalisation.  The producer left `parts` partial pairs (sum h, sum h^2) per row;
    // they are added in a fixed order: the KS waves and the two lane halves each take every (2 KS)-th pair
    // (eight loads in flight at a time), the halves are combined by one lane exchange and the waves through
    // LDS below.  The first operand chunks are already on their way, so these round trips overlap theirs.
    float w1[NF > 0 ? MT : 1] = {}, w2[NF > 0 ? MT : 1] = {};     // this wave's share, rows 32 t + r (both halves hold it)
    if constexpr (NF > 0) {
        typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
        constexpr int kStride = 2 * KS;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int row = m_base + 32 * t + r;
            float b1[4] = {0.f, 0.f, 0.f, 0.f}, b2[4] = {0.f, 0.f, 0.f, 0.f};
            if (row < M) {
                // eight pairs per round trip; loads past the end re-read the last pair and are not added
                const f32x2* sp = reinterpret_cast<const f32x2*>(nf.stats) + (size_t)row * nf.parts;
                for (int p = 2 * wk + half; p < nf.parts; p += 8 * kStride) {
                    f32x2 v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = sp[min(p + u * kStride, nf.parts - 1)];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const bool have = p + u * kStride < nf.parts;
                        b1[u & 3] += have ? v[u][0] : 0.f;
                        b2[u & 3] += have ? v[u][1] : 0.f;
                    }
                }
            }
            w1[t] = (b1[0] + b1[1]) + (b1[2] + b1[3]);
            w2[t] = (b2[0] + b2[1]) + (b2[2] + b2[3]);
            w1[t] += __shfl_xor(w1[t], 32, 64);
            w2[t] += __shfl_xor(w2[t], 32, 64);
        }
    }

    if (n_mine > 0) {
        bf16x8 f[2][TILES][4];
// LDS operations of one wave execute in order: the fragment reads see the writes before them, and
// the writes of the next chunk cannot overtake the reads of this one.
#define SD_STAGE_TO_FRAG(P, FB)                                                                          \
    {                                                                                                    \
        _Pragma("unroll") for (int t = 0; t < TILES; ++t) _Pragma("unroll") for (int i = 0; i < 4; ++i)  \
            stage[t * 256 + i * 64 + wslot2[i & 1]] = g[P][t][i];                                        \
        _Pragma("unroll") for (int t = 0; t < TILES; ++t) _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) \
            f[FB][t][s4] = __builtin_bit_cast(bf16x8, stage[t * 256 + r * 8 + ((2 * s4 + half) ^ rkey)]); \
    }
#define SD_MMA(FB)                                                                                       \
    {                                                                                                    \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) _Pragma("unroll") for (int i = 0; i < MT; ++i)  \
            _Pragma("unroll") for (int j = 0; j < NT; ++j)                                               \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[FB][i][s4], f[FB][MT + j][s4], acc[i][j], 0, 0, 0); \
    }
        const int full = n_mine / PD, rem = n_mine % PD;
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

    float* const lds_f = reinterpret_cast<float*>(&stage_all[0][0]);
    constexpr int kRedFloats = (KS - 1) * MT * NT * 16 * 64;
    constexpr int kStatFloats = KS > 1 ? KS * MT * 32 * 2 : 0; // the waves' shares of the row sums
    constexpr int kRowSumFloats = 32 * 33;                     // one 32 x 32 tile, padded rows (EPI_RESID_NORM)
    static_assert(sizeof(stage_all) >= (kRedFloats + kStatFloats + MT * 32 * 2 + kRowSumFloats) * sizeof(float), "epilogue scratch aliases the staging tiles");
    // KS > 1: scratch behind the reduction area (one wave is left); KS == 1: in the wave's own staging tile.
    float* const stat = lds_f + kRedFloats;
    float* const ab = KS > 1 ? stat + kStatFloats : reinterpret_cast<float*>(stage);
    float* const rowsum = ab + MT * 32 * 2;
    float S1 = 0.f, S2 = 0.f;          // row sums of row m_base + lane (lanes < 32 MT)

    if constexpr (KS > 1) {           // fixed-order reduction over the K-splitting waves
        float (*red)[MT * NT * 16][64] = reinterpret_cast<float (*)[MT * NT * 16][64]>(lds_f);
        __syncthreads();               // every wave has finished with its staging tile
        if constexpr (NF > 0) {
            if (half == 0) {
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    stat[((wk * MT + t) * 32 + r) * 2 + 0] = w1[t];
                    stat[((wk * MT + t) * 32 + r) * 2 + 1] = w2[t];
                }
            }
        }
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
        if constexpr (NF > 0) {
            if (lane < MT * 32) {
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    S1 += stat[(k * MT * 32 + lane) * 2 + 0];
                    S2 += stat[(k * MT * 32 + lane) * 2 + 1];
                }
            }
        }
    } else if constexpr (NF > 0) {
        S1 = w1[MT == 2 && lane >= 32 ? 1 : 0];
        S2 = w2[MT == 2 && lane >= 32 ? 1 : 0];
    }

    // K split across workgroups (one output tile set per workgroup, one wave left at this point).
    if constexpr (WM * WN == 1) {
        if (sk.gsplit > 1) {
            constexpr int kRec = MT * NT * 1024;            // accumulators [tile][e][lane]
            const int tile_id = tn * tiles_m + tm;
            float* const rec0 = sk.part + (size_t)tile_id * sk.gsplit * kRec;
            float* const mine = rec0 + (size_t)blockIdx.y * kRec;
            // Partials travel as device-scope accesses (they go past the caches that are private to one
            // XCD), so no cache-wide write-back or invalidation is needed: wait until the stores have
            // completed, then draw the ticket.
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        __hip_atomic_store(&mine[((i * NT + j) * 16 + e) * 64 + lane], acc[i][j][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // Hand-over without cache-wide operations: partials and ticket are device-scope accesses (they go past the caches
            // private to one XCD), the wait below completes every lane's partial stores before the ticket is drawn, and its
            // memory clobber keeps the compiler from moving accesses across it.  (An agent-scope release fence here is a
            // write-back of the whole L2, an acquire fence an invalidation: measured 1-2 us per kernel, and far more where
            // thousands of workgroups hand over, for data that never sat in those caches.)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            unsigned int old = 0;
            if (lane == 0) old = __hip_atomic_fetch_add(&sk.ticket[tile_id], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            old = __builtin_amdgcn_readfirstlane(old);
            if (old != (unsigned int)sk.gsplit - 1u) return;
            if (lane == 0) __hip_atomic_store(&sk.ticket[tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
            asm volatile("" ::: "memory");     // compiler barrier: the loads below stay behind the ticket
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
            // in split order, four splits per round trip to device-scope memory
            for (int g0 = 0; g0 < sk.gsplit; g0 += 4) {
                float v[4][MT * NT * 16];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float* rec = rec0 + (size_t)min(g0 + b, sk.gsplit - 1) * kRec;
#pragma unroll
                    for (int q = 0; q < MT * NT * 16; ++q)
                        v[b][q] = __hip_atomic_load(&rec[q * 64 + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const bool have = g0 + b < sk.gsplit;          // uniform
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < NT; ++j)
#pragma unroll
                            for (int e = 0; e < 16; ++e) acc[i][j][e] += have ? v[b][(i * NT + j) * 16 + e] : 0.f;
                }
            }
        }
    }

    float na[NF > 0 ? MT : 1][16], nb[NF > 0 ? MT : 1][16];   // per accumulator row: rstd and -rstd * mu
    if constexpr (NF > 0) {
        if (lane < MT * 32) {
            const float mu = NF == 1 ? S1 / (float)K : 0.f;
            const float var = fmaxf(S2 / (float)K - mu * mu, 0.f);
            const float rstd = rsqrtf(var + nf.eps);
            ab[lane * 2 + 0] = rstd;
            ab[lane * 2 + 1] = -rstd * mu;
        }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = 32 * i + 8 * (e >> 2) + 4 * half + (e & 3);
                na[i][e] = ab[row * 2 + 0];
                nb[i][e] = ab[row * 2 + 1];
            }
    }

    // Epilogue.  Accumulator e of a 32 x 32 tile: row m = 8*(e/4) + 4*half + e%4, column n = lane & 31,
    // so each store instruction writes runs of 32 consecutive columns.  No branches: rows >= M fall
    // behind the end of the buffer, columns >= N carry the out-of-range offset, and the hardware drops both.
    // (The epilogue kind is a template parameter: with a run-time switch the compiler puts a full
    // memory wait in front of every store and the 16 stores of a tile serialise.)
    const __amdgpu_buffer_rsrc_t rxg = __builtin_amdgcn_make_buffer_rsrc(fo.xg, 0, (EPI == EPI_RESID_NORM) ? (uint32_t)M * (uint32_t)N * 2u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rcs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(sk.rope_cs), 0, (EPI == EPI_STORE_ROPE) ? (uint32_t)M * (uint32_t)(sk.rope_dh / 2) * 8u : 0u, kBufFlags);
    const int parts_out = (N + 31) / 32;
    // Rotation angles of this lane's accumulator rows: all requested at once, without conditions (a load under a
    // condition is waited for on the spot); tiles outside the rotated columns read nothing and rotate by zero.
    float rope_c[EPI == EPI_STORE_ROPE ? MT : 1][16], rope_s[EPI == EPI_STORE_ROPE ? MT : 1][16];
    if constexpr (EPI == EPI_STORE_ROPE) {
        const uint32_t t0 = rotated ? ((uint32_t)(m_base + 4 * half) * (uint32_t)(sk.rope_dh / 2) + (uint32_t)(cm0 % sk.rope_dh + (r & 15))) * 8u : kOutOfRange;
        unsigned int cc[MT][16], ss[MT][16];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const uint32_t o_ = t0 + (uint32_t)(32 * i + 8 * (e >> 2) + (e & 3)) * (uint32_t)(sk.rope_dh / 2) * 8u;
                cc[i][e] = __builtin_amdgcn_raw_buffer_load_b32(rcs, o_, 0, 0);
                ss[i][e] = __builtin_amdgcn_raw_buffer_load_b32(rcs, o_ + 4u, 0, 0);
            }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                rope_c[i][e] = rotated ? __builtin_bit_cast(float, cc[i][e]) : 1.f;
                rope_s[i][e] = rotated ? __builtin_bit_cast(float, ss[i][e]) : 0.f;
            }
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const uint32_t n = EPI == EPI_STORE_ROPE ? (uint32_t)SD_COLMAP(r) : (uint32_t)(n_base + 32 * j + r);
        const uint32_t xgoff = n < (uint32_t)N ? ((uint32_t)(m_base + 4 * half) * (uint32_t)N + n) * 2u : kOutOfRange;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int lr = 32 * i + 8 * (e >> 2) + (e & 3);           // row within the wave's tiles, minus 4 * half
                const uint32_t so = (uint32_t)lr * (uint32_t)ldo * kOutBytes;
                float v = acc[i][j][e];
                if constexpr (NF > 0) v = fmaf(na[i][e], v, nb[i][e] * uv[j]);
                v += bv[j];
                if constexpr (EPI == EPI_GELU) v = gelu_fast(v);
                if constexpr (EPI == EPI_STORE_ROPE) {
                    // lanes r < 16 hold x_i, lanes r >= 16 hold x_{i + dh/2} of the same row: (a c - b s, b c + a s);
                    // tiles outside the rotated columns got (1, 0) above
                    const float other = __shfl_xor(v, 16, 64);
                    v = r < 16 ? v * rope_c[i][e] - other * rope_s[i][e] : v * rope_c[i][e] + other * rope_s[i][e];
                }
                if constexpr (kResid) {
                    if constexpr (kPrefetchResid) v += yres[i][j][e];
                    else v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ry, yoff[j] + so, 0, 0));
                }
                if constexpr (kOutBytes == 2)
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v)), ry, yoff[j] + so, 0, 0);
                else
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), ry, yoff[j] + so, 0, 0);
                if constexpr (EPI == EPI_RESID_NORM) {
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v * gv[j])), rxg,
                                                          xgoff + (uint32_t)lr * (uint32_t)N * 2u, 0, 0);
                    rowsum[(8 * (e >> 2) + 4 * half + (e & 3)) * 33 + r] = v;       // columns >= N hold 0
                }
            }
            if constexpr (EPI == EPI_RESID_NORM) {
                // Row sums of this 32 x 32 tile, columns in ascending order.  (LDS operations of one wave execute
                // in order: the reads see the stores above, the next tile's stores come after these reads.)
                const int row = m_base + 32 * i + lane;
                if (lane < 32 && row < M && n_base + 32 * j < N) {
                    float t1 = 0.f, t2 = 0.f;
#pragma unroll
                    for (int c = 0; c < 32; ++c) {
                        const float x = rowsum[lane * 33 + c];
                        t1 += x;
                        t2 = fmaf(x, x, t2);
                    }
                    float* so_ = fo.stats + ((size_t)row * parts_out + (n_base / 32 + j)) * 2;
                    so_[0] = t1;
                    so_[1] = t2;
                }
            }
        }
    }
}

static int g_variant_override = -1, g_split_override = -1;
void linear_mfma_set_variant(int v) { g_variant_override = v; }
void linear_mfma_set_split(int s) { g_split_override = s; }
int linear_mfma_get_variant() { return g_variant_override; }
int linear_mfma_get_split() { return g_split_override; }

template <int MT, int NT, int WM, int WN, int KS, int PD>
static hipError_t launch_variant(const void* x, const void* w, const float* bias, void* y, int m, int n, int k,
                                 int ldy, int epi, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws,
                                 hipStream_t st) {
    const int tiles_n = (n + 32 * NT * WN - 1) / (32 * NT * WN), tiles_m = (m + 32 * MT * WM - 1) / (32 * MT * WM);
    // K split over workgroups: only for the one-tile-set-per-workgroup shapes, when the tiles alone cannot
    // fill the chip, keeping at least two chunks per wave, within the workspace.
    SplitArgs sk{nullptr, nullptr, 1, 0, no.y1, no.y2, no.c1, no.c2, no.ld12, no.rope_cs, no.rope_cols, no.rope_dh};
    if (no.y1 && (NT != 1 || epi != EPI_STORE)) return hipErrorInvalidValue;
    sk.x_stationary = xcd_order(m, n, tiles_n);
    if constexpr (WM * WN == 1) {
        const long tiles = (long)tiles_n * tiles_m;
        const long part_floats = ws.base ? (ws.bytes - kSplitTicketBytes) / 4 : 0;
        constexpr long kRec = MT * NT * 1024;
        if (ws.base && tiles * 4 <= kSplitTicketBytes && part_floats > 0) {
            // Worth it only for long K (the ticket and the final pass over the partials cost about a
            // microsecond): aim at six chunks per wave, and stop splitting once the tiles fill the chip.
            const long chunks = k / 64;
            long want = g_split_override > 0 ? std::min((long)g_split_override, std::max(1L, chunks / (KS * 2)))
                                             : std::min(chunks / (KS * 6), 256 / tiles);
            want = std::min(want, part_floats / (tiles * kRec));
            want = std::min(want, 64L);
            if (want > 1) {
                sk.gsplit = (int)want;
                sk.ticket = static_cast<unsigned int*>(ws.base);
                sk.part = reinterpret_cast<float*>(static_cast<char*>(ws.base) + kSplitTicketBytes);
            }
        }
    }
    const dim3 grid(xcd_grid(tiles_m, tiles_n), sk.gsplit);
    const bf16_t* wb = (const bf16_t*)w;
    const FoldIn fi{ni.stats, ni.u, ni.parts, ni.eps};
    const FoldOut fo{no.gain, static_cast<bf16_t*>(no.xg), no.stats};
    const bool stream_w = WM * WN == 1 && tiles_m == 1;
#define SD_GO(EPI, NF)                                                                                                  \
    do {                                                                                                                \
        if constexpr (WM * WN == 1) {                                                                                   \
            if (stream_w) launch_kernel(k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI, NF, 1>, dim3(grid), dim3(256), 0, st, x, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n, fi, fo, sk); \
            else launch_kernel(k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI, NF, 0>, dim3(grid), dim3(256), 0, st, x, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n, fi, fo, sk); \
        } else {                                                                                                        \
            launch_kernel(k_linear_mfma<MT, NT, WM, WN, KS, PD, EPI, NF, 0>, dim3(grid), dim3(256), 0, st, x, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n, fi, fo, sk); \
        }                                                                                                               \
    } while (0)
    if (no.rope_cs) {      // rotary epilogue: few-row tiles with one column tile per wave, plain or RMS-folded input
        if constexpr (NT == 1 && WM * WN == 1) {
            if (epi != EPI_STORE || ni.kind == 1) return hipErrorInvalidValue;
            if (ni.kind == 0) SD_GO(EPI_STORE_ROPE, 0); else SD_GO(EPI_STORE_ROPE, 2);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (ni.kind == 0) {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 0); break;
            case EPI_GELU: SD_GO(EPI_GELU, 0); break;
            case EPI_RESID: if (no.gain) SD_GO(EPI_RESID_NORM, 0); else SD_GO(EPI_RESID, 0); break;
            default: SD_GO(EPI_F32, 0); break;
        }
    } else if (ni.kind == 1) {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 1); break;
            case EPI_GELU: SD_GO(EPI_GELU, 1); break;
            case EPI_F32: SD_GO(EPI_F32, 1); break;
            default: return hipErrorInvalidValue;
        }
    } else {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 2); break;
            case EPI_GELU: SD_GO(EPI_GELU, 2); break;
            case EPI_F32: SD_GO(EPI_F32, 2); break;
            default: return hipErrorInvalidValue;
        }
    }
#undef SD_GO
    return hipGetLastError();
}

bool linear_mfma_supported(int dtype, int m, int n, int k, int ldy) {
    const int64_t lim = (int64_t)1 << 31;       // every operand is addressed through a < 2 GiB buffer resource
    return dtype == SD_DTYPE_BF16 && k % 64 == 0 && m > 0 && n > 0 && (int64_t)m * k * 2 < lim && (int64_t)n * k * 2 < lim &&
           ((int64_t)m + 64) * ldy * 4 < lim;
}

static std::string g_names[8][7][3][2];   // [variant][epilogue][fold][streamed weights]: kernel names as rocprof prints them
static const char* variant_name(const char* params, int v, int epi, int nfk, int wnt) {
    std::string& s = g_names[v][epi][nfk][wnt];
    if (s.empty()) s = std::string("k_linear_mfma<") + params + "," + std::to_string(epi) + "," + std::to_string(nfk) + "," + std::to_string(wnt) + ">";
    return s.c_str();
}

// Tile choice by shape.  Up to 64 rows the weights are the whole cost: one workgroup column per 32 weight
// rows, all x rows in one wave (so W is fetched once), K split over the waves and over workgroups.
static int choose_variant(int m, int n, int k) {
    const long tiles64 = (long)((n + 63) / 64) * ((m + 63) / 64);
    const long tiles32 = (long)((n + 31) / 32) * ((m + 31) / 32);
    if (m <= 32) return 0;
    if (m <= 64) return 6;
    if (tiles64 < 160) return 0;                // few tiles: smallest tile, K split over the four waves
    if (k >= 2048 && tiles32 <= 1024) return 0; // long K, a few tiles per CU: the K split still wins (1056 x 768 x 3072: 22 vs 29 us)
    if (tiles64 < 4096) return 5;
    return 3;
}

#define SD_VARIANT(ID, MT, NT, WM, WN, KS, PD)                                                      \
    case ID:                                                                                        \
        if (kernel_name) *kernel_name = variant_name(#MT "," #NT "," #WM "," #WN "," #KS "," #PD, ID, kepi, ni.kind, WM * WN == 1 && m <= 32 * MT); \
        return launch_variant<MT, NT, WM, WN, KS, PD>(x, w, bias, y, m, n, k, ldy, epi, ni, no, ws, st);

// ni.kind != 0: x = bf16(h gain) and the row sums of h come from the producer of h (see FoldIn), bias = W beta + bias.
// no.gain != NULL (residual epilogue only): also emit x and row sums for the normalisation that follows (FoldOut).
hipError_t launch_linear_mfma(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epi, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws, hipStream_t st,
                              const char** kernel_name) {
    if (no.gain && epi != EPI_RESID) return hipErrorInvalidValue;
    if (ni.kind < 0 || ni.kind > 2 || (ni.kind && (epi == EPI_RESID || !ni.stats || ni.parts <= 0))) return hipErrorInvalidValue;
    const int kepi = no.gain ? (int)EPI_RESID_NORM : (no.rope_cs ? (int)EPI_STORE_ROPE : epi);
    if (no.rope_cs && (!no.y1 || (no.rope_dh != 64 && no.rope_dh != 128) || no.rope_cols % no.rope_dh || no.rope_cols > n || n % 32 ||
                       no.c1 % no.rope_dh || no.c2 % no.rope_dh))
        return hipErrorInvalidValue;                      // the rotary epilogue comes with the column split (q | k | v)
    if (no.y1) {       // a column split exists in the few-row kernel only
        if (epi != EPI_STORE || m > 64 || !no.y2 || no.c1 % 32 || no.c2 % 32 || no.c1 > no.c2 || no.c2 > n || no.ld12 <= 0) return hipErrorInvalidValue;
        switch (choose_variant(m, n, k)) {
            SD_VARIANT(0, 1, 1, 1, 1, 4, 2)
            SD_VARIANT(6, 2, 1, 1, 1, 4, 2)
            default: return hipErrorInvalidValue;
        }
    }
    if (g_variant_override == 9 || (g_variant_override < 0 && linear_stream_preferred(m, n, k, ni.kind != 0))) {
        const hipError_t e = launch_linear_stream(x, w, bias, y, m, n, k, ldy, epi, ni, no, ws, g_split_override, st, kernel_name);
        if (e != hipErrorNotSupported) return e;          // does not fit (K range vs. LDS, workspace): the kernels below
    }
    const int pipe = g_variant_override >= 10 && g_variant_override <= 15 ? g_variant_override - 10
                     : (g_variant_override < 0 ? linear_pipe_shape(m, n, k) : -1);
    if (pipe >= 0) {
        const hipError_t e = launch_linear_pipe(x, w, bias, y, m, n, k, ldy, epi, ni, no, pipe, st, kernel_name);
        if (e != hipErrorNotSupported) return e;          // K shorter than the ring: the kernels below
    }
    if (g_variant_override == 7 || g_variant_override == 8 || (g_variant_override < 0 && linear_tile_preferred(m, n, k)))
        return launch_linear_tile(x, w, bias, y, m, n, k, ldy, epi, ni, no, g_variant_override == 8 ? 64 : (g_variant_override == 7 ? 128 : 0), st, kernel_name);
    int v = (g_variant_override >= 0 && g_variant_override < 9) ? g_variant_override : choose_variant(m, n, k);
    if (ni.kind && v == 3) v = 5;               // the 128 x 128 wave-private tile is not instantiated with a fold
    switch (v) {
        SD_VARIANT(0, 1, 1, 1, 1, 4, 2)     // 32 x 32 tile, four waves split K
        SD_VARIANT(3, 2, 2, 2, 2, 1, 2)     // 128 x 128 tile, one 64 x 64 quadrant per wave
        SD_VARIANT(5, 1, 1, 2, 2, 1, 2)     // 64 x 64 tile, one 32 x 32 quadrant per wave
        SD_VARIANT(6, 2, 1, 1, 1, 4, 2)     // 64 x 32 tile (up to 64 x rows against 32 weight rows), four waves split K
        default: return hipErrorInvalidValue;
    }
}

// u[n] = sum_k g[k] W[n,k];  v[n] = sum_k beta[k] W[n,k] + bias[n]   (beta, bias may be NULL).  One wave per row.
__global__ __launch_bounds__(256) void k_fold_norm(const bf16_t* __restrict__ W, const float* __restrict__ g,
                                                   const float* __restrict__ beta, const float* __restrict__ bias,
                                                   float* __restrict__ u, float* __restrict__ v, int N, int K) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    float su = 0.f, sv = 0.f;
    for (int k = lane; k < K; k += 64) {
        const float w = static_cast<float>(W[(size_t)n * K + k]);
        su = fmaf(g[k], w, su);
        if (beta) sv = fmaf(beta[k], w, sv);
    }
    for (int o = 32; o > 0; o >>= 1) { su += __shfl_xor(su, o, 64); sv += __shfl_xor(sv, o, 64); }
    if (lane == 0) { u[n] = su; v[n] = sv + (bias ? bias[n] : 0.f); }
}

hipError_t launch_fold_norm(const void* w, const float* gain, const float* beta, const float* bias, float* u, float* v,
                            int n, int k, hipStream_t st) {
    launch_kernel(k_fold_norm, dim3((n + 3) / 4), dim3(256), 0, st, (const bf16_t*)w, gain, beta, bias, u, v, n, k);
    return hipGetLastError();
}

}  // namespace sd
