// bf16 contraction y = epilogue(x W^T + bias) for up to 64 rows against a large weight matrix (the target's
// gamma + 1 query rows, the LM heads): the weights are the whole cost and have to arrive at HBM speed.
//
// In the few-row kernel of gemm_mfma.hip every wave re-reads its x chunk from L2 next to each 4 KB of
// weights; with 64 x rows two thirds of the bytes that pass through the load path are x, and that path,
// not HBM, sets the rate (measured: 4.0 TB/s for a pure load loop with that mix against 6.1 TB/s for the
// weights alone).  Here the four waves of a workgroup own four neighbouring 32-column tiles and share x
// through LDS: K is walked in steps of kStep chunks of 64; the x rows of a step (the "slab", already in
// matrix-core operand order, rows beyond M replaced by one row of zeros) are fetched once per workgroup,
// one step ahead, into the other half of a double buffer, and one barrier per step publishes them.
// Between two barriers the waves run freely: wave w streams the 32 weight rows of column tile
// 4 blockIdx.x + w with non-temporal 16-byte loads (8 lanes per 128-byte line, PD chunks ahead, across the
// barriers), turns each chunk into MFMA operands through a wave-private swizzled LDS tile and reads the
// matching x operands from the slab.  Only weights cross the load path in quantity.
//
// Chunks past the end of the K range are multiplied as zeros (weight loads with an out-of-range offset fetch
// nothing and return 0), so the loop has no remainder code and no conditional loads.
//
// When the column tiles alone cannot fill the chip, the K range is split over gridDim.y: split s of column
// tile t writes its fp32 partial tile (rows < M only) to a workspace, takes a ticket, and whichever wave
// draws the last ticket of the tile adds the partials in split order (its own included, read back) and runs
// the epilogue: deterministic, and nobody waits for anybody.
//
// Normalisations folded around the contraction work as in gemm_mfma.hip (FoldIn / FoldOut in mfma_common.hip.h).
//
// EPI_ARGMAX (LM heads at temperature 0): no output matrix; a wave reduces its 32 columns per row to the largest value
// and its column (lowest column on ties) and writes one pair per row and tile.  No K split in this form.
//
// EPI_SWIGLU (the gated MLP of the Llama-shaped target): W holds the gate rows followed by the up rows; a workgroup
// takes 64 gate columns and the 64 up columns that belong to them -- waves 0, 1 the gate tiles, waves 2, 3 the up
// tiles --, the up waves hand their results over through LDS and the gate waves store silu(gate) * up.  The gate / up
// activations never reach memory and no separate gating kernel runs.  No K split in this form.
#include <algorithm>
#include <string>

#include "mfma_common.hip.h"

namespace sd {

constexpr int kStagePieces = 272;                    // per wave: 4 KB weight tile; reused as a 32 x 33 fp32 tile
constexpr int kAbPieces = 32;                        // 64 rows x (rstd, -rstd mu)
constexpr int kStreamPD = 4;                         // chunks in flight per wave (16 KB)
constexpr int kStep = 4;                             // chunks per slab step

struct StreamSplit {
    float* part;            // [column tile][split][MT * 16][64] fp32
    unsigned int* ticket;   // one counter per column tile, zero between launches
    int split_chunks;       // K chunks per workgroup (the last split may have fewer)
    float* am_v;            // EPI_ARGMAX: [M][ceil(N / 32)] largest value per row and column tile ...
    int32_t* am_i;          // ... and its column
};

template <int MT, int EPI, int NF>
__global__ __launch_bounds__(256) void k_linear_stream(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W,
                                                       const float* __restrict__ bias, void* Y, int M, int N, int K,
                                                       int ldy, FoldIn nf, FoldOut fo, StreamSplit sk) {
    constexpr int PD = kStreamPD, S = kStep;
    static_assert(S == PD && PD % 2 == 0, "one group of PD chunks per step; fragment double buffering needs an even PD");
    extern __shared__ u32x4 lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    u32x4* const stage = lds + wave * kStagePieces;
    float* const ab = reinterpret_cast<float*>(lds + 4 * kStagePieces);
    u32x4* const slab = lds + 4 * kStagePieces + kAbPieces;       // [buffer][chunk of the step][rows_s + 1][8 pieces]
    // Slab rows: all 32 of the first row tile (rows >= M arrive as zeros), of the second only up to M rounded up
    // to 8; everything beyond reads the row of zeros at index rows_s of each chunk block.
    const int rows_s = MT == 1 ? 32 : min(64, (M + 7) & ~7);
    const int blk = (rows_s + (MT == 2 ? 1 : 0)) * 8;             // pieces per chunk block
    const int buf_pieces = S * blk;

    // EPI_SWIGLU: wave -> (column pair 0 / 1, gate / up); W row n_base + r, output column o_base + r of N / 2.
    const int sw_pair = wave & 1, sw_up = wave >> 1;
    const int tile = EPI == EPI_SWIGLU ? (int)blockIdx.x * 2 + sw_pair : (int)blockIdx.x * 4 + wave;
    const int o_base = tile * 32;
    const int n_base = EPI == EPI_SWIGLU ? o_base + sw_up * (N / 2) : o_base;
    const int n_chunks = K / 64;
    const int c0 = blockIdx.y * sk.split_chunks, nck = min(sk.split_chunks, n_chunks - c0);   // >= 1 (host)
    const int steps = (nck + S - 1) / S;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(X), 0, (uint32_t)M * (uint32_t)K * 2u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W), 0, (uint32_t)N * (uint32_t)K * 2u, kBufFlags);
    // Weight loads: instruction i covers rows 8 i .. 8 i + 7 of the tile, lane -> (row 8 i + lrow, 16-byte piece pc).
    // (A wave whose tile lies beyond N loads nothing, multiplies zeros and stores nothing, but keeps the barriers.)
    const int lrow = lane >> 3, pc = lane & 7;
    uint32_t goff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t row = (uint32_t)(n_base + 8 * i + lrow);
        goff[i] = row < (uint32_t)N ? (row * (uint32_t)K + 8u * pc) * 2u : kOutOfRange;
    }
    // Piece c of tile row q sits at piece c ^ key(q), key(q) = (q & 7) ^ ((q >> 3) & 1): a fragment read covers 32
    // rows at one logical piece, rows are 128 bytes apart, and the key separates any 16 consecutive rows.
    const int wslot2[2] = {lrow * 8 + (pc ^ lrow), lrow * 8 + (pc ^ lrow ^ 1)};
    const int rkey = (r & 7) ^ ((r >> 3) & 1);
    // x fragment of row tile t, k step s4: piece (2 s4 + half) of row 32 t + r, or of the zero row.
    int xrow8[MT], xkey[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const bool have = 32 * t + r < rows_s;
        xrow8[t] = (have ? 32 * t + r : rows_s) * 8;
        xkey[t] = have ? rkey : 0;
    }

    u32x4 g[PD][4];
    // Workgroups start their walk over the chunks at different places and wrap around (a sum does not care):
    // when all of them read the same column of their rows at the same time, the requests crowd on a few
    // memory channels (measured on a pure load loop of this pattern: 5.4 -> 6.2 TB/s).
    const int start = (int)((blockIdx.x * 5u + blockIdx.y * 3u) % (unsigned)nck);
// walk position POS (chunk (start + POS) mod nck) into register slot P; past the end of the walk nothing is
// fetched and zeros arrive
#define SD_GLOAD(P, POS)                                                                            \
    {                                                                                               \
        const int pos_ = (POS);                                                                     \
        int ch_ = start + min(pos_, nck - 1);                                                       \
        ch_ = ch_ >= nck ? ch_ - nck : ch_;                                                         \
        const int lc_ = pos_ < nck ? ch_ : nck;                                                     \
        const uint32_t koff_ = (uint32_t)(c0 + ch_) * 128u;                                         \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                               \
            g[P][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, lc_ < nck ? goff[i] : kOutOfRange, koff_, 2 /* non-temporal */); \
    }
    // The weights do not depend on the slab: their first PD chunks are requested before it is filled.
#pragma unroll
    for (int p = 0; p < PD; ++p) SD_GLOAD(p, p)

    // What the epilogue needs from memory (bias, the residual stream) is requested now as well.
    constexpr bool kResid = EPI == EPI_RESID || EPI == EPI_RESID_NORM;
    constexpr uint32_t kOutBytes = (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_SWIGLU) ? 2u : 4u;
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(Y, 0, (uint32_t)M * (uint32_t)ldy * kOutBytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(nf.u), 0, (NF == 1) ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rgn = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(fo.gain), 0, (EPI == EPI_RESID_NORM) ? (uint32_t)N * 4u : 0u, kBufFlags);
    // Output element (row 32 t + 8 (e/4) + 4 half + e%4, column n_base + r).
    const uint32_t ncol = (uint32_t)(n_base + r);
    const uint32_t ocol = (uint32_t)(o_base + r);            // == ncol except for EPI_SWIGLU
    const uint32_t yoff = ncol < (uint32_t)N ? ((uint32_t)(4 * half) * (uint32_t)ldy + ocol) * kOutBytes : kOutOfRange;
    const float bv = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, ncol * 4u, 0, 0));
    const float uv = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ru, ncol * 4u, 0, 0));
    const float gv = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rgn, ncol * 4u, 0, 0));
    floatx16 yres[kResid ? MT : 1];
    if constexpr (kResid) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                yres[t][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                    ry, yoff + (uint32_t)(32 * t + 8 * (e >> 2) + (e & 3)) * (uint32_t)ldy * 4u, 0, 0));
    }

    // Slab traffic: thread -> (row 32 t + (threadIdx.x >> 3), piece threadIdx.x & 7) of each chunk of a step.
    const int srow = threadIdx.x >> 3, spc = threadIdx.x & 7;
    // Rows that the slab does not hold arrive as zeros like every row >= M and are written onto the row of
    // zeros: no store is conditional (the compiler would move the loads into the conditional blocks and wait
    // for each on the spot).
    uint32_t xoff[MT];
    int sslot[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int row = 32 * t + srow;
        xoff[t] = row < M ? ((uint32_t)row * (uint32_t)K + 8u * spc) * 2u : kOutOfRange;     // rows >= M read as 0
        sslot[t] = row < rows_s ? row * 8 + (spc ^ (row & 7) ^ ((row >> 3) & 1)) : rows_s * 8 + spc;
    }
    u32x4 xv[S][MT];
// the x rows of step ST of the walk (positions past its end repeat the last chunk: finite values against zero
// weights)
#define SD_XLOAD(ST)                                                                                \
    {                                                                                               \
        _Pragma("unroll") for (int u = 0; u < S; ++u) {                                             \
            int ch_ = start + min((ST) * S + u, nck - 1);                                           \
            ch_ = ch_ >= nck ? ch_ - nck : ch_;                                                     \
            _Pragma("unroll") for (int t = 0; t < MT; ++t)                                          \
                xv[u][t] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff[t], (uint32_t)(c0 + ch_) * 128u, 0); \
        }                                                                                           \
        __builtin_amdgcn_sched_barrier(0);          /* issued here, a step ahead of their use */  \
    }
#define SD_XWRITE(BUF)                                                                              \
    _Pragma("unroll") for (int u = 0; u < S; ++u) _Pragma("unroll") for (int t = 0; t < MT; ++t)    \
        slab[(BUF) * buf_pieces + u * blk + sslot[t]] = xv[u][t];
    SD_XLOAD(0)
    if constexpr (MT == 2) {             // the rows of zeros of both buffers, written once
        if (threadIdx.x < 2 * S * 8) slab[(threadIdx.x >> 3) * blk + rows_s * 8 + (threadIdx.x & 7)] = u32x4{0u, 0u, 0u, 0u};
    }
    SD_XWRITE(0)
    // Row statistics of a folded normalisation: thread -> row threadIdx.x >> 2, every fourth partial pair; the four
    // threads of a row are combined by two lane exchanges (a fixed order).
    if constexpr (NF > 0) {
        typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
        const int row = threadIdx.x >> 2;
        float b1[4] = {0.f, 0.f, 0.f, 0.f}, b2[4] = {0.f, 0.f, 0.f, 0.f};
        if (row < M) {
            const f32x2* sp = reinterpret_cast<const f32x2*>(nf.stats) + (size_t)row * nf.parts;
            // eight pairs per round trip; loads past the end re-read the last pair and are not added
            for (int p = threadIdx.x & 3; p < nf.parts; p += 32) {
                f32x2 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = sp[min(p + 4 * u, nf.parts - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool have = p + 4 * u < nf.parts;
                    b1[u & 3] += have ? v[u][0] : 0.f;
                    b2[u & 3] += have ? v[u][1] : 0.f;
                }
            }
        }
        float s1 = (b1[0] + b1[1]) + (b1[2] + b1[3]), s2 = (b2[0] + b2[1]) + (b2[2] + b2[3]);
        s1 += __shfl_xor(s1, 1, 64); s2 += __shfl_xor(s2, 1, 64);
        s1 += __shfl_xor(s1, 2, 64); s2 += __shfl_xor(s2, 2, 64);
        if ((threadIdx.x & 3) == 0) {
            const float mu = NF == 1 ? s1 / (float)K : 0.f;
            const float var = fmaxf(s2 / (float)K - mu * mu, 0.f);
            const float rstd = rsqrtf(var + nf.eps);
            ab[row * 2 + 0] = rstd;
            ab[row * 2 + 1] = -rstd * mu;
        }
    }
    __syncthreads();

    floatx16 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

    // Two software pipelines per wave: global -> registers runs PD chunks ahead (HBM latency), registers -> LDS ->
    // operand fragments one chunk ahead of the MFMAs (LDS round trip).  Chunk c of a step multiplies out of
    // fragment set c & 1.  The x fragments of a step's first chunk can only be read behind the barrier that
    // publishes its slab; everything else of the next chunk is staged while the current one multiplies.
    {
        bf16x8 fw[2][4], fx[2][MT][4];
// LDS operations of one wave execute in order: the fragment reads see the writes before them, and the
// writes of the next chunk cannot overtake the reads of this one.
#define SD_STAGE_W(P, FB)                                                                           \
    {                                                                                               \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) stage[i * 64 + wslot2[i & 1]] = g[P][i];      \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4)                                            \
            fw[FB][s4] = __builtin_bit_cast(bf16x8, stage[r * 8 + ((2 * s4 + half) ^ rkey)]);       \
    }
#define SD_FRAG_X(FB, BUF, U)                                                                       \
    {                                                                                               \
        const u32x4* xs_ = slab + (BUF) * buf_pieces + (U) * blk;                                   \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) _Pragma("unroll") for (int t = 0; t < MT; ++t) \
            fx[FB][t][s4] = __builtin_bit_cast(bf16x8, xs_[xrow8[t] + ((2 * s4 + half) ^ xkey[t])]); \
    }
#define SD_MMA(FB)                                                                                  \
    {                                                                                               \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) _Pragma("unroll") for (int t = 0; t < MT; ++t) \
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[FB][t][s4], fw[FB][s4], acc[t], 0, 0, 0); \
    }
        SD_STAGE_W(0, 0)
        SD_FRAG_X(0, 0, 0)
        for (int st = 0; st < steps; ++st) {
            const int buf = st & 1;
            SD_XLOAD(st + 1)
#pragma unroll
            for (int p = 0; p < PD; ++p) {
                SD_GLOAD(p, (st + 1) * PD + p)           // slot p was consumed one chunk ago
                SD_STAGE_W((p + 1) % PD, (p + 1) & 1)
                if (p + 1 < PD) SD_FRAG_X((p + 1) & 1, buf, p + 1)
                // all LDS traffic of the next chunk is on its way before the matrix cores start on this one
                // (left alone, the compiler pairs each fragment read with its MFMA and waits for every read)
                __builtin_amdgcn_sched_barrier(0);
                SD_MMA(p & 1)
                __builtin_amdgcn_sched_barrier(0);
            }
            SD_XWRITE(buf ^ 1)
            lds_barrier();
            SD_FRAG_X(0, buf ^ 1, 0)
        }
#undef SD_GLOAD
#undef SD_XLOAD
#undef SD_XWRITE
#undef SD_STAGE_W
#undef SD_FRAG_X
#undef SD_MMA
    }
    if constexpr (EPI != EPI_SWIGLU) {
        if (n_base >= N) return;         // wave-uniform; no barrier follows
    }

    // K split across workgroups.  Partials travel as device-scope accesses (past the caches that are private
    // to one XCD): wait until the stores have completed, then draw the ticket.
    if (gridDim.y > 1) {
        constexpr int kRec = MT * 1024;
        float* const rec0 = sk.part + (size_t)tile * gridDim.y * kRec;
        float* const mine = rec0 + (size_t)blockIdx.y * kRec;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (32 * t + 8 * (e >> 2) + (e & 3) + 4 * half < M)
                    __hip_atomic_store(&mine[(t * 16 + e) * 64 + lane], acc[t][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Hand-over without cache-wide operations: partials and ticket are device-scope accesses (they go past the caches
        // private to one XCD), the wait below completes every lane's partial stores before the ticket is drawn, and its
        // memory clobber keeps the compiler from moving accesses across it.  (An agent-scope release fence here is a
        // write-back of the whole L2, an acquire fence an invalidation: measured 1-2 us per kernel, and far more where
        // thousands of workgroups hand over, for data that never sat in those caches.)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        unsigned int old = 0;
        if (lane == 0) old = __hip_atomic_fetch_add(&sk.ticket[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        old = __builtin_amdgcn_readfirstlane(old);
        if (old != gridDim.y - 1u) return;
        if (lane == 0) __hip_atomic_store(&sk.ticket[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        asm volatile("" ::: "memory");     // compiler barrier: the loads below stay behind the ticket
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
        // The partials are fetched four splits at a time (one round trip to device-scope memory per group, not
        // per split) and added in split order.  Unconditional loads: a load under a per-lane condition would be
        // waited for on the spot; elements of rows >= M re-read element 0 of the lane instead, and whatever that
        // holds lands in accumulators of rows that are never stored.
        for (unsigned int s0 = 0; s0 < gridDim.y; s0 += 4) {
            floatx16 v[4][MT];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float* rec = rec0 + (size_t)min(s0 + j, gridDim.y - 1u) * kRec;
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const bool valid = 32 * t + 8 * (e >> 2) + (e & 3) + 4 * half < M;
                        v[j][t][e] = __hip_atomic_load(&rec[(valid ? (t * 16 + e) * 64 : 0) + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool have = s0 + j < gridDim.y;          // uniform
#pragma unroll
                for (int t = 0; t < MT; ++t)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[t][e] += have ? v[j][t][e] : 0.f;
            }
        }
    }

    if constexpr (EPI == EPI_ARGMAX) {
        // Through the wave's own staging tile (free after the loop; LDS operations of one wave execute in order): the
        // 32 x 32 tile is written [row][column] with padded rows, then lane -> (row lane & 31, column half lane >> 5)
        // scans 16 columns and one exchange between the halves finishes the row.
        const int n_tiles = (N + 31) / 32;
        float* const tl = reinterpret_cast<float*>(stage);            // 32 x 33 floats <= 4352 bytes
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int lr = 8 * (e >> 2) + (e & 3) + 4 * half;
                float v = acc[t][e];
                if constexpr (NF > 0) v = fmaf(ab[(32 * t + lr) * 2 + 0], v, ab[(32 * t + lr) * 2 + 1] * uv);
                v += bv;
                tl[lr * 33 + r] = ncol < (uint32_t)N ? v : -INFINITY;
            }
            float best = tl[r * 33 + 16 * half];
            int bc = 16 * half;
#pragma unroll
            for (int c = 1; c < 16; ++c) {
                const float x = tl[r * 33 + 16 * half + c];
                if (x > best) { best = x; bc = 16 * half + c; }      // ascending columns: the lowest column wins ties
            }
            const float ov = __shfl_xor(best, 32, 64);
            const int oc = __shfl_xor(bc, 32, 64);
            if (half == 0) {
                const bool take = ov > best;                           // the upper half only when strictly larger
                const int row = 32 * t + r;
                if (row < M) {
                    sk.am_v[(size_t)row * n_tiles + tile] = take ? ov : best;
                    sk.am_i[(size_t)row * n_tiles + tile] = n_base + (take ? oc : bc);
                }
            }
        }
        return;
    }

    if constexpr (EPI == EPI_SWIGLU) {
        // The up waves park their tiles (normalisation and bias applied) in LDS, the gate waves of the same column pair
        // pick them up.  The slabs are free once every wave has left the K loop.
        float* const xch = reinterpret_cast<float*>(slab) + sw_pair * (MT * 16 * 64);
        __syncthreads();
        floatx16 val[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int lr = 32 * t + 8 * (e >> 2) + (e & 3);
                float v = acc[t][e];
                if constexpr (NF > 0) v = fmaf(ab[(lr + 4 * half) * 2 + 0], v, ab[(lr + 4 * half) * 2 + 1] * uv);
                val[t][e] = v + bv;
            }
        if (sw_up) {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) xch[(t * 16 + e) * 64 + lane] = val[t][e];
        }
        __syncthreads();
        if (sw_up) return;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int lr = 32 * t + 8 * (e >> 2) + (e & 3);
                const float g = val[t][e], u = xch[(t * 16 + e) * 64 + lane];
                const float v = g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u;       // silu(g) * u; rounded to bf16 below
                __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v)), ry,
                                                      yoff + (uint32_t)lr * (uint32_t)ldy * 2u, 0, 0);
            }
        return;
    }

    // Epilogue (one 32-column tile per wave).  Rows >= M fall behind the end of the buffers, columns >= N carry the
    // out-of-range offset; the hardware drops both.
    const __amdgpu_buffer_rsrc_t rxg = __builtin_amdgcn_make_buffer_rsrc(fo.xg, 0, (EPI == EPI_RESID_NORM) ? (uint32_t)M * (uint32_t)N * 2u : 0u, kBufFlags);
    const uint32_t xgoff = ncol < (uint32_t)N ? ((uint32_t)(4 * half) * (uint32_t)N + ncol) * 2u : kOutOfRange;
    float* const rowsum = reinterpret_cast<float*>(stage);
    const int parts_out = (N + 31) / 32;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int lr = 32 * t + 8 * (e >> 2) + (e & 3);               // row, minus 4 * half
            const uint32_t so = (uint32_t)lr * (uint32_t)ldy * kOutBytes;
            float v = acc[t][e];
            if constexpr (NF > 0) v = fmaf(ab[(lr + 4 * half) * 2 + 0], v, ab[(lr + 4 * half) * 2 + 1] * uv);
            v += bv;
            if constexpr (EPI == EPI_GELU) v = gelu_fast(v);
            if constexpr (kResid) v += yres[t][e];
            if constexpr (kOutBytes == 2)
                __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v)), ry, yoff + so, 0, 0);
            else
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), ry, yoff + so, 0, 0);
            if constexpr (EPI == EPI_RESID_NORM) {
                __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, static_cast<bf16_t>(v * gv)), rxg,
                                                      xgoff + (uint32_t)lr * (uint32_t)N * 2u, 0, 0);
                rowsum[(8 * (e >> 2) + 4 * half + (e & 3)) * 33 + r] = v;           // columns >= N hold 0
            }
        }
        if constexpr (EPI == EPI_RESID_NORM) {
            // Row sums of this 32 x 32 tile, columns ascending (LDS operations of one wave execute in order).
            const int row = 32 * t + lane;
            if (lane < 32 && row < M) {
                float t1 = 0.f, t2 = 0.f;
#pragma unroll
                for (int c = 0; c < 32; ++c) {
                    const float x = rowsum[lane * 33 + c];
                    t1 += x;
                    t2 = fmaf(x, x, t2);
                }
                float* so_ = fo.stats + ((size_t)row * parts_out + tile) * 2;
                so_[0] = t1;
                so_[1] = t2;
            }
        }
    }
}

// ---- host side ---------------------------------------------------------------------------------

constexpr int kLdsBytes = 160 * 1024;
static int lds_bytes(int mt, int m) {
    const int rows_s = mt == 1 ? 32 : std::min(64, (m + 7) & ~7);
    return (4 * kStagePieces + kAbPieces + 2 * kStep * (rows_s + (mt == 2 ? 1 : 0)) * 8) * 16;
}

struct StreamPlan {
    int mt, split_chunks, gsplit;
};
// K split over workgroups: only when the column tiles alone leave CUs idle, keeping at least eight chunks
// (32 KB of weights per wave) per partial tile, within the workspace.
static bool plan_stream(int m, int n, int k, const SplitWorkspace& ws, int force_split, StreamPlan* out) {
    if (m > 64) return false;
    const int mt = m <= 32 ? 1 : 2;
    const int chunks = k / 64;
    const long tiles = (n + 31) / 32, groups = (tiles + 3) / 4;
    const long part_floats = ws.base ? (ws.bytes - kSplitTicketBytes) / 4 : 0;
    long gs = force_split > 0 ? std::min<long>(force_split, chunks)
                              : (groups >= 160 ? 1 : std::min<long>((256 + groups - 1) / groups, std::max(1, chunks / 8)));
    if (tiles * 4 > kSplitTicketBytes) gs = 1;
    gs = std::min(gs, part_floats / (tiles * mt * 1024));
    gs = std::max(gs, 1L);
    const int per = (int)((chunks + gs - 1) / gs);
    *out = StreamPlan{mt, per, (chunks + per - 1) / per};
    return true;
}

// Worth it when the column tiles alone keep the chip busy with long streams: 160 to 256 workgroups (one per CU,
// no second round) or several per CU.  In between, the uneven second round costs more than the kernel gains;
// with fewer column tiles K has to be split, and then the round trips of the split (partials, ticket, read-back:
// about 1.6 us each on this part) eat the gain -- the few-row kernel of gemm_mfma.hip serves both better
// (measured on 4096 x 14336, 6144 x 4096, 50257 x 1600).
// With a folded normalisation and up to 32 rows (the LM heads) it wins at any tile count: the row sums are gathered
// once per workgroup of four column tiles instead of once per tile (50257 x 768: 18.7 us against 21.5 us).
bool linear_stream_preferred(int m, int n, int k, bool folded) {
    if (m > 64 || (int64_t)n * k * 2 < ((int64_t)24 << 20)) return false;
    const long groups = ((n + 31) / 32 + 3) / 4;
    return (folded && m <= 32) || (groups >= 160 && groups <= 256) || groups >= 700;
}

static std::string g_stream_names[3][8][3];
static const char* stream_name(int mt, int epi, int nfk) {
    std::string& s = g_stream_names[mt][epi][nfk];
    if (s.empty()) s = "k_linear_stream<" + std::to_string(mt) + "," + std::to_string(epi) + "," + std::to_string(nfk) + ">";
    return s.c_str();
}

template <int MT, int EPI, int NF>
static hipError_t go(const dim3& grid, int bytes, hipStream_t st, const bf16_t* x, const bf16_t* w, const float* bias, void* y,
                     int m, int n, int k, int ldy, const FoldIn& fi, const FoldOut& fo, const StreamSplit& sk) {
    static bool raised = false;          // dynamic LDS beyond 64 KB has to be allowed once per kernel
    if (!raised) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_linear_stream<MT, EPI, NF>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    launch_kernel(k_linear_stream<MT, EPI, NF>, dim3(grid), dim3(256), bytes, st, x, w, bias, y, m, n, k, ldy, fi, fo, sk);
    return hipGetLastError();
}

template <int MT>
static hipError_t launch_mt(const dim3& grid, int bytes, hipStream_t st, const bf16_t* x, const bf16_t* w, const float* bias,
                            void* y, int m, int n, int k, int ldy, int epi, const NormIn& ni, const NormOut& no,
                            const StreamSplit& sk) {
    const FoldIn fi{ni.stats, ni.u, ni.parts, ni.eps};
    const FoldOut fo{no.gain, static_cast<bf16_t*>(no.xg), no.stats};
#define SD_GO(EPI, NF) return go<MT, EPI, NF>(grid, bytes, st, x, w, bias, y, m, n, k, ldy, fi, fo, sk)
    if (ni.kind == 0) {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 0);
            case EPI_GELU: SD_GO(EPI_GELU, 0);
            case EPI_RESID: if (no.gain) SD_GO(EPI_RESID_NORM, 0); else SD_GO(EPI_RESID, 0);
            case EPI_SWIGLU: SD_GO(EPI_SWIGLU, 0);
            case EPI_ARGMAX: SD_GO(EPI_ARGMAX, 0);
            default: SD_GO(EPI_F32, 0);
        }
    } else if (ni.kind == 1) {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 1);
            case EPI_GELU: SD_GO(EPI_GELU, 1);
            case EPI_F32: SD_GO(EPI_F32, 1);
            case EPI_ARGMAX: SD_GO(EPI_ARGMAX, 1);
            default: return hipErrorInvalidValue;
        }
    } else {
        switch (epi) {
            case EPI_STORE: SD_GO(EPI_STORE, 2);
            case EPI_GELU: SD_GO(EPI_GELU, 2);
            case EPI_F32: SD_GO(EPI_F32, 2);
            case EPI_SWIGLU: SD_GO(EPI_SWIGLU, 2);
            case EPI_ARGMAX: SD_GO(EPI_ARGMAX, 2);
            default: return hipErrorInvalidValue;
        }
    }
#undef SD_GO
}

// x bf16 [m, k] with m <= 64, w bf16 [n, k]; shape limits of linear_mfma_supported; ni / no as in launch_linear_mfma.
// Returns hipErrorNotSupported for more than 64 rows: the caller falls back.
hipError_t launch_linear_stream(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                                int epi, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws, int force_split,
                                hipStream_t st, const char** kernel_name) {
    if (epi < 0 || (epi > 3 && epi != EPI_SWIGLU && epi != EPI_ARGMAX)) return hipErrorInvalidValue;
    StreamPlan p;
    if (!plan_stream(m, n, k, ws, (epi == EPI_SWIGLU || epi == EPI_ARGMAX) ? 1 : force_split, &p)) return hipErrorNotSupported;
    if (epi == EPI_ARGMAX && (p.gsplit != 1 || !no.am_v || !no.am_i || no.gain)) return hipErrorNotSupported;
    // gate / up pairs of 64 columns per workgroup, no K split, LayerNorm folds not instantiated
    if (epi == EPI_SWIGLU && (n % 128 != 0 || p.gsplit != 1 || ni.kind == 1 || no.gain)) return hipErrorNotSupported;
    StreamSplit sk{nullptr, nullptr, p.split_chunks, no.am_v, no.am_i};
    if (p.gsplit > 1) {
        sk.ticket = static_cast<unsigned int*>(ws.base);
        sk.part = reinterpret_cast<float*>(static_cast<char*>(ws.base) + kSplitTicketBytes);
    }
    const dim3 grid(epi == EPI_SWIGLU ? (unsigned)(n / 128) : (unsigned)(((n + 31) / 32 + 3) / 4), (unsigned)p.gsplit);
    const int bytes = lds_bytes(p.mt, m);
    if (kernel_name) *kernel_name = stream_name(p.mt, no.gain ? (int)EPI_RESID_NORM : epi, ni.kind);
    return p.mt == 1 ? launch_mt<1>(grid, bytes, st, (const bf16_t*)x, (const bf16_t*)w, bias, y, m, n, k, ldy, epi, ni, no, sk)
                     : launch_mt<2>(grid, bytes, st, (const bf16_t*)x, (const bf16_t*)w, bias, y, m, n, k, ldy, epi, ni, no, sk);
}

}  // namespace sd
