// bf16 contraction y = epilogue(x W^T + bias) for many rows (batched passes): a workgroup of four waves
// owns a (64 WM) x 128 output tile and shares both operand tiles through LDS, so every byte fetched from
// L2 / HBM feeds 64 rows of matrix-core work per wave instead of 32 (the few-row kernel keeps its tiles
// private to a wave and pays for that with twice the loads per flop).  WM = 2: 128 x 128 tile, waves 2 x 2,
// 64 x 64 outputs each; WM = 1: 64 x 128 tile, waves 1 x 4, 64 x 32 outputs each (a few hundred rows).
//
// K is walked in chunks of 64.  All 256 threads fetch the two operand tiles of a chunk with
// 16-byte buffer loads (8 consecutive lanes per 128-byte line), hold them in registers for two chunks
// and then store them into one of two LDS stages, XOR-swizzled (see swizzle_key) so that neither the
// stores nor the operand reads conflict.  Wave (wm, wn) computes the
// 64 x 64 quadrant: per 16-wide k step two A and two B fragments, four v_mfma_f32_32x32x16_bf16.  One
// barrier per chunk; the global loads in the loop body are unconditional (past the end of K they
// repeat the last chunk), so the compiler's wait counts stay exact.
//
// A normalisation folded around the contraction works as in the few-row kernel: x = bf16(h gain) and the
// partial row sums come from the producer of h (NF), and the residual epilogue can prepare both for the
// normalisation that follows (EPI_RESID_NORM).
#include <string>

#include "mfma_common.hip.h"

namespace sd {

template <int EPI, int WM, int NF>
__global__ __launch_bounds__(256) void k_linear_tile(const void* __restrict__ Xv, const bf16_t* __restrict__ W,
                                                     const float* __restrict__ bias, void* Y, int M, int N, int K,
                                                     int ldy, int tiles_m, int tiles_n, int x_stationary,
                                                     FoldIn nf, FoldOut fo) {
    constexpr int BM = 64 * WM;            // rows of the workgroup tile
    constexpr int XI = BM / 32;            // x row groups per loader thread
    constexpr int NT = WM == 2 ? 2 : 1;    // 32-column tiles per wave
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    const int wm = wave % WM, wn = wave / WM;
    // XCD-aware tile order (workgroups go to the 8 XCDs round-robin): the larger operand is fetched by one XCD only.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    int tn, tm;
    if (x_stationary) {
        // x_stationary = number of column groups cg (1, 2 or 4): the XCDs form a cg x (8 / cg) grid, XCD (c, r) takes
        // the column tiles of group c and the row tiles r, r + 8 / cg, ...  With cg > 1 an XCD keeps 1 / cg of W in its
        // L2 while a (8 / cg)-th of x streams through once.
        const int cgn = x_stationary, rgn = 8 / cgn;
        const int cg = xcd % cgn, rg = xcd / cgn;
        const int per = (tiles_n + cgn - 1) / cgn;
        tn = cg * per + local % per;
        tm = rg + rgn * (local / per);
        if (tn >= (cg + 1) * per) return;
    } else {
        tn = xcd + 8 * (local / tiles_m);
        tm = local % tiles_m;
    }
    if (tn >= tiles_n || tm >= tiles_m) return;
    const int m_base = tm * BM, n_base = tn * 128;

    __shared__ u32x4 lds_x[2][BM * 8];                // [stage][rows x 8 pieces]
    __shared__ u32x4 lds_w[2][1024];

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(Xv), 0, (uint32_t)M * (uint32_t)K * 2u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W), 0, (uint32_t)N * (uint32_t)K * 2u, kBufFlags);

    // Loader geometry: thread t handles piece pc = t & 7 of rows 32 i + (t >> 3) of both tiles.
    const int lrow = threadIdx.x >> 3, pc = threadIdx.x & 7;
    uint32_t xoff[XI], woff[4];
    int slot[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t wr = (uint32_t)(n_base + 32 * i + lrow);
        woff[i] = wr < (uint32_t)N ? (wr * (uint32_t)K + 8u * pc) * 2u : kOutOfRange;
        const int row = 32 * i + lrow;
        slot[i] = row * 8 + (pc ^ swizzle_key(row));
        if (i < XI) {
            const uint32_t xr = (uint32_t)(m_base + 32 * i + lrow);
            xoff[i] = xr < (uint32_t)M ? (xr * (uint32_t)K + 8u * pc) * 2u : kOutOfRange;
        }
    }
    // rows of the operand fragments this lane reads, and their swizzle keys
    int ra[2], rbw[NT], ka[2], kb[NT];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        ra[i] = wm * 64 + 32 * i + r;
        ka[i] = swizzle_key(ra[i]);
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        rbw[j] = wn * 32 * NT + 32 * j + r;
        kb[j] = swizzle_key(rbw[j]);
    }
    bf16x8 fa[2][2], fb[2][NT];

    floatx16 acc[2][NT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // two register sets: the global loads run two chunks ahead of the LDS stores
    u32x4 gx[2][XI], gw[2][4];
    const int n_chunks = K / 64;

#define SD_TILE_GLOAD(S, CHUNK)                                                                     \
    {                                                                                               \
        const uint32_t koff_ = (uint32_t)(CHUNK) * 128u;                                            \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                             \
            if (i < XI) gx[S][i < XI ? i : 0] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff[i < XI ? i : 0], koff_, 0); \
            gw[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, woff[i], koff_, 0);                \
        }                                                                                           \
    }
#define SD_TILE_SWRITE(S, STAGE)                                                                    \
    {                                                                                               \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                             \
            if (i < XI) lds_x[STAGE][slot[i]] = gx[S][i < XI ? i : 0];                              \
            lds_w[STAGE][slot[i]] = gw[S][i];                                                       \
        }                                                                                           \
    }
// Operand fragments are double-buffered by hand: the LDS reads of k step s4 + 1 are in flight while the
// matrix cores work on step s4.
#define SD_TILE_FRAGS(STAGE, FB, S4)                                                                \
    {                                                                                               \
        _Pragma("unroll") for (int i = 0; i < 2; ++i)                                               \
            fa[FB][i] = __builtin_bit_cast(bf16x8, lds_x[STAGE][ra[i] * 8 + ((2 * (S4) + half) ^ ka[i])]); \
        _Pragma("unroll") for (int j = 0; j < NT; ++j)                                              \
            fb[FB][j] = __builtin_bit_cast(bf16x8, lds_w[STAGE][rbw[j] * 8 + ((2 * (S4) + half) ^ kb[j])]); \
    }
#define SD_TILE_COMPUTE(STAGE)                                                                      \
    {                                                                                               \
        SD_TILE_FRAGS(STAGE, 0, 0)                                                                  \
        _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {                                          \
            if (s4 < 3) SD_TILE_FRAGS(STAGE, (s4 + 1) & 1, s4 + 1)                                  \
            __builtin_amdgcn_sched_barrier(0);     /* keep the reads of the next step ahead of these MFMAs */ \
            _Pragma("unroll") for (int i = 0; i < 2; ++i) _Pragma("unroll") for (int j = 0; j < NT; ++j) \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s4 & 1][i], fb[s4 & 1][j], acc[i][j], 0, 0, 0); \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }                                                                                           \
    }

    // Step c: store chunk c + 1 (register set (c + 1) & 1) into LDS stage (c + 1) & 1 -- last read before the
    // barrier that ended step c - 1 --, refill that register set with chunk c + 3, multiply chunk c.  The
    // steady state is a branch-free pair of steps (with branches inside, the compiler's wait counts fall
    // back to "everything outstanding" and the two-chunk prefetch distance is lost); the scheduling fences
    // keep the global loads in front of the multiply phase instead of behind it.  Past the end of K the
    // loads repeat the last chunk (unconditional, nobody reads them).
#define SD_TILE_STEP(NEXT, CUR, C)                      \
    {                                                   \
        SD_TILE_SWRITE(NEXT, NEXT)                      \
        SD_TILE_GLOAD(NEXT, min((C) + 3, last))         \
        __builtin_amdgcn_sched_barrier(0);              \
        SD_TILE_COMPUTE(CUR)                            \
        lds_barrier();                                  \
    }
    const int last = n_chunks - 1;
    // Per-column operands of the epilogue, requested ahead of the operand tiles: their round trip is over long
    // before the loop ends.
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(bias), 0, bias ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(nf.u), 0, (NF == 1) ? (uint32_t)N * 4u : 0u, kBufFlags);
    const __amdgpu_buffer_rsrc_t rgn = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(fo.gain), 0, (EPI == EPI_RESID_NORM) ? (uint32_t)N * 4u : 0u, kBufFlags);
    float bvs[NT], uvs[NT], gvns[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const uint32_t n = (uint32_t)(n_base + wn * 32 * NT + 32 * j + r);
        bvs[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, n * 4u, 0, 0));
        uvs[j] = NF == 1 ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ru, n * 4u, 0, 0)) : 0.f;
        gvns[j] = EPI == EPI_RESID_NORM ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rgn, n * 4u, 0, 0)) : 0.f;
    }
    SD_TILE_GLOAD(0, 0)
    SD_TILE_GLOAD(1, min(1, last))
    __builtin_amdgcn_sched_barrier(0);
    // Row sums of a folded normalisation: thread t adds the partial pairs p = (t & 3), (t & 3) + 4, ... of row
    // t >> 2 (BM = 64) -- or of rows t >> 2 and 64 + (t >> 2) (BM = 128) --, eight loads in flight; the four
    // threads of a row are combined by two lane exchanges.  Requested behind the first two operand chunks, so that
    // its round trips overlap theirs; consumed in the epilogue.
    float fs1[NF > 0 ? WM : 1] = {}, fs2[NF > 0 ? WM : 1] = {};
    if constexpr (NF > 0) {
        typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
#pragma unroll
        for (int t = 0; t < WM; ++t) {
            const int row = m_base + 64 * t + (threadIdx.x >> 2);
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
            fs1[t] = (b1[0] + b1[1]) + (b1[2] + b1[3]);
            fs2[t] = (b2[0] + b2[1]) + (b2[2] + b2[3]);
            fs1[t] += __shfl_xor(fs1[t], 1, 64); fs2[t] += __shfl_xor(fs2[t], 1, 64);
            fs1[t] += __shfl_xor(fs1[t], 2, 64); fs2[t] += __shfl_xor(fs2[t], 2, 64);
        }
    }

    SD_TILE_SWRITE(0, 0)
    SD_TILE_GLOAD(0, min(2, last))
    __syncthreads();
    int c = 0;
    for (; c + 2 <= last; c += 2) {
        SD_TILE_STEP(1, 0, c)
        SD_TILE_STEP(0, 1, c + 1)
    }
    if (c < last) {
        SD_TILE_STEP(1, 0, c)
        SD_TILE_COMPUTE(1)
    } else {
        SD_TILE_COMPUTE(0)
    }
#undef SD_TILE_STEP
#undef SD_TILE_GLOAD
#undef SD_TILE_SWRITE
#undef SD_TILE_FRAGS
#undef SD_TILE_COMPUTE

    // Epilogue (shared with the kernel that feeds its tiles straight into LDS); its LDS scratch is the W staging area,
    // free once every wave has left the loop.
    shared_tile_epilogue<EPI, NF, 2, NT, BM>(acc, reinterpret_cast<float*>(&lds_w[0][0]), fs1, fs2, bvs, uvs, gvns, wave, wm, wn,
                                             m_base, n_base, Y, M, N, K, ldy, nf, fo);
}

static std::string g_tile_names[5][3][3];
static const char* tile_name(int epi, int wm, int nfk) {
    std::string& s = g_tile_names[epi][wm][nfk];
    if (s.empty()) s = "k_linear_tile<" + std::to_string(epi) + "," + std::to_string(wm) + "," + std::to_string(nfk) + ">";
    return s.c_str();
}

// Tile height for a shape (0: leave it to the few-row kernel).  Worth it from a few hundred rows on, when
// the tiles can still occupy a good part of the chip and there is enough arithmetic per output element
// (short, narrow contractions are bound by their fp32 output).
int linear_tile_rows(int m, int n, int k) {
    if (m < 192) return 0;
    const bool small = n < 2048 && k < 2048;         // short, narrow contractions are bound by their fp32 output
    const long tn = (n + 127) / 128;
    const long tiles128 = (long)((m + 127) / 128) * tn, tiles64 = (long)((m + 63) / 64) * tn;
    if (m >= 512 && tiles128 >= 200) {
        // When either height runs as a single round of resident workgroups (two per CU at 128 rows, three at 64),
        // the lower tiles spread over more CUs: 7424 x 768 x 3072 takes 60 us at 64 rows against 69 us at 128
        // (and 7424 x 768 x 768 27 us against 30 us for the wave-private tiles).
        if (tiles128 <= 512 && tiles64 <= 768) return 64;
        return small ? 0 : 128;
    }
    if (small) return 0;
    if (tiles64 >= 160) return 64;
    return 0;
}
bool linear_tile_preferred(int m, int n, int k) { return linear_tile_rows(m, n, k) != 0; }

// Column groups of the XCD grid when x is the larger operand (see the kernel): with two, an XCD keeps half of W in
// its L2 and a quarter of x streams through once (7424-row drafter passes: 1 % faster than one group; four: slower).
constexpr int kTileColumnGroups = 2;
template <int WM>
static hipError_t launch_tile(const void* x, const bf16_t* wb, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epi, const NormIn& ni, const NormOut& no, hipStream_t st) {
    const int tiles_m = (m + 64 * WM - 1) / (64 * WM), tiles_n = (n + 127) / 128;
    const int xs = (int64_t)m > (int64_t)n ? kTileColumnGroups : 0;
    const int grid = xs ? 8 * ((tiles_m + 8 / xs - 1) / (8 / xs)) * ((tiles_n + xs - 1) / xs) : 8 * ((tiles_n + 7) / 8) * tiles_m;
    const FoldIn fi{ni.stats, ni.u, ni.parts, ni.eps};
    const FoldOut fo{no.gain, static_cast<bf16_t*>(no.xg), no.stats};
#define SD_GO(EPI, NF) launch_kernel(k_linear_tile<EPI, WM, NF>, dim3(grid), dim3(256), 0, st, x, wb, bias, y, m, n, k, ldy, tiles_m, tiles_n, xs, fi, fo)
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

// x bf16 [m, k], w bf16 [n, k]; same shape limits as the few-row kernel (linear_mfma_supported); ni / no as there.
// rows: tile height, 64 or 128 (0: by shape, 128 if the shape has no preference).
hipError_t launch_linear_tile(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epi, const NormIn& ni, const NormOut& no, int rows, hipStream_t st,
                              const char** kernel_name) {
    if (epi < 0 || epi > 3) return hipErrorInvalidValue;
    if (rows == 0) rows = linear_tile_rows(m, n, k) == 64 ? 64 : 128;
    if (kernel_name) *kernel_name = tile_name(no.gain ? (int)EPI_RESID_NORM : epi, rows / 64, ni.kind);
    return rows == 64 ? launch_tile<1>(x, (const bf16_t*)w, bias, y, m, n, k, ldy, epi, ni, no, st)
                      : launch_tile<2>(x, (const bf16_t*)w, bias, y, m, n, k, ldy, epi, ni, no, st);
}

}  // namespace sd
