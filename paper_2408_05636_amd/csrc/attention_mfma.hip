// bf16 attention on the gfx950 matrix cores for both networks of the round: non-causal over
// prefix o block for the diffusion drafter, causal over the KV cache plus the new rows for the
// target.  Visibility is expressed per query row as a key count kv_len[r] (keys 0..kv_len-1 of the
// row's sequence), which covers both cases and ragged batches.
//
// One wave owns a tile of 32 query rows of one head and walks over blocks of 32 keys with an
// online softmax.  Everything is kept transposed so that no cross-lane traffic is needed:
//   S^T = K Q^T        A = K rows (d contiguous, from global), B = Q rows (registers, loaded once)
//                      -> lane = query, its 16 accumulators = 16 keys: row max / sum are in-lane,
//                         plus one exchange between the two lane halves;
//   O^T += V^T P^T     B = P^T comes straight from the S^T accumulators (cast to bf16);
//                      A = V^T needs keys contiguous per d: the 32 x d_head V block is transposed
//                      through a wave-private LDS tile (no workgroup barrier in the loop).
// The K rows are fed to the first MFMA in a permuted order chosen so that accumulator e of lane
// half h is key 16h + e of the block: then the P^T operand of MFMA step s is registers 8s..8s+7 and
// the matching V^T operand is 16 contiguous bytes of the LDS tile.
// A workgroup is 4 waves: either 4 query tiles (large batches) or 4 interleaved key ranges of one
// tile merged through LDS (few query rows: the target's gamma+1 rows, batch-1 drafter).
#include "common.h"

namespace sd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kVtLd = 40;    // LDS row stride of the transposed V tile (32 keys + 8 pad), in elements

typedef __attribute__((__vector_size__(4 * sizeof(unsigned int)))) unsigned int u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(unsigned int)))) unsigned int u32x2;
constexpr int kBufFlags = 0x00020000;          // raw buffer, 32-bit data format
constexpr uint32_t kOutOfRange = 0x80000000u;  // VGPR offset of accesses that must not happen (buffers are < 2 GiB)

template <int DH, bool KSPLIT>
__global__ __launch_bounds__(256) void k_attention_mfma(AttnArgs a) {
    constexpr int NCH = DH / 64;     // 64-wide chunks of a q / k row
    constexpr int DT = DH / 32;      // 32-row tiles of O^T
    constexpr int NV = DH / 16;      // 16-byte pieces of a V row handled per lane
    __shared__ __attribute__((aligned(16))) bf16_t vt_all[4][DH * kVtLd];
    __shared__ float mrg_m[KSPLIT ? 3 : 1][64], mrg_l[KSPLIT ? 3 : 1][64];
    __shared__ float mrg_o[KSPLIT ? 3 : 1][KSPLIT ? DT * 16 : 1][64];

    // wave-uniform values are kept in scalar registers (tile description, buffer descriptors, block counters)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    const int tile = KSPLIT ? (int)blockIdx.x : (int)blockIdx.x * 4 + wave;
    const int head = blockIdx.y;
    if (!KSPLIT && tile >= a.n_tiles) return;           // whole wave; this variant has no barriers

    // One scalar load brings everything that is uniform over the tile; the per-row key counts, the query
    // rows and the first key / value block are then requested together (two dependent round trips in all).
    const AttnTile tl = a.tiles[tile];
    const int row0 = tl.row0, nrows = tl.nrows, kv_max = tl.kv_max;
    const int qrow = row0 + min(r, nrows - 1);
    const int g = head / (a.n_head / a.n_kv_head);
    const uint32_t kv_bytes = ((uint32_t)(kv_max - 1) * (uint32_t)a.kv_ld + DH) * 2u;    // keys 0..kv_max-1 of this kv head
    bf16_t* kbase = const_cast<bf16_t*>(static_cast<const bf16_t*>(a.k)) + tl.kv_off + (size_t)g * DH;
    bf16_t* vbase = const_cast<bf16_t*>(static_cast<const bf16_t*>(a.v)) + tl.kv_off + (size_t)g * DH;
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(kbase, 0, kv_bytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(vbase, 0, kv_bytes, kBufFlags);
    const int kvl = a.kv_len[qrow];
    const bf16_t* Qp = static_cast<const bf16_t*>(a.q) + (size_t)qrow * a.q_ld + (size_t)head * DH + 32 * half;
    bf16_t* vt = vt_all[wave];

    bf16x8 qf[NCH][4];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int s = 0; s < 4; ++s) qf[c][s] = __builtin_bit_cast(bf16x8, reinterpret_cast<const u32x4*>(Qp + c * 64)[s]);

    // MFMA row rho of the S^T tile carries key pi(rho) of the block: rho = 8g' + 4h' + i -> 16h' + 4g' + i
    const int pi_r = 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
    // Byte offsets inside the key / value buffers of this lane's row of block 0.  Rows beyond kv_max fall
    // outside the buffer and read as 0 (they are masked below), so the last block needs no special case and
    // the block after the last can be prefetched unconditionally.
    const uint32_t k_lane = ((uint32_t)pi_r * (uint32_t)a.kv_ld + 32u * half) * 2u;
    const uint32_t v_lane = ((uint32_t)r * (uint32_t)a.kv_ld + 8u * half) * 2u;
    const uint32_t blk_bytes = 32u * (uint32_t)a.kv_ld * 2u;

    float m_run = -INFINITY, l_run = 0.f;
    floatx16 o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    const float scale = rsqrtf((float)DH) * 1.4426950408889634f;     // scores in log2 units

    const int n_blocks = (kv_max + 31) / 32;
    constexpr int kStep = KSPLIT ? 4 : 1;
    u32x4 kc[NCH][4], vc[NV], kn[NCH][4], vn[NV];
#define SD_LOAD_BLOCK(KR, VR, KB)                                                                        \
    {                                                                                                    \
        const uint32_t ko_ = k_lane + (uint32_t)(KB) * blk_bytes, vo_ = v_lane + (uint32_t)(KB) * blk_bytes; \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) _Pragma("unroll") for (int q4 = 0; q4 < 4; ++q4) \
            KR[c][q4] = __builtin_amdgcn_raw_buffer_load_b128(rk, ko_ + (uint32_t)(c * 128 + q4 * 16), 0, 0); \
        _Pragma("unroll") for (int i = 0; i < NV; ++i)                                                   \
            VR[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, vo_ + (uint32_t)(i * 32), 0, 0);            \
    }
    int kb = KSPLIT ? wave : 0;
    SD_LOAD_BLOCK(kc, vc, kb)
    for (; kb < n_blocks; kb += kStep) {
        SD_LOAD_BLOCK(kn, vn, kb + kStep)                               // prefetch; beyond the end it reads nothing
        // ---- S^T = K Q^T
        floatx16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kc[c][q4]), qf[c][q4], s, 0, 0, 0);
        // ---- stage V^T of this key block in the wave's LDS tile (piece i of this lane: key r, d = 8 (half + 2i) ..)
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const bf16x8 tv = __builtin_bit_cast(bf16x8, vc[i]);
#pragma unroll
            for (int u = 0; u < 8; ++u) vt[(8 * (half + 2 * i) + u) * kVtLd + r] = tv[u];
        }
        // ---- online softmax; accumulator e of this lane is key kb*32 + 16*half + e
        float mb = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            s[e] = (kb * 32 + 16 * half + e < kvl) ? s[e] * scale : -INFINITY;
            mb = fmaxf(mb, s[e]);
        }
        mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
        const float m_new = fmaxf(m_run, mb);
        const bool dead = m_new == -INFINITY;                         // no visible key so far
        const float alpha = dead ? 1.f : exp2f(m_run - m_new);
        float psum = 0.f;
        bf16x8 pf[2];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float p = dead ? 0.f : exp2f(s[e] - m_new);
            psum += p;
            pf[e >> 3][e & 7] = static_cast<bf16_t>(p);
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
        // ---- O^T += V^T P^T
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vt + (t * 32 + r) * kVtLd + 16 * half + 8 * s2);
                o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s2], o[t], 0, 0, 0);
            }
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) kc[c][q4] = kn[c][q4];
#pragma unroll
        for (int i = 0; i < NV; ++i) vc[i] = vn[i];
    }
#undef SD_LOAD_BLOCK

    if constexpr (KSPLIT) {            // merge the four key ranges in a fixed order
        if (wave > 0) {
            mrg_m[wave - 1][lane] = m_run;
            mrg_l[wave - 1][lane] = l_run;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) mrg_o[wave - 1][t * 16 + e][lane] = o[t][e];
        }
        __syncthreads();
        if (wave > 0) return;
        float m_all = m_run;
#pragma unroll
        for (int w = 0; w < 3; ++w) m_all = fmaxf(m_all, mrg_m[w][lane]);
        const float f0 = m_run == -INFINITY ? 0.f : exp2f(m_run - m_all);
        l_run *= f0;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[t][e] *= f0;
#pragma unroll
        for (int w = 0; w < 3; ++w) {
            const float mw = mrg_m[w][lane];
            const float fw = mw == -INFINITY ? 0.f : exp2f(mw - m_all);
            l_run += mrg_l[w][lane] * fw;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[t][e] += mrg_o[w][t * 16 + e][lane] * fw;
        }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.f / l_tot;
    // Output row qrow, columns head*DH + d: accumulators 4*e4 .. 4*e4+3 are 4 consecutive d.  Lanes of rows
    // beyond the tile carry the out-of-range offset and their stores are dropped.
    const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (uint32_t)a.rows * (uint32_t)a.out_ld * 2u, kBufFlags);
    const uint32_t o_lane = r < nrows ? ((uint32_t)qrow * (uint32_t)a.out_ld + (uint32_t)head * DH + 4u * half) * 2u : kOutOfRange;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            union { bf16_t h[4]; u32x2 u; } pk;
#pragma unroll
            for (int i = 0; i < 4; ++i) pk.h[i] = static_cast<bf16_t>(o[t][4 * e4 + i] * inv);
            __builtin_amdgcn_raw_buffer_store_b64(pk.u, ro, o_lane + (uint32_t)(t * 32 + 8 * e4) * 2u, 0, 0);
        }
}

bool attention_mfma_supported(int dtype, const AttnArgs& a) {
    return dtype == SD_DTYPE_BF16 && (a.d_head == 64 || a.d_head == 128) && a.tiles != nullptr && a.n_tiles > 0 &&
           a.q_ld % 8 == 0 && a.kv_ld % 8 == 0 && a.out_ld % 4 == 0 && (int64_t)a.max_kv * a.kv_ld * 2 < ((int64_t)1 << 31) &&
           (int64_t)a.rows * a.out_ld * 2 < ((int64_t)1 << 31);
}

hipError_t launch_attention_mfma(const AttnArgs& a, hipStream_t st, const char** kernel_name) {
    const bool ksplit = (long)a.n_tiles * a.n_head < 1024 && a.max_kv > 64;
    const dim3 grid(ksplit ? a.n_tiles : (a.n_tiles + 3) / 4, a.n_head);
    if (a.d_head == 64) {
        if (ksplit) { if (kernel_name) *kernel_name = "k_attention_mfma<64,true>"; k_attention_mfma<64, true><<<grid, 256, 0, st>>>(a); }
        else { if (kernel_name) *kernel_name = "k_attention_mfma<64,false>"; k_attention_mfma<64, false><<<grid, 256, 0, st>>>(a); }
    } else {
        if (ksplit) { if (kernel_name) *kernel_name = "k_attention_mfma<128,true>"; k_attention_mfma<128, true><<<grid, 256, 0, st>>>(a); }
        else { if (kernel_name) *kernel_name = "k_attention_mfma<128,false>"; k_attention_mfma<128, false><<<grid, 256, 0, st>>>(a); }
    }
    return hipGetLastError();
}

}  // namespace sd
