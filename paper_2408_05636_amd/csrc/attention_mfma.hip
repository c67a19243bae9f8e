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

template <int DH, bool KSPLIT>
__global__ __launch_bounds__(256) void k_attention_mfma(AttnArgs a) {
    constexpr int NCH = DH / 64;     // 64-wide chunks of a q / k row
    constexpr int DT = DH / 32;      // 32-row tiles of O^T
    __shared__ __attribute__((aligned(16))) bf16_t vt_all[4][DH * kVtLd];
    __shared__ float mrg_m[KSPLIT ? 3 : 1][64], mrg_l[KSPLIT ? 3 : 1][64];
    __shared__ float mrg_o[KSPLIT ? 3 : 1][KSPLIT ? DT * 16 : 1][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, half = lane >> 5;
    const int tile = KSPLIT ? (int)blockIdx.x : (int)blockIdx.x * 4 + wave;
    const int head = blockIdx.y;
    if (!KSPLIT && tile >= a.n_tiles) return;           // whole wave; this variant has no barriers

    const int row0 = a.tile_row0[tile], nrows = a.tile_rows[tile];
    const int qrow = row0 + min(r, nrows - 1);
    const int kvl = a.kv_len[qrow];
    int kv_max = kvl;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) kv_max = max(kv_max, __shfl_xor(kv_max, o, 64));
    const int g = head / (a.n_head / a.n_kv_head);
    const bf16_t* Kp = static_cast<const bf16_t*>(a.k) + a.kv_off[row0] + (size_t)g * DH;
    const bf16_t* Vp = static_cast<const bf16_t*>(a.v) + a.kv_off[row0] + (size_t)g * DH;
    const bf16_t* Qp = static_cast<const bf16_t*>(a.q) + (size_t)qrow * a.q_ld + (size_t)head * DH + 32 * half;
    bf16_t* vt = vt_all[wave];

    bf16x8 qf[NCH][4];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4 t = reinterpret_cast<const uint4*>(Qp + c * 64)[s];
            qf[c][s] = *reinterpret_cast<const bf16x8*>(&t);
        }

    // MFMA row rho of the S^T tile carries key pi(rho) of the block: rho = 8g' + 4h' + i -> 16h' + 4g' + i
    const int pi_r = 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);

    float m_run = -INFINITY, l_run = 0.f;
    floatx16 o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    const float scale = rsqrtf((float)DH) * 1.4426950408889634f;     // scores in log2 units

    const int n_blocks = (kv_max + 31) / 32;
    for (int kb = KSPLIT ? wave : 0; kb < n_blocks; kb += KSPLIT ? 4 : 1) {
        // ---- S^T = K Q^T
        const int krow = min(kb * 32 + pi_r, kv_max - 1);             // clamped: masked below
        const bf16_t* kr = Kp + (size_t)krow * a.kv_ld + 32 * half;
        floatx16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const uint4 t = reinterpret_cast<const uint4*>(kr + c * 64)[q4];
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&t), qf[c][q4], s, 0, 0, 0);
            }
        // ---- stage V^T of this key block in the wave's LDS tile
        const int vrow = min(kb * 32 + r, kv_max - 1);
        const bf16_t* vr = Vp + (size_t)vrow * a.kv_ld;
#pragma unroll
        for (int i = 0; i < DH / 16; ++i) {
            const int dg = half + 2 * i;
            const uint4 t = *reinterpret_cast<const uint4*>(vr + 8 * dg);
            const bf16_t* tv = reinterpret_cast<const bf16_t*>(&t);
#pragma unroll
            for (int u = 0; u < 8; ++u) vt[(8 * dg + u) * kVtLd + r] = tv[u];
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
    }

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
    if (r >= nrows) return;
    const float inv = 1.f / l_tot;
    bf16_t* op = static_cast<bf16_t*>(a.out) + (size_t)qrow * a.out_ld + (size_t)head * DH;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {       // accumulators 4*e4 .. 4*e4+3 are 4 consecutive d
            const int d0 = t * 32 + 8 * e4 + 4 * half;
            union { bf16_t h[4]; uint2 u; } pk;
#pragma unroll
            for (int i = 0; i < 4; ++i) pk.h[i] = static_cast<bf16_t>(o[t][4 * e4 + i] * inv);
            *reinterpret_cast<uint2*>(op + d0) = pk.u;
        }
}

bool attention_mfma_supported(int dtype, const AttnArgs& a) {
    return dtype == SD_DTYPE_BF16 && (a.d_head == 64 || a.d_head == 128) && a.tile_row0 != nullptr && a.n_tiles > 0 &&
           a.q_ld % 8 == 0 && a.kv_ld % 8 == 0 && a.out_ld % 4 == 0;
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
