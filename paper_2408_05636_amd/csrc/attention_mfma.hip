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
//                      A = V^T needs keys contiguous per d, while the block sits in LDS as loaded (rows = keys).
//                      The transposing LDS read of gfx950 (ds_read_b64_tr_b16) delivers exactly that: within
//                      each group of 16 lanes, lane 4a + c receives element c of the 8-byte pieces addressed by
//                      lanes a, a + 4, a + 8, a + 12.  Lanes a + 4j point at key j of a run of four keys and at
//                      the four d values 4a .. 4a + 3, so lane 4a + c ends up with four consecutive keys of
//                      d = 4a + c; two such reads make the 8-key operand.  No extra MFMA, no conversion and no
//                      cross-lane traffic in the loop.
// The K rows are fed to the score MFMAs in a permuted order chosen so that accumulator e of lane half h is
// key 16h + e of the block: then the P^T operand of MFMA step s is registers 8s..8s+7 of the scores, and the
// matching V^T operand is keys 16h + 8s .. 16h + 8s + 7.
// A workgroup is 4 waves: either 4 query tiles (large batches) or 4 interleaved key ranges of one
// tile merged through LDS (few query rows: the target's gamma+1 rows, batch-1 drafter).
#include "mfma_common.hip.h"

namespace sd {

typedef __attribute__((__vector_size__(2 * sizeof(unsigned int)))) unsigned int u32x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
// Offsets (in 2-byte units from the start of a V tile in LDS: [64-wide d chunk][32 keys][8 pieces of 16 bytes],
// piece p of key row x at p ^ swz(x)) of the two transposing reads that give this lane the V^T operand of d tile t,
// MFMA step s2: keys 16 half + 8 s2 + 0..3 and + 4..7 of d = 32 t + (lane & 31).
__device__ inline void vt_offsets(int lane, int t, int s2, int* off) {
    const int s = lane & 15, grp = lane >> 4;
    const int d = 32 * t + 16 * (grp & 1) + 4 * (s & 3);
#pragma unroll
    for (int u4 = 0; u4 < 2; ++u4) {
        const int row = 16 * (grp >> 1) + 8 * s2 + (s >> 2) + 4 * u4;
        const int piece = ((d & 63) >> 3) ^ ((row & 7) ^ ((row >> 4) & 1));
        off[u4] = ((d >> 6) * 256 + row * 8 + piece) * 8 + ((d & 7) >> 2) * 4;
    }
}
__device__ inline bf16x8 vt_operand(const u32x4* v_tile, const int* off) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const short* base = reinterpret_cast<const short*>(v_tile);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(base + off[0]));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(base + off[1]));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// KW: 0 -- the waves of a workgroup take four query tiles; 4 -- the four waves share the key range of one tile.
template <int DH, int KW>
constexpr int attention_lds_bytes() {
    constexpr int stage = (KW ? KW : 4) * 2 * (DH / 64) * 256 * 16;
    constexpr int merge = KW ? (KW - 1) * (2 + DH / 32 * 16) * 64 * 4 : 0;
    return stage > merge ? stage : merge;
}
template <int DH, int KW>
__global__ __launch_bounds__(256, (DH == 64 ? 2 : 1)) void k_attention_mfma(AttnArgs a) {
    static_assert(KW == 0 || KW == 4, "a workgroup is four waves");
    constexpr bool KSPLIT = KW > 0;
    constexpr int NCH = DH / 64;     // 64-wide chunks of a q / k row
    constexpr int DT = DH / 32;      // 32-row tiles of O^T
    // Per wave: a K tile and a V tile of 32 keys (NCH x 4 KB each), private to the wave.  After the loop the
    // key-splitting variant reuses the memory to merge its partial results.
    extern __shared__ u32x4 smem[];

    // wave-uniform values are kept in scalar registers (tile description, buffer descriptors, block counters)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    int tile = KSPLIT ? (int)blockIdx.x : (int)blockIdx.x * 4 + wave;
    int head = blockIdx.y;
    if (KSPLIT && a.order != nullptr) {                 // XCD-aware launch order
        if (a.regular) {
            // one sequence, tiles of (nearly) equal work: the host's order is the list (head, tile) cut into eight equal
            // pieces -- computed here instead of fetched, which takes a dependent load off the start of the kernel
            if (!xcd_tile(a.n_tiles, a.n_head, 0, tile, head)) return;
        } else {
            const int ent = a.order[blockIdx.x];
            if (ent < 0) return;                        // padding entry (whole workgroup)
            tile = ent & 0xFFFFF;
            head = ent >> 20;
        }
    }
    if (!KSPLIT && tile >= a.n_tiles) return;           // whole wave; this variant has no barriers

    // One scalar load brings everything that is uniform over the tile; the per-row key counts, the query
    // rows and the first key / value block are then requested together (two dependent round trips in all;
    // one for a regular single sequence, whose tile needs no description).
    AttnTile tl;
    if (a.regular == 1) {
        tl.row0 = 32 * tile; tl.nrows = min(32, a.rows - 32 * tile); tl.kv_max = a.max_kv; tl.kv_off = 0;
    } else if (a.regular == 2) {          // one sequence, causal: row q sees kv_base + q keys
        tl.row0 = 32 * tile; tl.nrows = min(32, a.rows - 32 * tile); tl.kv_max = a.kv_base + tl.row0 + tl.nrows - 1; tl.kv_off = 0;
    } else {
        tl = a.tiles[tile];
    }
    const int row0 = tl.row0, nrows = tl.nrows, kv_max = tl.kv_max;
    const int qrow = row0 + min(r, nrows - 1);
    const int g = head / (a.n_head / a.n_kv_head);
    const uint32_t kv_bytes = ((uint32_t)(kv_max - 1) * (uint32_t)a.kv_ld + DH) * 2u;    // keys 0..kv_max-1 of this kv head
    bf16_t* kbase = const_cast<bf16_t*>(static_cast<const bf16_t*>(a.k)) + tl.kv_off + (size_t)g * DH;
    bf16_t* vbase = const_cast<bf16_t*>(static_cast<const bf16_t*>(a.v)) + tl.kv_off + (size_t)g * DH;
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(kbase, 0, kv_bytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(vbase, 0, kv_bytes, kBufFlags);
    const int kvl = a.regular == 1 ? a.max_kv : (a.regular == 2 ? a.kv_base + qrow : a.kv_len[qrow]);
    int kv_min = kvl;                                    // smallest key count among the tile's rows (wave-uniform)
    if (a.regular == 2) {
        kv_min = a.kv_base + row0;
    } else if (!a.regular) {
#pragma unroll
        for (int o_ = 32; o_ > 0; o_ >>= 1) kv_min = min(kv_min, __shfl_xor(kv_min, o_, 64));
        kv_min = __builtin_amdgcn_readfirstlane(kv_min);
    }
    const bf16_t* Qp = static_cast<const bf16_t*>(a.q) + (size_t)qrow * a.q_ld + (size_t)head * DH + 32 * half;

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
    // Global loads are coalesced (8 consecutive lanes cover one 128-byte piece of a key row; one row per lane
    // would leave the loads bound by the address unit, 32 cache lines per instruction) and pass through the
    // wave-private LDS tile, XOR-swizzled by 16-byte pieces, into the operand layout -- lane = key pi(r).
    const int lrow = lane >> 3, pc = lane & 7;
    const uint32_t kv_lane = ((uint32_t)lrow * (uint32_t)a.kv_ld + 8u * pc) * 2u;
    const uint32_t row8_bytes = 8u * (uint32_t)a.kv_ld * 2u;
    u32x4* const stage_k = smem + wave * (2 * NCH * 256);
    u32x4* const stage_v = stage_k + NCH * 256;
    // piece p of tile row x sits at piece p ^ key(x); the 16 rows a fragment read touches per cycle group are
    // {0..7, 16..23} or {8..15, 24..31} (pi of 16 consecutive lanes): bit 4 of the row separates the two halves.
    int wslot[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 8 * i + lrow;
        wslot[i] = row * 8 + (pc ^ ((row & 7) ^ ((row >> 4) & 1)));
    }
    const int rkey = (pi_r & 7) ^ ((pi_r >> 4) & 1);
    int voff[DT][2][2];                  // transposing reads of the V^T operands, see vt_offsets
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) vt_offsets(lane, t, s2, voff[t][s2]);
    const uint32_t blk_bytes = 32u * (uint32_t)a.kv_ld * 2u;

    float m_run = -INFINITY, l_run = 0.f;
    floatx16 o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    const float scale = rsqrtf((float)DH) * 1.4426950408889634f;     // scores in log2 units

    const int n_blocks = (kv_max + 31) / 32;
    constexpr int kStep = KSPLIT ? KW : 1;
    u32x4 kc[NCH][4], vc[NCH][4], kn[NCH][4], vn[NCH][4];
#define SD_LOAD_BLOCK(KR, VR, KB)                                                                        \
    {                                                                                                    \
        const uint32_t o_ = kv_lane + (uint32_t)(KB) * blk_bytes;                                        \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) _Pragma("unroll") for (int i = 0; i < 4; ++i) {  \
            KR[c][i] = __builtin_amdgcn_raw_buffer_load_b128(rk, o_ + (uint32_t)i * row8_bytes + (uint32_t)(c * 128), 0, 0); \
            VR[c][i] = __builtin_amdgcn_raw_buffer_load_b128(rv, o_ + (uint32_t)i * row8_bytes + (uint32_t)(c * 128), 0, 0); \
        }                                                                                                \
    }
// One key block: scores, online softmax, transpose of the V block, accumulation.  KC / VC: registers of
// this block; the caller has already requested the next block into the other register set.
#define SD_ATTN_BLOCK(KC, VC, KB)                                                                        \
    {                                                                                                    \
        /* LDS operations of one wave execute in order: no barrier around the private tiles */           \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) _Pragma("unroll") for (int i = 0; i < 4; ++i) {  \
            stage_k[c * 256 + wslot[i]] = KC[c][i];                                                      \
            stage_v[c * 256 + wslot[i]] = VC[c][i];                                                      \
        }                                                                                                \
        floatx16 s;                                                                                      \
        _Pragma("unroll") for (int e = 0; e < 16; ++e) s[e] = 0.f;                                       \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) _Pragma("unroll") for (int q4 = 0; q4 < 4; ++q4) \
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                                 \
                __builtin_bit_cast(bf16x8, stage_k[c * 256 + pi_r * 8 + ((4 * half + q4) ^ rkey)]), qf[c][q4], s, 0, 0, 0); \
        /* V^T operands of the block, requested now so that they arrive during the softmax */            \
        bf16x8 vfa_[DT][2];                                                                              \
        _Pragma("unroll") for (int t = 0; t < DT; ++t) _Pragma("unroll") for (int s2 = 0; s2 < 2; ++s2)  \
            vfa_[t][s2] = vt_operand(stage_v, voff[t][s2]);                                              \
        /* online softmax on the raw scores (the scale is positive and is applied inside the exponent);     \
           accumulator e of this lane is key KB*32 + 16*half + e.  Only blocks that reach past the smallest \
           key count of the tile need masking. */                                                         \
        if ((KB) * 32 + 32 > kv_min) {                                                                   \
            _Pragma("unroll") for (int e = 0; e < 16; ++e)                                               \
                s[e] = ((KB) * 32 + 16 * half + e < kvl) ? s[e] : -INFINITY;                             \
        }                                                                                                \
        float mb_ = fmaxf(s[0], s[1]);                                                                   \
        _Pragma("unroll") for (int e = 2; e < 16; ++e) mb_ = fmaxf(mb_, s[e]);                           \
        mb_ = fmaxf(mb_, __shfl_xor(mb_, 32, 64));                                                       \
        const float m_new_ = fmaxf(m_run, mb_);                                                          \
        const float m_fin_ = fmaxf(m_new_, -1e30f);              /* finite even if no key was visible yet */ \
        const float msc_ = m_fin_ * scale;                                                               \
        const float alpha_ = __builtin_amdgcn_exp2f((m_run - m_fin_) * scale);   /* 0 on the first visible block */ \
        float psum_ = 0.f;                                                                               \
        bf16x8 pf_[2];                                                                                   \
        _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                                 \
            const float p_ = __builtin_amdgcn_exp2f(fmaf(s[e], scale, -msc_));                           \
            psum_ += p_;                                                                                 \
            pf_[e >> 3][e & 7] = static_cast<bf16_t>(p_);                                                \
        }                                                                                                \
        l_run = l_run * alpha_ + psum_;                                                                  \
        m_run = m_new_;                                                                                  \
        if (__builtin_amdgcn_ballot_w64(alpha_ != 1.f) != 0) {    /* some row's maximum moved */          \
            _Pragma("unroll") for (int t = 0; t < DT; ++t) _Pragma("unroll") for (int e = 0; e < 16; ++e) o[t][e] *= alpha_; \
        }                                                                                                \
        _Pragma("unroll") for (int t = 0; t < DT; ++t) _Pragma("unroll") for (int s2 = 0; s2 < 2; ++s2) { \
            o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfa_[t][s2], pf_[s2], o[t], 0, 0, 0);         \
        }                                                                                                \
    }
    // Two register sets alternate (no copies): while one block is processed the next is in flight; the block
    // after the last is requested too and reads nothing.
    int kb = KSPLIT ? wave : 0;
    SD_LOAD_BLOCK(kc, vc, kb)
    for (; kb < n_blocks; kb += 2 * kStep) {
        SD_LOAD_BLOCK(kn, vn, kb + kStep)
        SD_ATTN_BLOCK(kc, vc, kb)
        if (kb + kStep >= n_blocks) break;
        SD_LOAD_BLOCK(kc, vc, kb + 2 * kStep)
        SD_ATTN_BLOCK(kn, vn, kb + kStep)
    }
#undef SD_ATTN_BLOCK
#undef SD_LOAD_BLOCK

    if constexpr (KSPLIT) {            // merge the key ranges in a fixed order
        float* const mf = reinterpret_cast<float*>(smem);
        constexpr int NP = KW - 1;     // partial results besides wave 0's own
        float (*mrg_m)[64] = reinterpret_cast<float (*)[64]>(mf);                       // [NP][64]
        float (*mrg_l)[64] = reinterpret_cast<float (*)[64]>(mf + NP * 64);             // [NP][64]
        float (*mrg_o)[DT * 16][64] = reinterpret_cast<float (*)[DT * 16][64]>(mf + 2 * NP * 64);   // [NP][DT*16][64]
        __syncthreads();               // every wave is done with its staging tiles
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
        for (int w = 0; w < NP; ++w) m_all = fmaxf(m_all, mrg_m[w][lane]);
        const float f0 = m_run == -INFINITY ? 0.f : exp2f((m_run - m_all) * scale);
        l_run *= f0;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[t][e] *= f0;
#pragma unroll
        for (int w = 0; w < NP; ++w) {
            const float mw = mrg_m[w][lane];
            const float fw = mw == -INFINITY ? 0.f : exp2f((mw - m_all) * scale);
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

// ---------------------------------------------------------------------------------------------------
// Query tiles that share their keys: a workgroup takes up to four consecutive query tiles of one sequence
// and one head (one tile per wave) and walks the key blocks once for all of them.  A key / value block is
// fetched by the whole workgroup (one 16-byte piece of K and of V per thread and 64-wide chunk), parked in
// one of two LDS stages shared by the waves, and each wave runs the same block step as above on its own
// queries.  This divides the L2 -> CU traffic of K and V by the number of tiles per group -- at a few
// hundred keys and more the one-tile-per-workgroup variants are bound by exactly that traffic -- at the
// price of one barrier per key block.  Global loads run two blocks ahead through two register sets.
template <int DH>
__global__ __launch_bounds__(256, (DH == 64 ? 2 : 1)) void k_attention_group(AttnArgs a) {
    constexpr int NCH = DH / 64, DT = DH / 32;
    constexpr int kStageStride = 2 * NCH * 256;                // one stage: K tile, V tile (u32x4 units)
    __shared__ u32x4 smem[2 * kStageStride];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, half = lane >> 5;
    const int ent = a.groups[blockIdx.x];
    if (ent < 0) return;                                       // padding entry (whole workgroup)
    const int tile0 = ent & 0x3FFFF, nt = ((ent >> 18) & 3) + 1, head = ent >> 20;
    const bool has_tile = wave < nt;                           // the other waves only help loading
    const AttnTile tl = a.tiles[tile0 + min(wave, nt - 1)];
    int kv_all = 0;                                            // keys any tile of the group can see
    for (int t = 0; t < nt; ++t) kv_all = max(kv_all, a.tiles[tile0 + t].kv_max);
    const int row0 = tl.row0, nrows = tl.nrows, kv_max = tl.kv_max;
    const int qrow = row0 + min(r, nrows - 1);
    const int g = head / (a.n_head / a.n_kv_head);
    const uint32_t kv_bytes = ((uint32_t)(kv_all - 1) * (uint32_t)a.kv_ld + DH) * 2u;
    bf16_t* kbase = const_cast<bf16_t*>(static_cast<const bf16_t*>(a.k)) + tl.kv_off + (size_t)g * DH;
    bf16_t* vbase = const_cast<bf16_t*>(static_cast<const bf16_t*>(a.v)) + tl.kv_off + (size_t)g * DH;
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(kbase, 0, kv_bytes, kBufFlags);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(vbase, 0, kv_bytes, kBufFlags);
    const int kvl = a.kv_len[qrow];
    int kv_min = kvl;
#pragma unroll
    for (int o_ = 32; o_ > 0; o_ >>= 1) kv_min = min(kv_min, __shfl_xor(kv_min, o_, 64));
    kv_min = __builtin_amdgcn_readfirstlane(kv_min);
    const bf16_t* Qp = static_cast<const bf16_t*>(a.q) + (size_t)qrow * a.q_ld + (size_t)head * DH + 32 * half;
    bf16x8 qf[NCH][4];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int s = 0; s < 4; ++s) qf[c][s] = __builtin_bit_cast(bf16x8, reinterpret_cast<const u32x4*>(Qp + c * 64)[s]);

    const int pi_r = 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);      // see k_attention_mfma
    const int rkey = (pi_r & 7) ^ ((pi_r >> 4) & 1);
    int voff[DT][2][2];                  // transposing reads of the V^T operands, see vt_offsets
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) vt_offsets(lane, t, s2, voff[t][s2]);
    // cooperative loader: thread t brings piece t & 7 of key row t >> 3 of the block (per 64-wide chunk)
    const int lrow = threadIdx.x >> 3, pc = threadIdx.x & 7;
    const uint32_t kv_lane = ((uint32_t)lrow * (uint32_t)a.kv_ld + 8u * pc) * 2u;
    const uint32_t blk_bytes = 32u * (uint32_t)a.kv_ld * 2u;
    const int wslot = lrow * 8 + (pc ^ ((lrow & 7) ^ ((lrow >> 4) & 1)));

    float m_run = -INFINITY, l_run = 0.f;
    floatx16 o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
    const float scale = rsqrtf((float)DH) * 1.4426950408889634f;
    const int n_blocks = (kv_all + 31) / 32;
    const int my_blocks = has_tile ? (kv_max + 31) / 32 : 0;

    u32x4 gk[2][NCH], gv[2][NCH];
#define SD_G_LOAD(S, KB)                                                                                 \
    {                                                                                                    \
        const uint32_t o_ = kv_lane + (uint32_t)(KB) * blk_bytes;                                        \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) {                                                \
            gk[S][c] = __builtin_amdgcn_raw_buffer_load_b128(rk, o_ + (uint32_t)(c * 128), 0, 0);         \
            gv[S][c] = __builtin_amdgcn_raw_buffer_load_b128(rv, o_ + (uint32_t)(c * 128), 0, 0);         \
        }                                                                                                \
    }
#define SD_G_STAGE(S, STG)                                                                               \
    {                                                                                                    \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) {                                                \
            smem[(STG) * kStageStride + c * 256 + wslot] = gk[S][c];                                     \
            smem[(STG) * kStageStride + NCH * 256 + c * 256 + wslot] = gv[S][c];                         \
        }                                                                                                \
    }
#define SD_G_BLOCK(STG, KB)                                                                              \
    if ((KB) < my_blocks) {                                                                              \
        const u32x4* sk_ = smem + (STG) * kStageStride;                                                  \
        const u32x4* sv_ = sk_ + NCH * 256;                                                              \
        floatx16 s;                                                                                      \
        _Pragma("unroll") for (int e = 0; e < 16; ++e) s[e] = 0.f;                                       \
        _Pragma("unroll") for (int c = 0; c < NCH; ++c) _Pragma("unroll") for (int q4 = 0; q4 < 4; ++q4) \
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                                 \
                __builtin_bit_cast(bf16x8, sk_[c * 256 + pi_r * 8 + ((4 * half + q4) ^ rkey)]), qf[c][q4], s, 0, 0, 0); \
        bf16x8 vfa_[DT][2];                                                                              \
        _Pragma("unroll") for (int t = 0; t < DT; ++t) _Pragma("unroll") for (int s2 = 0; s2 < 2; ++s2)  \
            vfa_[t][s2] = vt_operand(sv_, voff[t][s2]);                                                  \
        if ((KB) * 32 + 32 > kv_min) {                                                                   \
            _Pragma("unroll") for (int e = 0; e < 16; ++e)                                               \
                s[e] = ((KB) * 32 + 16 * half + e < kvl) ? s[e] : -INFINITY;                             \
        }                                                                                                \
        float mb_ = fmaxf(s[0], s[1]);                                                                   \
        _Pragma("unroll") for (int e = 2; e < 16; ++e) mb_ = fmaxf(mb_, s[e]);                           \
        mb_ = fmaxf(mb_, __shfl_xor(mb_, 32, 64));                                                       \
        const float m_new_ = fmaxf(m_run, mb_);                                                          \
        const float m_fin_ = fmaxf(m_new_, -1e30f);                                                      \
        const float msc_ = m_fin_ * scale;                                                               \
        const float alpha_ = __builtin_amdgcn_exp2f((m_run - m_fin_) * scale);                           \
        float psum_ = 0.f;                                                                               \
        bf16x8 pf_[2];                                                                                   \
        _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                                 \
            const float p_ = __builtin_amdgcn_exp2f(fmaf(s[e], scale, -msc_));                           \
            psum_ += p_;                                                                                 \
            pf_[e >> 3][e & 7] = static_cast<bf16_t>(p_);                                                \
        }                                                                                                \
        l_run = l_run * alpha_ + psum_;                                                                  \
        m_run = m_new_;                                                                                  \
        if (__builtin_amdgcn_ballot_w64(alpha_ != 1.f) != 0) {                                           \
            _Pragma("unroll") for (int t = 0; t < DT; ++t) _Pragma("unroll") for (int e = 0; e < 16; ++e) o[t][e] *= alpha_; \
        }                                                                                                \
        _Pragma("unroll") for (int t = 0; t < DT; ++t) _Pragma("unroll") for (int s2 = 0; s2 < 2; ++s2) { \
            o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfa_[t][s2], pf_[s2], o[t], 0, 0, 0);         \
        }                                                                                                \
    }
    // Step kb: park block kb + 1 (register set (kb + 1) & 1) in LDS stage (kb + 1) & 1 -- last read before the
    // barrier that ended step kb - 1 --, refill that set with block kb + 3, work on block kb.  Blocks past the
    // end are requested too and read nothing.
    SD_G_LOAD(0, 0)
    SD_G_LOAD(1, 1)
    SD_G_STAGE(0, 0)
    SD_G_LOAD(0, 2)
    __syncthreads();
    for (int kb = 0; kb < n_blocks; kb += 2) {
        SD_G_STAGE(1, 1)
        SD_G_LOAD(1, kb + 3)
        SD_G_BLOCK(0, kb)
        lds_barrier();
        if (kb + 1 >= n_blocks) break;
        SD_G_STAGE(0, 0)
        SD_G_LOAD(0, kb + 4)
        SD_G_BLOCK(1, kb + 1)
        lds_barrier();
    }
#undef SD_G_LOAD
#undef SD_G_STAGE
#undef SD_G_BLOCK
    if (!has_tile) return;

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.f / l_tot;
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

template <int DH, int KW>
static hipError_t launch_attention_kernel(dim3 grid, hipStream_t st, const AttnArgs& a) {
    constexpr int kLds = attention_lds_bytes<DH, KW>();
    static bool raised = false;                   // more than the default 64 KB of LDS: allowed once per kernel
    if (kLds > 65536 && !raised) {
        const hipError_t e = hipFuncSetAttribute((const void*)k_attention_mfma<DH, KW>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    launch_kernel(k_attention_mfma<DH, KW>, grid, dim3(256), kLds, st, a);
    return hipGetLastError();
}

bool attention_mfma_supported(int dtype, const AttnArgs& a) {
    return dtype == SD_DTYPE_BF16 && (a.d_head == 64 || a.d_head == 128) && a.tiles != nullptr && a.n_tiles > 0 &&
           a.q_ld % 8 == 0 && a.kv_ld % 8 == 0 && a.out_ld % 4 == 0 && (int64_t)a.max_kv * a.kv_ld * 2 < ((int64_t)1 << 31) &&
           (int64_t)a.rows * a.out_ld * 2 < ((int64_t)1 << 31);
}

hipError_t launch_attention_mfma(const AttnArgs& a, hipStream_t st, const char** kernel_name) {
    // several query tiles per sequence: share the key / value blocks among up to four of them
    if (a.groups != nullptr && a.n_groups > 0 && a.group_tiles >= 2 && (long)a.n_tiles * a.n_head >= 1024 && a.max_kv > 64) {
        if (a.d_head == 64) { if (kernel_name) *kernel_name = "k_attention_group<64>"; launch_kernel(k_attention_group<64>, dim3(a.n_groups), dim3(256), 0, st, a); }
        else { if (kernel_name) *kernel_name = "k_attention_group<128>"; launch_kernel(k_attention_group<128>, dim3(a.n_groups), dim3(256), 0, st, a); }
        return hipGetLastError();
    }
    // few tiles: the four waves of a workgroup share the key range of one tile.  (Eight waves per tile were measured too:
    // slower -- 256 registers per lane leave one workgroup per CU, and the chip then needs two rounds of them.)
    const int kw = (long)a.n_tiles * a.n_head < 1024 && a.max_kv > 64 ? 4 : 0;
    const dim3 grid = kw ? (a.order ? dim3(a.regular ? xcd_grid(a.n_tiles, a.n_head) : a.n_order, 1) : dim3(a.n_tiles, a.n_head))
                         : dim3((a.n_tiles + 3) / 4, a.n_head);
#define SD_GO(DH, KW)                                                                                          \
    {                                                                                                          \
        if (kernel_name) *kernel_name = "k_attention_mfma<" #DH "," #KW ">";                                   \
        return launch_attention_kernel<DH, KW>(grid, st, a);                                                   \
    }
    if (a.d_head == 64) {
        if (kw == 4) SD_GO(64, 4) else SD_GO(64, 0)
    } else {
        if (kw == 4) SD_GO(128, 4) else SD_GO(128, 0)
    }
#undef SD_GO
}

}  // namespace sd
