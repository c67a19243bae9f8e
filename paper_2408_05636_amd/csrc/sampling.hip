// Vocabulary-row kernels of Algorithm 1: softmax statistics, the reveal / categorical-sampling
// step of the diffusion drafter, and the acceptance test with residual resampling.
//
// All probability-space arithmetic is fp64 (exp, normalisers, CDF prefix sums): these kernels
// stream fp32 rows from HBM/L2 and are nowhere near ALU-bound, and fp64 keeps every integer
// decision (which token, how many accepted) independent of the summation tree.  No float
// atomics anywhere: every reduction has a fixed order, so results are run-to-run identical.
//
// A row of `vocab` logits is cut into chunks of kChunk columns; one 256-thread workgroup owns
// one chunk (4 consecutive columns per thread), so a single row is spread over many CUs.
#include "common.h"
#include "philox.hip.h"

namespace sd {

constexpr int kThreads = 256;
constexpr int kMaxChunks = 512;   // vocab <= 524288

// ---------------------------------------------------------------- block-wide primitives (256 threads)
__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;   // valid in lane 0
}
__device__ inline double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;   // all lanes
}
__device__ inline double block_sum(double v, double* sh /*[4]*/) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}
__device__ inline double block_max(double v, double* sh) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmax(fmax(sh[0], sh[1]), fmax(sh[2], sh[3]));
}
__device__ inline int block_min_int(int v, int* sh) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return min(min(sh[0], sh[1]), min(sh[2], sh[3]));
}
__device__ inline int block_max_int(int v, int* sh) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return max(max(sh[0], sh[1]), max(sh[2], sh[3]));
}
// exclusive prefix sum over the 256 threads, in thread order
__device__ inline double block_excl_scan(double v, double* sh /*[4]*/) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    double inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) sh[wv] = inc;
    __syncthreads();
    double base = 0.0;
    for (int i = 0; i < wv; ++i) base += sh[i];
    return base + (inc - v);
}

// 4 consecutive logits of this thread; columns >= vocab read as -inf
__device__ inline void load4(const float* row, int col, int vocab, float (&l)[4]) {
    if (col + 3 < vocab) {
        const float4 t = *reinterpret_cast<const float4*>(row + col);
        l[0] = t.x; l[1] = t.y; l[2] = t.z; l[3] = t.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) l[i] = (col + i < vocab) ? row[col + i] : -INFINITY;
    }
}

// ---------------------------------------------------------------- chunk statistics
// grid (n_chunks, rows).  z != NULL: drafter mode, rows that are not revealed at this step are skipped.
__global__ __launch_bounds__(kThreads) void k_row_stats(const float* __restrict__ logits, int ld, int vocab,
                                                        const int32_t* __restrict__ z, int gamma, int step,
                                                        const uint64_t* __restrict__ seed_p, double* __restrict__ part_m,
                                                        double* __restrict__ part_s, int32_t* __restrict__ active) {
    __shared__ double sh[4];
    const int row = blockIdx.y, c = blockIdx.x, nch = gridDim.x;
    if (z != nullptr) {
        const bool act = (z[row] == vocab) && reveal_now(row % gamma, step, row / gamma, STREAM_DRAFT, *seed_p);
        if (c == 0 && threadIdx.x == 0) active[row] = act ? 1 : 0;
        if (!act) return;
    }
    float l[4];
    load4(logits + (size_t)row * ld, c * kChunk + threadIdx.x * 4, vocab, l);
    const double m = block_max((double)fmaxf(fmaxf(l[0], l[1]), fmaxf(l[2], l[3])), sh);
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += exp((double)l[i] - m);   // exp(-inf) = 0 for padding columns
    s = block_sum(s, sh);
    if (threadIdx.x == 0) {
        part_m[(size_t)row * nch + c] = m;
        part_s[(size_t)row * nch + c] = s;
    }
}

// Combine a row's chunk statistics: m = max_c m_c, sS[c] = s_c exp(m_c - m).  Block-uniform result.
__device__ inline double combine_chunks(const double* pm, const double* ps, int nch, double* sS, double* sh) {
    double m = -INFINITY;
    for (int i = threadIdx.x; i < nch; i += kThreads) m = fmax(m, pm[i]);
    m = block_max(m, sh);
    for (int i = threadIdx.x; i < nch; i += kThreads) sS[i] = ps[i] * exp(pm[i] - m);
    __syncthreads();
    return m;
}

// Thread 0: total of sS[0..nch) in chunk order, the chunk where the running sum first exceeds
// u * total and the running sum before that chunk.
struct ChunkPick { double total, target, before; int chunk; };
__device__ inline ChunkPick pick_chunk(const double* sS, int nch, double u) {
    ChunkPick p;
    double tot = 0.0;
    for (int i = 0; i < nch; ++i) tot += sS[i];
    p.total = tot;
    p.target = u * tot;
    double run = 0.0;
    p.chunk = -1;
    p.before = 0.0;
    int last_pos = 0;
    for (int i = 0; i < nch; ++i) {
        if (sS[i] > 0.0) last_pos = i;
        if (run + sS[i] > p.target) { p.chunk = i; p.before = run; break; }
        run += sS[i];
    }
    if (p.chunk < 0) {          // rounding only: last chunk that carries mass
        p.chunk = last_pos;
        double r2 = 0.0;
        for (int i = 0; i < last_pos; ++i) r2 += sS[i];
        p.before = r2;
    }
    return p;
}

// Within one chunk: smallest column whose inclusive running sum exceeds target; if none (rounding),
// the last column of the chunk with positive weight.  w: this thread's 4 weights.  Block-uniform result.
__device__ inline int select_in_chunk(const double (&w)[4], int col0, double before, double target, double* sh,
                                      int* shi) {
    const double mine = ((w[0] + w[1]) + w[2]) + w[3];
    double run = before + block_excl_scan(mine, sh);
    int cand = INT_MAX, lastpos = -1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        run += w[i];
        if (w[i] > 0.0) lastpos = col0 + i;
        if (cand == INT_MAX && run > target && w[i] > 0.0) cand = col0 + i;
    }
    cand = block_min_int(cand, shi);
    if (cand != INT_MAX) return cand;
    return block_max_int(lastpos, shi);
}

// ---------------------------------------------------------------- reveal + sample (drafter)
// grid (n_chunks, rows).  Writes the full q row of every revealed slot; the workgroup owning the
// chunk where the CDF crosses u picks the token.
__global__ __launch_bounds__(kThreads) void k_unmask_sample(const float* __restrict__ logits, int ld, int vocab,
                                                            int gamma, int step, const uint64_t* __restrict__ seed_p,
                                                            const double* __restrict__ part_m,
                                                            const double* __restrict__ part_s,
                                                            const int32_t* __restrict__ active, int32_t* __restrict__ z,
                                                            float* __restrict__ q, float* __restrict__ qtok, int sps_k) {
    __shared__ double sS[kMaxChunks];
    __shared__ double sh[4];
    __shared__ int shi[4];
    __shared__ ChunkPick pick;
    // sps_k >= 0: step sps_k of the autoregressive drafter -- logits row = sequence, every row draws, with its own
    // Philox stream, and the results go to slot (sequence, sps_k) of the [batch, gamma] outputs.
    const int lrow = blockIdx.y, c = blockIdx.x, nch = gridDim.x;
    const int row = sps_k >= 0 ? lrow * gamma + sps_k : lrow;
    if (sps_k < 0 && !active[lrow]) return;
    const double m = combine_chunks(part_m + (size_t)lrow * nch, part_s + (size_t)lrow * nch, nch, sS, sh);
    if (threadIdx.x == 0) {
        const Philox4 r = sps_k >= 0 ? philox4x32_10((uint32_t)sps_k, 0u, (uint32_t)lrow, STREAM_SPS, *seed_p)
                                     : philox4x32_10((uint32_t)(row % gamma), (uint32_t)step, (uint32_t)(row / gamma), STREAM_DRAFT, *seed_p);
        pick = pick_chunk(sS, nch, uniform_f64(r.y));
    }
    __syncthreads();
    const double Z = pick.total;
    const int col0 = c * kChunk + threadIdx.x * 4;
    float l[4];
    load4(logits + (size_t)lrow * ld, col0, vocab, l);
    double w[4];
    float qv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        w[i] = exp((double)l[i] - m);
        qv[i] = (float)(w[i] / Z);
    }
    if (col0 < ld) *reinterpret_cast<float4*>(q + (size_t)row * ld + col0) = make_float4(qv[0], qv[1], qv[2], qv[3]);
    if (c != pick.chunk) return;
    const int v = select_in_chunk(w, col0, pick.before, pick.target, sh, shi);
    if (v >= col0 && v < col0 + 4) {
        z[row] = v;
        qtok[row] = qv[v - col0];
    }
}

// ---------------------------------------------------------------- acceptance + final token (target)
// Weight of column i of the row the final token is drawn from: residual max(0, p - q) after a
// rejection, p itself after full acceptance (or when the residual carries no mass).
__device__ inline double final_weight(float l, float qv, double m, double Z, bool use_residual) {
    const double p = exp((double)l - m) / Z;
    return use_residual ? fmax(0.0, p - (double)qv) : p;
}

// grid (n_chunks, batch), after k_row_stats has left the chunk statistics of the gamma + 1 target rows.
//  0. Every workgroup of a sequence combines the chunk statistics of the sequence's gamma + 1 rows (maximum, normaliser)
//     and  1. runs the gamma acceptance tests r_k q_k(x_k) <= p_k(x_k) (fp32 product), n = the first rejection: a few
//     thousand exponentials and gamma lookups, cheaper done by every workgroup than handed around.
//  2. It sums the final-token weights of its chunk of row n -- max(0, p_n - q_n) after a rejection, p_gamma after full
//     acceptance --, leaves the sum in part_r and draws a ticket (device-scope accesses, complete before the ticket).
//  3. The last arrival of the sequence picks the chunk whose running sum passes u * total, then the token inside it, and
//     writes n and the token; nobody waits.  Fixed orders throughout: run-to-run identical.
__global__ __launch_bounds__(kThreads) void k_accept_final(const float* __restrict__ p_logits, const float* __restrict__ q,
                                                           const int32_t* __restrict__ draft, int ld, int vocab, int gamma,
                                                           const uint64_t* __restrict__ seed_p, const double* __restrict__ part_m,
                                                           const double* __restrict__ part_s, double* __restrict__ part_r,
                                                           unsigned int* __restrict__ ticket, int32_t* __restrict__ n_acc,
                                                           int32_t* __restrict__ token) {
    extern __shared__ double dyn[];          // [gamma+1] maxima, [gamma+1] normalisers
    __shared__ double sS[kMaxChunks];
    __shared__ double sh[4];
    __shared__ int shi[4];
    __shared__ ChunkPick pick;
    __shared__ int s_resid;
    __shared__ unsigned int s_last;
    double* const row_m = dyn;
    double* const row_z = dyn + (gamma + 1);
    const int b = blockIdx.y, c = blockIdx.x, nch = gridDim.x;
    // 0. row statistics of P[0..gamma] (one wave per row, lanes stride over the chunks)
    {
        const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
        for (int k = wv; k <= gamma; k += kThreads / 64) {
            const size_t o = ((size_t)b * (gamma + 1) + k) * nch;
            double mm = -INFINITY;
            for (int i = lane; i < nch; i += 64) mm = fmax(mm, part_m[o + i]);
            mm = wave_max(mm);
            double ss = 0.0;
            for (int i = lane; i < nch; i += 64) ss += part_s[o + i] * exp(part_m[o + i] - mm);
            ss = wave_sum(ss);
            if (lane == 0) { row_m[k] = mm; row_z[k] = ss; }
        }
    }
    __syncthreads();
    // 1. acceptance tests
    int first_reject = gamma;
    for (int k = threadIdx.x; k < gamma; k += kThreads) {
        const int x = draft[b * gamma + k];
        bool ok = false;
        if ((unsigned)x < (unsigned)vocab) {
            const size_t prow = (size_t)b * (gamma + 1) + k, qrow = (size_t)b * gamma + k;
            const float px = (float)(exp((double)p_logits[prow * ld + x] - row_m[k]) / row_z[k]);
            const float qx = q[qrow * ld + x];
            const Philox4 r = philox4x32_10((uint32_t)k, 0u, (uint32_t)b, STREAM_VERIFY, *seed_p);
            ok = __fmul_rn(uniform_f32(r.x), qx) <= px;        // accept iff r q(x) <= p(x), fp32 product
        }
        if (!ok) first_reject = min(first_reject, k);
    }
    const int n = block_min_int(first_reject, shi);
    // 2. this chunk's share of the final-token weights
    const size_t nrow = (size_t)b * (gamma + 1) + n;
    const double m = row_m[n], Z = row_z[n];
    bool resid = n < gamma;
    int col0 = c * kChunk + threadIdx.x * 4;
    float l[4], qv[4] = {0.f, 0.f, 0.f, 0.f};
    load4(p_logits + nrow * ld, col0, vocab, l);
    if (resid && col0 < ld) {
        const float4 t = *reinterpret_cast<const float4*>(q + ((size_t)b * gamma + n) * ld + col0);
        qv[0] = t.x; qv[1] = t.y; qv[2] = t.z; qv[3] = t.w;
    }
    double w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (col0 + i < vocab) ? final_weight(l[i], qv[i], m, Z, resid) : 0.0;
    const double s = block_sum(((w[0] + w[1]) + w[2]) + w[3], sh);
    if (threadIdx.x == 0) {
        __hip_atomic_store(&part_r[(size_t)b * nch + c], s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        s_last = __hip_atomic_fetch_add(&ticket[b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned int)nch - 1u;
    }
    __syncthreads();
    if (!s_last) return;
    asm volatile("" ::: "memory");     // compiler barrier: the loads below stay behind the ticket
    // 3. the last arrival draws the token
    for (int i = threadIdx.x; i < nch; i += kThreads)
        sS[i] = __hip_atomic_load(&part_r[(size_t)b * nch + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_store(&ticket[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);       // ready for the next launch
        const Philox4 r = philox4x32_10((uint32_t)n, 0u, (uint32_t)b, STREAM_VERIFY, *seed_p);
        const double u = uniform_f64(r.y);
        int rs = resid ? 1 : 0;
        if (rs) {
            double tot = 0.0;
            for (int i = 0; i < nch; ++i) tot += sS[i];
            if (!(tot > 0.0)) {      // empty residual (cannot happen in exact arithmetic): draw from p
                rs = 0;
                const size_t o = nrow * nch;
                for (int i = 0; i < nch; ++i) sS[i] = part_s[o + i] * exp(part_m[o + i] - m) / Z;
            }
        }
        s_resid = rs;
        pick = pick_chunk(sS, nch, u);
        n_acc[b] = n;
    }
    __syncthreads();
    resid = s_resid != 0;
    col0 = pick.chunk * kChunk + threadIdx.x * 4;
    qv[0] = qv[1] = qv[2] = qv[3] = 0.f;
    load4(p_logits + nrow * ld, col0, vocab, l);
    if (resid && col0 < ld) {
        const float4 t = *reinterpret_cast<const float4*>(q + ((size_t)b * gamma + n) * ld + col0);
        qv[0] = t.x; qv[1] = t.y; qv[2] = t.z; qv[3] = t.w;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (col0 + i < vocab) ? final_weight(l[i], qv[i], m, Z, resid) : 0.0;
    const int v = select_in_chunk(w, col0, pick.before, pick.target, sh, shi);
    if (threadIdx.x == 0) token[b] = v;
}

__global__ void k_zero_u32(unsigned int* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ---------------------------------------------------------------- temperature 0
// The one-hot limit of the rule: a revealed slot takes the argmax of its row, a drafted token is accepted
// iff it is the argmax of the target's row, and the extra token is the argmax of row n.  Arg-maxima are
// taken on the stored fp32 logits, lowest column on ties.
struct MaxAt { float v; int i; };
__device__ inline MaxAt better(MaxAt a, MaxAt b) { return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a; }
__device__ inline MaxAt wave_best(MaxAt a) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        MaxAt b;
        b.v = __shfl_xor(a.v, o, 64);
        b.i = __shfl_xor(a.i, o, 64);
        a = better(a, b);
    }
    return a;
}

// grid (n_chunks, rows): per chunk the largest logit and its column.  z != NULL: drafter mode, rows that are
// not revealed at this step are skipped (and flagged in active[]).
__global__ __launch_bounds__(kThreads) void k_chunk_argmax(const float* __restrict__ logits, int ld, int vocab,
                                                           const int32_t* __restrict__ z, int gamma, int step,
                                                           const uint64_t* __restrict__ seed_p, float* __restrict__ part_v,
                                                           int32_t* __restrict__ part_i, int32_t* __restrict__ active) {
    __shared__ float shv[4];
    __shared__ int shi[4];
    const int row = blockIdx.y, c = blockIdx.x, nch = gridDim.x;
    if (z != nullptr) {
        const bool act = (z[row] == vocab) && reveal_now(row % gamma, step, row / gamma, STREAM_DRAFT, *seed_p);
        if (c == 0 && threadIdx.x == 0) active[row] = act ? 1 : 0;
        if (!act) return;
    }
    const int col0 = c * kChunk + threadIdx.x * 4;
    float l[4];
    load4(logits + (size_t)row * ld, col0, vocab, l);            // columns >= vocab read as -inf
    MaxAt m{l[0], col0};
#pragma unroll
    for (int i = 1; i < 4; ++i) m = better(m, MaxAt{l[i], col0 + i});
    m = wave_best(m);
    if ((threadIdx.x & 63) == 0) { shv[threadIdx.x >> 6] = m.v; shi[threadIdx.x >> 6] = m.i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        MaxAt b{shv[0], shi[0]};
        for (int w = 1; w < 4; ++w) b = better(b, MaxAt{shv[w], shi[w]});
        part_v[(size_t)row * nch + c] = b.v;
        part_i[(size_t)row * nch + c] = b.i;
    }
}

// One wave: best chunk of a row.
__device__ inline MaxAt row_best(const float* pv, const int32_t* pi, int nch, int lane) {
    MaxAt m{-INFINITY, INT_MAX};
    for (int i = lane; i < nch; i += 64) m = better(m, MaxAt{pv[i], pi[i]});
    return wave_best(m);
}

// grid (rows), one wave: revealed slots take the argmax of their row.
__global__ __launch_bounds__(64) void k_greedy_reveal(const float* __restrict__ part_v, const int32_t* __restrict__ part_i,
                                                      int nch, const int32_t* __restrict__ active,
                                                      int32_t* __restrict__ z, float* __restrict__ qtok, int gamma, int sps_k) {
    const int lrow = blockIdx.x;                                   // sps_k >= 0: see k_unmask_sample
    if (sps_k < 0 && !active[lrow]) return;
    const int row = sps_k >= 0 ? lrow * gamma + sps_k : lrow;
    const MaxAt m = row_best(part_v + (size_t)lrow * nch, part_i + (size_t)lrow * nch, nch, threadIdx.x);
    if (threadIdx.x == 0) { z[row] = m.i; qtok[row] = 1.f; }
}

// Best (value, column) of a row's tiles by a whole workgroup: thread t takes tiles t, t + 256, ..., then a fixed tree.
__device__ inline MaxAt row_best_block(const float* pv, const int32_t* pi, int nch, float* shv, int* shi) {
    MaxAt m{-INFINITY, INT_MAX};
    for (int i = threadIdx.x; i < nch; i += kThreads) m = better(m, MaxAt{pv[i], pi[i]});
    m = wave_best(m);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { shv[threadIdx.x >> 6] = m.v; shi[threadIdx.x >> 6] = m.i; }
    __syncthreads();
    MaxAt b{shv[0], shi[0]};
    for (int w = 1; w < 4; ++w) b = better(b, MaxAt{shv[w], shi[w]});
    return b;
}

// grid (rows), on per-tile maxima of all rows (an LM head with EPI_ARGMAX): the reveal decision is taken here.
__global__ __launch_bounds__(kThreads) void k_greedy_reveal_tiles(const float* __restrict__ part_v, const int32_t* __restrict__ part_i,
                                                                  int nch, int vocab, int gamma, int step, int sps_k,
                                                                  const uint64_t* __restrict__ seed_p, int32_t* __restrict__ z,
                                                                  float* __restrict__ qtok) {
    __shared__ float shv[4];
    __shared__ int shi[4];
    const int lrow = blockIdx.x;
    const int row = sps_k >= 0 ? lrow * gamma + sps_k : lrow;
    if (sps_k < 0 && !((z[row] == vocab) && reveal_now(row % gamma, step, row / gamma, STREAM_DRAFT, *seed_p))) return;   // block-uniform
    const MaxAt m = row_best_block(part_v + (size_t)lrow * nch, part_i + (size_t)lrow * nch, nch, shv, shi);
    if (threadIdx.x == 0) { z[row] = m.i; qtok[row] = 1.f; }
}

// grid (gamma + 1, batch), on per-tile maxima: top[b][k] = argmax of target row k of sequence b.
__global__ __launch_bounds__(kThreads) void k_row_argmax_tiles(const float* __restrict__ part_v, const int32_t* __restrict__ part_i,
                                                               int nch, int32_t* __restrict__ top) {
    __shared__ float shv[4];
    __shared__ int shi[4];
    const size_t row = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
    const MaxAt m = row_best_block(part_v + row * nch, part_i + row * nch, nch, shv, shi);
    if (threadIdx.x == 0) top[row] = m.i;
}

// grid (batch), one wave: n = first drafted token that differs from its row's argmax, token = argmax of row n.
__global__ __launch_bounds__(64) void k_greedy_accept_top(const int32_t* __restrict__ top, const int32_t* __restrict__ draft, int gamma,
                                                          int32_t* __restrict__ n_acc, int32_t* __restrict__ token) {
    const int b = blockIdx.x;
    int first = gamma;
    for (int k = threadIdx.x; k < gamma; k += 64)
        if (draft[b * gamma + k] != top[(size_t)b * (gamma + 1) + k]) { first = k; break; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) first = min(first, __shfl_xor(first, o, 64));
    if (threadIdx.x == 0) { n_acc[b] = first; token[b] = top[(size_t)b * (gamma + 1) + first]; }
}

// grid (batch), one wave: n = first drafted token that is not the argmax of its target row, token = argmax of row n.
__global__ __launch_bounds__(64) void k_greedy_accept(const float* __restrict__ part_v, const int32_t* __restrict__ part_i,
                                                      int nch, const int32_t* __restrict__ draft, int gamma,
                                                      int32_t* __restrict__ n_acc, int32_t* __restrict__ token) {
    const int b = blockIdx.x;
    int n = gamma, tok = 0;
    for (int k = 0; k <= gamma; ++k) {
        const size_t o = ((size_t)b * (gamma + 1) + k) * nch;
        const MaxAt m = row_best(part_v + o, part_i + o, nch, threadIdx.x);
        tok = m.i;
        if (k < gamma && draft[b * gamma + k] != m.i) { n = k; break; }
    }
    if (threadIdx.x == 0) { n_acc[b] = n; token[b] = tok; }
}

// z <- value (the all-[MASK] start state of the block); a kernel rather than a memset so that it can
// live inside a captured graph.
__global__ void k_fill_i32(int32_t* __restrict__ p, int n, int v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t* p, int n, int v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    launch_kernel(k_fill_i32, dim3((n + 255) / 256), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------- host side
int64_t sampling_scratch_bytes(int rows, int vocab) {
    if (rows <= 0 || vocab <= 0) return 0;
    const int64_t nch = n_chunks(vocab);
    int64_t b = 0;
    b += align_up(rows * nch * 8, 256) * 3;   // part_m, part_s, part_r
    b += align_up((int64_t)rows * 8, 256) * 2; // row_m, row_z
    b += align_up((int64_t)rows * 4, 256);     // active
    b += align_up((int64_t)rows * 8, 256);     // arrival counters (rows + batch <= 2 rows)
    b += 256;                                  // seed slot
    return b;
}

SampleScratch sampling_scratch(void* base, int rows, int vocab) {
    const int64_t nch = n_chunks(vocab);
    char* p = static_cast<char*>(base);
    SampleScratch s;
    const int64_t big = align_up(rows * nch * 8, 256), small = align_up((int64_t)rows * 8, 256);
    s.part_m = reinterpret_cast<double*>(p); p += big;
    s.part_s = reinterpret_cast<double*>(p); p += big;
    s.part_r = reinterpret_cast<double*>(p); p += big;
    s.row_m = reinterpret_cast<double*>(p); p += small;
    s.row_z = reinterpret_cast<double*>(p); p += small;
    s.active = reinterpret_cast<int32_t*>(p); p += align_up((int64_t)rows * 4, 256);
    s.ticket = reinterpret_cast<unsigned int*>(p); p += align_up((int64_t)rows * 8, 256);
    s.seed = reinterpret_cast<uint64_t*>(p);
    return s;
}

hipError_t launch_unmask_sample(const float* logits, int batch, int gamma, int vocab, int step, const uint64_t* seed,
                                int32_t* z, float* q, float* qtok, const SampleScratch& s, hipStream_t st) {
    const int rows = batch * gamma, nch = n_chunks(vocab), ld = vocab_pad(vocab);
    const dim3 grid(nch, rows);
    launch_kernel(k_row_stats, dim3(grid), dim3(kThreads), 0, st, logits, ld, vocab, z, gamma, step, seed, s.part_m, s.part_s, s.active);
    launch_kernel(k_unmask_sample, dim3(grid), dim3(kThreads), 0, st, logits, ld, vocab, gamma, step, seed, s.part_m, s.part_s, s.active, z,
                  q, qtok, -1);
    return hipGetLastError();
}

hipError_t launch_unmask_greedy(const float* logits, int batch, int gamma, int vocab, int step, const uint64_t* seed,
                                int32_t* z, float* qtok, const SampleScratch& s, hipStream_t st) {
    const int rows = batch * gamma, nch = n_chunks(vocab), ld = vocab_pad(vocab);
    float* pv = reinterpret_cast<float*>(s.part_m);          // the fp64 partial arrays are free in this mode
    int32_t* pi = reinterpret_cast<int32_t*>(s.part_s);
    launch_kernel(k_chunk_argmax, dim3(dim3(nch, rows)), dim3(kThreads), 0, st, logits, ld, vocab, z, gamma, step, seed, pv, pi, s.active);
    launch_kernel(k_greedy_reveal, dim3(rows), dim3(64), 0, st, pv, pi, nch, s.active, z, qtok, gamma, -1);
    return hipGetLastError();
}

hipError_t launch_sps_sample(const float* logits, int batch, int gamma, int vocab, int k, const uint64_t* seed, int32_t* z,
                             float* q, float* qtok, bool greedy, const SampleScratch& s, hipStream_t st) {
    const int nch = n_chunks(vocab), ld = vocab_pad(vocab);
    const dim3 grid(nch, batch);
    if (greedy) {
        float* pv = reinterpret_cast<float*>(s.part_m);
        int32_t* pi = reinterpret_cast<int32_t*>(s.part_s);
        launch_kernel(k_chunk_argmax, dim3(grid), dim3(kThreads), 0, st, logits, ld, vocab, nullptr, gamma, 0, nullptr, pv, pi, s.active);
        launch_kernel(k_greedy_reveal, dim3(batch), dim3(64), 0, st, pv, pi, nch, s.active, z, qtok, gamma, k);
        return hipGetLastError();
    }
    launch_kernel(k_row_stats, dim3(grid), dim3(kThreads), 0, st, logits, ld, vocab, nullptr, gamma, 0, seed, s.part_m, s.part_s, s.active);
    launch_kernel(k_unmask_sample, dim3(grid), dim3(kThreads), 0, st, logits, ld, vocab, gamma, 0, seed, s.part_m, s.part_s, s.active, z, q, qtok, k);
    return hipGetLastError();
}

hipError_t launch_greedy_from_tiles(const float* pv, const int32_t* pi, int tiles, int batch, int gamma, int vocab, int step, int sps_k,
                                    const uint64_t* seed, int32_t* z, float* qtok, hipStream_t st) {
    launch_kernel(k_greedy_reveal_tiles, dim3(sps_k >= 0 ? batch : batch * gamma), dim3(kThreads), 0, st, pv, pi, tiles, vocab, gamma, step, sps_k, seed, z, qtok);
    return hipGetLastError();
}

// top: int32 [batch * (gamma + 1)] scratch
hipError_t launch_accept_greedy_from_tiles(const float* pv, const int32_t* pi, int tiles, const int32_t* draft, int batch, int gamma,
                                           int32_t* top, int32_t* n_acc, int32_t* token, hipStream_t st) {
    launch_kernel(k_row_argmax_tiles, dim3(gamma + 1, batch), dim3(kThreads), 0, st, pv, pi, tiles, top);
    launch_kernel(k_greedy_accept_top, dim3(batch), dim3(64), 0, st, top, draft, gamma, n_acc, token);
    return hipGetLastError();
}

hipError_t launch_accept_greedy(const float* p_logits, const int32_t* draft, int batch, int gamma, int vocab,
                                int32_t* n_acc, int32_t* token, const SampleScratch& s, hipStream_t st) {
    const int rows = batch * (gamma + 1), nch = n_chunks(vocab), ld = vocab_pad(vocab);
    float* pv = reinterpret_cast<float*>(s.part_m);
    int32_t* pi = reinterpret_cast<int32_t*>(s.part_s);
    launch_kernel(k_chunk_argmax, dim3(dim3(nch, rows)), dim3(kThreads), 0, st, p_logits, ld, vocab, nullptr, gamma, 0, nullptr, pv, pi, s.active);
    launch_kernel(k_greedy_accept, dim3(batch), dim3(64), 0, st, pv, pi, nch, draft, gamma, n_acc, token);
    return hipGetLastError();
}

hipError_t launch_sampling_reset(const SampleScratch& s, int rows, hipStream_t st) {
    launch_kernel(k_zero_u32, dim3((rows + 255) / 256), dim3(256), 0, st, s.ticket, rows);
    return hipGetLastError();
}

// Two launches: chunk statistics, then the acceptance tests, the final-token weights and -- by the last arrival per
// sequence -- the token.
hipError_t launch_accept_resample(const float* p_logits, const float* q, const int32_t* draft, int batch,
                                  int gamma, int vocab, const uint64_t* seed, int32_t* n_acc, int32_t* token,
                                  const SampleScratch& s, hipStream_t st) {
    const int rows = batch * (gamma + 1), nch = n_chunks(vocab), ld = vocab_pad(vocab);
    launch_kernel(k_row_stats, dim3(dim3(nch, rows)), dim3(kThreads), 0, st, p_logits, ld, vocab, nullptr, gamma, 0, seed, s.part_m,
                  s.part_s, s.active);
    launch_kernel(k_accept_final, dim3(dim3(nch, batch)), dim3(kThreads), 2 * (gamma + 1) * sizeof(double), st, p_logits, q, draft, ld, vocab,
                  gamma, seed, s.part_m, s.part_s, s.part_r, s.ticket, n_acc, token);
    return hipGetLastError();
}

}  // namespace sd
