// Shared declarations of the gfx950 SpecDiff library: element types, launch helpers and the
// prototypes of the kernel launchers (one translation unit per kernel family).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/specdiff.h"

namespace sd {

typedef __bf16 bf16_t;

constexpr int kWave = 64;            // CDNA wavefront
constexpr int kChunk = 1024;         // vocabulary columns handled by one workgroup of the sampling kernels
constexpr uint32_t STREAM_DRAFT = 1; // Philox counter word 3
constexpr uint32_t STREAM_VERIFY = 2;
constexpr uint32_t STREAM_SPS = 3;   // token samples of the autoregressive drafter of standard speculative decoding

__host__ __device__ inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
__host__ __device__ inline int vocab_pad(int v) { return (v + 255) / 256 * 256; }
__host__ __device__ inline int n_chunks(int vocab) { return (vocab + kChunk - 1) / kChunk; }

enum Epilogue {
    EPI_STORE = 0, EPI_GELU = 1, EPI_RESID = 2, EPI_F32 = 3,
    EPI_RESID_NORM = 4,  // kernels only: EPI_RESID with NormOut
    EPI_ARGMAX = 7,      // no output rows at all: per row and 32-column tile the largest value and its column (NormOut::am_v / am_i;
                         // temperature 0 needs nothing else of an LM head); the few-row streaming kernel only (launch_linear_stream)
    EPI_STORE_ROPE = 6,  // kernels only: EPI_STORE with NormOut::rope_cs (rotary embedding in the epilogue)
    EPI_SWIGLU = 5       // W = [gate rows | up rows] ([n, k], n even): y[m, n / 2] (dtype) = silu(gate part) * (up part); the few-row
                         // streaming kernel only (launch_linear_stream), callers fall back to EPI_STORE + launch_swiglu
};

// A normalisation folded around a contraction  y = W norm(h) + bias  (bf16 models).  Whoever produces the
// residual stream h also writes x = bf16(h * gain) and partial row sums (sum h, sum h^2); the contraction
// multiplies x and applies mean and variance in its epilogue:
//   LayerNorm (kind 1): y_n = rstd_m (sum_k x_mk W_nk - mu_m u_n) + v_n, u = W gain, v = W beta + bias;
//   RMSNorm   (kind 2): y_n = rstd_m  sum_k x_mk W_nk + bias_n.
struct NormIn {              // consumer: how to finish the contraction
    int kind = 0;            // 0: plain contraction
    const float* stats = nullptr;   // [m][parts][2] partial (sum h, sum h^2) of every row, added in order
    int parts = 0;
    const float* u = nullptr;       // W gain [n] (kind 1); the bias argument then carries v
    float eps = 0.f;
};
struct NormOut {             // producer (residual epilogue): what to prepare for the normalisation after it
    const float* gain = nullptr;    // [n] gain of that normalisation; NULL: nothing to prepare
    void* xg = nullptr;             // bf16 [m][n] = bf16(y * gain)
    float* stats = nullptr;         // [m][ceil(n / 32)][2]
    // Output columns from c1 on go elsewhere (plain bf16 store epilogue of the few-row matrix-core kernel only; c1, c2
    // multiples of 32): columns [c1, c2) to y1[row * ld12 + col - c1], columns >= c2 to y2[row * ld12 + col - c2] -- the
    // K and V parts of a QKV contraction written straight into the KV cache.  y1 == NULL: everything goes to y.
    void* y1 = nullptr;
    void* y2 = nullptr;
    int c1 = 0, c2 = 0, ld12 = 0;
    // Rotary embedding of the output columns [0, rope_cols) (the q and k parts of a QKV contraction; same kernel and
    // epilogue as the column split): heads of rope_dh columns (64 or 128), the pair (i, i + rope_dh / 2) of row m is
    // rotated by the angle whose (cos, sin) is rope_cs[m * rope_dh / 2 + i] (launch_rope_table).  NULL: no rotation.
    const float* rope_cs = nullptr;
    int rope_cols = 0, rope_dh = 0;
    // EPI_ARGMAX: am_v[row * ceil(n / 32) + tile] = largest value of the row within columns 32 tile .. 32 tile + 31,
    // am_i[...] = its column (lowest on ties).
    float* am_v = nullptr;
    int32_t* am_i = nullptr;
};

// Every kernel of the library is launched through launch_kernel().  Ordinarily that is a plain launch.  While a
// handle's per-kernel timing is on (sd_profile_begin), g_launch_hook hands out a pair of HIP events per launch and the
// launch goes through hipExtLaunchKernelGGL, which stamps them with the kernel's own start and end of execution (what
// a profiler's kernel trace shows): events recorded around a launch would also count the gap in front of it.
// The hook is process-wide: one handle profiles at a time.
typedef void (*launch_hook_t)(void* ctx, hipEvent_t* start, hipEvent_t* stop);
extern launch_hook_t g_launch_hook;
extern void* g_launch_hook_ctx;

template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), const dim3& grid, const dim3& block, size_t lds_bytes, hipStream_t st,
                          Args&&... args) {
    if (g_launch_hook != nullptr) {
        hipEvent_t e0 = nullptr, e1 = nullptr;
        g_launch_hook(g_launch_hook_ctx, &e0, &e1);
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, st, e0, e1, 0u, static_cast<KArgs>(args)...);
    } else {
        kernel<<<grid, block, lds_bytes, st>>>(static_cast<KArgs>(args)...);
    }
}

// ---- launchers (all asynchronous on `st`; return hipGetLastError()) ------------------------

// y = epilogue(x W^T + bias); see sd_linear in specdiff.h.
// *kernel_name (optional) receives the name of the kernel variant that was launched.
struct SplitWorkspace;
hipError_t launch_linear(int dtype, const void* x, const void* w, const float* bias, void* y, int m, int n,
                         int k, int ldy, int epilogue, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws,
                         hipStream_t st, const char** kernel_name);

// h[r, :] = wte[token(r)] + wpe[pos[r]] + temb, fp32 residual stream.  token(r) = src[r] >= 0 ?
// prefix[src[r]] : block[-src[r] - 1].  wpe, temb may be NULL.  gain != NULL: also xg = bf16(h * gain) and
// stats[r] = (sum h, sum h^2) for a normalisation folded into the first contraction (see NormIn).
hipError_t launch_embed(int dtype, const int32_t* src, const int32_t* pos, const int32_t* prefix,
                        const int32_t* block, const void* wte, const void* wpe, const float* temb,
                        float* h, int rows, int d, const float* gain, void* xg, float* stats, hipStream_t st);

// temb[j-1, :] = W2 silu(W1 s(j/T) + b1) + b2 for j = 1..T  (sinusoidal s of 1000 t).
hipError_t launch_timestep_embed(int dtype, const void* w1, const float* b1, const void* w2, const float* b2,
                                 float* hidden, float* temb, int T, int d, hipStream_t st);

// out[i, :] = norm(h[idx ? idx[i] : i, :]) * gain (+ bias): LayerNorm if bias != NULL else RMSNorm.
hipError_t launch_norm(int dtype, const float* h, const int32_t* idx, const float* gain, const float* bias,
                       void* out, int rows, int d, float eps, hipStream_t st);

// In-place rotary embedding of the q and k parts of qkv rows (llama), positions pos[r].
hipError_t launch_rope(int dtype, void* qkv, const int32_t* pos, int rows, int n_head, int n_kv_head, int d_head,
                       float theta, hipStream_t st);

// cs[r * d_head / 2 + i] = (cos, sin) of pos[r] * theta^(-2 i / d_head): the rotation angles of `rows` rows, for the
// contraction epilogue that rotates q and k itself (NormOut::rope_cs).  The angles depend on the positions only, so one
// table serves every layer of a forward.
hipError_t launch_rope_table(const int32_t* pos, int rows, int d_head, float theta, float* cs, hipStream_t st);

// Both of the above in one pass (rotary embedding, then the cache append of the rotated k and of v).
hipError_t launch_rope_kv_store(int dtype, void* qkv, const int32_t* seq, const int32_t* pos, void* kcache, void* vcache,
                                int rows, int n_head, int n_kv_head, int d_head, float theta, int n_ctx, hipStream_t st);

// Copy the k and v parts of qkv rows into the cache at (seq[r], pos[r]).
hipError_t launch_kv_store(int dtype, const void* qkv, const int32_t* seq, const int32_t* pos, void* kcache,
                           void* vcache, int rows, int n_head, int n_kv_head, int d_head, int n_ctx, hipStream_t st);

// out[r, h*dh:(h+1)*dh] = softmax(q_r k^T / sqrt(dh)) v over keys 0..kv_len[r]-1 of r's sequence.
// Keys/values of sequence s start at kbase + kv_off[r] elements with row stride kv_ld.
struct AttnTile;
struct AttnArgs {
    const void* q; int q_ld;                 // query rows, head h at column h*dh
    const void* k; const void* v; int kv_ld; // key / value rows, kv head g at column g*dh
    const int64_t* kv_off;                   // per query row: element offset of its sequence's key row 0
    const int32_t* kv_len;                   // per query row: number of visible keys
    void* out; int out_ld;
    int rows, n_head, n_kv_head, d_head;
    int max_kv;                              // upper bound of kv_len over the rows
    // Query tiles for the matrix-core kernel (NULL / 0 when not provided).
    const struct AttnTile* tiles = nullptr;
    int n_tiles = 0;
    // Launch order of the key-splitting variant: workgroup i handles tile order[i] & 0xFFFFF of head
    // order[i] >> 20 (negative: nothing).  NULL: workgroup (x, y) handles tile x of head y.
    const int32_t* order = nullptr;
    int n_order = 0;
    // Launch order of the key-sharing variant: workgroup i handles tiles t0 .. t0 + n - 1 (consecutive tiles
    // of one sequence, n <= 4) of one head, groups[i] = t0 | (n - 1) << 18 | head << 20 (negative: nothing).
    // group_tiles: the largest n (the variant is used from 2 on).
    const int32_t* groups = nullptr;
    int n_groups = 0, group_tiles = 0;
    // 1: one sequence whose rows all see all max_kv keys (the drafter at batch 1): tile t is rows 32 t .. of it, key offset
    // 0.  2: one sequence with causal visibility (the target's query rows at batch 1): row q sees its first kv_base + q
    // keys.  The kernels then take nothing from tiles / kv_off / kv_len and save the round trip for them.
    int regular = 0;
    int kv_base = 0;
};
// Rows row0 .. row0 + nrows - 1 (<= 32, all of one sequence); kv_max = largest kv_len among them;
// kv_off = element offset of the sequence's key row 0 (the kv_off of its rows).
struct AttnTile {
    int32_t row0, nrows, kv_max, pad;
    int64_t kv_off, pad2;
};
bool attention_mfma_supported(int dtype, const AttnArgs& a);
hipError_t launch_attention_mfma(const AttnArgs& a, hipStream_t st, const char** kernel_name);
hipError_t launch_attention(int dtype, const AttnArgs& a, hipStream_t st, const char** kernel_name);
hipError_t launch_attention_generic(int dtype, const AttnArgs& a, int max_kv, hipStream_t st);
hipError_t launch_linear_generic(int dtype, const void* x, const void* w, const float* bias, void* y, int m, int n,
                                 int k, int ldy, int epilogue, hipStream_t st);

// Device workspace of the contractions that split K over workgroups: kSplitTicketBytes of counters
// (zero between launches) followed by the partial-sum records.  base == nullptr: no such split.
constexpr int64_t kSplitTicketBytes = 16384;
struct SplitWorkspace {
    void* base = nullptr;
    int64_t bytes = 0;
};
bool linear_mfma_supported(int dtype, int m, int n, int k, int ldy);
void linear_mfma_set_variant(int v);     // tuning hook: force a tile variant (-1 = choose by shape)
void linear_mfma_set_split(int s);       // tuning hook: force the K split over workgroups (<= 0 = choose by shape)
int linear_mfma_get_variant();
int linear_mfma_get_split();
hipError_t launch_fold_norm(const void* w, const float* gain, const float* beta, const float* bias, float* u, float* v,
                            int n, int k, hipStream_t st);
hipError_t launch_linear_mfma(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epilogue, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws,
                              hipStream_t st, const char** kernel_name);
// x = bf16(h * gain) and one pair (sum h, sum h^2) per row (parts = 1): prepares a folded normalisation for
// rows that no contraction epilogue produced (after the embedding).  d % 4 == 0.
hipError_t launch_norm_prep(const float* h, const float* gain, void* xg, float* stats, int rows, int d, hipStream_t st);

// Up to 64 rows against a long weight stream: x parked in LDS, weights streamed (gemm_stream.hip).  Returns
// hipErrorNotSupported when the shape does not fit (the caller then uses another kernel).
bool linear_stream_preferred(int m, int n, int k, bool folded);
hipError_t launch_linear_stream(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                                int epilogue, const NormIn& ni, const NormOut& no, const SplitWorkspace& ws,
                                int force_split, hipStream_t st, const char** kernel_name);

// Many-row contraction with workgroup-shared 64 x 128 or 128 x 128 tiles (x bf16); rows = 0: height by shape.
bool linear_tile_preferred(int m, int n, int k);
hipError_t launch_linear_tile(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epilogue, const NormIn& ni, const NormOut& no, int rows, hipStream_t st,
                              const char** kernel_name);

// Many-row contraction whose operand tiles go from global memory straight into a ring of LDS stages
// (gemm_pipe.hip).  shape: 0 = 64 x 64, 1 = 64 x 128, 2 = 128 x 128, 3 = 256 x 128 workgroup tiles, one 64-wide
// chunk of K per stage; 4 = 64 x 64, 5 = 64 x 128 with two chunks per stage (K a multiple of 128).
// hipErrorNotSupported: K shorter than the ring or not a multiple of the stage width (the caller then uses another kernel).
int linear_pipe_shape(int m, int n, int k);     // shape this kernel wants for a contraction, -1: none
hipError_t launch_linear_pipe(const void* x, const void* w, const float* bias, void* y, int m, int n, int k, int ldy,
                              int epilogue, const NormIn& ni, const NormOut& no, int shape, hipStream_t st,
                              const char** kernel_name);

// act[r, c] = silu(gu[r, c]) * gu[r, F + c]
hipError_t launch_swiglu(int dtype, const void* gu, void* act, int rows, int F, hipStream_t st);

// ---- sampling family ------------------------------------------------------------------------
struct SampleScratch {       // carved from one device buffer by sampling_scratch()
    double* part_m;          // [rows, n_chunks] chunk maxima
    double* part_s;          // [rows, n_chunks] chunk sums of exp(l - chunk max)
    double* part_r;          // [batch, n_chunks] chunk sums of the residual / bonus weights
    double* row_m;           // [batch] max of the row the final token is drawn from
    double* row_z;           // [batch] its softmax normaliser
    int32_t* active;         // [rows]
    unsigned int* ticket;    // [batch] arrival counters of the acceptance path: zero before a launch, zero again after it
    uint64_t* seed;          // Philox key of the current call (kernels read it from memory so that a
                             // captured graph can be replayed with a new seed)
};
int64_t sampling_scratch_bytes(int rows, int vocab);
SampleScratch sampling_scratch(void* base, int rows, int vocab);
// Zero the arrival counters (scratch memory of unknown content; the kernels leave them zero afterwards).
hipError_t launch_sampling_reset(const SampleScratch& s, int rows, hipStream_t st);

hipError_t launch_fill_i32(int32_t* p, int n, int v, hipStream_t st);
hipError_t launch_unmask_sample(const float* logits, int batch, int gamma, int vocab, int step, const uint64_t* seed,
                                int32_t* z, float* q, float* qtok, const SampleScratch& s, hipStream_t st);
hipError_t launch_accept_resample(const float* p_logits, const float* q, const int32_t* draft, int batch,
                                  int gamma, int vocab, const uint64_t* seed, int32_t* n_acc, int32_t* token,
                                  const SampleScratch& s, hipStream_t st);

// Step k of the autoregressive drafter (standard speculative decoding): logits [batch, ld], one row per sequence;
// x_k ~ softmax(row b) by inverse CDF with the Philox draw (position k, step 0, sequence b, STREAM_SPS) word 1;
// z[b * gamma + k] <- x_k, q row b * gamma + k <- the softmax row, qtok[b * gamma + k] <- its probability.
// greedy: x_k = argmax (lowest id on ties), qtok = 1, no q row.
hipError_t launch_sps_sample(const float* logits, int batch, int gamma, int vocab, int k, const uint64_t* seed, int32_t* z,
                             float* q, float* qtok, bool greedy, const SampleScratch& s, hipStream_t st);

// Temperature 0 on per-tile maxima left by an LM head with EPI_ARGMAX (pv, pi: [rows][tiles]) instead of on logits:
// the reveal step of the diffusion drafter (step >= 1), step k of the autoregressive drafter (sps_k >= 0, logits row =
// sequence), and the acceptance (rows = batch * (gamma + 1)).
hipError_t launch_greedy_from_tiles(const float* pv, const int32_t* pi, int tiles, int batch, int gamma, int vocab, int step, int sps_k,
                                    const uint64_t* seed, int32_t* z, float* qtok, hipStream_t st);
hipError_t launch_accept_greedy_from_tiles(const float* pv, const int32_t* pi, int tiles, const int32_t* draft, int batch, int gamma,
                                           int32_t* top /* int32 [batch * (gamma + 1)] scratch */, int32_t* n_acc, int32_t* token, hipStream_t st);

// Temperature 0: argmax at reveal (qtok = 1, no q row); accept iff the drafted token is the target's argmax.
hipError_t launch_unmask_greedy(const float* logits, int batch, int gamma, int vocab, int step, const uint64_t* seed,
                                int32_t* z, float* qtok, const SampleScratch& s, hipStream_t st);
hipError_t launch_accept_greedy(const float* p_logits, const int32_t* draft, int batch, int gamma, int vocab,
                                int32_t* n_acc, int32_t* token, const SampleScratch& s, hipStream_t st);

}  // namespace sd
