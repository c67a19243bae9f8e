// Row-wise kernels around the contractions: token / position / timestep embedding, LayerNorm and
// RMSNorm, rotary embedding, KV-cache append and the SwiGLU gate.  The residual stream is fp32
// for every storage type; normalised activations are emitted in the storage type, ready to be the
// A operand of the next contraction.
#include "common.h"

namespace sd {

template <typename T> __device__ inline float to_f(T v) { return static_cast<float>(v); }
template <typename T> __device__ inline T from_f(float v) { return static_cast<T>(v); }

// ---------------------------------------------------------------- embedding
// One wave per row (four rows per workgroup), 4 elements per lane and step (d % 4 == 0).  The drafter adds
// the timestep embedding to every row.  gain != NULL: the first layer's normalisation is folded into its
// QKV contraction, which wants x = bf16(h * gain) and the row sums (sum h, sum h^2) of every row.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float emb_f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 emb_bf16x4;
template <typename T>
__device__ inline emb_f32x4 load4_as_f32(const T* p) {
    if constexpr (sizeof(T) == 2) {
        const emb_bf16x4 v = *reinterpret_cast<const emb_bf16x4*>(p);
        return emb_f32x4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
    } else {
        return *reinterpret_cast<const emb_f32x4*>(p);
    }
}
template <typename T>
__global__ __launch_bounds__(256) void k_embed(const int32_t* __restrict__ src, const int32_t* __restrict__ pos,
                                               const int32_t* __restrict__ prefix, const int32_t* __restrict__ block,
                                               const T* __restrict__ wte, const T* __restrict__ wpe,
                                               const float* __restrict__ temb, float* __restrict__ h, int rows, int d,
                                               const float* __restrict__ gain, bf16_t* __restrict__ xg,
                                               float* __restrict__ stats) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= rows) return;
    const int s = src[r];
    const int tok = s >= 0 ? prefix[s] : block[-s - 1];
    const T* e = wte + (size_t)tok * d;
    const T* p = wpe ? wpe + (size_t)pos[r] * d : nullptr;
    float s1 = 0.f, s2 = 0.f;
    for (int c = lane * 4; c < d; c += 256) {
        emb_f32x4 v = load4_as_f32(e + c);
        if (p) v += load4_as_f32(p + c);
        if (temb) v += *reinterpret_cast<const emb_f32x4*>(temb + c);
        *reinterpret_cast<emb_f32x4*>(h + (size_t)r * d + c) = v;
        if (gain) {
            const emb_f32x4 g = *reinterpret_cast<const emb_f32x4*>(gain + c);
            emb_bf16x4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                s1 += v[u];
                s2 = fmaf(v[u], v[u], s2);
                o[u] = static_cast<bf16_t>(v[u] * g[u]);
            }
            *reinterpret_cast<emb_bf16x4*>(xg + (size_t)r * d + c) = o;
        }
    }
    if (gain) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) { s1 += __shfl_xor(s1, off, 64); s2 += __shfl_xor(s2, off, 64); }
        if (lane == 0) { stats[2 * (size_t)r] = s1; stats[2 * (size_t)r + 1] = s2; }
    }
}

// x = bf16(h * gain) and (sum h, sum h^2) per row for rows that already sit in the residual stream.
__global__ __launch_bounds__(256) void k_norm_prep(const float* __restrict__ h, const float* __restrict__ gain,
                                                   bf16_t* __restrict__ xg, float* __restrict__ stats, int rows, int d) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= rows) return;
    float s1 = 0.f, s2 = 0.f;
    for (int c = lane * 4; c < d; c += 256) {
        const emb_f32x4 v = *reinterpret_cast<const emb_f32x4*>(h + (size_t)r * d + c);
        const emb_f32x4 g = *reinterpret_cast<const emb_f32x4*>(gain + c);
        emb_bf16x4 o;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            s1 += v[u];
            s2 = fmaf(v[u], v[u], s2);
            o[u] = static_cast<bf16_t>(v[u] * g[u]);
        }
        *reinterpret_cast<emb_bf16x4*>(xg + (size_t)r * d + c) = o;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { s1 += __shfl_xor(s1, off, 64); s2 += __shfl_xor(s2, off, 64); }
    if (lane == 0) { stats[2 * (size_t)r] = s1; stats[2 * (size_t)r + 1] = s2; }
}

// ---------------------------------------------------------------- timestep embedding (drafter)
// temb(j/T) = W2 silu(W1 s + b1) + b2 with s_i = sin(1000 t f_i), s_{i+d/2} = cos(1000 t f_i),
// f_i = 10000^(-2i/d), for all T steps of a round at once.  Three small launches: the sinusoid table
// (fp64 arguments, one thread per (step, frequency)), then twice the same mat-vec kernel in which one
// wave owns one output row of the weight matrix, keeps it in registers and applies it to all T inputs.
__global__ __launch_bounds__(256) void k_timestep_sinusoid(float* __restrict__ s, int n_steps, int d) {
    const int half = d / 2;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_steps * half) return;
    const int j = idx / half + 1, i = idx % half;
    const double t = (double)j / (double)n_steps;
    const double f = exp(-log(10000.0) * 2.0 * (double)i / (double)d);
    s[(size_t)(j - 1) * d + i] = (float)sin(1000.0 * t * f);
    s[(size_t)(j - 1) * d + i + half] = (float)cos(1000.0 * t * f);
}

constexpr int kMatvecMax = 32;     // register-resident weight row: d <= 64 * 4 * kMatvecMax
template <typename T, bool SILU>
__global__ __launch_bounds__(256) void k_timestep_matvec(const T* __restrict__ w, const float* __restrict__ b,
                                                         const float* __restrict__ in, float* __restrict__ out,
                                                         int n_steps, int d) {
    const int o = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (o >= d) return;
    emb_f32x4 wr[kMatvecMax];
    int cnt = 0;
    for (int c = lane * 4; c < d; c += 256) wr[cnt++] = load4_as_f32(w + (size_t)o * d + c);
    const float bias = b[o];
    for (int j = 0; j < n_steps; ++j) {
        float acc = 0.f;
        int q = 0;
        for (int c = lane * 4; c < d; c += 256, ++q) {
            const emb_f32x4 x = *reinterpret_cast<const emb_f32x4*>(in + (size_t)j * d + c);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = fmaf(wr[q][u], x[u], acc);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) {
            const float x = acc + bias;
            out[(size_t)j * d + o] = SILU ? x / (1.f + expf(-x)) : x;
        }
    }
}

// ---------------------------------------------------------------- LayerNorm / RMSNorm
// One wave per output row (four rows per workgroup), the row held in registers as 16-byte pieces
// (d % 4 == 0, d <= 64 * 4 * kNormPieces); reductions by lane shuffles only, no LDS and no barrier.
constexpr int kNormPieces = 32;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float norm_f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 norm_bf16x4;
template <typename T, int P>
__global__ __launch_bounds__(256) void k_norm(const float* __restrict__ h, const int32_t* __restrict__ idx,
                                              const float* __restrict__ gain, const float* __restrict__ bias,
                                              T* __restrict__ out, int rows, int d, float eps) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= rows) return;
    const float* x = h + (size_t)(idx ? idx[r] : r) * d;
    const int n4 = d >> 2;
    norm_f32x4 v[P];
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = lane + 64 * p;
        if (c < n4) {
            v[p] = *reinterpret_cast<const norm_f32x4*>(x + 4 * c);
            s += (v[p][0] + v[p][1]) + (v[p][2] + v[p][3]);
        }
    }
    auto wsum = [](float a) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
        return a;
    };
    float mean = 0.f;
    if (bias) mean = wsum(s) / (float)d;           // LayerNorm centres; RMSNorm does not
    float ss = 0.f;
#pragma unroll
    for (int p = 0; p < P; ++p)
        if (lane + 64 * p < n4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) { const float t = v[p][u] - mean; ss = fmaf(t, t, ss); }
        }
    const float rstd = rsqrtf(wsum(ss) / (float)d + eps);
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = lane + 64 * p;
        if (c < n4) {
            const norm_f32x4 g = *reinterpret_cast<const norm_f32x4*>(gain + 4 * c);
            norm_f32x4 y;
#pragma unroll
            for (int u = 0; u < 4; ++u) y[u] = (v[p][u] - mean) * rstd * g[u];
            if (bias) {
                const norm_f32x4 b = *reinterpret_cast<const norm_f32x4*>(bias + 4 * c);
#pragma unroll
                for (int u = 0; u < 4; ++u) y[u] += b[u];
            }
            T* o = out + (size_t)r * d + 4 * c;
            if constexpr (sizeof(T) == 2) {
                norm_bf16x4 pk;
#pragma unroll
                for (int u = 0; u < 4; ++u) pk[u] = static_cast<bf16_t>(y[u]);
                *reinterpret_cast<norm_bf16x4*>(o) = pk;
            } else {
                *reinterpret_cast<norm_f32x4*>(o) = y;
            }
        }
    }
}

// ---------------------------------------------------------------- rotary embedding (llama)
// One thread per (row, head, pair): rotates (x_i, x_{i+dh/2}) of q and k by pos * theta^(-2i/dh).
template <typename T>
__global__ __launch_bounds__(256) void k_rope(T* __restrict__ qkv, const int32_t* __restrict__ pos, int rows,
                                              int n_head, int n_kv_head, int d_head, float theta) {
    const int half = d_head / 2;
    const int heads = n_head + n_kv_head;          // q heads then k heads are contiguous in a qkv row
    const long total = (long)rows * heads * half;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const int i = (int)(t % half);
    const int hd = (int)((t / half) % heads);
    const int r = (int)(t / ((long)half * heads));
    const int ld = (n_head + 2 * n_kv_head) * d_head;
    T* x = qkv + (size_t)r * ld + (size_t)hd * d_head;
    const double inv = exp(-log((double)theta) * 2.0 * (double)i / (double)d_head);
    const double ang = (double)pos[r] * inv;
    const float c = (float)cos(ang), s = (float)sin(ang);
    const float a = to_f(x[i]), b = to_f(x[i + half]);
    x[i] = from_f<T>(a * c - b * s);
    x[i + half] = from_f<T>(b * c + a * s);
}

// (cos, sin) of pos[r] * theta^(-2 i / d_head), the arithmetic of k_rope; one thread per (row, pair).
__global__ __launch_bounds__(256) void k_rope_table(const int32_t* __restrict__ pos, int rows, int d_head, float theta,
                                                    float* __restrict__ cs) {
    const int half = d_head / 2;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= rows * half) return;
    const int i = t % half, r = t / half;
    const double inv = exp(-log((double)theta) * 2.0 * (double)i / (double)d_head);
    const double ang = (double)pos[r] * inv;
    cs[2 * t + 0] = (float)cos(ang);
    cs[2 * t + 1] = (float)sin(ang);
}

// Rotary embedding and KV-cache append in one pass over the qkv rows (the causal Llama-shaped target): q is rotated
// in place, k is rotated on its way into the cache (and in place), v is copied.  Thread -> one (i, i + d_head/2)
// pair of one head of one row; the arithmetic is that of k_rope.
template <typename T>
__global__ __launch_bounds__(256) void k_rope_kv_store(T* __restrict__ qkv, const int32_t* __restrict__ seq,
                                                       const int32_t* __restrict__ pos, T* __restrict__ kc, T* __restrict__ vc,
                                                       int rows, int n_head, int n_kv_head, int d_head, float theta, int n_ctx) {
    const int half = d_head / 2;
    const int heads = n_head + 2 * n_kv_head;      // q heads, k heads, v heads of a qkv row
    const long total = (long)rows * heads * half;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const int i = (int)(t % half);
    const int hd = (int)((t / half) % heads);
    const int r = (int)(t / ((long)half * heads));
    const int dkv = n_kv_head * d_head;
    T* x = qkv + (size_t)r * ((size_t)heads * d_head) + (size_t)hd * d_head;
    const int p = pos[r];
    const size_t o = ((size_t)seq[r] * n_ctx + p) * dkv;
    if (hd >= n_head + n_kv_head) {                // v: copy
        T* dst = vc + o + (size_t)(hd - n_head - n_kv_head) * d_head;
        dst[i] = x[i];
        dst[i + half] = x[i + half];
        return;
    }
    const double inv = exp(-log((double)theta) * 2.0 * (double)i / (double)d_head);
    const double ang = (double)p * inv;
    const float c = (float)cos(ang), s = (float)sin(ang);
    const float a = to_f(x[i]), b = to_f(x[i + half]);
    const T lo = from_f<T>(a * c - b * s), hi = from_f<T>(b * c + a * s);
    x[i] = lo;
    x[i + half] = hi;
    if (hd >= n_head) {                            // k: also into the cache
        T* dst = kc + o + (size_t)(hd - n_head) * d_head;
        dst[i] = lo;
        dst[i + half] = hi;
    }
}

// ---------------------------------------------------------------- KV-cache append
// cache layout [max_batch, n_ctx, n_kv_head * d_head]; one workgroup per row.
template <typename T>
__global__ __launch_bounds__(256) void k_kv_store(const T* __restrict__ qkv, const int32_t* __restrict__ seq,
                                                  const int32_t* __restrict__ pos, T* __restrict__ kc,
                                                  T* __restrict__ vc, int dq, int dkv, int n_ctx) {
    const int r = blockIdx.x;
    const T* k = qkv + (size_t)r * (dq + 2 * dkv) + dq;
    const T* v = k + dkv;
    const size_t o = ((size_t)seq[r] * n_ctx + pos[r]) * dkv;
    for (int i = threadIdx.x; i < dkv; i += blockDim.x) {
        kc[o + i] = k[i];
        vc[o + i] = v[i];
    }
}

// ---------------------------------------------------------------- SwiGLU gate
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu(const T* __restrict__ gu, T* __restrict__ act, long total, int F) {
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const long r = t / F;
    const int c = (int)(t % F);
    const float g = to_f(gu[r * 2 * F + c]), u = to_f(gu[r * 2 * F + F + c]);
    act[t] = from_f<T>(g / (1.f + expf(-g)) * u);
}

// ---------------------------------------------------------------- launchers
#define SD_DISPATCH(dtype, CALL)                   \
    if ((dtype) == SD_DTYPE_F32) { using T = float; CALL; } else { using T = bf16_t; CALL; }

hipError_t launch_embed(int dtype, const int32_t* src, const int32_t* pos, const int32_t* prefix,
                        const int32_t* block, const void* wte, const void* wpe, const float* temb, float* h,
                        int rows, int d, const float* gain, void* xg, float* stats, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    if (d % 4) return hipErrorInvalidValue;
    SD_DISPATCH(dtype, (launch_kernel(k_embed<T>, dim3((rows + 3) / 4), dim3(256), 0, st, src, pos, prefix, block, (const T*)wte, (const T*)wpe, temb, h,
                                                                 rows, d, gain, (bf16_t*)xg, stats)));
    return hipGetLastError();
}

hipError_t launch_norm_prep(const float* h, const float* gain, void* xg, float* stats, int rows, int d, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    if (d % 4) return hipErrorInvalidValue;
    launch_kernel(k_norm_prep, dim3((rows + 3) / 4), dim3(256), 0, st, h, gain, (bf16_t*)xg, stats, rows, d);
    return hipGetLastError();
}

hipError_t launch_timestep_embed(int dtype, const void* w1, const float* b1, const void* w2, const float* b2,
                                 float* hidden, float* temb, int T_steps, int d, hipStream_t st) {
    if (d % 4 || d > 64 * 4 * kMatvecMax) return hipErrorInvalidValue;
    const int n_sin = T_steps * (d / 2);
    launch_kernel(k_timestep_sinusoid, dim3((n_sin + 255) / 256), dim3(256), 0, st, temb, T_steps, d);               // temb doubles as the sinusoid table
    SD_DISPATCH(dtype, (launch_kernel(k_timestep_matvec<T, true>, dim3((d + 3) / 4), dim3(256), 0, st, (const T*)w1, b1, temb, hidden, T_steps, d)));
    SD_DISPATCH(dtype, (launch_kernel(k_timestep_matvec<T, false>, dim3((d + 3) / 4), dim3(256), 0, st, (const T*)w2, b2, hidden, temb, T_steps, d)));
    return hipGetLastError();
}

hipError_t launch_norm(int dtype, const float* h, const int32_t* idx, const float* gain, const float* bias,
                       void* out, int rows, int d, float eps, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    if (d % 4 || d > 64 * 4 * kNormPieces) return hipErrorInvalidValue;
    const int pieces = (d / 4 + 63) / 64, grid = (rows + 3) / 4;
    // register-resident row: instantiate a few row lengths so that short rows do not carry 32 pieces
    if (pieces <= 4) { SD_DISPATCH(dtype, (launch_kernel(k_norm<T, 4>, dim3(grid), dim3(256), 0, st, h, idx, gain, bias, (T*)out, rows, d, eps))); }
    else if (pieces <= 8) { SD_DISPATCH(dtype, (launch_kernel(k_norm<T, 8>, dim3(grid), dim3(256), 0, st, h, idx, gain, bias, (T*)out, rows, d, eps))); }
    else if (pieces <= 16) { SD_DISPATCH(dtype, (launch_kernel(k_norm<T, 16>, dim3(grid), dim3(256), 0, st, h, idx, gain, bias, (T*)out, rows, d, eps))); }
    else { SD_DISPATCH(dtype, (launch_kernel(k_norm<T, kNormPieces>, dim3(grid), dim3(256), 0, st, h, idx, gain, bias, (T*)out, rows, d, eps))); }
    return hipGetLastError();
}

hipError_t launch_rope(int dtype, void* qkv, const int32_t* pos, int rows, int n_head, int n_kv_head, int d_head,
                       float theta, hipStream_t st) {
    const long total = (long)rows * (n_head + n_kv_head) * (d_head / 2);
    if (total <= 0) return hipSuccess;
    const int grid = (int)((total + 255) / 256);
    SD_DISPATCH(dtype, (launch_kernel(k_rope<T>, dim3(grid), dim3(256), 0, st, (T*)qkv, pos, rows, n_head, n_kv_head, d_head, theta)));
    return hipGetLastError();
}

hipError_t launch_rope_table(const int32_t* pos, int rows, int d_head, float theta, float* cs, hipStream_t st) {
    const int total = rows * (d_head / 2);
    if (total <= 0) return hipSuccess;
    launch_kernel(k_rope_table, dim3((total + 255) / 256), dim3(256), 0, st, pos, rows, d_head, theta, cs);
    return hipGetLastError();
}

hipError_t launch_rope_kv_store(int dtype, void* qkv, const int32_t* seq, const int32_t* pos, void* kcache, void* vcache,
                                int rows, int n_head, int n_kv_head, int d_head, float theta, int n_ctx, hipStream_t st) {
    const long total = (long)rows * (n_head + 2 * n_kv_head) * (d_head / 2);
    if (total <= 0) return hipSuccess;
    const int grid = (int)((total + 255) / 256);
    SD_DISPATCH(dtype, (launch_kernel(k_rope_kv_store<T>, dim3(grid), dim3(256), 0, st, (T*)qkv, seq, pos, (T*)kcache, (T*)vcache, rows, n_head, n_kv_head, d_head, theta, n_ctx)));
    return hipGetLastError();
}

hipError_t launch_kv_store(int dtype, const void* qkv, const int32_t* seq, const int32_t* pos, void* kcache,
                           void* vcache, int rows, int n_head, int n_kv_head, int d_head, int n_ctx, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    SD_DISPATCH(dtype, (launch_kernel(k_kv_store<T>, dim3(rows), dim3(256), 0, st, (const T*)qkv, seq, pos, (T*)kcache, (T*)vcache, n_head * d_head, n_kv_head * d_head, n_ctx)));
    return hipGetLastError();
}

hipError_t launch_swiglu(int dtype, const void* gu, void* act, int rows, int F, hipStream_t st) {
    const long total = (long)rows * F;
    if (total <= 0) return hipSuccess;
    const int grid = (int)((total + 255) / 256);
    SD_DISPATCH(dtype, (launch_kernel(k_swiglu<T>, dim3(grid), dim3(256), 0, st, (const T*)gu, (T*)act, total, F)));
    return hipGetLastError();
}

}  // namespace sd
