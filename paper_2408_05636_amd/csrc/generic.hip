// Storage-type-generic contraction and attention kernels on the vector ALUs.  They serve the
// fp32 workload (whose matrices are a few hundred KB and whose round is launch-latency bound)
// and are the fallback shapes of the bf16 path; the bf16 hot shapes run on the MFMA kernels.
#include "common.h"

namespace sd {

template <typename T> __device__ inline float to_f(T v) { return static_cast<float>(v); }
template <typename T> __device__ inline T from_f(float v) { return static_cast<T>(v); }

__device__ inline float gelu_tanh(float x) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.f + tanhf(u));
}

// ---------------------------------------------------------------- y = epilogue(x W^T + bias)
// 64 x 64 output tile per 256-thread workgroup, K in steps of 16 through LDS, 4 x 4 outputs per thread.
constexpr int GT = 64, GK = 16;
template <typename T>
__global__ __launch_bounds__(256) void k_linear_generic(const T* __restrict__ x, const T* __restrict__ w,
                                                        const float* __restrict__ bias, void* __restrict__ y, int m,
                                                        int n, int k, int ldy, int epi) {
    __shared__ float xs[GK][GT + 4];
    __shared__ float ws[GK][GT + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
    const int lr = tid >> 2, lk = (tid & 3) * 4;      // this thread stages row lr, k-offsets lk..lk+3
    float acc[4][4] = {};
    for (int k0 = 0; k0 < k; k0 += GK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + lk + i;
            xs[lk + i][lr] = (m0 + lr < m && kk < k) ? to_f(x[(size_t)(m0 + lr) * k + kk]) : 0.f;
            ws[lk + i][lr] = (n0 + lr < n && kk < k) ? to_f(w[(size_t)(n0 + lr) * k + kk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = xs[kk][ty * 4 + i]; b[i] = ws[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = m0 + ty * 4 + i;
        if (r >= m) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = n0 + tx * 4 + j;
            if (c >= n) continue;
            float v = acc[i][j] + (bias ? bias[c] : 0.f);
            const size_t o = (size_t)r * ldy + c;
            if (epi == EPI_STORE) static_cast<T*>(y)[o] = from_f<T>(v);
            else if (epi == EPI_GELU) static_cast<T*>(y)[o] = from_f<T>(gelu_tanh(v));
            else if (epi == EPI_RESID) static_cast<float*>(y)[o] += v;
            else static_cast<float*>(y)[o] = v;
        }
    }
}

hipError_t launch_linear_generic(int dtype, const void* x, const void* w, const float* bias, void* y, int m, int n,
                                 int k, int ldy, int epilogue, hipStream_t st) {
    if (m <= 0 || n <= 0) return hipSuccess;
    const dim3 grid((n + GT - 1) / GT, (m + GT - 1) / GT);
    if (dtype == SD_DTYPE_F32)
        launch_kernel(k_linear_generic<float>, dim3(grid), dim3(256), 0, st, (const float*)x, (const float*)w, bias, y, m, n, k, ldy, epilogue);
    else
        launch_kernel(k_linear_generic<bf16_t>, dim3(grid), dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)w, bias, y, m, n, k, ldy, epilogue);
    return hipGetLastError();
}

// ---------------------------------------------------------------- attention, one wave per (row, head)
// Pass 1: lane j computes the scores of keys j, j+64, ... into LDS; pass 2: lanes own output
// dimensions and accumulate softmax-weighted values.  d_head in {32, 64, 128}.
template <typename T>
__global__ __launch_bounds__(256) void k_attention_generic(AttnArgs a, int max_kv) {
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int dh = a.d_head;
    float* sc = smem + (size_t)wv * (max_kv + dh);
    float* qs = sc + max_kv;
    const long pair = (long)blockIdx.x * 4 + wv;
    const bool valid = pair < (long)a.rows * a.n_head;
    const int r = valid ? (int)(pair / a.n_head) : 0, hd = valid ? (int)(pair % a.n_head) : 0;
    const int g = hd / (a.n_head / a.n_kv_head);
    const int kv = valid ? a.kv_len[r] : 0;
    const T* q = static_cast<const T*>(a.q) + (size_t)r * a.q_ld + (size_t)hd * dh;
    const T* kb = static_cast<const T*>(a.k) + a.kv_off[r] + (size_t)g * dh;
    const T* vb = static_cast<const T*>(a.v) + a.kv_off[r] + (size_t)g * dh;
    const float scale = rsqrtf((float)dh);
    if (valid)
        for (int i = lane; i < dh; i += 64) qs[i] = to_f(q[i]) * scale;
    __syncthreads();
    float mx = -INFINITY;
    for (int j = lane; j < kv; j += 64) {
        const T* kr = kb + (size_t)j * a.kv_ld;
        float s = 0.f;
        for (int i = 0; i < dh; ++i) s = fmaf(qs[i], to_f(kr[i]), s);
        sc[j] = s;
        mx = fmaxf(mx, s);
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float sum = 0.f;
    for (int j = lane; j < kv; j += 64) {
        const float p = expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    __syncthreads();
    const int width = dh < 64 ? dh : 64;               // lanes that own distinct dimensions
    const int groups = 64 / width;                     // key-interleaved lane groups when dh < 64
    const int dim = lane % width, grp = lane / width;
    float acc0 = 0.f, acc1 = 0.f;
    for (int j = grp; j < kv; j += groups) {
        const float p = sc[j];
        const T* vr = vb + (size_t)j * a.kv_ld;
        acc0 = fmaf(p, to_f(vr[dim]), acc0);
        if (dh > 64) acc1 = fmaf(p, to_f(vr[dim + 64]), acc1);
    }
    for (int o = width; o < 64; o <<= 1) acc0 += __shfl_xor(acc0, o, 64);
    if (valid && grp == 0) {
        T* out = static_cast<T*>(a.out) + (size_t)r * a.out_ld + (size_t)hd * dh;
        const float inv = 1.f / sum;
        out[dim] = from_f<T>(acc0 * inv);
        if (dh > 64) out[dim + 64] = from_f<T>(acc1 * inv);
    }
}

hipError_t launch_attention_generic(int dtype, const AttnArgs& a, int max_kv, hipStream_t st) {
    const long pairs = (long)a.rows * a.n_head;
    if (pairs <= 0) return hipSuccess;
    if (a.d_head != 32 && a.d_head != 64 && a.d_head != 128) return hipErrorInvalidValue;
    const int grid = (int)((pairs + 3) / 4);
    const size_t shm = (size_t)4 * (max_kv + a.d_head) * sizeof(float);
    if (shm > 64 * 1024) return hipErrorInvalidValue;
    if (dtype == SD_DTYPE_F32) launch_kernel(k_attention_generic<float>, dim3(grid), dim3(256), shm, st, a, max_kv);
    else launch_kernel(k_attention_generic<bf16_t>, dim3(grid), dim3(256), shm, st, a, max_kv);
    return hipGetLastError();
}

}  // namespace sd
