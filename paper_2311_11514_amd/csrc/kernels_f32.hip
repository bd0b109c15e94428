// fp32 stage path: plain row-major layouts and vector-ALU kernels.  It exists for the small
// full-precision configuration (tight 1e-4 parity, identical greedy tokens); the whole model sits in
// cache there, so these kernels are written for clarity and exact fp32 accumulation, not for a roofline.
#include "kernels.h"

__global__ __launch_bounds__(256) void f32_rmsnorm_kernel(const float *__restrict__ in, const float *__restrict__ g,
                                                         float *__restrict__ out, int H, float eps) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    float ss = 0.f;
    for (int c = threadIdx.x; c < H; c += 256) { float x = in[(size_t)t * H + c]; ss += x * x; }
    ss = block_sum_256(ss, red);
    const float rstd = 1.0f / sqrtf(ss / (float)H + eps);
    for (int c = threadIdx.x; c < H; c += 256) out[(size_t)t * H + c] = in[(size_t)t * H + c] * rstd * g[c];
}
void f32_launch_rmsnorm(const float *in, const float *g, float *out, int T, int H, float eps, hipStream_t s) {
    if (T <= 0) return;
    hipLaunchKernelGGL(f32_rmsnorm_kernel, dim3(T), dim3(256), 0, s, in, g, out, H, eps);
}

// out[T][N] = X[T][K] . W[K][N]; 64 x 64 block tile, 16-deep k steps through LDS, 4 x 4 per thread.
__global__ __launch_bounds__(256) void f32_gemm_kernel(const float *__restrict__ X, const float *__restrict__ W,
                                                      float *__restrict__ out, int T, int K, int N) {
    __shared__ float sX[16][64 + 1];
    __shared__ float sW[16][64 + 1];
    const int bt = blockIdx.y * 64, bn = blockIdx.x * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int kk = e & 15, r = e >> 4;          // X: consecutive threads walk k (contiguous)
            const int t = bt + r, k = k0 + kk;
            sX[kk][r] = (t < T && k < K) ? X[(size_t)t * K + k] : 0.f;
            const int c = e & 63, kw = e >> 6;          // W: consecutive threads walk n (contiguous)
            const int n = bn + c, k2 = k0 + kw;
            sW[kw][c] = (n < N && k2 < K) ? W[(size_t)k2 * N + n] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sX[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = sW[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = bt + ty * 4 + i;
        if (t >= T) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = bn + tx * 4 + j;
            if (n < N) out[(size_t)t * N + n] = acc[i][j];
        }
    }
}
void f32_launch_gemm(const float *X, const float *W, float *out, int T, int K, int N, hipStream_t s) {
    if (T <= 0 || N <= 0) return;
    hipLaunchKernelGGL(f32_gemm_kernel, dim3((N + 63) / 64, (T + 63) / 64), dim3(256), 0, s, X, W, out, T, K, N);
}

// cache layout per layer: [seq][hkv_l][smax][d]
__global__ void f32_rope_append_kernel(const float *__restrict__ qkv, int hq_l, int hkv_l, int d, int smax, RowMap rm,
                                       const float *__restrict__ cos_tab, const float *__restrict__ sin_tab,
                                       float *__restrict__ q_out, float *__restrict__ kc, float *__restrict__ vc) {
    const int t = blockIdx.x, head = blockIdx.y, i = threadIdx.x, half = d >> 1;
    const int N = (hq_l + 2 * hkv_l) * d;
    float lo = qkv[(size_t)t * N + head * d + i], hi = qkv[(size_t)t * N + head * d + i + half];
    const int seq = rm.row_seq[t], pos = rm.row_pos[t];
    if (head < hq_l + hkv_l) {
        const float c = cos_tab[(size_t)pos * half + i], sn = sin_tab[(size_t)pos * half + i];
        const float rlo = lo * c - hi * sn, rhi = hi * c + lo * sn;
        lo = rlo; hi = rhi;
    }
    float *dst;
    if (head < hq_l) dst = q_out + ((size_t)t * hq_l + head) * d;
    else if (head < hq_l + hkv_l) dst = kc + (((size_t)seq * hkv_l + (head - hq_l)) * smax + pos) * d;
    else dst = vc + (((size_t)seq * hkv_l + (head - hq_l - hkv_l)) * smax + pos) * d;
    dst[i] = lo;
    dst[i + half] = hi;
}
void f32_launch_rope_append(const float *qkv, int T, int hq_l, int hkv_l, int d, int smax, RowMap rm,
                            const float *cos_tab, const float *sin_tab, float *q_out, float *kc, float *vc,
                            hipStream_t s) {
    if (T <= 0) return;
    hipLaunchKernelGGL(f32_rope_append_kernel, dim3(T, hq_l + 2 * hkv_l), dim3(d / 2), 0, s, qkv, hq_l, hkv_l, d, smax,
                       rm, cos_tab, sin_tab, q_out, kc, vc);
}

// one block per (row, query head): scores of positions 0..pos in LDS, softmax, weighted V sum
__global__ __launch_bounds__(256) void f32_attn_kernel(const float *__restrict__ q, const float *__restrict__ kc,
                                                      const float *__restrict__ vc, int hq_l, int hkv_l, int d,
                                                      int smax, RowMap rm, float *__restrict__ o) {
    extern __shared__ float sc[];     // [smax] scores, then [256] partial sums
    __shared__ float red[4];
    __shared__ float sq[128];
    const int t = blockIdx.x, head = blockIdx.y;
    const int seq = rm.row_seq[t], pos = rm.row_pos[t];
    const int G = hq_l / hkv_l, c = head / G;
    const float *K = kc + ((size_t)seq * hkv_l + c) * smax * d;
    const float *V = vc + ((size_t)seq * hkv_l + c) * smax * d;
    if (threadIdx.x < d) sq[threadIdx.x] = q[((size_t)t * hq_l + head) * d + threadIdx.x];
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int p = threadIdx.x; p <= pos; p += 256) {
        float s = 0.f;
        for (int e = 0; e < d; ++e) s = fmaf(K[(size_t)p * d + e], sq[e], s);
        s *= scale;
        sc[p] = s;
        mx = fmaxf(mx, s);
    }
    mx = block_max_256(mx, red);
    float sum = 0.f;
    for (int p = threadIdx.x; p <= pos; p += 256) { float w = expf(sc[p] - mx); sc[p] = w; sum += w; }
    sum = block_sum_256(sum, red);
    // thread (e = tid % d, slice = tid / d) sums its slice of positions; slices are added in order
    const int e = threadIdx.x % d, slice = threadIdx.x / d, nslice = 256 / d;
    float acc = 0.f;
    for (int p = slice; p <= pos; p += nslice) acc = fmaf(sc[p], V[(size_t)p * d + e], acc);
    float *ps = sc + smax;
    ps[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < d) {
        float tot = 0.f;
        for (int sl = 0; sl < nslice; ++sl) tot += ps[sl * d + threadIdx.x];
        o[((size_t)t * hq_l + head) * d + threadIdx.x] = tot / sum;
    }
}
void f32_launch_attn(const float *q, const float *kc, const float *vc, int T, int hq_l, int hkv_l, int d, int smax,
                     RowMap rm, float *o, hipStream_t s) {
    if (T <= 0) return;
    size_t shm = (size_t)(smax + 256) * sizeof(float);
    hipLaunchKernelGGL(f32_attn_kernel, dim3(T, hq_l), dim3(256), shm, s, q, kc, vc, hq_l, hkv_l, d, smax, rm, o);
}

// ab = [T][2*F_l] with W1 columns then W3 columns
__global__ void f32_swiglu_kernel(const float *__restrict__ ab, float *__restrict__ u, int T, int F_l) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)T * F_l) return;
    const int t = (int)(i / F_l), f = (int)(i % F_l);
    const float a = ab[(size_t)t * 2 * F_l + f], b = ab[(size_t)t * 2 * F_l + F_l + f];
    u[i] = a / (1.0f + expf(-a)) * b;
}
void f32_launch_swiglu(const float *ab, float *u, int T, int F_l, hipStream_t s) {
    int64_t n = (int64_t)T * F_l;
    if (n <= 0) return;
    hipLaunchKernelGGL(f32_swiglu_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ab, u, T, F_l);
}

// staging [n][hkv_l][d] <-> cache rows pos0.. of sequence seq
__global__ void f32_kv_copy_kernel(float *kc, float *vc, float *k, float *v, int hkv_l, int d, int smax, int seq,
                                   int pos0, int n, int to_cache) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)n * hkv_l * d) return;
    const int e = (int)(i % d), c = (int)((i / d) % hkv_l), p = pos0 + (int)(i / ((int64_t)d * hkv_l));
    const size_t o = (((size_t)seq * hkv_l + c) * smax + p) * d + e;
    if (to_cache) { kc[o] = k[i]; vc[o] = v[i]; } else { k[i] = kc[o]; v[i] = vc[o]; }
}
void f32_launch_kv_copy(float *kc, float *vc, float *k, float *v, int hkv_l, int d, int smax, int seq, int pos0,
                        int n, int to_cache, hipStream_t s) {
    int64_t tot = (int64_t)n * hkv_l * d;
    if (tot <= 0) return;
    hipLaunchKernelGGL(f32_kv_copy_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, kc, vc, k, v, hkv_l, d,
                       smax, seq, pos0, n, to_cache);
}
