// Element-type conversions at the library's edges: norm gains to fp32, cache rows <-> fp32 staging.
// Compiled once per 16-bit element type (see common.h) into namespace HX_NS.
#include "kernels.h"
#include "kvlayout.h"

namespace HX_NS {

__global__ void cvt_h16_to_f32_kernel(const h16_t *__restrict__ src, float *__restrict__ dst, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = h16_to_f32(src[i]);
}
void launch_cvt_h16_to_f32(const h16_t *src, float *dst, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    hipLaunchKernelGGL(cvt_h16_to_f32_kernel, dim3(blocks), dim3(256), 0, s, src, dst, n);
}

// staging [n][hkv_l][d] fp32  <->  packed cache slabs of sequence `seq`
__global__ void kv_scatter_kernel(const float *__restrict__ k, const float *__restrict__ v, h16_t *__restrict__ kc,
                                  h16_t *__restrict__ vc, KvGeom kg, int seq, int pos0, int n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)n * kg.hkv_l * kg.d;
    if (i >= total) return;
    int dd = (int)(i % kg.d);
    int c = (int)((i / kg.d) % kg.hkv_l);
    int p = pos0 + (int)(i / ((int64_t)kg.d * kg.hkv_l));
    size_t slab = (size_t)seq * kg.seq_stride + (size_t)c * kg.smax * kg.d;
    kc[slab + kv_k_offset(p, dd, kg.d)] = f32_to_h16(k[i]);
    vc[slab + kv_v_offset(p, dd, kg.d)] = f32_to_h16(v[i]);
}
void launch_kv_scatter(const float *k, const float *v, h16_t *kc, h16_t *vc, KvGeom kg, int seq, int pos0,
                       int n, hipStream_t s) {
    int64_t total = (int64_t)n * kg.hkv_l * kg.d;
    if (total <= 0) return;
    hipLaunchKernelGGL(kv_scatter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, k, v, kc, vc, kg,
                       seq, pos0, n);
}
__global__ void kv_gather_kernel(const h16_t *__restrict__ kc, const h16_t *__restrict__ vc, KvGeom kg, int seq,
                                 int pos0, int n, float *__restrict__ k, float *__restrict__ v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)n * kg.hkv_l * kg.d;
    if (i >= total) return;
    int dd = (int)(i % kg.d);
    int c = (int)((i / kg.d) % kg.hkv_l);
    int p = pos0 + (int)(i / ((int64_t)kg.d * kg.hkv_l));
    size_t slab = (size_t)seq * kg.seq_stride + (size_t)c * kg.smax * kg.d;
    k[i] = h16_to_f32(kc[slab + kv_k_offset(p, dd, kg.d)]);
    v[i] = h16_to_f32(vc[slab + kv_v_offset(p, dd, kg.d)]);
}
void launch_kv_gather(const h16_t *kc, const h16_t *vc, KvGeom kg, int seq, int pos0, int n, float *k, float *v,
                      hipStream_t s) {
    int64_t total = (int64_t)n * kg.hkv_l * kg.d;
    if (total <= 0) return;
    hipLaunchKernelGGL(kv_gather_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, kc, vc, kg, seq,
                       pos0, n, k, v);
}

}  // namespace HX_NS
