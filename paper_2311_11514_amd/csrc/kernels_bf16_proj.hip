// bf16 projections of the prefill path: RMSNorm fused with the cast into the GEMM operand layout, the
// epilogue kernels of the MFMA GEMM (kernels_bf16_gemm.hip) (RoPE + cache append, residual + next norm, SwiGLU).
// The decode path (T <= 32 rows) lives in kernels_bf16_decode.hip.
//
// Every contraction is computed "transposed": D^T[n][t] = sum_k Wp[n][k] * Xp[t][k] with the weight
// tile as MFMA operand A and the activation tile as operand B.  In the 16x16 result each lane then
// owns 4 consecutive output features of one token, which is exactly a 16-byte (fp32) or 8-byte
// (bf16) piece of the next operand -- no shuffle between one GEMM's output and the next one's input.
#include "kernels.h"
#include "kvlayout.h"

// -------------------------------------------------------------------------------------------------
// RMSNorm (+ optional fp32 copy of the input) -> packed bf16.  One 256-thread block per row.
// -------------------------------------------------------------------------------------------------
template <bool IN_BF16>
__global__ __launch_bounds__(256) void rmsnorm_pack_kernel(const void *__restrict__ in, float *__restrict__ h_out,
                                                          const float *__restrict__ g, bf16_t *__restrict__ np,
                                                          bf16_t *__restrict__ np_lo, int H, float eps) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    const int chunks = H >> 3;
    float ss = 0.f;
    for (int c = threadIdx.x; c < chunks; c += 256) {
        float x[8];
        if (IN_BF16) {
            uint4 raw = *reinterpret_cast<const uint4 *>(reinterpret_cast<const bf16_t *>(in) + (size_t)t * H + c * 8);
            const bf16_t *e = reinterpret_cast<const bf16_t *>(&raw);
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = bf16_to_f32(e[j]);
        } else {
            const float4 *p = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(in) + (size_t)t * H + c * 8);
            float4 a = p[0], b = p[1];
            x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += x[j] * x[j];
        if (h_out) {
            float4 *o = reinterpret_cast<float4 *>(h_out + (size_t)t * H + c * 8);
            o[0] = make_float4(x[0], x[1], x[2], x[3]);
            o[1] = make_float4(x[4], x[5], x[6], x[7]);
        }
    }
    ss = block_sum_256(ss, red);
    const float rstd = 1.0f / sqrtf(ss / (float)H + eps);
    const int k_tiles = H >> 5;
    for (int c = threadIdx.x; c < chunks; c += 256) {
        float x[8];
        if (IN_BF16) {
            uint4 raw = *reinterpret_cast<const uint4 *>(reinterpret_cast<const bf16_t *>(in) + (size_t)t * H + c * 8);
            const bf16_t *e = reinterpret_cast<const bf16_t *>(&raw);
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = bf16_to_f32(e[j]);
        } else {
            const float4 *p = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(in) + (size_t)t * H + c * 8);
            float4 a = p[0], b = p[1];
            x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        }
        const float4 *gp = reinterpret_cast<const float4 *>(g + c * 8);
        float4 g0 = gp[0], g1 = gp[1];
        uint4 o, ol;
        split_pack2(x[0] * rstd * g0.x, x[1] * rstd * g0.y, o.x, ol.x);
        split_pack2(x[2] * rstd * g0.z, x[3] * rstd * g0.w, o.y, ol.y);
        split_pack2(x[4] * rstd * g1.x, x[5] * rstd * g1.y, o.z, ol.z);
        split_pack2(x[6] * rstd * g1.z, x[7] * rstd * g1.w, o.w, ol.w);
        const size_t off = frag_offset(t, c * 8, k_tiles);
        *reinterpret_cast<uint4 *>(np + off) = o;
        if (np_lo) *reinterpret_cast<uint4 *>(np_lo + off) = ol;
    }
}

void launch_rmsnorm_pack(const void *in, int in_is_bf16, float *h_out, const float *g, bf16_t *n_packed,
                         bf16_t *n_lo, int T, int H, float eps, hipStream_t s) {
    if (T <= 0) return;
    if (in_is_bf16)
        hipLaunchKernelGGL(rmsnorm_pack_kernel<true>, dim3(T), dim3(256), 0, s, in, h_out, g, n_packed, n_lo, H, eps);
    else
        hipLaunchKernelGGL(rmsnorm_pack_kernel<false>, dim3(T), dim3(256), 0, s, in, h_out, g, n_packed, n_lo, H, eps);
}

// -------------------------------------------------------------------------------------------------
// Epilogues.  `part` is [ksplit][T][N] fp32; partials are always summed in split order.
// -------------------------------------------------------------------------------------------------
// grid (T, hq_l + 2*hkv_l), block d/2: thread i owns the rotary pair (i, i + d/2) of one head.
__global__ void qkv_rope_append_kernel(const float *__restrict__ part, int ksplit, int T, int hq_l, KvGeom kg,
                                       RowMap rm, const float *__restrict__ cos_tab,
                                       const float *__restrict__ sin_tab, bf16_t *__restrict__ q_out,
                                       bf16_t *__restrict__ q_lo, bf16_t *__restrict__ kc,
                                       bf16_t *__restrict__ vc) {
    const int t = blockIdx.x, head = blockIdx.y, i = threadIdx.x;
    const int d = kg.d, half = d >> 1;
    const int N = (hq_l + 2 * kg.hkv_l) * d;
    // projection output columns are rope-interleaved: pair (i, i + d/2) sits at (8 apart) in one tile
    const int col = head * d + (i >> 3) * 16 + (i & 7);
    float lo = 0.f, hi = 0.f;
    for (int ks = 0; ks < ksplit; ++ks) {
        const float *p = part + ((size_t)ks * T + t) * N + col;
        lo += p[0];
        hi += p[8];
    }
    const int seq = rm.row_seq[t], pos = rm.row_pos[t];
    if (head < hq_l + kg.hkv_l) {
        const float c = cos_tab[(size_t)pos * half + i], sn = sin_tab[(size_t)pos * half + i];
        const float rlo = lo * c - hi * sn, rhi = hi * c + lo * sn;
        lo = rlo; hi = rhi;
    }
    if (head < hq_l) {
        const size_t qo = (size_t)t * hq_l * d + head * d;
        bf16_t a_hi, a_lo, b_hi, b_lo;
        split_bf16(lo, a_hi, a_lo);
        split_bf16(hi, b_hi, b_lo);
        q_out[qo + i] = a_hi;
        q_out[qo + i + half] = b_hi;
        if (q_lo) { q_lo[qo + i] = a_lo; q_lo[qo + i + half] = b_lo; }
    } else {
        const bool is_k = head < hq_l + kg.hkv_l;
        const int c = is_k ? head - hq_l : head - hq_l - kg.hkv_l;
        const size_t slab = (size_t)seq * kg.seq_stride + (size_t)c * kg.smax * d;
        if (is_k) {
            kc[slab + kv_k_offset(pos, i, d)] = f32_to_bf16(lo);
            kc[slab + kv_k_offset(pos, i + half, d)] = f32_to_bf16(hi);
        } else {
            vc[slab + kv_v_offset(pos, i, d)] = f32_to_bf16(lo);
            vc[slab + kv_v_offset(pos, i + half, d)] = f32_to_bf16(hi);
        }
    }
}
void launch_qkv_rope_append(const float *part, int ksplit, int T, int hq_l, KvGeom kg, RowMap rm,
                            const float *cos_tab, const float *sin_tab, bf16_t *q_out, bf16_t *q_lo, bf16_t *kc,
                            bf16_t *vc, hipStream_t s) {
    if (T <= 0) return;
    hipLaunchKernelGGL(qkv_rope_append_kernel, dim3(T, hq_l + 2 * kg.hkv_l), dim3(kg.d / 2), 0, s, part, ksplit, T,
                       hq_l, kg, rm, cos_tab, sin_tab, q_out, q_lo, kc, vc);
}

// one block per row: h += sum of partials; optional RMSNorm of the new h into packed bf16
__global__ __launch_bounds__(256) void reduce_resid_norm_kernel(const float *__restrict__ part, int ksplit,
                                                               float *__restrict__ h, const float *__restrict__ g,
                                                               bf16_t *__restrict__ np, bf16_t *__restrict__ np_lo,
                                                               int T, int H, float eps) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    const int quads = H >> 2;
    float ss = 0.f;
    for (int c = threadIdx.x; c < quads; c += 256) {
        float4 v = *reinterpret_cast<const float4 *>(h + (size_t)t * H + c * 4);
        for (int ks = 0; ks < ksplit; ++ks) {
            float4 p = *reinterpret_cast<const float4 *>(part + ((size_t)ks * T + t) * H + c * 4);
            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        }
        *reinterpret_cast<float4 *>(h + (size_t)t * H + c * 4) = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    if (g == nullptr) return;
    ss = block_sum_256(ss, red);   // the barrier inside also orders the h writes above
    const float rstd = 1.0f / sqrtf(ss / (float)H + eps);
    const int k_tiles = H >> 5, chunks = H >> 3;
    for (int c = threadIdx.x; c < chunks; c += 256) {
        const float4 *p = reinterpret_cast<const float4 *>(h + (size_t)t * H + c * 8);
        float4 a = p[0], b = p[1];
        const float4 *gp = reinterpret_cast<const float4 *>(g + c * 8);
        float4 g0 = gp[0], g1 = gp[1];
        uint4 o, ol;
        split_pack2(a.x * rstd * g0.x, a.y * rstd * g0.y, o.x, ol.x);
        split_pack2(a.z * rstd * g0.z, a.w * rstd * g0.w, o.y, ol.y);
        split_pack2(b.x * rstd * g1.x, b.y * rstd * g1.y, o.z, ol.z);
        split_pack2(b.z * rstd * g1.z, b.w * rstd * g1.w, o.w, ol.w);
        const size_t off = frag_offset(t, c * 8, k_tiles);
        *reinterpret_cast<uint4 *>(np + off) = o;
        if (np_lo) *reinterpret_cast<uint4 *>(np_lo + off) = ol;
    }
}
void launch_reduce_resid_norm(const float *part, int ksplit, float *h, const float *g, bf16_t *n_packed,
                              bf16_t *n_lo, int T, int H, float eps, hipStream_t s) {
    if (T <= 0) return;
    hipLaunchKernelGGL(reduce_resid_norm_kernel, dim3(T), dim3(256), 0, s, part, ksplit, h, g, n_packed, n_lo, T, H,
                       eps);
}

__global__ void reduce_partial_kernel(const float *__restrict__ part, int ksplit, float *__restrict__ dst,
                                      int64_t TH) {
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= TH) return;
    float4 v = *reinterpret_cast<const float4 *>(part + i);
    for (int ks = 1; ks < ksplit; ++ks) {
        float4 p = *reinterpret_cast<const float4 *>(part + (size_t)ks * TH + i);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    *reinterpret_cast<float4 *>(dst + i) = v;
}
void launch_reduce_partial(const float *part, int ksplit, float *dst, int T, int H, hipStream_t s) {
    int64_t TH = (int64_t)T * H;
    if (TH <= 0) return;
    hipLaunchKernelGGL(reduce_partial_kernel, dim3((unsigned)((TH / 4 + 255) / 256)), dim3(256), 0, s, part, ksplit,
                       dst, TH);
}

// The W1/W3 projection output interleaves 16-column tiles: tile 2i = W1 (gate) columns 16i..16i+15,
// tile 2i+1 = W3 (up) columns of the same range.  One thread produces 8 consecutive u values.
__global__ void reduce_swiglu_kernel(const float *__restrict__ part, int ksplit, bf16_t *__restrict__ up,
                                     bf16_t *__restrict__ up_lo, int T, int F_l) {
    const int t = blockIdx.x;
    const int chunk = blockIdx.y * blockDim.x + threadIdx.x;
    if (chunk >= (F_l >> 3)) return;
    const int f0 = chunk * 8;
    const int N = 2 * F_l;
    const int ca = (f0 >> 4) * 32 + (f0 & 15);
    float a[8], b[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { a[j] = 0.f; b[j] = 0.f; }
    for (int ks = 0; ks < ksplit; ++ks) {
        const float4 *pa = reinterpret_cast<const float4 *>(part + ((size_t)ks * T + t) * N + ca);
        const float4 *pb = reinterpret_cast<const float4 *>(part + ((size_t)ks * T + t) * N + ca + 16);
        float4 a0 = pa[0], a1 = pa[1], b0 = pb[0], b1 = pb[1];
        a[0] += a0.x; a[1] += a0.y; a[2] += a0.z; a[3] += a0.w; a[4] += a1.x; a[5] += a1.y; a[6] += a1.z; a[7] += a1.w;
        b[0] += b0.x; b[1] += b0.y; b[2] += b0.z; b[3] += b0.w; b[4] += b1.x; b[5] += b1.y; b[6] += b1.z; b[7] += b1.w;
    }
    float u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) u[j] = a[j] / (1.0f + __expf(-a[j])) * b[j];
    uint4 o, ol;
    split_pack2(u[0], u[1], o.x, ol.x); split_pack2(u[2], u[3], o.y, ol.y);
    split_pack2(u[4], u[5], o.z, ol.z); split_pack2(u[6], u[7], o.w, ol.w);
    const size_t off = frag_offset(t, f0, F_l >> 5);
    *reinterpret_cast<uint4 *>(up + off) = o;
    if (up_lo) *reinterpret_cast<uint4 *>(up_lo + off) = ol;
}
void launch_reduce_swiglu(const float *part, int ksplit, bf16_t *u_packed, bf16_t *u_lo, int T, int F_l,
                          hipStream_t s) {
    if (T <= 0) return;
    const int chunks = F_l >> 3;
    hipLaunchKernelGGL(reduce_swiglu_kernel, dim3(T, (chunks + 255) / 256), dim3(256), 0, s, part, ksplit, u_packed,
                       u_lo, T, F_l);
}
