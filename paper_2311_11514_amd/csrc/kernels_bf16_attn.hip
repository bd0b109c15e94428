// bf16 attention on the matrix cores: split-KV GQA decode attention and flash-style causal prefill
// attention.  Both compute scores transposed, S^T = K . Q^T (operand A = a K fragment of the cache,
// operand B = query rows), so one lane owns one query row / query head and 4 consecutive positions;
// softmax statistics are per lane plus two cross-lane steps; and O^T = V^T . P^T takes P straight from
// the score accumulators (see kvlayout.h for the matching V layout).
//
// Decode: the G query heads that share a KV head are the 16 columns of operand B, so every K and V
// fragment is fetched from HBM exactly once per sequence and serves the whole query group inside one
// MFMA.  The KV range of a sequence is split across blockIdx.x; partial (m, l, o) triples are merged
// by log-sum-exp in a second kernel, in split order.
#include "kernels.h"
#include "kvlayout.h"

#define NEG_INF (-INFINITY)

template <int D>
__global__ __launch_bounds__(64) void attn_decode_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ q_lo,
                                                        const bf16_t *__restrict__ kc,
                                                        const bf16_t *__restrict__ vc, KvGeom kg, int hq_l, int G,
                                                        const int32_t *__restrict__ row_pos, int nsplit,
                                                        float *__restrict__ part_o, float *__restrict__ part_ml,
                                                        float scale_log2e) {
    constexpr int KT = D / 32, DT = D / 16;
    const int split = blockIdx.x, c = blockIdx.y, sq = blockIdx.z;
    const int lane = threadIdx.x, j = lane & 15, g = lane >> 4;
    const int n_pos = row_pos[sq] + 1;   // cached context plus the row appended in this step
    const int n_t32 = (n_pos + 31) >> 5;
    const int per = (n_t32 + nsplit - 1) / nsplit;
    const int t0 = split * per, t1 = min(n_t32, t0 + per);
    const int head = c * G + j;
    const bool hv = j < G;

    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    // the query is carried as hi + lo bf16 parts (decode is HBM-bound: the second MFMA is free)
    bf16x8 qf[KT], ql[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
        const size_t qo = ((size_t)sq * hq_l + head) * D + kt * 32 + 8 * g;
        qf[kt] = hv ? *reinterpret_cast<const bf16x8 *>(q + qo) : zero;
        ql[kt] = hv ? *reinterpret_cast<const bf16x8 *>(q_lo + qo) : zero;
    }

    floatx4 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = NEG_INF, lsum = 0.f;

    const size_t slab = (size_t)sq * kg.seq_stride + (size_t)c * kg.smax * D;
    const bf16x8 *ks = reinterpret_cast<const bf16x8 *>(kc + slab) + lane;
    const bf16x8 *vs = reinterpret_cast<const bf16x8 *>(vc + slab) + lane;

    for (int t = t0; t < t1; ++t) {
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
        bf16x8 ka[KT], kb[KT], va[DT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            ka[kt] = ks[(size_t)((2 * t) * KT + kt) * 64];
            kb[kt] = ks[(size_t)((2 * t + 1) * KT + kt) * 64];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) va[dt] = vs[(size_t)(t * DT + dt) * 64];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt], ql[kt], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[kt], ql[kt], s1, 0, 0, 0);
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt], qf[kt], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[kt], qf[kt], s1, 0, 0, 0);
        }
        const int pbase = t * 32 + 4 * g;
        float mx = NEG_INF;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s0[r] = (pbase + r < n_pos) ? s0[r] * scale_log2e : NEG_INF;
            s1[r] = (pbase + 16 + r < n_pos) ? s1[r] * scale_log2e : NEG_INF;
            mx = fmaxf(mx, fmaxf(s0[r], s1[r]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);          // finite: position t*32 < n_pos is never masked
        const float alpha = exp2f(m - m_new);
        m = m_new;
        float p0[4], p1[4], ps = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p0[r] = exp2f(s0[r] - m_new);
            p1[r] = exp2f(s1[r] - m_new);
            ps += p0[r] + p1[r];
        }
        lsum = lsum * alpha + ps;
        union { uint32_t u[4]; bf16x8 v; } pb, pl;
        split_pack2(p0[0], p0[1], pb.u[0], pl.u[0]); split_pack2(p0[2], p0[3], pb.u[1], pl.u[1]);
        split_pack2(p1[0], p1[1], pb.u[2], pl.u[2]); split_pack2(p1[2], p1[3], pb.u[3], pl.u[3]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            oacc[dt] *= alpha;
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pl.v, oacc[dt], 0, 0, 0);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pb.v, oacc[dt], 0, 0, 0);
        }
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (hv) {
        const size_t e = ((size_t)sq * hq_l + head) * nsplit + split;
        if (g == 0) { part_ml[e * 2] = m; part_ml[e * 2 + 1] = lsum; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            *reinterpret_cast<floatx4 *>(part_o + e * D + dt * 16 + 4 * g) = oacc[dt];
    }
}

// grid (b, hq_l), block D threads: log-sum-exp merge in split order -> packed bf16 o
template <int D>
__global__ void attn_decode_merge_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                         int hq_l, int nsplit, bf16_t *__restrict__ o_act) {
    const int sq = blockIdx.x, head = blockIdx.y, dd = threadIdx.x;
    const size_t e0 = ((size_t)sq * hq_l + head) * nsplit;
    float M = NEG_INF;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part_ml[(e0 + s) * 2]);
    float L = 0.f, o = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float ms = part_ml[(e0 + s) * 2];
        const float w = (ms == NEG_INF) ? 0.f : exp2f(ms - M);
        L += part_ml[(e0 + s) * 2 + 1] * w;
        o += part_o[(e0 + s) * D + dd] * w;
    }
    bf16_t hi, lo;
    split_bf16(o / L, hi, lo);
    const size_t off = dec_act_offset(sq, head * D + dd, (hq_l * D) >> 5, 0);
    o_act[off] = hi;
    o_act[off + 32] = lo;
}

// Single-kernel variant: one 8-wave block per (sequence, kv head); the waves interleave over the
// 32-position tiles of the context and their (m, l, o) triples are merged through LDS in wave order.
// Used when there are enough (sequence, kv head) pairs to fill the chip or the context is short.
template <int D>
__global__ __launch_bounds__(512) void attn_decode_block_kernel(const bf16_t *__restrict__ q,
                                                               const bf16_t *__restrict__ q_lo,
                                                               const bf16_t *__restrict__ kc,
                                                               const bf16_t *__restrict__ vc, KvGeom kg, int hq_l, int G,
                                                               const int32_t *__restrict__ row_pos,
                                                               bf16_t *__restrict__ o_act, float scale_log2e) {
    constexpr int KT = D / 32, DT = D / 16, W = 8;
    __shared__ float s_m[W][16], s_l[W][16];
    __shared__ float s_o[W][16][D];
    const int c = blockIdx.x, sq = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
    const int n_pos = row_pos[sq] + 1;
    const int n_t32 = (n_pos + 31) >> 5;
    const int head = c * G + j;
    const bool hv = j < G;

    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8 qf[KT], ql[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
        const size_t qo = ((size_t)sq * hq_l + head) * D + kt * 32 + 8 * g;
        qf[kt] = hv ? *reinterpret_cast<const bf16x8 *>(q + qo) : zero;
        ql[kt] = hv ? *reinterpret_cast<const bf16x8 *>(q_lo + qo) : zero;
    }
    floatx4 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = NEG_INF, lsum = 0.f;
    const size_t slab = (size_t)sq * kg.seq_stride + (size_t)c * kg.smax * D;
    const bf16x8 *ks = reinterpret_cast<const bf16x8 *>(kc + slab) + lane;
    const bf16x8 *vs = reinterpret_cast<const bf16x8 *>(vc + slab) + lane;

    for (int t = wave; t < n_t32; t += W) {
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
        bf16x8 ka[KT], kb[KT], va[DT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            ka[kt] = ks[(size_t)((2 * t) * KT + kt) * 64];
            kb[kt] = ks[(size_t)((2 * t + 1) * KT + kt) * 64];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) va[dt] = vs[(size_t)(t * DT + dt) * 64];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt], ql[kt], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[kt], ql[kt], s1, 0, 0, 0);
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt], qf[kt], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[kt], qf[kt], s1, 0, 0, 0);
        }
        const int pbase = t * 32 + 4 * g;
        float mx = NEG_INF;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s0[r] = (pbase + r < n_pos) ? s0[r] * scale_log2e : NEG_INF;
            s1[r] = (pbase + 16 + r < n_pos) ? s1[r] * scale_log2e : NEG_INF;
            mx = fmaxf(mx, fmaxf(s0[r], s1[r]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float alpha = exp2f(m - m_new);
        m = m_new;
        float p0[4], p1[4], ps = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p0[r] = exp2f(s0[r] - m_new);
            p1[r] = exp2f(s1[r] - m_new);
            ps += p0[r] + p1[r];
        }
        lsum = lsum * alpha + ps;
        union { uint32_t u[4]; bf16x8 v; } pb, pl;
        split_pack2(p0[0], p0[1], pb.u[0], pl.u[0]); split_pack2(p0[2], p0[3], pb.u[1], pl.u[1]);
        split_pack2(p1[0], p1[1], pb.u[2], pl.u[2]); split_pack2(p1[2], p1[3], pb.u[3], pl.u[3]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            oacc[dt] *= alpha;
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pl.v, oacc[dt], 0, 0, 0);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pb.v, oacc[dt], 0, 0, 0);
        }
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (g == 0) { s_m[wave][j] = m; s_l[wave][j] = lsum; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<floatx4 *>(&s_o[wave][j][dt * 16 + 4 * g]) = oacc[dt];
    __syncthreads();
    const int k_tiles = (hq_l * D) >> 5;
    for (int idx = threadIdx.x * 4; idx < G * D; idx += 512 * 4) {
        const int hh = idx / D, dd = idx % D;
        float M = NEG_INF;
#pragma unroll
        for (int w = 0; w < W; ++w) M = fmaxf(M, s_m[w][hh]);
        float L = 0.f;
        floatx4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const float mw = s_m[w][hh];
            const float wt = (mw == NEG_INF) ? 0.f : exp2f(mw - M);
            L += s_l[w][hh] * wt;
            o += *reinterpret_cast<const floatx4 *>(&s_o[w][hh][dd]) * wt;
        }
        const float inv = 1.0f / L;
        uint2 ph, pl;
        split_pack2(o[0] * inv, o[1] * inv, ph.x, pl.x);
        split_pack2(o[2] * inv, o[3] * inv, ph.y, pl.y);
        const size_t off = dec_act_offset(sq, (c * G + hh) * D + dd, k_tiles, 0);
        *reinterpret_cast<uint2 *>(o_act + off) = ph;
        *reinterpret_cast<uint2 *>(o_act + off + 32) = pl;
    }
}

void launch_attn_decode(const bf16_t *q, const bf16_t *q_lo, const bf16_t *kc, const bf16_t *vc, KvGeom kg,
                        int hq_l, const int32_t *row_pos, int b, int nsplit, float *part_o, float *part_ml,
                        bf16_t *o_act, hipStream_t s) {
    const int G = hq_l / kg.hkv_l;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)kg.d);
    if (nsplit <= 1) {       // single kernel, LDS merge
        dim3 grid(kg.hkv_l, b);
        if (kg.d == 128)
            hipLaunchKernelGGL(attn_decode_block_kernel<128>, grid, dim3(512), 0, s, q, q_lo, kc, vc, kg, hq_l, G,
                               row_pos, o_act, scale_log2e);
        else
            hipLaunchKernelGGL(attn_decode_block_kernel<64>, grid, dim3(512), 0, s, q, q_lo, kc, vc, kg, hq_l, G,
                               row_pos, o_act, scale_log2e);
        return;
    }
    dim3 grid(nsplit, kg.hkv_l, b);
    if (kg.d == 128) {
        hipLaunchKernelGGL(attn_decode_kernel<128>, grid, dim3(64), 0, s, q, q_lo, kc, vc, kg, hq_l, G, row_pos, nsplit,
                           part_o, part_ml, scale_log2e);
        hipLaunchKernelGGL(attn_decode_merge_kernel<128>, dim3(b, hq_l), dim3(128), 0, s, part_o, part_ml, hq_l,
                           nsplit, o_act);
    } else {
        hipLaunchKernelGGL(attn_decode_kernel<64>, grid, dim3(64), 0, s, q, q_lo, kc, vc, kg, hq_l, G, row_pos, nsplit,
                           part_o, part_ml, scale_log2e);
        hipLaunchKernelGGL(attn_decode_merge_kernel<64>, dim3(b, hq_l), dim3(64), 0, s, part_o, part_ml, hq_l, nsplit,
                           o_act);
    }
}

// -------------------------------------------------------------------------------------------------
// Prefill: grid (ceil(max_new / 64), hq_l, batch), 4 waves per block, each wave owns 16 query rows of
// one head of one sequence and walks the cache in 32-position steps up to its last row's position
// (causal: later tiles are never touched).  Rows of the call sit at positions pos0[seq] + i.
// -------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_prefill_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ kc,
                                                          const bf16_t *__restrict__ vc, KvGeom kg, int hq_l, int G,
                                                          const int32_t *__restrict__ cu_rows,
                                                          const int32_t *__restrict__ pos0,
                                                          bf16_t *__restrict__ o_packed, float scale_log2e) {
    constexpr int KT = D / 32, DT = D / 16;
    const int seq = blockIdx.z, head = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
    const int row0 = cu_rows[seq], n_new = cu_rows[seq + 1] - row0, p0s = pos0[seq];
    const int qbase = blockIdx.x * 64 + wave * 16;
    if (qbase >= n_new) return;               // whole wave leaves; no block-level barrier below
    const int ri = qbase + j;
    const bool valid = ri < n_new;
    const int qpos = valid ? p0s + ri : 0x3fffffff;    // padded rows: nothing masked, nothing stored
    const int last_pos = p0s + min(qbase + 15, n_new - 1);
    const int n_t32 = (last_pos >> 5) + 1;
    const int c = head / G;

    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8 qf[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
        qf[kt] = valid ? *reinterpret_cast<const bf16x8 *>(q + frag_offset(row0 + ri, head * D + kt * 32 + 8 * g,
                                                                            (hq_l * D) >> 5))
                       : zero;
    floatx4 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = NEG_INF, lsum = 0.f;

    const size_t slab = (size_t)seq * kg.seq_stride + (size_t)c * kg.smax * D;
    const bf16x8 *ks = reinterpret_cast<const bf16x8 *>(kc + slab) + lane;
    const bf16x8 *vs = reinterpret_cast<const bf16x8 *>(vc + slab) + lane;

    for (int t = 0; t < n_t32; ++t) {
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
        bf16x8 ka[KT], kb[KT], va[DT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            ka[kt] = ks[(size_t)((2 * t) * KT + kt) * 64];
            kb[kt] = ks[(size_t)((2 * t + 1) * KT + kt) * 64];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) va[dt] = vs[(size_t)(t * DT + dt) * 64];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[kt], qf[kt], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[kt], qf[kt], s1, 0, 0, 0);
        }
        const int pbase = t * 32 + 4 * g;
        float mx = NEG_INF;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s0[r] = (pbase + r <= qpos) ? s0[r] * scale_log2e : NEG_INF;
            s1[r] = (pbase + 16 + r <= qpos) ? s1[r] * scale_log2e : NEG_INF;
            mx = fmaxf(mx, fmaxf(s0[r], s1[r]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);     // finite from the first tile on: position 0 <= qpos
        const float alpha = exp2f(m - m_new);
        m = m_new;
        float p0[4], p1[4], ps = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p0[r] = exp2f(s0[r] - m_new);
            p1[r] = exp2f(s1[r] - m_new);
            ps += p0[r] + p1[r];
        }
        lsum = lsum * alpha + ps;
        union { uint32_t u[4]; bf16x8 v; } pb;
        pb.u[0] = pack_bf16x2(p0[0], p0[1]); pb.u[1] = pack_bf16x2(p0[2], p0[3]);
        pb.u[2] = pack_bf16x2(p1[0], p1[1]); pb.u[3] = pack_bf16x2(p1[2], p1[3]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            oacc[dt] *= alpha;
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pb.v, oacc[dt], 0, 0, 0);
        }
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (valid) {
        const float inv = 1.0f / lsum;
        const int k_tiles = (hq_l * D) >> 5;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            uint2 o;
            o.x = pack_bf16x2(oacc[dt][0] * inv, oacc[dt][1] * inv);
            o.y = pack_bf16x2(oacc[dt][2] * inv, oacc[dt][3] * inv);
            *reinterpret_cast<uint2 *>(o_packed + frag_offset(row0 + ri, head * D + dt * 16 + 4 * g, k_tiles)) = o;
        }
    }
}

void launch_attn_prefill(const bf16_t *q, const bf16_t *kc, const bf16_t *vc, KvGeom kg, int hq_l,
                         const int32_t *cu_rows, const int32_t *pos0, int batch, int max_new, bf16_t *o_packed,
                         hipStream_t s) {
    if (batch <= 0 || max_new <= 0) return;
    const int G = hq_l / kg.hkv_l;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)kg.d);
    dim3 grid((max_new + 63) / 64, hq_l, batch);
    if (kg.d == 128)
        hipLaunchKernelGGL(attn_prefill_kernel<128>, grid, dim3(256), 0, s, q, kc, vc, kg, hq_l, G, cu_rows, pos0,
                           o_packed, scale_log2e);
    else
        hipLaunchKernelGGL(attn_prefill_kernel<64>, grid, dim3(256), 0, s, q, kc, vc, kg, hq_l, G, cu_rows, pos0,
                           o_packed, scale_log2e);
}
