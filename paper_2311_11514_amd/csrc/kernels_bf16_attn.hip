// bf16 attention on the matrix cores: split-KV GQA decode attention and flash-style causal prefill
// attention.  Both compute scores transposed, S^T = K . Q^T (operand A = a K fragment of the cache,
// operand B = query rows), so one lane owns one query row / query head and 4 consecutive positions;
// softmax statistics are per lane plus two cross-lane steps; and O^T = V^T . P^T takes P straight from
// the score accumulators (see kvlayout.h for the matching V layout).
//
// Decode: the G query heads that share a KV head are the 16 columns of operand B, so every K and V
// fragment is fetched from HBM exactly once per sequence and serves the whole query group inside one
// MFMA.  A long context with few sequences is split over several blocks, whose partial (m, l, o) triples the
// last block to finish merges by log-sum-exp, in split order.
#include "kernels.h"
#include "kvlayout.h"

#define NEG_INF (-INFINITY)

namespace HX_NS {



// ---- finishing a split QKV projection inside the decode attention (QkvTail) ---------------------------------------
// LDS staging of what a block computes for its own (sequence, kv head): the G query heads as the MFMA's B operand
// (hi and lo parts, heads beyond G zero) and the new K / V row.
template <int D>
struct QkvStage {
    h16_t qh[16][D], ql[16][D];
    h16_t kn[D], vn[D];
};

// Every thread of the block: adds up the split partial sums of the block's G query heads and of its K and V head for
// row `sq` (in split order), applies 1/rms and the rotary embedding at position `pos`, and leaves q (hi + lo) and the
// new K / V row in LDS; `append` blocks also write the row to the cache.  The QKV weight tiles are packed so that a
// 16-feature tile holds 8 rotary pairs: features 0..7 of the tile are elements 8 tl .. 8 tl + 7 of the head, features
// 8..15 the elements half a head further (the layout decode_epilogue<DEC_QKV> reads as well).  Ends with a barrier.
template <int D, int NT>
__device__ __forceinline__ void qkv_tail_stage(const QkvTail &tail, QkvStage<D> &st, int sq, int c, int G, int hq_l,
                                               const KvGeom &kg, int pos, bool append, h16_t *kc, h16_t *vc) {
    constexpr int TPH = D / 16, HALF = D / 2;
    const float r = tail.rstd[sq];
    const size_t slab = (size_t)sq * kg.seq_stride + (size_t)c * kg.smax * D;
    for (int idx = threadIdx.x; idx < (G + 2) * TPH * 2; idx += NT) {
        const int hh = idx / (TPH * 2), rem = idx - hh * TPH * 2, tl = rem >> 1, q2 = rem & 1;
        const int head_g = hh < G ? c * G + hh : (hh == G ? hq_l + c : hq_l + kg.hkv_l + c);
        const size_t col = ((size_t)head_g * TPH + tl) * 16 + 4 * q2;
        floatx4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
        for (int ks0 = 0; ks0 < tail.splits; ks0 += 8) {         // eight splits' partials in flight at a time
            floatx4 pl[8], ph[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float *p = tail.part + ((size_t)min(ks0 + u, tail.splits - 1) * tail.T + sq) * tail.N + col;
                pl[u] = *reinterpret_cast<const floatx4 *>(p);
                ph[u] = *reinterpret_cast<const floatx4 *>(p + 8);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)                           // added in split order
                if (ks0 + u < tail.splits) { lo += pl[u]; hi += ph[u]; }
        }
        lo *= r;
        hi *= r;
        const int i0 = tl * 8 + 4 * q2;              // first of this thread's four rotary pairs
        float ol[4], oh[4];
        if (hh <= G) {
            const floatx4 c4 = *reinterpret_cast<const floatx4 *>(tail.cos_tab + (size_t)pos * HALF + i0);
            const floatx4 s4 = *reinterpret_cast<const floatx4 *>(tail.sin_tab + (size_t)pos * HALF + i0);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                ol[x] = lo[x] * c4[x] - hi[x] * s4[x];
                oh[x] = hi[x] * c4[x] + lo[x] * s4[x];
            }
        } else {
#pragma unroll
            for (int x = 0; x < 4; ++x) { ol[x] = lo[x]; oh[x] = hi[x]; }
        }
        if (hh < G) {
            uint2 a, al, b, bl;
            split_pack2(ol[0], ol[1], a.x, al.x); split_pack2(ol[2], ol[3], a.y, al.y);
            split_pack2(oh[0], oh[1], b.x, bl.x); split_pack2(oh[2], oh[3], b.y, bl.y);
            *reinterpret_cast<uint2 *>(&st.qh[hh][i0]) = a;
            *reinterpret_cast<uint2 *>(&st.ql[hh][i0]) = al;
            *reinterpret_cast<uint2 *>(&st.qh[hh][HALF + i0]) = b;
            *reinterpret_cast<uint2 *>(&st.ql[hh][HALF + i0]) = bl;
        } else {
            uint2 a, b;
            a.x = pack_h16x2(ol[0], ol[1]); a.y = pack_h16x2(ol[2], ol[3]);
            b.x = pack_h16x2(oh[0], oh[1]); b.y = pack_h16x2(oh[2], oh[3]);
            h16_t *dst = hh == G ? st.kn : st.vn;
            *reinterpret_cast<uint2 *>(dst + i0) = a;
            *reinterpret_cast<uint2 *>(dst + HALF + i0) = b;
            if (append) {
                if (hh == G) {
                    *reinterpret_cast<uint2 *>(kc + slab + kv_k_offset(pos, i0, D)) = a;
                    *reinterpret_cast<uint2 *>(kc + slab + kv_k_offset(pos, HALF + i0, D)) = b;
                } else {
                    const h16_t *av = reinterpret_cast<const h16_t *>(&a), *bv = reinterpret_cast<const h16_t *>(&b);
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        vc[slab + kv_v_offset(pos, i0 + x, D)] = av[x];
                        vc[slab + kv_v_offset(pos, HALF + i0 + x, D)] = bv[x];
                    }
                }
            }
        }
    }
    for (int idx = threadIdx.x; idx < (16 - G) * (D / 8); idx += NT) {      // operand columns beyond the group: zero
        const int hh = G + idx / (D / 8), e8 = (idx % (D / 8)) * 8;
        *reinterpret_cast<uint4 *>(&st.qh[hh][e8]) = uint4{0u, 0u, 0u, 0u};
        *reinterpret_cast<uint4 *>(&st.ql[hh][e8]) = uint4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
}

// The tile that holds the new row's position takes that row from LDS instead of the cache (the row is being written
// by this very block): K fragments hold position 32 t + 16 sub + lane % 16, V^T fragments positions 4 g .. 4 g + 3 and
// 16 + 4 g .. + 3 of the tile (kvlayout.h).
template <int D>
__device__ __forceinline__ void qkv_tail_patch(const QkvStage<D> &st, int p32, int j, int g, h16x8 (&ka)[D / 32],
                                               h16x8 (&kb)[D / 32], h16x8 (&va)[D / 16]) {
    const int sub = p32 >> 4, jp = p32 & 15;
    if (j == jp) {
#pragma unroll
        for (int kt = 0; kt < D / 32; ++kt) {
            const h16x8 nk = *reinterpret_cast<const h16x8 *>(&st.kn[kt * 32 + 8 * g]);
            if (sub) kb[kt] = nk;
            else ka[kt] = nk;
        }
    }
    const int gp = (p32 & 15) >> 2, ep = (p32 & 3) + 4 * (p32 >> 4);
    if (g == gp) {
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            union { h16x8 v; h16_t e[8]; } u;
            u.v = va[dt];
            const h16_t nv = st.vn[dt * 16 + j];
#pragma unroll
            for (int x = 0; x < 8; ++x) u.e[x] = x == ep ? nv : u.e[x];
            va[dt] = u.v;
        }
    }
}

// One 8-wave block per (sequence, kv head); the waves interleave over the 32-position tiles of the context and
// their (m, l, o) triples are merged through LDS in wave order.
// Used when there are enough (sequence, kv head) pairs to fill the chip or the context is short.
// PF: the layouts of the prefill path on both ends (used when more than 32 sequences decode one row each, which the
// prefill kernels otherwise serve): q is read from fragment tiles (row = sequence, no lo part), o is written to them.
// FUSE: the QKV projection of this step left split partial sums (QkvTail): the block finishes them for its own heads
// first, appends the new K / V row to the cache and takes q and that row from LDS.
template <int D, bool PF, bool FUSE>
__global__ __launch_bounds__(512) void attn_decode_block_kernel(const h16_t *__restrict__ q,
                                                               const h16_t *__restrict__ q_lo, h16_t *kc, h16_t *vc,
                                                               KvGeom kg, int hq_l, int G,
                                                               const int32_t *__restrict__ row_pos,
                                                               h16_t *__restrict__ o_act, float scale_log2e, QkvTail tail) {
    constexpr int KT = D / 32, DT = D / 16, W = 8;
    static_assert(!(PF && FUSE), "the prefill path finishes its projections in their own epilogues");
    __shared__ float s_m[W][16], s_l[W][16];
    __shared__ float s_o[W][16][D];
    __shared__ __align__(16) QkvStage<FUSE ? D : 8> s_qkv;
    const int c = blockIdx.x, sq = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
    const int n_pos = row_pos[sq] + 1;
    const int n_t32 = (n_pos + 31) >> 5;
    const int head = c * G + j;
    const bool hv = j < G;

    const h16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    h16x8 qf[KT], ql[KT];
    const size_t slab = (size_t)sq * kg.seq_stride + (size_t)c * kg.smax * D;
    const h16x8 *ks = reinterpret_cast<const h16x8 *>(kc + slab) + lane;
    const h16x8 *vs = reinterpret_cast<const h16x8 *>(vc + slab) + lane;
    h16x8 ka[KT], kb[KT], va[DT];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            ka[kt] = ks[(size_t)((2 * t) * KT + kt) * 64];
            kb[kt] = ks[(size_t)((2 * t + 1) * KT + kt) * 64];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) va[dt] = vs[(size_t)(t * DT + dt) * 64];
    };
    if constexpr (FUSE) {
        // the wave's first tile is requested before the projection's tail is finished: the two wait side by side
        if (wave < n_t32) load_tile(wave);
        qkv_tail_stage<D, 512>(tail, reinterpret_cast<QkvStage<D> &>(s_qkv), sq, c, G, hq_l, kg, n_pos - 1, true, kc, vc);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            qf[kt] = *reinterpret_cast<const h16x8 *>(&reinterpret_cast<QkvStage<D> &>(s_qkv).qh[j][kt * 32 + 8 * g]);
            ql[kt] = *reinterpret_cast<const h16x8 *>(&reinterpret_cast<QkvStage<D> &>(s_qkv).ql[j][kt * 32 + 8 * g]);
        }
    } else {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            const size_t qo = PF ? frag_offset(sq, head * D + kt * 32 + 8 * g, (hq_l * D) >> 5)
                                 : ((size_t)sq * hq_l + head) * D + kt * 32 + 8 * g;
            qf[kt] = hv ? *reinterpret_cast<const h16x8 *>(q + qo) : zero;
            ql[kt] = (hv && !PF) ? *reinterpret_cast<const h16x8 *>(q_lo + qo) : zero;
        }
    }
    floatx4 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = NEG_INF, lsum = 0.f;

    for (int t = wave; t < n_t32; t += W) {
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
        if (!FUSE || t != wave) load_tile(t);
        if constexpr (FUSE) {
            if (t == n_t32 - 1) qkv_tail_patch<D>(reinterpret_cast<const QkvStage<D> &>(s_qkv), (n_pos - 1) & 31, j, g, ka, kb, va);
        }
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            s0 = hx_mfma16(ka[kt], ql[kt], s0);
            s1 = hx_mfma16(kb[kt], ql[kt], s1);
            s0 = hx_mfma16(ka[kt], qf[kt], s0);
            s1 = hx_mfma16(kb[kt], qf[kt], s1);
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
        union { uint32_t u[4]; h16x8 v; } pb, pl;
        split_pack2(p0[0], p0[1], pb.u[0], pl.u[0]); split_pack2(p0[2], p0[3], pb.u[1], pl.u[1]);
        split_pack2(p1[0], p1[1], pb.u[2], pl.u[2]); split_pack2(p1[2], p1[3], pb.u[3], pl.u[3]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            oacc[dt] *= alpha;
            oacc[dt] = hx_mfma16(va[dt], pl.v, oacc[dt]);
            oacc[dt] = hx_mfma16(va[dt], pb.v, oacc[dt]);
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
        if (PF) {
            *reinterpret_cast<uint2 *>(o_act + frag_offset(sq, (c * G + hh) * D + dd, k_tiles)) = ph;
        } else {
            const size_t off = dec_act_offset(sq, (c * G + hh) * D + dd, k_tiles, 0);
            *reinterpret_cast<uint2 *>(o_act + off) = ph;
            *reinterpret_cast<uint2 *>(o_act + off + 32) = pl;
        }
    }
}

// Split-KV variant in ONE kernel: grid (nsplit, kv heads, sequences).  A block takes a contiguous run of the
// sequence's 32-position tiles (its waves interleave over them; with few sequences the run is 8 tiles, one per wave,
// so the whole context is requested at once), merges its waves through LDS and writes one (m, l, o) partial per query
// head.  Blocks of one (sequence, kv head) then count themselves on a device counter; whichever arrives LAST merges
// the partials -- in split order, so the result does not depend on who that was -- and resets the counter for the
// next launch.  Nobody waits for anybody: every block runs straight to its end.
// The partials cross the chip's L2 slices: they are written with device-scope stores and read with device-scope
// loads (no fence: a fence would write back and invalidate the die's whole L2); a block counts itself once every
// lane's store counter has drained.
template <int D, bool FUSE>
__global__ __launch_bounds__(512) void attn_decode_split_kernel(const h16_t *__restrict__ q,
                                                               const h16_t *__restrict__ q_lo, h16_t *kc, h16_t *vc,
                                                               KvGeom kg, int hq_l, int G,
                                                               const int32_t *__restrict__ row_pos, int nsplit,
                                                               float *part_o, float *part_ml, unsigned int *arrived,
                                                               h16_t *__restrict__ o_act, float scale_log2e, QkvTail tail) {
    constexpr int KT = D / 32, DT = D / 16, W = 8, NT = 64 * W;
    __shared__ float s_m[W][16], s_l[W][16];
    __shared__ float s_o[W][16][D];
    __shared__ int s_last;
    __shared__ __align__(16) QkvStage<FUSE ? D : 8> s_qkv;
    const int split = blockIdx.x, c = blockIdx.y, sq = blockIdx.z;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
    const int n_pos = row_pos[sq] + 1;
    const int n_t32 = (n_pos + 31) >> 5;
    // tiles per block: the sequence's own even share; nb = blocks of this (sequence, kv head) that have tiles -- the
    // others (short contexts in a ragged batch) leave at once and are never counted
    const int per = (n_t32 + nsplit - 1) / nsplit;
    const int nb = min(nsplit, (n_t32 + per - 1) / per);
    if (split >= nb) return;
    const int t0 = split * per, t1 = (split == nb - 1) ? n_t32 : t0 + per;
    const int head = c * G + j;
    const bool hv = j < G;

    const h16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    h16x8 qf[KT], ql[KT];
    const size_t slab = (size_t)sq * kg.seq_stride + (size_t)c * kg.smax * D;
    const h16x8 *ks = reinterpret_cast<const h16x8 *>(kc + slab) + lane;
    const h16x8 *vs = reinterpret_cast<const h16x8 *>(vc + slab) + lane;
    h16x8 ka[KT], kb[KT], va[DT];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            ka[kt] = ks[(size_t)((2 * t) * KT + kt) * 64];
            kb[kt] = ks[(size_t)((2 * t + 1) * KT + kt) * 64];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) va[dt] = vs[(size_t)(t * DT + dt) * 64];
    };
    if constexpr (FUSE) {
        // every block of the pair finishes q for itself; the block that holds the last tile appends the new row; the
        // wave's first tile is requested before that, so that the two wait side by side
        if (t0 + wave < t1) load_tile(t0 + wave);
        qkv_tail_stage<D, 512>(tail, reinterpret_cast<QkvStage<D> &>(s_qkv), sq, c, G, hq_l, kg, n_pos - 1, split == nb - 1, kc, vc);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            qf[kt] = *reinterpret_cast<const h16x8 *>(&reinterpret_cast<QkvStage<D> &>(s_qkv).qh[j][kt * 32 + 8 * g]);
            ql[kt] = *reinterpret_cast<const h16x8 *>(&reinterpret_cast<QkvStage<D> &>(s_qkv).ql[j][kt * 32 + 8 * g]);
        }
    } else {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            const size_t qo = ((size_t)sq * hq_l + head) * D + kt * 32 + 8 * g;
            qf[kt] = hv ? *reinterpret_cast<const h16x8 *>(q + qo) : zero;
            ql[kt] = hv ? *reinterpret_cast<const h16x8 *>(q_lo + qo) : zero;
        }
    }
    floatx4 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = NEG_INF, lsum = 0.f;

    for (int t = t0 + wave; t < t1; t += W) {
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
        if (!FUSE || t != t0 + wave) load_tile(t);
        if constexpr (FUSE) {
            if (t == n_t32 - 1) qkv_tail_patch<D>(reinterpret_cast<const QkvStage<D> &>(s_qkv), (n_pos - 1) & 31, j, g, ka, kb, va);
        }
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            s0 = hx_mfma16(ka[kt], ql[kt], s0);
            s1 = hx_mfma16(kb[kt], ql[kt], s1);
            s0 = hx_mfma16(ka[kt], qf[kt], s0);
            s1 = hx_mfma16(kb[kt], qf[kt], s1);
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
        const float m_new = fmaxf(m, mx);          // finite: position t * 32 < n_pos is never masked
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
        union { uint32_t u[4]; h16x8 v; } pb, pl;
        split_pack2(p0[0], p0[1], pb.u[0], pl.u[0]); split_pack2(p0[2], p0[3], pb.u[1], pl.u[1]);
        split_pack2(p1[0], p1[1], pb.u[2], pl.u[2]); split_pack2(p1[2], p1[3], pb.u[3], pl.u[3]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            oacc[dt] *= alpha;
            oacc[dt] = hx_mfma16(va[dt], pl.v, oacc[dt]);
            oacc[dt] = hx_mfma16(va[dt], pb.v, oacc[dt]);
        }
    }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (g == 0) { s_m[wave][j] = m; s_l[wave][j] = lsum; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<floatx4 *>(&s_o[wave][j][dt * 16 + 4 * g]) = oacc[dt];
    __syncthreads();
    // the block's result per query head: waves merged in wave order
    for (int idx = threadIdx.x * 4; idx < G * D; idx += NT * 4) {
        const int hh = idx / D, dd = idx % D;
        const size_t e = ((size_t)sq * hq_l + c * G + hh) * nsplit + split;
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
        if (nb == 1) {          // the whole context was this block's: final result, as in the one-block kernel
            const float inv = 1.0f / L;
            uint2 ph, pl;
            split_pack2(o[0] * inv, o[1] * inv, ph.x, pl.x);
            split_pack2(o[2] * inv, o[3] * inv, ph.y, pl.y);
            const size_t off = dec_act_offset(sq, (c * G + hh) * D + dd, (hq_l * D) >> 5, 0);
            *reinterpret_cast<uint2 *>(o_act + off) = ph;
            *reinterpret_cast<uint2 *>(o_act + off + 32) = pl;
            continue;
        }
        float *po = part_o + e * D + dd;
#pragma unroll
        for (int r = 0; r < 4; ++r) dev_store(po + r, o[r]);
        if (dd == 0) { dev_store(part_ml + e * 2, M); dev_store(part_ml + e * 2 + 1, L); }
    }
    if (nb == 1) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this lane's device-scope stores have completed ...
    __syncthreads();                                      // ... and so have every other lane's of the block ...
    if (threadIdx.x == 0) {                               // ... before the block counts itself
        const unsigned int before = __hip_atomic_fetch_add(&arrived[sq * gridDim.y + c], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = before + 1 == (unsigned int)nb;
        // all blocks have counted: ready for the next launch
        if (s_last) __hip_atomic_store(&arrived[sq * gridDim.y + c], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;
    for (int idx = threadIdx.x * 4; idx < G * D; idx += NT * 4) {
        const int hh = idx / D, dd = idx % D;
        const size_t e0 = ((size_t)sq * hq_l + c * G + hh) * nsplit;
        float M = NEG_INF;
        for (int sp = 0; sp < nb; ++sp) M = fmaxf(M, dev_load(part_ml + (e0 + sp) * 2));
        float L = 0.f;
        floatx4 o = {0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < nb; ++sp) {
            const float ms = dev_load(part_ml + (e0 + sp) * 2);
            const float wt = (ms == NEG_INF) ? 0.f : exp2f(ms - M);
            L += dev_load(part_ml + (e0 + sp) * 2 + 1) * wt;
            const float *po = part_o + (e0 + sp) * D + dd;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] += dev_load(po + r) * wt;
        }
        const float inv = 1.0f / L;
        uint2 ph, pl;
        split_pack2(o[0] * inv, o[1] * inv, ph.x, pl.x);
        split_pack2(o[2] * inv, o[3] * inv, ph.y, pl.y);
        const size_t off = dec_act_offset(sq, (c * G + hh) * D + dd, (hq_l * D) >> 5, 0);
        *reinterpret_cast<uint2 *>(o_act + off) = ph;
        *reinterpret_cast<uint2 *>(o_act + off + 32) = pl;
    }
}

void launch_attn_decode(const h16_t *q, const h16_t *q_lo, h16_t *kc, h16_t *vc, KvGeom kg,
                        int hq_l, const int32_t *row_pos, int b, int nsplit, float *part_o, float *part_ml,
                        unsigned int *arrived, h16_t *o_act, const QkvTail &tail, hipStream_t s) {
    const int G = hq_l / kg.hkv_l;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)kg.d);
    const bool fuse = tail.part != nullptr;
#define HX_BLK(DD, FF)                                                                                                   \
    hipLaunchKernelGGL((attn_decode_block_kernel<DD, false, FF>), grid, dim3(512), 0, s, q, q_lo, kc, vc, kg, hq_l, G, row_pos, \
                       o_act, scale_log2e, tail)
#define HX_SPL(DD, FF)                                                                                                   \
    hipLaunchKernelGGL((attn_decode_split_kernel<DD, FF>), grid, dim3(512), 0, s, q, q_lo, kc, vc, kg, hq_l, G, row_pos, nsplit, \
                       part_o, part_ml, arrived, o_act, scale_log2e, tail)
    if (nsplit <= 1) {       // one block per (sequence, kv head), LDS merge
        dim3 grid(kg.hkv_l, b);
        if (kg.d == 128) { if (fuse) HX_BLK(128, true); else HX_BLK(128, false); }
        else { if (fuse) HX_BLK(64, true); else HX_BLK(64, false); }
        return;
    }
    dim3 grid(nsplit, kg.hkv_l, b);
    if (kg.d == 128) { if (fuse) HX_SPL(128, true); else HX_SPL(128, false); }
    else { if (fuse) HX_SPL(64, true); else HX_SPL(64, false); }
#undef HX_BLK
#undef HX_SPL
}

// one new row per sequence on the prefill path's layouts: q and o in fragment tiles (row = sequence)
void launch_attn_decode_rows(const h16_t *q, const h16_t *kc, const h16_t *vc, KvGeom kg, int hq_l,
                             const int32_t *row_pos, int b, h16_t *o_packed, hipStream_t s) {
    const int G = hq_l / kg.hkv_l;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)kg.d);
    const QkvTail none{nullptr, 0, 0, 0, nullptr, nullptr, nullptr};
    h16_t *kw = const_cast<h16_t *>(kc), *vw = const_cast<h16_t *>(vc);       // read only without a QkvTail
    dim3 grid(kg.hkv_l, b);
    if (kg.d == 128)
        hipLaunchKernelGGL((attn_decode_block_kernel<128, true, false>), grid, dim3(512), 0, s, q, q, kw, vw, kg, hq_l, G, row_pos,
                           o_packed, scale_log2e, none);
    else
        hipLaunchKernelGGL((attn_decode_block_kernel<64, true, false>), grid, dim3(512), 0, s, q, q, kw, vw, kg, hq_l, G, row_pos,
                           o_packed, scale_log2e, none);
}

// -------------------------------------------------------------------------------------------------
// Prefill: grid (G n_items, kv heads); a block of 4 waves owns 128 query rows of one head of one sequence, a wave 32 of
// them, and walks the cache in 32-position tiles up to its last row's position (causal: later tiles are never
// touched).  Rows of the call sit at positions pos0[seq] + i.  The (sequence, row block) pairs come from a work list
// built on the host, longest walks first; the G query heads of a kv head run next to each other on one XCD, so the
// blocks that walk the same K and V do so at the same time and share them in that XCD's L2.
//
// Everything runs on v_mfma_f32_32x32x16_bf16.  S^T (32 positions x 32 query rows) = K . Q^T: operand A is gathered
// from the two 16-position K tiles, operand B is the wave's query block, held in registers for the whole walk.
// In the result a lane owns query row lane % 32 and positions 8 q + 4 (lane / 32) + r: register quads q = 0, 2 are
// exactly the position slots (4 g .. 4 g + 3, 16 + 4 g .. 16 + 4 g + 3) of k-group g = lane / 32 of the V^T tiles
// (see kvlayout.h), quads 1, 3 those of k-group 2 + lane / 32 -- so P goes from the score registers straight into the
// two 16-slot MFMAs of O^T = V^T . P^T, with no cross-lane traffic, on the cache layout the decode kernels use.
// The K and V tiles of a step (16 KB at d = 128) are shared by the block's waves through LDS (direct-to-LDS loads,
// three stages); two blocks fit a CU, so one wave's softmax arithmetic hides behind the other's MFMAs.
// -------------------------------------------------------------------------------------------------
#define HX_AS1(p) ((const __attribute__((address_space(1))) void *)(p))
#define HX_AS3(p) ((__attribute__((address_space(3))) void *)(p))
#define HX_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

template <int D, int NWV>
__global__ __launch_bounds__(64 * NWV, 2) void attn_prefill_kernel(const h16_t *__restrict__ q, const h16_t *__restrict__ kc,
                                                             const h16_t *__restrict__ vc, KvGeom kg, int hq_l, int G,
                                                             const int32_t *__restrict__ cu_rows,
                                                             const int32_t *__restrict__ pos0,
                                                             const int32_t *__restrict__ items, int n_items,
                                                             h16_t *__restrict__ o_packed, float scale_log2e) {
    constexpr int KT = D / 32, DT = D / 16, DB = D / 32;     // K d-tiles, V^T d-tiles, 32-wide output blocks
    constexpr int TILES = 2 * KT + DT;                       // 1 KB tiles per 32-position step: K then V^T
    constexpr int LPT = TILES / NWV;                         // loads per wave and step
    constexpr int ROWS = 32 * NWV;                           // query rows per block
    constexpr int S = 3;
    static_assert(TILES % NWV == 0, "tiles must divide over the waves");
    __shared__ h16x8 smem[S][TILES][64];
    // Consecutive block ids are dealt to the 8 XCDs in turn, each with its own L2: block id = 8 slot + xcd.  An XCD takes
    // every eighth item, and the G heads of an item occupy consecutive slots of that XCD.
    const int slot = blockIdx.x >> 3, xcd = blockIdx.x & 7;
    const int item = (slot / G) * 8 + xcd, c = blockIdx.y, head = c * G + slot % G;
    if (item >= n_items) return;                             // the whole block leaves
    const int seq = items[2 * item], rb = items[2 * item + 1];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int row0 = cu_rows[seq], n_new = cu_rows[seq + 1] - row0, p0s = pos0[seq];
    if (rb * ROWS >= n_new) return;                          // the whole block leaves
    const int qbase = rb * ROWS + wave * 32;
    const int hl = lane >> 5;
    const int ri = qbase + (lane & 31);
    const bool valid = ri < n_new;
    const int qpos = valid ? p0s + ri : 0x3fffffff;          // padded rows: nothing masked, nothing stored
    const int nt = ((p0s + min(rb * ROWS + ROWS - 1, n_new - 1)) >> 5) + 1;                      // steps of the block
    const int nt_w = qbase < n_new ? ((p0s + min(qbase + 31, n_new - 1)) >> 5) + 1 : 0;    // steps this wave computes
    const int first_masked = (p0s + qbase) >> 5;             // tiles before it lie wholly in every row's past

    // 32x32x16 operand gather from a pair of 16-row fragment tiles: lane l takes row l % 32, k-group 2 kh + l / 32
    const int sub = (lane & 31) >> 4;                        // which tile of the pair
    const int fl = (lane & 15) + 16 * hl;                    // lane slot inside the tile for kh = 0 (+ 32 for kh = 1)
    const int qkt = (hq_l * D) >> 5;
    h16x8 qf[2 * KT];
    {
        const h16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        const int qr = row0 + min(ri, n_new - 1);
#pragma unroll
        for (int kk = 0; kk < 2 * KT; ++kk)
            qf[kk] = qbase < n_new ? *reinterpret_cast<const h16x8 *>(
                                          q + frag_offset(qr, head * D + (kk >> 1) * 32 + 8 * (2 * (kk & 1) + hl), qkt))
                                    : zero;
    }
    floatx16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m = NEG_INF, lsum = 0.f;

    const size_t slab = (size_t)seq * kg.seq_stride + (size_t)c * kg.smax * D;
    const h16x8 *ks = reinterpret_cast<const h16x8 *>(kc + slab);
    const h16x8 *vs = reinterpret_cast<const h16x8 *>(vc + slab);
    // tiles of step t: K tiles (2 t) KT .. (2 t + 2) KT - 1 and V^T tiles t DT .. (t + 1) DT - 1, both contiguous.
    // The loads are written in their scalar-base form as asm: besides saving a vector add per load, that keeps
    // them out of the compiler's memory model, which would otherwise drain vmcnt to 0 in front of every LDS
    // read of the array they target and so undo the prefetch.  Every wait on them is explicit (HX_WAIT_VM).
    const unsigned lane_bytes = (unsigned)lane * 16u;
    auto issue = [&](int t) {
#pragma unroll
        for (int x = 0; x < LPT; ++x) {
            const int tile = wave + NWV * x;
            const h16x8 *src = tile < 2 * KT ? ks + (size_t)(2 * t * KT + tile) * 64 : vs + (size_t)(t * DT + tile - 2 * KT) * 64;
            const unsigned lds_addr = (unsigned)reinterpret_cast<uintptr_t>(HX_AS3(&smem[t % S][tile][0]));
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_addr), "v"(lane_bytes), "s"(src)
                         : "memory");
        }
    };
    // the query block has landed before the first hidden load is issued: the compiler, which does not see those
    // loads, would otherwise place its own wait for the query registers (a full drain) inside the loop
    HX_WAIT_VM(0);
    issue(0);
    if (nt > 1) issue(1);
    for (int t = 0; t < nt; ++t) {
        if (t + 1 < nt) HX_WAIT_VM(LPT);      // step t has landed; the loads of step t + 1 stay in flight
        else HX_WAIT_VM(0);
        __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));       // this wave's LDS reads are complete
        asm volatile("s_barrier" ::: "memory");
        if (t + 2 < nt) issue(t + 2);         // into the buffer of step t - 1, which every wave has left
        if (t >= nt_w) continue;              // this wave's rows end before the tile (it still feeds the others)
        const h16x8(*st)[64] = smem[t % S];
        floatx16 sc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 2 * KT; ++kk)
            sc = hx_mfma32(st[sub * KT + (kk >> 1)][fl + 32 * (kk & 1)], qf[kk], sc);
        // causal mask (only tiles that reach a row's own position) and running max on the raw scores; the softmax
        // scale is folded into the exponent's multiply-add (scale > 0, so the max commutes with it)
        float mx = NEG_INF;
        if (t >= first_masked) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int pos = t * 32 + 8 * (r >> 2) + 4 * hl + (r & 3);
                sc[r] = pos <= qpos ? sc[r] : NEG_INF;
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);     // finite from the first tile on: position 0 <= qpos
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * scale_log2e);
        m = m_new;
        const float mb = -m_new * scale_log2e;
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sc[r] = __builtin_amdgcn_exp2f(fmaf(sc[r], scale_log2e, mb));
            ps += sc[r];
        }
        lsum = lsum * alpha + ps;
        union { uint32_t u[4]; h16x8 v; } pb0, pb1;      // P for k-groups hl (quads 0, 2) and 2 + hl (quads 1, 3)
        pb0.u[0] = pack_h16x2(sc[0], sc[1]);   pb0.u[1] = pack_h16x2(sc[2], sc[3]);
        pb0.u[2] = pack_h16x2(sc[8], sc[9]);   pb0.u[3] = pack_h16x2(sc[10], sc[11]);
        pb1.u[0] = pack_h16x2(sc[4], sc[5]);   pb1.u[1] = pack_h16x2(sc[6], sc[7]);
        pb1.u[2] = pack_h16x2(sc[12], sc[13]); pb1.u[3] = pack_h16x2(sc[14], sc[15]);
        // rescale the running output only when some row's maximum moved (rare after the first tiles)
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            oacc[db] = hx_mfma32(st[2 * KT + 2 * db + sub][fl], pb0.v, oacc[db]);
            oacc[db] = hx_mfma32(st[2 * KT + 2 * db + sub][fl + 32], pb1.v, oacc[db]);
        }
    }
    lsum += __shfl_xor(lsum, 32, 64);
    if (valid) {
        const float inv = 1.0f / lsum;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 o;
                o.x = pack_h16x2(oacc[db][4 * qd] * inv, oacc[db][4 * qd + 1] * inv);
                o.y = pack_h16x2(oacc[db][4 * qd + 2] * inv, oacc[db][4 * qd + 3] * inv);
                *reinterpret_cast<uint2 *>(o_packed + frag_offset(row0 + ri, head * D + 32 * db + 8 * qd + 4 * hl, qkt)) = o;
            }
    }
}

void launch_attn_prefill(const h16_t *q, const h16_t *kc, const h16_t *vc, KvGeom kg, int hq_l,
                         const int32_t *cu_rows, const int32_t *pos0, const int32_t *items, int n_items, h16_t *o_packed,
                         hipStream_t s) {
    if (n_items <= 0) return;
    const int G = hq_l / kg.hkv_l;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)kg.d);
    dim3 grid((unsigned)G * ((n_items + 7) / 8 * 8), kg.hkv_l);
    if (kg.d == 128)
        hipLaunchKernelGGL((attn_prefill_kernel<128, 4>), grid, dim3(256), 0, s, q, kc, vc, kg, hq_l, G, cu_rows, pos0, items,
                           n_items, o_packed, scale_log2e);
    else
        hipLaunchKernelGGL((attn_prefill_kernel<64, 4>), grid, dim3(256), 0, s, q, kc, vc, kg, hq_l, G, cu_rows, pos0, items,
                           n_items, o_packed, scale_log2e);
}

}  // namespace HX_NS
