// Decode projections (T <= 32 token rows): weight-streaming skinny GEMMs on the matrix cores with the
// whole sub-layer glue fused into their tails.  Two forms: decode_proj_kernel (one or two rows, small or short
// matrices: one kernel, complete dot products per block, no scratch buffers, no atomics) and, further down,
// decode_splitk_kernel + decode_finish_kernel (3 to 32 rows: operand shared through LDS, contraction split over
// blocks); launch_decode_proj chooses.
//
// Main loop of decode_proj_kernel.  Each wave streams 1 KB weight tiles with one 128-bit load per lane (fully coalesced,
// non-temporal) and feeds them to v_mfma_f32_16x16x32_bf16 against a 16-token activation tile: 16 MFMA
// cycles per KB, a quarter of what unpacking bf16 on the vector ALU would cost, so the kernel stays
// HBM-bound up to 32 rows.  Activations arrive as hi + lo bf16 pairs (two MFMAs per tile, free here).
// A block owns one unit = UT 16-feature tiles over the WHOLE contraction; its waves interleave over the
// k-tiles and are summed through LDS in wave order (bit-reproducible).  Because a block holds complete
// dot products, the epilogue runs in registers on the 16x16 accumulator layout (lane = one token, four
// consecutive features):
//   QKV    : x rstd of the input rows, RoPE, q -> hi/lo rows, k / v -> KV cache.  The QKV weight tiles are
//            packed so that a tile holds 8 rotary pairs (features i and i + d/2), which lie 32 lanes apart.
//   RESID  : h += partial; (h * gain of the next norm) -> hi/lo operand of the next projection (compact
//            token-major layout, see dec_act_offset);
//            per-unit sum of squares of the new h, from which the next kernel derives rstd
//   SWIGLU : x rstd, silu(gate) * up -> hi/lo operand of the W2 projection (gate / up tiles interleaved)
//   RAW    : x rstd (if the input is a normalised stream), plain fp32 partial (validation surface)
// RMSNorm is thus never a kernel of its own in decode: y = rstd * ((h*g) . W), with rstd a per-row
// scalar applied after the contraction.
#include <algorithm>
#include <cstdlib>

#include "kernels.h"
#include "kvlayout.h"

namespace HX_NS {


// rstd of a token row from the per-unit sums of squares of the residual stream
__device__ inline void rstd_row(const DecodeEpi &e, int t, int lane, float *s_rstd) {
    float r = 1.0f;
    if (e.ssq_in) {
        float ss = 0.f;
        for (int i = lane; i < e.ssq_units; i += 64) ss += e.ssq_in[i * DEC_SSQ_STRIDE + t];
        ss = wave_sum(ss);
        r = 1.0f / sqrtf(ss / (float)e.norm_dim + e.eps);
    }
    if (lane == 0) s_rstd[t] = r;
}
// wave w handles tokens w, w + WAVES, ...
template <int WAVES>
__device__ inline void load_rstd(const DecodeEpi &e, int T, int wave, int lane, float *s_rstd) {
    for (int t = wave; t < T; t += WAVES) rstd_row(e, t, lane, s_rstd);
}
// The same in two halves, so that the loads can be requested ahead of other memory traffic and summed later: the
// first RSTD_REGS * 64 units wait in registers (hidden sizes up to 8192), any further ones are fetched in the second half.
constexpr int RSTD_REGS = 8;
__device__ inline void rstd_request(const DecodeEpi &e, int t, int lane, float (&sv)[RSTD_REGS]) {
#pragma unroll
    for (int j = 0; j < RSTD_REGS; ++j) sv[j] = e.ssq_in[min(lane + 64 * j, e.ssq_units - 1) * DEC_SSQ_STRIDE + t];
}
__device__ inline void rstd_finish(const DecodeEpi &e, int t, int lane, const float (&sv)[RSTD_REGS], float *s_rstd) {
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < RSTD_REGS; ++j) ss += lane + 64 * j < e.ssq_units ? sv[j] : 0.f;      // lane's units ascending
    for (int i = lane + 64 * RSTD_REGS; i < e.ssq_units; i += 64) ss += e.ssq_in[i * DEC_SSQ_STRIDE + t];
    ss = wave_sum(ss);
    if (lane == 0) s_rstd[t] = 1.0f / sqrtf(ss / (float)e.norm_dim + e.eps);
}

__device__ inline void store_split4(const float x[4], h16_t *hi, h16_t *lo, size_t off) {
    uint2 o, ol;
    split_pack2(x[0], x[1], o.x, ol.x);
    split_pack2(x[2], x[3], o.y, ol.y);
    *reinterpret_cast<uint2 *>(hi + off) = o;
    *reinterpret_cast<uint2 *>(lo + off) = ol;
}
// 4 consecutive features k..k+3 of one token into a compact decode operand (hi and lo planes)
__device__ inline void store_act4(const float x[4], h16_t *xa, int token, int k, int k_tiles) {
    const size_t off = dec_act_offset(token, k, k_tiles, 0);
    uint2 o, ol;
    split_pack2(x[0], x[1], o.x, ol.x);
    split_pack2(x[2], x[3], o.y, ol.y);
    *reinterpret_cast<uint2 *>(xa + off) = o;
    *reinterpret_cast<uint2 *>(xa + off + 32) = ol;
}

// What the register epilogue reads from memory, requested long before it is used (the finishing wave asks for it at
// kernel start, so the answers arrive behind the first weights instead of adding two memory round trips to the
// block's tail).  Rows beyond T re-read row T - 1, so that no request sits behind a branch.
//   QKV   : first the row's position, then (once it is known) the rotary table entries of this lane's four pairs
//   RESID : the residual stream and the next norm's gain at this lane's four columns
struct EpiPre {
    floatx4 a, b;
    int pos;
};
template <int MODE>
__device__ inline void epi_request_first(EpiPre &p, int unit, int b, int lane, int N, int T, const DecodeEpi &e) {
    const int token = min((lane & 15) + 16 * b, T - 1), g = lane >> 4;
    if (MODE == DEC_QKV) p.pos = e.row_pos[token];
    if (MODE == DEC_RESID) {
        const int n0 = unit * 16 + 4 * g;
        p.a = *reinterpret_cast<const floatx4 *>(e.h + (size_t)token * N + n0);
        if (!e.last_layer) p.b = *reinterpret_cast<const floatx4 *>(e.g_next + n0);
    }
}
template <int MODE>
__device__ inline void epi_request_second(EpiPre &p, int unit, int lane, const DecodeEpi &e) {
    if (MODE == DEC_QKV) {
        const int d = e.kg.d, half = d >> 1, tiles_per_head = d >> 4, g = lane >> 4;
        const int head = unit / tiles_per_head, tl = unit - head * tiles_per_head;
        if (head < e.hq_l + e.kg.hkv_l) {
            const int i0 = tl * 8 + 4 * (g & 1);
            p.a = *reinterpret_cast<const floatx4 *>(e.cos_tab + (size_t)p.pos * half + i0);
            p.b = *reinterpret_cast<const floatx4 *>(e.sin_tab + (size_t)p.pos * half + i0);
        }
    }
}

// Register epilogue of one unit (UT 16-feature tiles) and one 16-token tile, on complete dot products in the
// 16x16 accumulator layout: lane = (token j = lane % 16, row group g = lane / 16) holds rows 4g .. 4g+3 of each tile.
// Must be called by a whole wave (it shuffles across the row groups).
template <int MODE, int UT>
__device__ inline void decode_epilogue(const floatx4 (&v)[UT], int unit, int b, int lane, int N, int T, const DecodeEpi &e,
                                       const float *s_rstd, const EpiPre &pre) {
    const int token = (lane & 15) + 16 * b, g = lane >> 4;
    const bool valid = token < T;
    const float r = (MODE != DEC_RESID && valid) ? s_rstd[token] : 1.0f;

    if (MODE == DEC_RAW) {
#pragma unroll
        for (int u = 0; u < UT; ++u) {
            const int n0 = (unit * UT + u) * 16 + 4 * g;
            if (valid) *reinterpret_cast<floatx4 *>(e.raw_out + (size_t)token * N + n0) = v[u] * r;
        }
    } else if (MODE == DEC_RESID) {
        const int n0 = unit * 16 + 4 * g;
        float ss = 0.f;
        if (valid) {
            const floatx4 h4 = pre.a;
            if (e.last_layer) {
                // stage output: the partial without residual, and the residual it belongs to
                uint2 po;
                po.x = pack_h16x2(v[0][0], v[0][1]);
                po.y = pack_h16x2(v[0][2], v[0][3]);
                *reinterpret_cast<uint2 *>(e.out_partial + (size_t)token * N + n0) = po;
                if (e.out_resid) {
                    uint2 ro;
                    ro.x = pack_h16x2(h4[0], h4[1]);
                    ro.y = pack_h16x2(h4[2], h4[3]);
                    *reinterpret_cast<uint2 *>(e.out_resid + (size_t)token * N + n0) = ro;
                }
            } else {
                const floatx4 hn = h4 + v[0];
                *reinterpret_cast<floatx4 *>(e.h + (size_t)token * N + n0) = hn;
                const floatx4 g4 = pre.b;
                const float x[4] = {hn[0] * g4[0], hn[1] * g4[1], hn[2] * g4[2], hn[3] * g4[3]};
                store_act4(x, e.hg, token, n0, N >> 5);
                ss = hn[0] * hn[0] + hn[1] * hn[1] + hn[2] * hn[2] + hn[3] * hn[3];
            }
        }
        if (!e.last_layer) {
            ss += __shfl_xor(ss, 16, 64);
            ss += __shfl_xor(ss, 32, 64);
            if (g == 0 && valid) e.ssq_out[unit * DEC_SSQ_STRIDE + token] = ss;
        }
    } else if (MODE == DEC_SWIGLU) {
        // unit = one gate tile (v[0]) and the matching up tile (v[1]): 16 features of u
        if (valid) {
            const int f0 = unit * 16 + 4 * g;
            float uu[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float aa = v[0][j] * r;
                uu[j] = aa / (1.0f + __expf(-aa)) * (v[UT - 1][j] * r);
            }
            store_act4(uu, e.u, token, f0, e.F_l >> 5);
        }
    } else {   // DEC_QKV
        const int d = e.kg.d, half = d >> 1, tiles_per_head = d >> 4;
        const int head = unit / tiles_per_head, tl = unit - head * tiles_per_head;
        floatx4 mine = v[0] * r, other;
#pragma unroll
        for (int j = 0; j < 4; ++j) other[j] = __shfl_xor(mine[j], 32, 64);
        const bool low = g < 2;                       // rows 0-7 of the tile: features i; rows 8-15: i + d/2
        const int i0 = tl * 8 + 4 * (g & 1);          // first rotary pair index held by this lane
        if (valid) {
            const int pos = pre.pos;
            float out[4];
            if (head < e.hq_l + e.kg.hkv_l) {
                const floatx4 c4 = pre.a, s4 = pre.b;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float lo = low ? mine[j] : other[j], hi = low ? other[j] : mine[j];
                    out[j] = low ? lo * c4[j] - hi * s4[j] : hi * c4[j] + lo * s4[j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) out[j] = mine[j];
            }
            const int e0 = i0 + (low ? 0 : half);     // element index inside the head
            if (head < e.hq_l) {
                store_split4(out, e.q_hi, e.q_lo, ((size_t)token * e.hq_l + head) * d + e0);
            } else if (head < e.hq_l + e.kg.hkv_l) {
                const size_t slab = (size_t)token * e.kg.seq_stride + (size_t)(head - e.hq_l) * e.kg.smax * d;
                uint2 o;
                o.x = pack_h16x2(out[0], out[1]);
                o.y = pack_h16x2(out[2], out[3]);
                *reinterpret_cast<uint2 *>(e.kc + slab + kv_k_offset(pos, e0, d)) = o;
            } else {
                const size_t slab =
                    (size_t)token * e.kg.seq_stride + (size_t)(head - e.hq_l - e.kg.hkv_l) * e.kg.smax * d;
#pragma unroll
                for (int j = 0; j < 4; ++j) e.vc[slab + kv_v_offset(pos, e0 + j, d)] = f32_to_h16(out[j]);
            }
        }
    }
}

constexpr int kXldsMaxBytes = 64 * 1024;      // activation operand staged in LDS up to this size

// XLDS: the whole activation operand (T <= 2 rows) is staged once per block in LDS, so the main loop
// issues nothing but weight loads; otherwise each lane fetches its 16-byte pieces per k-tile (L2 hits).
template <int NB, int UT, int WAVES, int UNROLL, int MODE, bool XLDS, int XR>
__global__ __launch_bounds__(WAVES * 64) void decode_proj_kernel(const h16_t *__restrict__ Wp,
                                                                const h16_t *__restrict__ Xa, int N, int k_tiles,
                                                                int T, DecodeEpi e) {
    __shared__ floatx4 red[WAVES][UT * NB][64];
    __shared__ float s_rstd[32];
    extern __shared__ h16x8 xs[];          // XLDS: copy of Xa, [token][k_tile][plane][lane group]
    const int unit = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;

    floatx4 acc[UT][NB];
#pragma unroll
    for (int u = 0; u < UT; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[u][b] = floatx4{0.f, 0.f, 0.f, 0.f};

    const h16x8 *wp[UT];
#pragma unroll
    for (int u = 0; u < UT; ++u)
        wp[u] = reinterpret_cast<const h16x8 *>(Wp) + (size_t)(unit * UT + u) * 64 + lane;
    const size_t kstride = (size_t)(N >> 4) * 64;          // k-tile-major weights: one k-tile of all features
    // operand B of lane (token j, group g) for k-tile kt: hi at x[b][kt * 8], lo at x[b][kt * 8 + 4]
    const h16x8 *xg[NB];
    bool xv[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int token = (lane & 15) + 16 * b;
        xv[b] = token < T;
        xg[b] = (XLDS ? xs : reinterpret_cast<const h16x8 *>(Xa)) + (size_t)(xv[b] ? token : 0) * k_tiles * 8 + (lane >> 4);
    }
    const h16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    // Wave w owns k-tiles w, w + WAVES, ...; it holds a ring of UNROLL of them per feature tile in registers.  The
    // first ring round is requested before anything else, so the weights are already on their way while the block
    // stages the activation operand and derives the rows' rstd.
    const int rounds = (k_tiles - wave + WAVES - 1) / WAVES / UNROLL;
    // request order = arrival order: the operand copy and the sums of squares (L2 hits) go out first and are
    // waited for first; the weights requested right behind them stay in flight meanwhile
    // (every request below is unconditional, out-of-range ones re-read a valid address: the compiler can only count
    // requests in flight exactly, and so wait for the oldest alone, when none of them sits behind a branch)
    EpiPre pre;
    const bool finisher = wave < NB;          // wave b finishes token tile b
    if (finisher) epi_request_first<MODE>(pre, unit, wave, lane, N, T, e);
    h16x8 xr[XLDS ? XR : 1];
    const int n16 = T * k_tiles * 8;
    if (XLDS) {
#pragma unroll
        for (int j = 0; j < XR; ++j)
            xr[j] = reinterpret_cast<const h16x8 *>(Xa)[min((int)threadIdx.x + j * WAVES * 64, n16 - 1)];
    }
    float sv[RSTD_REGS];
    const bool rstd_wave = MODE != DEC_RESID && wave < T && e.ssq_in != nullptr;       // wave t derives rstd of row t
    if (rstd_wave) rstd_request(e, wave, lane, sv);
    // ring slot = the weight tiles of one k-tile and, when the operand is not staged in LDS, its hi / lo pieces too
    // (requested together, so that no wait for an operand piece ever drains the weight requests behind it)
    h16x8 a[UNROLL][UT], xq[XLDS ? 1 : UNROLL][NB][2];
    auto request = [&](int i, int kt) {
        if (!XLDS) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                // unconditional (see above): lanes past the last row re-read row 0 and feed output columns nobody stores
                xq[i][b][0] = xg[b][kt * 8];
                xq[i][b][1] = xg[b][kt * 8 + 4];
            }
        }
#pragma unroll
        for (int u = 0; u < UT; ++u) a[i][u] = __builtin_nontemporal_load(wp[u] + (size_t)kt * kstride);
    };
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) request(i, min(wave + i * WAVES, k_tiles - 1));
    if (finisher) epi_request_second<MODE>(pre, unit, lane, e);
    if (XLDS) {
#pragma unroll
        for (int j = 0; j < XR; ++j) {
            const int idx = threadIdx.x + j * WAVES * 64;
            if (idx < n16) xs[idx] = xr[j];
        }
    }
    if (rstd_wave) rstd_finish(e, wave, lane, sv, s_rstd);
    if (MODE != DEC_RESID)
        for (int t = rstd_wave ? wave + WAVES : wave; t < T; t += WAVES) rstd_row(e, t, lane, s_rstd);
    if (XLDS) __syncthreads();       // (s_rstd is read behind the barrier of the reduction below)

    // the k-tile held by ring slot i against the operand
    auto contract = [&](int i, int kt) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            h16x8 x, y;
            if (XLDS) {
                x = xv[b] ? xg[b][kt * 8] : zero;
                y = xv[b] ? xg[b][kt * 8 + 4] : zero;
            } else {
                x = xq[i][b][0];
                y = xq[i][b][1];
            }
#pragma unroll
            for (int u = 0; u < UT; ++u) {
                acc[u][b] = hx_mfma16(a[i][u], y, acc[u][b]);
                acc[u][b] = hx_mfma16(a[i][u], x, acc[u][b]);
            }
        }
    };
    // steady state: slot i is consumed and at once refilled with the tile one ring round ahead, so UNROLL - 1
    // requests per feature tile stay in flight all the time
    for (int rd = 1; rd < rounds; ++rd) {
#pragma unroll
        for (int i = 0; i < UNROLL; ++i) {
            const int kt = wave + ((rd - 1) * UNROLL + i) * WAVES;
            contract(i, kt);
            request(i, kt + UNROLL * WAVES);
            if (!XLDS) __builtin_amdgcn_sched_barrier(0);       // keep each refill right behind its slot's use
        }
    }
    // The last full round is refilled as well, with the wave's remaining (fewer than UNROLL) k-tiles, so that those are
    // in flight while the round is consumed instead of being fetched one by one behind it; slots past the last k-tile
    // re-read it (unconditional requests, see above) and are not used.  With no full round at all the first ring round,
    // requested at kernel start, already is this remainder.
    const int kt_rem = wave + rounds * UNROLL * WAVES;       // the wave's first k-tile beyond its full rounds
    if (rounds > 0) {
        if (kt_rem < k_tiles) {       // (uniform over the wave; a wave without remainder issues no request it does not use)
#pragma unroll
            for (int i = 0; i < UNROLL; ++i) {
                contract(i, wave + ((rounds - 1) * UNROLL + i) * WAVES);
                request(i, min(kt_rem + i * WAVES, k_tiles - 1));
                if (!XLDS) __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < UNROLL; ++i) contract(i, wave + ((rounds - 1) * UNROLL + i) * WAVES);
        }
    }
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const int kt = kt_rem + i * WAVES;       // uniform over the wave
        if (kt < k_tiles) contract(i, kt);
    }

#pragma unroll
    for (int u = 0; u < UT; ++u)
#pragma unroll
        for (int b = 0; b < NB; ++b) red[wave][u * NB + b][lane] = acc[u][b];
    __syncthreads();
    if (!finisher) return;

    const int b = wave;
    floatx4 v[UT];
#pragma unroll
    for (int u = 0; u < UT; ++u) {
        v[u] = red[0][u * NB + b][lane];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) v[u] += red[w][u * NB + b][lane];
    }
    decode_epilogue<MODE, UT>(v, unit, b, lane, N, T, e, s_rstd, pre);
}

// -------------------------------------------------------------------------------------------------
// Batched decode (3 <= T <= 32 rows).  With more than a couple of rows the activation operand outweighs the
// weights a block streams (32 rows of hi + lo pairs are 4 KB per k-tile against 1 KB of weights per 16 features),
// and fetching it per wave from L2 in 64-byte pieces leaves the kernel at a quarter of the HBM rate.  Here the
// eight waves of a block own eight neighbouring feature tiles and walk the SAME k-tiles, so the block stages each
// 8-k-tile chunk of the operand once in LDS (global -> registers -> LDS, double-buffered) and all waves read it
// from there; a k-tile's weights for the block are one contiguous 8 KB run.  To still fill the chip the
// contraction is split over blockIdx.y; the fp32 partial sums go to a scratch buffer [split][token][feature] and
// decode_finish_kernel adds them in split order (bit-reproducible) and runs the same register epilogue as the
// single-kernel path.
// -------------------------------------------------------------------------------------------------
constexpr int SK_CH = 8;                       // k-tiles per chunk: 1 KB of one token's compact operand
constexpr int SK_TOK_STRIDE = 1024 + 16;       // LDS bytes per token and chunk; the pad spreads tokens over the banks

template <int NB>
__global__ __launch_bounds__(512) void decode_splitk_kernel(const h16_t *__restrict__ Wp, const h16_t *__restrict__ Xa,
                                                           int n_tiles, int k_tiles, int T,
                                                           float *__restrict__ part, const float *__restrict__ ssq_in,
                                                           int ssq_units, int norm_dim, float eps,
                                                           float *__restrict__ rstd_out) {
    constexpr int TOK = 16 * NB, LPW = TOK / 8;        // token rows staged per chunk; rows copied per wave
    constexpr int BUF = TOK * SK_TOK_STRIDE;
    extern __shared__ unsigned char sk_lds[];          // [2][TOK][SK_TOK_STRIDE]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
    const int tile = blockIdx.x * 8 + wave;
    const bool tile_ok = tile < n_tiles;
    // the chunks of the contraction are dealt out evenly over the splits (blockIdx.y)
    const int chunks = (k_tiles + SK_CH - 1) / SK_CH;
    const int kt0 = (int)((long)blockIdx.y * chunks / gridDim.y) * SK_CH;
    const int kt1 = min(k_tiles, (int)((long)(blockIdx.y + 1) * chunks / gridDim.y) * SK_CH);
    const int n_chunks = (kt1 - kt0 + SK_CH - 1) / SK_CH;
    const int N = n_tiles * 16;

    // chunk c of the operand rows this wave copies: lane l carries bytes 16 l .. 16 l + 15 of the row's 1 KB
    const h16x8 *xsrc[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i)
        xsrc[i] = reinterpret_cast<const h16x8 *>(Xa) + (size_t)min(wave + 8 * i, T - 1) * k_tiles * 8 + lane;
    auto load_x = [&](int c, h16x8(&x)[LPW]) {
        const int kc = kt0 + c * SK_CH;
        const bool ok = c < n_chunks && kc + (lane >> 3) < kt1;         // 8 lanes per k-tile line
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            if (ok) x[i] = xsrc[i][(size_t)kc * 8];
    };
    auto store_x = [&](int c, const h16x8(&x)[LPW]) {
        unsigned char *buf = sk_lds + (c & 1) * BUF;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            *reinterpret_cast<h16x8 *>(buf + (wave + 8 * i) * SK_TOK_STRIDE + lane * 16) = x[i];
    };
    // this wave's weight tile for the k-tiles of chunk c
    const h16x8 *wsrc = reinterpret_cast<const h16x8 *>(Wp) + (size_t)min(tile, n_tiles - 1) * 64 + lane;
    const size_t kstride = (size_t)n_tiles * 64;
    const h16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    auto load_w = [&](int c, h16x8(&w)[SK_CH]) {
        const int kc = kt0 + c * SK_CH;
#pragma unroll
        for (int i = 0; i < SK_CH; ++i)
            w[i] = (c < n_chunks && kc + i < kt1) ? __builtin_nontemporal_load(wsrc + (size_t)(kc + i) * kstride) : zero;
    };

    // On the side: the rows' rstd for the finishing kernel, each row by one wave of one block of the launch (the
    // sums of squares are requested now and added up after the main loop, when they have long arrived).
    const int n_blocks = gridDim.x * gridDim.y, bid = blockIdx.y * gridDim.x + blockIdx.x;
    const int rstd_row = bid + wave * n_blocks;
    const bool rstd_mine = rstd_out != nullptr && rstd_row < T;
    float sv[RSTD_REGS];
    if (rstd_mine && ssq_in != nullptr) {
#pragma unroll
        for (int q = 0; q < RSTD_REGS; ++q) sv[q] = ssq_in[min(lane + 64 * q, ssq_units - 1) * DEC_SSQ_STRIDE + rstd_row];
    }

    floatx4 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
    h16x8 xr[LPW], wc[SK_CH], wn[SK_CH];
#pragma unroll
    for (int i = 0; i < LPW; ++i) xr[i] = zero;
    load_x(0, xr);
    load_w(0, wc);
    store_x(0, xr);
    load_x(1, xr);
    for (int c = 0; c < n_chunks; ++c) {
        // chunk c is complete in LDS for every wave, and nobody reads the other buffer (chunk c - 1) any more;
        // a bare s_barrier: __syncthreads() would also drain the weight loads in flight
        __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
        asm volatile("s_barrier" ::: "memory");
        store_x(c + 1, xr);
        load_x(c + 2, xr);
        load_w(c + 1, wn);
        const unsigned char *buf = sk_lds + (c & 1) * BUF;
        const int nk = min(SK_CH, kt1 - (kt0 + c * SK_CH));
#pragma unroll
        for (int i = 0; i < SK_CH; ++i) {
            if (i < nk) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const unsigned char *row = buf + (j + 16 * b) * SK_TOK_STRIDE + i * 128 + g * 16;
                    const h16x8 x = *reinterpret_cast<const h16x8 *>(row);
                    const h16x8 y = *reinterpret_cast<const h16x8 *>(row + 64);
                    acc[b] = hx_mfma16(wc[i], y, acc[b]);
                    acc[b] = hx_mfma16(wc[i], x, acc[b]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < SK_CH; ++i) wc[i] = wn[i];
    }
    if (rstd_mine) {
        float r = 1.0f;
        if (ssq_in != nullptr) {
            float ss = 0.f;
#pragma unroll
            for (int q = 0; q < RSTD_REGS; ++q) ss += lane + 64 * q < ssq_units ? sv[q] : 0.f;
            for (int i = lane + 64 * RSTD_REGS; i < ssq_units; i += 64) ss += ssq_in[i * DEC_SSQ_STRIDE + rstd_row];
            ss = wave_sum(ss);
            r = 1.0f / sqrtf(ss / (float)norm_dim + eps);
        }
        if (lane == 0) rstd_out[rstd_row] = r;
    }
    if (rstd_out != nullptr)           // a launch of fewer than T / 8 blocks: the rows not dealt out above
        for (int row = rstd_row + 8 * n_blocks; row < T; row += 8 * n_blocks) {
            float r = 1.0f;
            if (ssq_in != nullptr) {
                float ss = 0.f;
                for (int i = lane; i < ssq_units; i += 64) ss += ssq_in[i * DEC_SSQ_STRIDE + row];
                ss = wave_sum(ss);
                r = 1.0f / sqrtf(ss / (float)norm_dim + eps);
            }
            if (lane == 0) rstd_out[row] = r;
        }
    if (!tile_ok) return;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int token = j + 16 * b;
        if (token < T)
            *reinterpret_cast<floatx4 *>(part + ((size_t)blockIdx.y * T + token) * N + tile * 16 + 4 * g) = acc[b];
    }
}

// Sums the split partials in split order and runs the register epilogue; one wave per (unit, 16-token tile).
// rstd[T]: the rows' reciprocal rms, left by the split kernel of the same projection.
template <int MODE, int UT>
__global__ __launch_bounds__(256) void decode_finish_kernel(const float *__restrict__ part, int splits, int N, int T,
                                                           int n_units, DecodeEpi e, const float *__restrict__ rstd) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nbt = (T + 15) >> 4;
    const int idx = blockIdx.x * 4 + wave;
    if (idx >= n_units * nbt) return;
    const int unit = idx / nbt, b = idx - unit * nbt;
    const int token = (lane & 15) + 16 * b, g = lane >> 4;
    EpiPre pre;
    epi_request_first<MODE>(pre, unit, b, lane, N, T, e);
    epi_request_second<MODE>(pre, unit, lane, e);
    floatx4 v[UT];
#pragma unroll
    for (int u = 0; u < UT; ++u) {
        v[u] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (token < T)
#pragma unroll 4
            for (int ks = 0; ks < splits; ++ks)
                v[u] += *reinterpret_cast<const floatx4 *>(part + ((size_t)ks * T + token) * N + (unit * UT + u) * 16 + 4 * g);
    }
    decode_epilogue<MODE, UT>(v, unit, b, lane, N, T, e, rstd, pre);
}

namespace {

template <int NB, int UT, int UNR, int MODE, bool XLDS, int XR>
void launch_one(const h16_t *Wp, const h16_t *Xa, int N, int k_tiles, int T, const DecodeEpi &e, hipStream_t s) {
    constexpr int WAVES = 8;
    auto kern = decode_proj_kernel<NB, UT, WAVES, UNR, MODE, XLDS, XR>;
    size_t dyn = 0;
    if (XLDS) {
        dyn = (size_t)T * k_tiles * 8 * sizeof(h16x8);
        static bool raised = false;       // static + dynamic LDS may exceed the default 64 KB per block
        if (!raised) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      kXldsMaxBytes);
            raised = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3(N / 16 / UT), dim3(WAVES * 64), dyn, s, Wp, Xa, N, k_tiles, T, e);
}

template <int UT, int MODE>
void launch_mode(const h16_t *Wp, const h16_t *Xa, int N, int k_tiles, int T, const DecodeEpi &e, hipStream_t s) {
    const size_t xbytes = (size_t)T * k_tiles * 8 * sizeof(h16x8);
    // staged operand: XR 16-byte pieces per thread (512 threads), 4 up to 32 KB, 8 up to 64 KB
    // With one or two rows each wave of the residual projections (W_O, W2) and of W1/W3 fetches its operand pieces
    // through its request ring instead of the block staging the operand in LDS behind a barrier (measured: W_O
    // 17.9 -> 16.6 us and W2 44.0 -> 43.4 at one row, W1/W3 81.0 -> 77.9 at two rows and unchanged at one).  The
    // QKV projection keeps the staged operand: through the ring it loses 3.5 us.
    if ((MODE == DEC_RESID || MODE == DEC_SWIGLU) && T <= 2) {
        // (a contraction of at most 32 k-tiles gives a wave 4 of them: a ring of 4 requests nothing it does not use)
        if constexpr (UT == 1) {
            if (k_tiles <= 32) { launch_one<1, 1, 4, MODE, false, 1>(Wp, Xa, N, k_tiles, T, e, s); return; }
        }
        launch_one<1, UT, 8 / UT, MODE, false, 1>(Wp, Xa, N, k_tiles, T, e, s);
        return;
    }
    if (T <= 2 && xbytes <= (size_t)kXldsMaxBytes / 2) launch_one<1, UT, 8 / UT, MODE, true, 4>(Wp, Xa, N, k_tiles, T, e, s);
    else if (T <= 2 && xbytes <= (size_t)kXldsMaxBytes) launch_one<1, UT, 8 / UT, MODE, true, 8>(Wp, Xa, N, k_tiles, T, e, s);
    else if (T <= 16) launch_one<1, UT, 8 / UT, MODE, false, 1>(Wp, Xa, N, k_tiles, T, e, s);
    else launch_one<2, UT, 8 / UT, MODE, false, 1>(Wp, Xa, N, k_tiles, T, e, s);
}
}  // namespace

namespace {
template <int MODE, int UT>
void launch_splitk(const h16_t *Wp, const h16_t *Xa, int N, int k_tiles, int T, const DecodeEpi &e, float *scratch,
                   size_t scratch_floats, hipStream_t s, hipEvent_t mid, QkvTail *tail = nullptr) {
    const int n_tiles = N / 16, groups = (n_tiles + 7) / 8;
    // Two blocks fit a CU (registers), 512 on the chip.  The number of splits (at most 8, or 16 for a matrix of fewer than 64
    // feature groups: the finishing kernel walks them one after the other; partials within the scratch) minimises rounds of blocks x chunks per block, the time
    // of the launch in units of one chunk per block; on a tie the fewer splits (less partial-sum traffic) win.
    const int chunks = (k_tiles + SK_CH - 1) / SK_CH;
    const size_t part_floats = scratch_floats - 32;      // the last 32 floats of the scratch carry the rows' rstd
    float *rstd = scratch + part_floats;
    int splits = 1;
    long best = -1;
    const int cap = groups * 8 < 512 ? 16 : 8;      // a narrow matrix (TP8 QKV: 10 groups) fills more of the chip with 16
    for (int c = 1; c <= std::min(cap, chunks); ++c) {
        if (c > 1 && (size_t)c * T * N > part_floats) break;
        const long cost = (long)((groups * c + 511) / 512) * ((chunks + c - 1) / c) * 16 + c;
        if (best < 0 || cost < best) { best = cost; splits = c; }
    }
    const int nb = T > 16 ? 2 : 1;
    const size_t lds = (size_t)2 * 16 * nb * SK_TOK_STRIDE;
    const dim3 grid(groups, splits);
    if (nb == 2) {
        static bool raised = false;           // 65 KB: above the default limit
        if (!raised) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(decode_splitk_kernel<2>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            raised = true;
        }
        hipLaunchKernelGGL(decode_splitk_kernel<2>, grid, dim3(512), lds, s, Wp, Xa, n_tiles, k_tiles, T, scratch, e.ssq_in,
                           e.ssq_units, e.norm_dim, e.eps, rstd);
    } else {
        hipLaunchKernelGGL(decode_splitk_kernel<1>, grid, dim3(512), lds, s, Wp, Xa, n_tiles, k_tiles, T, scratch, e.ssq_in,
                           e.ssq_units, e.norm_dim, e.eps, rstd);
    }
    if (mid) (void)hipEventRecord(mid, s);
    if (tail != nullptr) {          // the consumer finishes the projection (QKV -> decode attention)
        *tail = QkvTail{scratch, splits, T, N, rstd, e.cos_tab, e.sin_tab};
        return;
    }
    const int n_units = n_tiles / UT, nbt = (T + 15) / 16;
    hipLaunchKernelGGL((decode_finish_kernel<MODE, UT>), dim3((n_units * nbt + 3) / 4), dim3(256), 0, s, scratch, splits, N, T,
                       n_units, e, rstd);
}
}  // namespace

void launch_decode_proj(const h16_t *Wp, const h16_t *Xa, int N, int K, int T, const DecodeEpi &e, float *scratch,
                        size_t scratch_floats, hipStream_t s, hipEvent_t mid) {
    const int k_tiles = K / 32;
    // one or two rows: one kernel, complete dot products per block; more: shared operand, split contraction
    // A small matrix (launch-bound) with a handful of rows is better off without the second kernel: each block then
    // fetches the rows' operand pieces itself (an L2 read of T x K x 4 bytes per block, which is what limits this to
    // few rows, fewer when the contraction is long), and needs enough k-tiles per wave to fill its request ring.
    const bool small = (size_t)N * K * sizeof(h16_t) <= ((size_t)72 << 20) && k_tiles >= 64 && T <= (K <= 4096 ? 8 : 4);
    // A residual projection with a short contraction (W_O of a narrow shard: 1024 or 2048 long) is one kernel as well:
    // a block holds complete dot products after 4 (8) k-tiles per wave, its ring sized to exactly that, and what the
    // split path adds -- partial sums, a second launch -- costs more than the rows' operand pieces fetched per block.
    // Measured on 70B shards, W_O per layer: TP8 (32 k-tiles) 3 / 8 / 16 / 17 / 32 rows 11.3 / 12.0 / 12.3 / 12.9 / 13.0 ->
    // 8.1 / 8.5 / 9.7 / 10.8 / 12.8 us; TP4 (64 k-tiles) 9 / 16 rows 15.3 / 15.9 -> 12.6 / 14.4, but 32 rows 17.7 -> 21.8.
    const bool short_k = e.mode == DEC_RESID && T > 2 && !small && k_tiles >= 8 &&
                         ((k_tiles <= 32 && T <= 32) || (k_tiles <= 64 && T <= 16));
    if (short_k) {
        if (k_tiles <= 32) {
            if (T <= 16) launch_one<1, 1, 4, DEC_RESID, false, 1>(Wp, Xa, N, k_tiles, T, e, s);
            else launch_one<2, 1, 4, DEC_RESID, false, 1>(Wp, Xa, N, k_tiles, T, e, s);
        } else {
            launch_one<1, 1, 8, DEC_RESID, false, 1>(Wp, Xa, N, k_tiles, T, e, s);
        }
        if (mid) (void)hipEventRecord(mid, s);
        return;
    }
    if (T > 2 && !small && scratch != nullptr && scratch_floats >= (size_t)T * N + 32 && k_tiles >= SK_CH) {
        switch (e.mode) {
            case DEC_RAW: launch_splitk<DEC_RAW, 1>(Wp, Xa, N, k_tiles, T, e, scratch, scratch_floats, s, mid); break;
            case DEC_QKV: launch_splitk<DEC_QKV, 1>(Wp, Xa, N, k_tiles, T, e, scratch, scratch_floats, s, mid); break;
            case DEC_RESID: launch_splitk<DEC_RESID, 1>(Wp, Xa, N, k_tiles, T, e, scratch, scratch_floats, s, mid); break;
            case DEC_SWIGLU: launch_splitk<DEC_SWIGLU, 2>(Wp, Xa, N, k_tiles, T, e, scratch, scratch_floats, s, mid); break;
        }
        return;
    }
    switch (e.mode) {
        case DEC_RAW:
            // two feature tiles per block (2 KB of weights per wave and k-tile) stream a few percent faster than one
            if ((N / 16) % 2 == 0 && N / 32 >= 512) launch_mode<2, DEC_RAW>(Wp, Xa, N, k_tiles, T, e, s);
            else launch_mode<1, DEC_RAW>(Wp, Xa, N, k_tiles, T, e, s);
            break;
        case DEC_QKV: launch_mode<1, DEC_QKV>(Wp, Xa, N, k_tiles, T, e, s); break;
        case DEC_RESID: launch_mode<1, DEC_RESID>(Wp, Xa, N, k_tiles, T, e, s); break;
        case DEC_SWIGLU: launch_mode<2, DEC_SWIGLU>(Wp, Xa, N, k_tiles, T, e, s); break;
    }
    if (mid) (void)hipEventRecord(mid, s);
}

void launch_decode_qkv(const h16_t *Wp, const h16_t *Xa, int N, int K, int T, const DecodeEpi &e, float *scratch,
                       size_t scratch_floats, QkvTail *tail, hipStream_t s) {
    *tail = QkvTail{nullptr, 0, T, N, nullptr, e.cos_tab, e.sin_tab};
    const int k_tiles = K / 32;
    // the same choice between the single-kernel and the split path as launch_decode_proj makes
    // (a matrix of fewer than 128 feature tiles would run the single kernel on that many blocks: TP8's 80 tiles with
    // 3 / 4 rows took 14.8 / 15.0 us against 10.0 / 10.4 split, 2.5 us per layer after the attention's longer start)
    const bool small = (size_t)N * K * sizeof(h16_t) <= ((size_t)72 << 20) && k_tiles >= 64 && T <= (K <= 4096 ? 8 : 4) && N / 16 >= 128;
    if (e.mode == DEC_QKV && T > 2 && !small && scratch != nullptr && scratch_floats >= (size_t)T * N + 32 && k_tiles >= SK_CH)
        launch_splitk<DEC_QKV, 1>(Wp, Xa, N, k_tiles, T, e, scratch, scratch_floats, s, nullptr, tail);
    else
        launch_decode_proj(Wp, Xa, N, K, T, e, scratch, scratch_floats, s, nullptr);
}

// -------------------------------------------------------------------------------------------------
// Per-step prologue: stage input rows (bf16, or fp32 for the validation surface) -> fp32 residual
// stream, (x * gain) hi/lo operand of the first projection, per-unit sums of squares (one unit = 16
// columns, as written by the RESID epilogue).  Block 0 also publishes each row's position (the
// sequence's committed length) and, when asked, advances the lengths.
// grid = H / 128 blocks of 512 threads; thread = (token, 4-column group).
// -------------------------------------------------------------------------------------------------
template <bool IN_H16>
__global__ __launch_bounds__(512) void decode_prologue_kernel(const void *__restrict__ in, const void *__restrict__ in2,
                                                             float *__restrict__ h_out,
                                                             const float *__restrict__ g, h16_t *__restrict__ hg,
                                                             float *__restrict__ ssq_out,
                                                             int T, int H, int32_t *lens, int32_t *row_pos,
                                                             int advance) {
    if (blockIdx.x == 0 && lens != nullptr && threadIdx.x < T) {
        const int l = lens[threadIdx.x];
        row_pos[threadIdx.x] = l;
        if (advance) lens[threadIdx.x] = l + 1;
    }
    // 32 column quads per block (128 columns), 16 tokens per pass
    const int quad = threadIdx.x & 31, tsub = threadIdx.x >> 5;
    const int col = blockIdx.x * 128 + quad * 4;
    for (int t = tsub; t < T; t += 16) {
        float ss = 0.f;
        if (col < H) {
            float x[4];
            if (IN_H16) {
                uint2 raw = *reinterpret_cast<const uint2 *>(reinterpret_cast<const h16_t *>(in) + (size_t)t * H + col);
                h16x2_to_f32(raw.x, x[0], x[1]);
                h16x2_to_f32(raw.y, x[2], x[3]);
                if (in2) {      // second addend (e.g. a stage's partial on top of its residual stream)
                    raw = *reinterpret_cast<const uint2 *>(reinterpret_cast<const h16_t *>(in2) + (size_t)t * H + col);
                    float y0, y1, y2, y3;
                    h16x2_to_f32(raw.x, y0, y1);
                    h16x2_to_f32(raw.y, y2, y3);
                    x[0] += y0; x[1] += y1; x[2] += y2; x[3] += y3;
                }
            } else {
                const floatx4 a = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const float *>(in) + (size_t)t * H + col);
                x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3];
                if (in2) {
                    const floatx4 c = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const float *>(in2) + (size_t)t * H + col);
                    x[0] += c[0]; x[1] += c[1]; x[2] += c[2]; x[3] += c[3];
                }
            }
            if (h_out) *reinterpret_cast<floatx4 *>(h_out + (size_t)t * H + col) = floatx4{x[0], x[1], x[2], x[3]};
            const floatx4 g4 = *reinterpret_cast<const floatx4 *>(g + col);
            const float y[4] = {x[0] * g4[0], x[1] * g4[1], x[2] * g4[2], x[3] * g4[3]};
            store_act4(y, hg, t, col, H >> 5);
            ss = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
        }
        // the 4 quads of one 16-column unit are 4 consecutive lanes
        ss += __shfl_xor(ss, 1, 64);
        ss += __shfl_xor(ss, 2, 64);
        if ((quad & 3) == 0 && col < H) ssq_out[(col >> 4) * DEC_SSQ_STRIDE + t] = ss;
    }
}

void launch_decode_prologue(const void *in, const void *in2, int in_is_h16, float *h_out, const float *g, h16_t *hg,
                            float *ssq_out, int T, int H, int32_t *lens, int32_t *row_pos, int advance, hipStream_t s) {
    const int blocks = (H + 127) / 128;
    if (in_is_h16)
        hipLaunchKernelGGL(decode_prologue_kernel<true>, dim3(blocks), dim3(512), 0, s, in, in2, h_out, g, hg, ssq_out, T, H,
                           lens, row_pos, advance);
    else
        hipLaunchKernelGGL(decode_prologue_kernel<false>, dim3(blocks), dim3(512), 0, s, in, in2, h_out, g, hg, ssq_out, T, H,
                           lens, row_pos, advance);
}

}  // namespace HX_NS
