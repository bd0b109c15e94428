// Prefill projection: LDS-staged MFMA GEMM, D^T[n][t] = sum_k Wp[n][k] * Xp[t][k].
//
// A block is a WM x WT grid of waves; each wave owns FM x FT tiles of 32 features x 32 tokens computed with
// v_mfma_f32_32x32x16_bf16 (measured on this chip: 89 % of the datasheet rate from registers against 64 % for
// the 16x16x32 form, which is issue-limited).  The large configurations cover 256 x 256 per block: 8 waves of
// 128 x 64 (two waves per SIMD, 128 accumulator registers each) or 4 waves of 128 x 128 (256 accumulators).
// Operands stay in the 16 x 32 fragment tiles shared with the decode kernels (see common.h): global -> LDS
// is a straight copy, and a 32x32x16 operand is gathered from two neighbouring 16-row tiles with per-lane
// LDS addresses (every 16 lanes read 256 contiguous bytes: conflict-free).  Both MFMA inputs use the
// same gather, so the k-order inside a tile cancels.
// Weights are k-tile-major, so the weight tiles of a block's k-step are one contiguous run of HBM.
//
// blockIdx.x is remapped so that each XCD (blocks are dealt round-robin to the 8 XCDs) works on a
// contiguous range of tiles, token-block fastest: tiles resident on one XCD share weight panels in
// that XCD's L2.
#include <atomic>
#include <type_traits>

#include "kernels.h"
#include "kvlayout.h"

#define HX_AS1(p) ((const __attribute__((address_space(1))) void *)(p))
#define HX_AS3(p) ((__attribute__((address_space(3))) void *)(p))
// s_waitcnt that only constrains vmcnt (gfx9 encoding: vmcnt[3:0] | expcnt<<4 | lgkmcnt<<8 | vmcnt[5:4]<<14)
#define HX_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
// s_waitcnt lgkmcnt(0) alone (vmcnt and expcnt left at "no wait")
#define HX_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14))
// Workgroup barrier WITHOUT the device-memory release a __syncthreads() carries: that release would make
// the compiler drain every outstanding direct-to-LDS load (vmcnt(0)) at each k-step and undo the
// pipelining.  LDS reads of the previous step have been consumed by MFMAs before this point; the loads
// of the step about to be read are covered by the explicit vmcnt wait issued just before.
#define HX_LDS_BARRIER()                        \
    do {                                        \
        HX_WAIT_LGKM0();                        \
        asm volatile("s_barrier" ::: "memory"); \
    } while (0)

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

namespace HX_NS {


// ---- epilogue, in registers.  32 x 32 result: lane l holds token column l % 32 and, per register quad q,
// features 8 q + 4 (l / 32) .. + 3 of the 32-feature block, i.e. of the 16-row tile q / 2 its rows
// (q % 2) * 8 + 4 (l / 32) .. + 3.  Rotary pairs (tile rows r, r + 8) and gate / up pairs (tiles 2m, 2m + 1)
// therefore sit in the same lane, in quads q and q ^ 1 respectively q and q + 2: no cross-lane traffic.
// acc_of(i, j): the wave's result tile (i, j) of its FM x FT tiles of block (bm, bt), wave (wm, wt), each asked for once
// (the two-phase loop converts its 16 x 16 results tile by tile on demand); rstd_s: 1 / rms of the block's token columns.
template <int FM, int FT, int WM, int WT, int MODE, typename AccF>
__device__ __forceinline__ void gemm_epilogue(AccF acc_of, int bm, int bt, int wm, int wt, int lane, int N,
                                              int n_tiles, int T, const GemmEpi &e, const float *rstd_s,
                                              float *ssq_lds = nullptr) {
    constexpr int TA = 2 * FM * WM, TB = 2 * FT * WT, NTOK = TB * 16;
    const int hl = lane >> 5;
    if (MODE == DEC_RESID) {
        // Residual read-modify-write.  Walks the wave tile one 32-feature block (i) at a time and fetches the
        // residual values of block i + 1 before the stores of block i: the stream is loaded and stored through
        // the same pointer, so the compiler would not move a load above a store by itself, and with one or
        // two waves per SIMD nothing else hides the latency.
        float ssq[FT];
        int token[FT];
#pragma unroll
        for (int j = 0; j < FT; ++j) {
            ssq[j] = 0.f;
            token[j] = (bt * TB + (wt * FT + j) * 2) * 16 + (lane & 31);
        }
        floatx4 hv[2][FT][4];
        auto load_h = [&](floatx4(&dst)[FT][4], int i) {
#pragma unroll
            for (int j = 0; j < FT; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = (bm * TA + (wm * FM + i) * 2) * 16 + 8 * q + 4 * hl;
                    dst[j][q] = (token[j] < T && n < N)
                                    ? *reinterpret_cast<const floatx4 *>(e.h + h_tile_offset(token[j], n, N))
                                    : floatx4{0.f, 0.f, 0.f, 0.f};
                }
        };
        load_h(hv[0], 0);
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            floatx4 gv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = (bm * TA + (wm * FM + i) * 2) * 16 + 8 * q + 4 * hl;
                gv[q] = (n < N && !e.last_layer) ? *reinterpret_cast<const floatx4 *>(e.g_next + n)
                                                 : floatx4{0.f, 0.f, 0.f, 0.f};
            }
            if (i + 1 < FM) load_h(hv[(i + 1) & 1], i + 1);
#pragma unroll
            for (int j = 0; j < FT; ++j) {
                const floatx16 c = acc_of(i, j);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = (bm * TA + (wm * FM + i) * 2) * 16 + 8 * q + 4 * hl;
                    if (token[j] >= T || n >= N) continue;
                    const floatx4 h4 = hv[i & 1][j][q];
                    const floatx4 v = {c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]};
                    if (e.last_layer) {
                        uint2 po;
                        po.x = pack_h16x2(v[0], v[1]);
                        po.y = pack_h16x2(v[2], v[3]);
                        *reinterpret_cast<uint2 *>(e.out_partial + (size_t)token[j] * N + n) = po;
                        if (e.out_resid) {
                            uint2 ro;
                            ro.x = pack_h16x2(h4[0], h4[1]);
                            ro.y = pack_h16x2(h4[2], h4[3]);
                            *reinterpret_cast<uint2 *>(e.out_resid + (size_t)token[j] * N + n) = ro;
                        }
                    } else {
                        const floatx4 hn = h4 + v;
                        *reinterpret_cast<floatx4 *>(e.h + h_tile_offset(token[j], n, N)) = hn;
                        const floatx4 g4 = gv[q];
                        uint2 o;
                        o.x = pack_h16x2(hn[0] * g4[0], hn[1] * g4[1]);
                        o.y = pack_h16x2(hn[2] * g4[2], hn[3] * g4[3]);
                        *reinterpret_cast<uint2 *>(e.hg + frag_offset(token[j], n, N >> 5)) = o;
                        ssq[j] += hn[0] * hn[0] + hn[1] * hn[1] + hn[2] * hn[2] + hn[3] * hn[3];
                    }
                }
            }
        }
        if (!e.last_layer) {
            // sum of squares of each token over the 128 features of one partial: the two lane halves hold disjoint rows
            static_assert(MODE != DEC_RESID || 32 * FM == GEMM_SSQ_COLS || (32 * FM * WM == GEMM_SSQ_COLS && WT == 1),
                          "one partial per wave, or per block, and token");
            if constexpr (32 * FM == GEMM_SSQ_COLS) {
                const int grp = (bm * TA + wm * FM * 2) * 16 / GEMM_SSQ_COLS;
#pragma unroll
                for (int j = 0; j < FT; ++j) {
                    const float tot = ssq[j] + __shfl_xor(ssq[j], 32, 64);
                    if (hl == 0 && token[j] < T) e.ssq_out[(size_t)grp * T + token[j]] = tot;
                }
            } else {
                // the block's WM waves each hold a quarter of the partial's features: summed through LDS in wave order
#pragma unroll
                for (int j = 0; j < FT; ++j) {
                    const float tot = ssq[j] + __shfl_xor(ssq[j], 32, 64);
                    if (hl == 0) ssq_lds[wm * NTOK + j * 32 + (lane & 31)] = tot;
                }
                __syncthreads();
                if (wm == 0) {
#pragma unroll
                    for (int j = 0; j < FT; ++j) {
                        float tot = 0.f;
#pragma unroll
                        for (int w = 0; w < WM; ++w) tot += ssq_lds[w * NTOK + j * 32 + (lane & 31)];
                        if (hl == 0 && token[j] < T) e.ssq_out[(size_t)bm * T + token[j]] = tot;
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < FT; ++j) {
        const int tl = (wt * FT + j) * 32 + (lane & 31);       // token column inside the block tile
        const int token = bt * NTOK + tl;
        const bool tv = token < T;
        const float r = e.ssq_in != nullptr ? rstd_s[tl] : 1.0f;
        int seq = 0, pos = 0;
        if (MODE == DEC_QKV && tv) { seq = e.rm.row_seq[token]; pos = e.rm.row_pos[token]; }
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int t16 = bm * TA + (wm * FM + i) * 2;        // first 16-row tile of this 32-feature block
            const floatx16 c = acc_of(i, j);
            if (MODE == DEC_RAW) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = t16 * 16 + 8 * q + 4 * hl;
                    if (tv && n < N)
                        *reinterpret_cast<floatx4 *>(e.raw_out + (size_t)token * N + n) =
                            floatx4{c[4 * q] * r, c[4 * q + 1] * r, c[4 * q + 2] * r, c[4 * q + 3] * r};
                }
            } else if (MODE == DEC_SWIGLU) {
                // tile t16 = gate, t16 + 1 = up (interleaved packing): quads 0, 1 against quads 2, 3
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int f = (t16 >> 1) * 16 + 8 * q + 4 * hl;
                    if (!tv || f >= e.F_l) continue;
                    float u[4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const float aa = c[4 * q + x] * r;
                        u[x] = aa / (1.0f + __expf(-aa)) * (c[4 * (q + 2) + x] * r);
                    }
                    uint2 o;
                    o.x = pack_h16x2(u[0], u[1]);
                    o.y = pack_h16x2(u[2], u[3]);
                    *reinterpret_cast<uint2 *>(e.u + frag_offset(token, f, e.F_l >> 5)) = o;
                }
            } else {   // DEC_QKV: each 16-row tile holds 8 rotary pairs (rows r, r + 8)
                const int d = e.kg.d, half = d >> 1, tph = d >> 4;
#pragma unroll
                for (int m = 0; m < 2; ++m) {              // the two 16-row tiles of this block
                    const int tile = t16 + m;
                    if (!tv || tile >= n_tiles) continue;
                    const int head = tile / tph, tl16 = tile - head * tph;
                    const int i0 = tl16 * 8 + 4 * hl;            // first rotary pair index of this lane
                    float lo[4], hi[4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) { lo[x] = c[4 * (2 * m) + x] * r; hi[x] = c[4 * (2 * m + 1) + x] * r; }
                    if (head < e.hq_l + e.kg.hkv_l) {
                        const floatx4 c4 = *reinterpret_cast<const floatx4 *>(e.cos_tab + (size_t)pos * half + i0);
                        const floatx4 s4 = *reinterpret_cast<const floatx4 *>(e.sin_tab + (size_t)pos * half + i0);
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            const float a = lo[x], b = hi[x];
                            lo[x] = a * c4[x] - b * s4[x];
                            hi[x] = b * c4[x] + a * s4[x];
                        }
                    }
                    uint2 plo, phi;
                    plo.x = pack_h16x2(lo[0], lo[1]); plo.y = pack_h16x2(lo[2], lo[3]);
                    phi.x = pack_h16x2(hi[0], hi[1]); phi.y = pack_h16x2(hi[2], hi[3]);
                    if (head < e.hq_l) {
                        const int qkt = (e.hq_l * d) >> 5;
                        *reinterpret_cast<uint2 *>(e.q + frag_offset(token, head * d + i0, qkt)) = plo;
                        *reinterpret_cast<uint2 *>(e.q + frag_offset(token, head * d + i0 + half, qkt)) = phi;
                    } else if (head < e.hq_l + e.kg.hkv_l) {
                        const size_t slab = (size_t)seq * e.kg.seq_stride + (size_t)(head - e.hq_l) * e.kg.smax * d;
                        *reinterpret_cast<uint2 *>(e.kc + slab + kv_k_offset(pos, i0, d)) = plo;
                        *reinterpret_cast<uint2 *>(e.kc + slab + kv_k_offset(pos, i0 + half, d)) = phi;
                    } else {
                        const size_t slab =
                            (size_t)seq * e.kg.seq_stride + (size_t)(head - e.hq_l - e.kg.hkv_l) * e.kg.smax * d;
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            e.vc[slab + kv_v_offset(pos, i0 + x, d)] = f32_to_h16(lo[x]);
                            e.vc[slab + kv_v_offset(pos, i0 + half + x, d)] = f32_to_h16(hi[x]);
                        }
                    }
                }
            }
        }
    }
}

// Linear tile id -> (feature block bm, token block bt).  Ids are dealt out patch by patch: a patch is pm_h feature
// blocks x pt_w token blocks (lower / narrower at the edges), patches run along the token blocks first, and inside a
// patch the feature block varies fastest.  pm_h = 1, pt_w = t_blocks is the plain row-major order.
__device__ __forceinline__ void gemm_tile_of_id(int id, int n_blocks, int t_blocks, int pm_h, int pt_w, int &bm, int &bt) {
    const int row = pm_h * t_blocks;                       // tiles of a full patch row
    const int pm = id / row, rem = id - pm * row;
    const int hm = min(pm_h, n_blocks - pm * pm_h);        // height of this patch row (the last one may be lower)
    const int pt = rem / (hm * pt_w), rem2 = rem - pt * hm * pt_w;
    bm = pm * pm_h + rem2 % hm;
    bt = pt * pt_w + rem2 / hm;
}

// Operand tiles travel HBM -> LDS with direct-to-LDS loads (no registers in between): a wave copies one
// 1 KB fragment tile per instruction, lane l's 16 bytes landing at tile base + 16 l.  S stages of the k-loop
// are resident; the wait before a step only covers that step's loads (vmcnt counts the rest).
//
// Block = WM x WT waves; each wave owns FM x FT tiles of 32 features x 32 tokens, so the block tile is
// (32 FM WM) features x (32 FT WT) tokens.
//
// PP = true (8 waves, two per SIMD): the two waves of a SIMD run the k-loop half a step out of phase.  Every wave
// alternates a MEMORY phase (all operand fragments of one 32-deep k-step from LDS into registers, its share of the
// direct-to-LDS loads of a later stage) and a COMPUTE phase (the k-step's MFMAs back to back, nothing else in the
// stream), each closed by a workgroup barrier; waves 4..7 pass one extra barrier before their loop, waves 0..3 one
// after it.  So while one wave of a SIMD waits for LDS data, for its loads or at a barrier, the other one is inside
// its MFMA run: the barriers and waits that idle the matrix core in the lock-stepped loop below fall into the
// shadow of the other wave's MFMAs.
//
// ABL (measurement only; results are garbage, every access stays in bounds and every barrier is kept): the same kernel
// with one activity of its k-loop taken out, to price that activity on a power-limited chip.  1: no direct-to-LDS
// loads inside the loop (the MFMAs run on the stages the prologue fetched); 2: the loads are issued but every k-step
// re-reads the block's first k-step (cache hits, no new bytes from HBM); 3: the operand fragments are read from LDS
// for the first k-step only.
template <int FM, int FT, int WM, int WT, int S, int MODE, bool PP = false, int ABL = 0>
__global__ __launch_bounds__(64 * WM * WT) void gemm_mfma_kernel(const h16_t *__restrict__ Wp,
                                                                 const h16_t *__restrict__ Xp, int N, int k_tiles,
                                                                 int n_tiles, int t_tiles, int T, int n_blocks,
                                                                 int t_blocks, GemmEpi e, float *__restrict__ part,
                                                                 int pm_h, int pt_w, int nb0) {
    constexpr int NW = WM * WT, NT = 64 * NW;
    constexpr int TA = 2 * FM * WM, TB = 2 * FT * WT;   // 16-row operand tiles per block and k-step
    constexpr int LA = TA / NW, LB = TB / NW;         // direct-to-LDS loads per wave and stage, per operand
    constexpr int LPT = LA + LB;
    constexpr int STAGE = (TA + TB) * 64;            // h16x8 elements per stage
    constexpr int NTOK = TB * 16;                    // token columns of the block tile
    static_assert(TA % NW == 0 && TB % NW == 0, "operand tiles must divide evenly over the waves");
    extern __shared__ h16x8 smem[];                 // [S][TA + TB][64], then NTOK floats
    float *rstd_s = reinterpret_cast<float *>(smem + (size_t)S * STAGE);
    // XCD-aware remap of the linear block id
    const int total = n_blocks * t_blocks;
    int id = blockIdx.x;
    const int per_xcd = (total + 7) / 8;
    id = (id & 7) * per_xcd + (id >> 3);
    if (id >= total) return;                     // only when total is not a multiple of 8
    // Consecutive ids (the blocks one XCD runs at the same time) form a patch of pm_h feature blocks x pt_w token
    // blocks: per k-step the patch fetches (pm_h + pt_w) operand slices into that XCD's L2 for pm_h x pt_w tiles.
    int bm, bt;
    gemm_tile_of_id(id, n_blocks, t_blocks, pm_h, pt_w, bm, bt);
    bm += nb0;               // the launch covers feature blocks nb0 .. nb0 + n_blocks - 1 of the matrix
    // the wave index is made provably uniform: tile addresses and LDS destinations then stay in scalar registers
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wm = wave % WM, wt = wave / WM;
    // split contraction (few token tiles, see launch_cfg): blockIdx.y takes k-steps [k0, k0 + k_len) and leaves its
    // fp32 result tiles in `part`; gemm_finish_kernel adds the splits up and runs the epilogue
    const int k0 = (int)((long)blockIdx.y * k_tiles / gridDim.y);
    const int k_len = (int)((long)(blockIdx.y + 1) * k_tiles / gridDim.y) - k0;

    floatx16 acc[FM][FT];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const h16x8 *A = reinterpret_cast<const h16x8 *>(Wp);
    const h16x8 *B = reinterpret_cast<const h16x8 *>(Xp);
    // this wave copies tiles wave, wave + NW, ... of both operands; out-of-range tiles are clamped to the last
    // valid tile (their products are never stored) so that every wave issues LPT loads per stage.  Tile bases
    // are uniform (scalar registers); the lane adds its 16-byte slot as a 32-bit offset.
    const h16x8 *asrc[LA], *bsrc[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) asrc[i] = A + (size_t)min(bm * TA + wave + NW * i, n_tiles - 1) * 64 + (size_t)k0 * n_tiles * 64;
#pragma unroll
    for (int i = 0; i < LB; ++i) bsrc[i] = B + ((size_t)min(bt * TB + wave + NW * i, t_tiles - 1) * k_tiles + k0) * 64;
    const size_t astep = (size_t)n_tiles * 64;       // k-tile-major weights
    // One direct-to-LDS load: index x < LA is a weight tile, the rest are activation tiles.  k-steps past
    // the end are clamped to the last one (they land in a buffer nobody reads any more), so that every
    // k-step issues exactly LPT loads and the loop body stays one basic block.
    // One direct-to-LDS load of a 1 KB tile: index x < LA is a weight tile, the rest are activation tiles.
    // k-steps past the end are clamped to the last one (they land in a buffer nobody reads any more), so that
    // every k-step issues exactly LPT loads and the loop body stays one basic block.  The load is written in
    // its scalar-base form (tile address in scalar registers, the lane's 16-byte slot as the 32-bit vector
    // offset, LDS destination in M0), which the compiler does not select for this instruction by itself: it
    // would spend a 64-bit vector add per load inside the MFMA stream.  The compiler does not see these
    // loads in its own vmcnt bookkeeping; every wait on them is explicit (HX_WAIT_VM), and vmcnt is drained
    // before the epilogue issues ordinary loads.  M0 is written here and cannot be named as clobbered: it is a
    // reserved register (the compiler rejects it in a clobber list as undefined behaviour) that the compiler never
    // allocates and only sets itself immediately in front of an instruction of its own that reads it; this kernel
    // contains no such instruction (no LDS-direct builtin, no movrel, no message), so nothing relies on its value.
    const unsigned lane_bytes = (unsigned)lane * 16u;
    auto issue_one = [&](int kt, int x) {
        const int kc = ABL == 2 ? 0 : min(kt, k_len - 1);
        h16x8 *st = smem + (size_t)(kt % S) * STAGE;
        const h16x8 *src = x < LA ? asrc[x] + kc * astep : bsrc[x - LA] + (size_t)kc * 64;
        h16x8 *dst = x < LA ? st + (wave + NW * x) * 64 : st + (TA + wave + NW * (x - LA)) * 64;
        const unsigned lds_addr = (unsigned)reinterpret_cast<uintptr_t>(HX_AS3(dst));
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(lds_addr), "v"(lane_bytes), "s"(src)
                     : "memory");
    };
    // 32x32x16 operand for k-half kh of a pair of 16-row tiles: lane l takes row l % 32, k-group 2 kh + l / 32
    const int frag = ((lane & 31) >> 4) * 64 + (lane & 15) + 16 * (lane >> 5);
    // Software pipeline.  (1) The operand registers of one 16-deep half step are fetched from LDS while the
    // MFMAs of the previous half step run.  (2) The barrier sits in the MIDDLE of a k-step: it publishes stage
    // kt + 1, whose first half is then fetched under the second half of stage kt, and frees the buffer of
    // stage kt - 1.  (3) The loads of stage kt + S - 1 into that buffer are spread over one whole step, half
    // behind the barrier of step kt and half in front of the barrier of step kt + 1, one load every few MFMAs.
    if constexpr (PP) {
        static_assert(NW == 8 && S >= 3, "ping-pong: two waves per SIMD");
        const int grp = wave >> 2;                 // waves w and w + 4 share a SIMD
#pragma unroll
        for (int p2 = 0; p2 < S - 1; ++p2)
#pragma unroll
            for (int x = 0; x < LPT; ++x) issue_one(p2, x);
        if (MODE != DEC_RESID && e.ssq_in != nullptr && part == nullptr) {
            const int groups = e.norm_dim / GEMM_SSQ_COLS;
            for (int t = tid; t < NTOK; t += NT) {
                const int token = bt * NTOK + t;
                float ss = 0.f;
                if (token < T) {
#pragma unroll 16
                    for (int gI = 0; gI < groups; ++gI) ss += e.ssq_in[(size_t)gI * T + token];
                }
                rstd_s[t] = 1.0f / sqrtf(ss / (float)e.norm_dim + e.eps);
            }
        }
        HX_WAIT_VM((S - 2) * LPT);                 // stage 0 has landed (this wave's share of it)
        HX_LDS_BARRIER();                          // ... and everybody's
        if (grp == 1) asm volatile("s_barrier" ::: "memory");       // half a step behind waves 0..3 from here on
        // The MFMAs of this loop are v_mfma_f32_16x16x32_bf16 on the fragment tiles as they lie in LDS (one 128-bit read per
        // 16-row tile and k-step, lane l reads entry l): on operands whose bits toggle the chip is power-limited, and this
        // form sustains about 12 % more flops than 32x32x16 at the same socket power (register-only probe,
        // profiles/hbm_mfma_calibration.txt).  Same LDS traffic and MFMA cycles per k-step as the 32x32x16 form: 12 reads,
        // 32 x 16 cycles.  a16[i][j] = features 16 i .. + 15 of the wave tile x tokens 16 j .. + 15; lane l holds token
        // l % 16 and features 4 (l / 16) .. + 3.
        floatx4 a16[2 * FM][2 * FT];
#pragma unroll
        for (int i = 0; i < 2 * FM; ++i)
#pragma unroll
            for (int j = 0; j < 2 * FT; ++j) a16[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        h16x8 pa[2 * FM], pb[2 * FT];
        for (int kt = 0; kt < k_len; ++kt) {
            // memory phase: the whole k-step's operands, then this wave's loads of stage kt + S - 1 into the buffer
            // of stage kt - 1, which both halves of the block have finished reading (barriers below)
            const h16x8 *sa = smem + (size_t)(kt % S) * STAGE + (wm * FM * 2) * 64 + lane;
            const h16x8 *sb = smem + (size_t)(kt % S) * STAGE + (TA + wt * FT * 2) * 64 + lane;
            if (ABL != 3 || kt == 0) {
#pragma unroll
                for (int x = 0; x < 2 * FT; ++x) pb[x] = sb[x * 64];
#pragma unroll
                for (int x = 0; x < 2 * FM; ++x) pa[x] = sa[x * 64];
            }
            if (ABL != 1) {
#pragma unroll
                for (int x = 0; x < LPT; ++x) issue_one(kt + S - 1, x);
            }
            __builtin_amdgcn_sched_barrier(0);
            HX_WAIT_VM(ABL == 1 ? 0 : (S - 2) * LPT);      // this wave's loads of stage kt + 1 have landed
            HX_LDS_BARRIER();                      // operands in registers; barrier
            __builtin_amdgcn_sched_barrier(0);
            // compute phase
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int i = 0; i < 2 * FM; ++i)
#pragma unroll
                for (int j = 0; j < 2 * FT; ++j)
                    a16[i][j] = hx_mfma16(pa[i], pb[j], a16[i][j]);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_barrier" ::: "memory");
        }
        if (grp == 0) asm volatile("s_barrier" ::: "memory");       // the barrier waves 4..7 passed ahead of their loop
        HX_WAIT_VM(0);
        // Into the register layout of a 32 x 32 MFMA result, which the epilogues are written for: lane L holds token
        // L % 32 and, in register 4 q + r, feature 8 q + 4 (L / 32) + r of the 32 x 32 block.  That value sits in the
        // 16 x 16 tile (q / 2, (L % 32) / 16) of the block, register r, lane 16 (2 (q % 2) + L / 32) + L % 16.  Converted
        // tile by tile when the epilogue asks for it, so that the two layouts never hold the whole wave tile at once.
        auto acc_of = [&](int i, int j) {
            floatx16 c;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int src = 16 * (2 * (q & 1) + (lane >> 5)) + (lane & 15);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float v0 = __shfl(a16[2 * i + (q >> 1)][2 * j][r], src, 64);
                    const float v1 = __shfl(a16[2 * i + (q >> 1)][2 * j + 1][r], src, 64);
                    c[4 * q + r] = (lane & 16) ? v1 : v0;
                }
            }
            return c;
        };
        if (part != nullptr) {
            float *dst = part + ((((size_t)blockIdx.y * total + id) * NW + wave) * (FM * FT)) * 1024 + lane * 4;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FT; ++j) {
                    const floatx16 c = acc_of(i, j);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<floatx4 *>(dst + (i * FT + j) * 1024 + q * 256) = floatx4{c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]};
                }
            return;
        }
        gemm_epilogue<FM, FT, WM, WT, MODE>(acc_of, bm, bt, wm, wt, lane, N, n_tiles, T, e, rstd_s);
        return;
    }
    constexpr int H1 = (LPT + 1) / 2, H2 = LPT / 2;  // loads issued behind / in front of the barrier
    constexpr int HL = H1;
    // MFMA slots of a half step: the first FM + FT also carry an LDS fetch; the loads go behind them when
    // there is room, else they are spread over all slots
    constexpr int FREE = FM * FT - (FM + FT);
    constexpr int LOAD0 = FREE >= HL ? FM + FT : 0;
    constexpr int GAP = FREE >= HL ? FREE / HL : ((FM * FT) / HL > 0 ? (FM * FT) / HL : 1);
    static_assert(S >= 3, "the pipeline needs three stages");
#pragma unroll
    for (int p = 0; p < S - 2; ++p)
#pragma unroll
        for (int x = 0; x < LPT; ++x) issue_one(p, x);
#pragma unroll
    for (int x = 0; x < H1; ++x) issue_one(S - 2, x);
    // 1 / rms of the block's token columns from the producer's partial sums of squares, once per block (the
    // values are the youngest loads in flight: the compiler's wait for them also covers the stages above)
    if (MODE != DEC_RESID && e.ssq_in != nullptr && part == nullptr) {
        const int groups = e.norm_dim / GEMM_SSQ_COLS;
        for (int t = tid; t < NTOK; t += NT) {
            const int token = bt * NTOK + t;
            float ss = 0.f;
            if (token < T) {
#pragma unroll 16
                for (int gI = 0; gI < groups; ++gI) ss += e.ssq_in[(size_t)gI * T + token];
            }
            rstd_s[t] = 1.0f / sqrtf(ss / (float)e.norm_dim + e.eps);
        }
    }
    h16x8 fa0[FM], fb0[FT], fa1[FM], fb1[FT];
    // x-th operand fetch of a half step: the FT token operands first, then the FM feature operands
    auto fetch_one = [&](h16x8(&fa)[FM], h16x8(&fb)[FT], int kt, int kh, int x) {
        const h16x8 *sa = smem + (size_t)(kt % S) * STAGE + (wm * FM * 2) * 64 + frag + kh * 32;
        const h16x8 *sb = smem + (size_t)(kt % S) * STAGE + (TA + wt * FT * 2) * 64 + frag + kh * 32;
        if (x < FT) fb[x] = sb[x * 128];
        else fa[x - FT] = sa[(x - FT) * 128];
    };
    auto fetch = [&](h16x8(&fa)[FM], h16x8(&fb)[FT], int kt, int kh) {
#pragma unroll
        for (int x = 0; x < FM + FT; ++x) fetch_one(fa, fb, kt, kh, x);
    };
    static_assert(PP || FM + FT <= FM * FT, "one operand fetch per MFMA slot");
    HX_WAIT_VM((S - 3) * LPT + H1);
    HX_LDS_BARRIER();
    fetch(fa0, fb0, 0, 0);
    HX_WAIT_LGKM0();
    // The memory pipeline of a CU accepts one wave-wide 1 KB load every ~26 cycles and hardly queues: waves
    // that issue their loads at the same point of the (lock-stepped) MFMA stream block each other for tens of
    // cycles with the matrix core idle.  Each wave therefore runs a copy of the loop whose loads sit OFF
    // MFMAs later than its neighbour's, which gives the CU one load per MFMA slot.
    auto k_loop = [&](auto off_c) {
        constexpr int OFF = decltype(off_c)::value;
    for (int kt = 0; kt < k_len; ++kt) {
        // one slot = one MFMA, at most one LDS fetch for the NEXT half step and at most one global load; the
        // slots are fenced so that the order below is the order in the instruction stream
#pragma unroll
        for (int m = 0; m < FM * FT; ++m) {
            acc[m / FT][m % FT] = hx_mfma32(fa0[m / FT], fb0[m % FT], acc[m / FT][m % FT]);
            if (m < FM + FT) fetch_one(fa1, fb1, kt, 1, m);
            if (m >= LOAD0 && (m - LOAD0) % GAP == OFF && (m - LOAD0) / GAP < H2) issue_one(kt + S - 2, H1 + (m - LOAD0) / GAP);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
        HX_WAIT_VM((S - 3) * LPT);      // stage kt + 1 has landed; later stages stay in flight
        HX_LDS_BARRIER();
#pragma unroll
        for (int m = 0; m < FM * FT; ++m) {
            acc[m / FT][m % FT] = hx_mfma32(fa1[m / FT], fb1[m % FT], acc[m / FT][m % FT]);
            if (m < FM + FT) fetch_one(fa0, fb0, kt + 1, 0, m);
            if (m >= LOAD0 && (m - LOAD0) % GAP == OFF && (m - LOAD0) / GAP < H1) issue_one(kt + S - 1, (m - LOAD0) / GAP);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the fetch of the next half step has had FM FT MFMAs to complete: waiting here, instead of where
        // the compiler would place it (behind the next fetch), costs nothing and keeps that fetch covered
        __builtin_amdgcn_sched_barrier(0);
        HX_WAIT_LGKM0();
    }
    };
    {
        const int off = (wave * GAP) / NW;
        if (GAP > 3 && off == 3) k_loop(std::integral_constant<int, (GAP > 3 ? 3 : 0)>{});
        else if (GAP > 2 && off == 2) k_loop(std::integral_constant<int, (GAP > 2 ? 2 : 0)>{});
        else if (GAP > 1 && off == 1) k_loop(std::integral_constant<int, (GAP > 1 ? 1 : 0)>{});
        else k_loop(std::integral_constant<int, 0>{});
    }
    HX_WAIT_VM(0);
    if (part != nullptr) {
        // result tiles as they sit in the registers: per tile 4 quads x 64 lanes x 4 floats, 1 KB per store
        float *dst = part + ((((size_t)blockIdx.y * total + id) * NW + wave) * (FM * FT)) * 1024 + lane * 4;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FT; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<floatx4 *>(dst + (i * FT + j) * 1024 + q * 256) =
                        floatx4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        return;
    }
    gemm_epilogue<FM, FT, WM, WT, MODE>([&](int i, int j) { return acc[i][j]; }, bm, bt, wm, wt, lane, N, n_tiles, T, e, rstd_s);
}

// Second pass of a split contraction: block `id` (the same tile and wave layout as gemm_mfma_kernel) adds its result
// tiles up over the splits, in split order, and runs the epilogue.  parts > 1 (a power of two that divides the waves;
// only where the epilogue needs nothing from another wave): a tile is finished by `parts` blocks, each with a
// contiguous share of the waves -- a split launch has few tiles, and one block per tile would leave most of the chip
// idle while each block reads its tile's partial sums alone.
template <int FM, int FT, int WM, int WT, int MODE>
__global__ __launch_bounds__(64 * WM * WT) void gemm_finish_kernel(const float *__restrict__ part, int splits, int N,
                                                                   int n_tiles, int T, int total, int t_blocks, GemmEpi e,
                                                                   int pm_h, int pt_w, int nb0, int parts) {
    constexpr int NW = WM * WT, NT = 64 * NW, TB = 2 * FT * WT, NTOK = TB * 16;
    __shared__ float rstd_s[NTOK];
    __shared__ float ssq_lds[(MODE == DEC_RESID && 32 * FM != GEMM_SSQ_COLS) ? WM * NTOK : 1];
    const int id = blockIdx.x / parts;
    int bm, bt;
    gemm_tile_of_id(id, total / t_blocks, t_blocks, pm_h, pt_w, bm, bt);      // as in the pass that wrote the partials
    bm += nb0;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wm = wave % WM, wt = wave / WM;
    const bool mine = wave / (NW / parts) == (int)blockIdx.x - id * parts;      // this block's share of the tile's waves
    if (MODE != DEC_RESID && e.ssq_in != nullptr) {
        const int groups = e.norm_dim / GEMM_SSQ_COLS;
        for (int t = tid; t < NTOK; t += NT) {
            const int token = bt * NTOK + t;
            float ss = 0.f;
            if (token < T) {
#pragma unroll 16
                for (int gI = 0; gI < groups; ++gI) ss += e.ssq_in[(size_t)gI * T + token];
            }
            rstd_s[t] = 1.0f / sqrtf(ss / (float)e.norm_dim + e.eps);
        }
    }
    floatx16 acc[FM][FT];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int z = 0; z < (mine ? splits : 0); ++z) {
        const float *src = part + ((((size_t)z * total + id) * NW + wave) * (FM * FT)) * 1024 + lane * 4;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FT; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 v = *reinterpret_cast<const floatx4 *>(src + (i * FT + j) * 1024 + q * 256);
#pragma unroll
                    for (int x = 0; x < 4; ++x) acc[i][j][4 * q + x] += v[x];
                }
    }
    __syncthreads();
    if (!mine) return;       // (parts > 1 only with an epilogue that has no block barrier)
    gemm_epilogue<FM, FT, WM, WT, MODE>([&](int i, int j) { return acc[i][j]; }, bm, bt, wm, wt, lane, N, n_tiles, T, e, rstd_s, ssq_lds);
}

// -------------------------------------------------------------------------------------------------
// Skinny form for one 128-token tile (a short prompt): the launch is bound by streaming the weights, not by the matrix
// cores, so it is built like the decode projections.  A block of 4 waves owns 128 features x 128 tokens, a wave 32
// features x 128 tokens; the weights never touch LDS: a lane requests the 16 bytes of the two 16-row tiles that the
// 32x32x16 operand wants from it (two 512-byte runs per request), RING k-steps ahead, in a register ring that is
// refilled slot by slot.  The activations of a k-step (8 KB, L2 hits) are shared by the block's waves through LDS,
// global -> registers (same ring) -> LDS one k-step before use.  The contraction is split over blockIdx.y; result
// tiles go to `part` in the layout gemm_finish_kernel<1, 1, 4, 1> reads (four 32-token blocks per feature block).
// -------------------------------------------------------------------------------------------------
constexpr int SKINNY_RING = 6;          // measured: 4, 6 and 8 run alike (the CU's load issue rate paces the kernel)
// KG = 2: a block of 8 waves = two groups of 4, each group walking one half of the block's share of the contraction
// in step with the other (one barrier serves both) and the second group's results added to the first's through LDS
// before anything is stored: as many waves and k-steps per wave as two blocks of 4 on two splits, half the partial sums.
template <int KG>
__global__ __launch_bounds__(256 * KG) void gemm_skinny_kernel(const h16_t *__restrict__ Wp, const h16_t *__restrict__ Xp,
                                                              int k_tiles, int n_tiles, int t_tiles, int total,
                                                              float *__restrict__ part) {
    constexpr int RING = SKINNY_RING;
    __shared__ h16x8 xs[KG][2][8 * 64];             // per group: two k-steps of the 8 token tiles
    const int id = blockIdx.x;                       // 128-feature block
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int kg = wave >> 2, w4 = wave & 3;         // k-group, wave inside the group (32 features each)
    const int b0 = (int)((long)blockIdx.y * k_tiles / gridDim.y);
    const int b_len = (int)((long)(blockIdx.y + 1) * k_tiles / gridDim.y) - b0;       // the block's k-steps ...
    const int g0 = (int)((long)kg * b_len / KG);
    const int k0 = b0 + g0, k_len = (int)((long)(kg + 1) * b_len / KG) - g0;          // ... and this group's
    const int steps = (b_len + KG - 1) / KG;         // k-steps every wave of the block walks (the longer group's)

    // weights: lane l of k-half kh takes slot (l % 16) + 16 (l / 32) + 32 kh of tile t16 + (l % 32) / 16
    const int t16 = min(id * 8 + w4 * 2 + ((lane & 31) >> 4), n_tiles - 1);
    const h16x8 *wsrc = reinterpret_cast<const h16x8 *>(Wp) + ((size_t)k0 * n_tiles + t16) * 64 + (lane & 15) + 16 * (lane >> 5);
    const size_t wstep = (size_t)n_tiles * 64;
    // activations: wave w of a group copies token tiles 2 w and 2 w + 1 of each k-step (clamped to the last valid tile)
    const h16x8 *xsrc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        xsrc[i] = reinterpret_cast<const h16x8 *>(Xp) + ((size_t)min(w4 * 2 + i, t_tiles - 1) * k_tiles + k0) * 64 + lane;
    const int frag = ((lane & 31) >> 4) * 64 + (lane & 15) + 16 * (lane >> 5);

    floatx16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    // Ring slot = one k-step: the wave's two weight operands and its two pieces of the activations.  Every request is
    // unconditional (k-steps past the end re-read the last one, an L2 hit, unused), so the compiler counts requests in
    // flight exactly; because loads return in order, a piece of the activations must not be requested later than the
    // weights it is used with, or the wait for it would drain the weight requests behind which it sits.
    h16x8 a[RING][2], xq[RING][2];
    auto request = [&](int slot, int kt) {
        const int kc = min(kt, k_len - 1);
        xq[slot][0] = xsrc[0][(size_t)kc * 64];
        xq[slot][1] = xsrc[1][(size_t)kc * 64];
        const h16x8 *src = wsrc + (size_t)kc * wstep;
        a[slot][0] = __builtin_nontemporal_load(src);
        a[slot][1] = __builtin_nontemporal_load(src + 32);
    };
    auto store_x = [&](int slot, int kt) {
        xs[kg][kt & 1][(w4 * 2) * 64 + lane] = xq[slot][0];
        xs[kg][kt & 1][(w4 * 2 + 1) * 64 + lane] = xq[slot][1];
    };
    auto step = [&](int slot, int kt) {
        if (KG > 1 && kt >= k_len) return;          // the shorter group's last k-step (uniform over the wave)
        const h16x8 *sb = xs[kg][kt & 1] + frag;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = hx_mfma32(a[slot][kh], sb[j * 128 + kh * 32], acc[j]);
    };
    // the barrier of a k-step waits for the LDS stores only: __syncthreads() would also drain the requests in flight
    auto lds_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14));
        asm volatile("s_barrier" ::: "memory");
    };
#pragma unroll
    for (int i = 0; i < RING; ++i) request(i, i);
    store_x(0, 0);
    const int rounds = steps / RING;
    for (int rd = 0; rd < rounds; ++rd) {
#pragma unroll
        for (int i = 0; i < RING; ++i) {
            const int kt = rd * RING + i;
            lds_barrier();                // k-step kt is complete in LDS; the other buffer (k-step kt - 1) is free
            store_x((i + 1) % RING, kt + 1);
            step(i, kt);
            request(i, kt + RING);
        }
    }
    // fewer than RING k-steps left: k-step rounds * RING + i already sits in slot i
#pragma unroll
    for (int i = 0; i < RING; ++i) {
        const int kt = rounds * RING + i;
        if (kt < steps) {                 // uniform over the block
            lds_barrier();
            store_x((i + 1) % RING, kt + 1);
            step(i, kt);
        }
    }
    if constexpr (KG == 2) {
        // group 1 hands its results to group 0, two of the four token blocks at a time, through the 32 KB of the staging
        // buffers (4 waves x 2 tiles x 16 registers x 64 lanes of fp32); group 0 + group 1, in that order, every time
        float *red = reinterpret_cast<float *>(&xs[0][0][0]);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            __syncthreads();              // the staging buffers (first pass) or the previous pass's values are no longer read
            if (kg == 1) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[((w4 * 2 + jj) * 16 + r) * 64 + lane] = acc[2 * half + jj][r];
            }
            __syncthreads();
            if (kg == 0) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[2 * half + jj][r] += red[((w4 * 2 + jj) * 16 + r) * 64 + lane];
            }
        }
        if (kg != 0) return;
    }
    // result tile (32 features x token block j) of this wave, in the layout gemm_finish_kernel<1, 1, 4, 1> reads with
    // four token blocks per feature block: the finishing pass then has four times as many (smaller) blocks
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<floatx4 *>(part + ((((size_t)blockIdx.y * total + id) * 4 + j) * 4 + w4) * 1024 + q * 256 + lane * 4) =
                floatx4{acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]};
}

template <int FM, int FT, int WM, int WT, int S, int MODE, bool PP = false, int ABL = 0>
static void launch_cfg(const h16_t *Wp, const h16_t *Xp, int N, int k_tiles, int n_tiles, int t_tiles, int T,
                       const GemmEpi &e, float *part, size_t part_floats, hipStream_t s, int nb0 = 0, int nb_count = -1) {
    constexpr int TA = 2 * FM * WM, TB = 2 * FT * WT;
    // feature blocks nb0 .. nb0 + nb_count - 1 of the matrix (all of them by default)
    const int n_blocks = nb_count >= 0 ? nb_count : (n_tiles + TA - 1) / TA, t_blocks = (t_tiles + TB - 1) / TB;
    const int total = n_blocks * t_blocks;
    const int grid = (total + 7) / 8 * 8;
    auto kern = gemm_mfma_kernel<FM, FT, WM, WT, S, MODE, PP, ABL>;
    const int pm_h = 4, pt_w = 8;         // patch of tiles one XCD works on at a time: 4 feature blocks x 8 token blocks
    const size_t dyn = (size_t)S * (TA + TB) * 64 * sizeof(h16x8) + (size_t)TB * 16 * sizeof(float);
    static bool raised = false;           // more than the default 64 KB of LDS per block
    if (!raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)dyn);
        raised = true;
    }
    // A short prompt gives few tiles, each walking the whole contraction while most of the chip idles and the weights
    // arrive at a fraction of the HBM rate: the contraction is then split over blockIdx.y (at most 8 ways, at least
    // 16 k-steps each, partials within the scratch) until the chip holds as many blocks as it can.
    int splits = 1;
    const size_t tile_floats = (size_t)64 * WM * WT * FM * FT * 16;
    const int resident = dyn <= 72 * 1024 ? 512 : 256;       // blocks the chip holds at once (LDS: two per CU or one)
    if (part != nullptr && 2 * total <= resident && k_tiles >= 32) {
        splits = std::max(1, std::min({8, resident / total, k_tiles / 16}));
        while (splits > 1 && (size_t)splits * total * tile_floats > part_floats) --splits;
    }
    hipLaunchKernelGGL(kern, dim3(grid, splits), dim3(64 * WM * WT), dyn, s, Wp, Xp, N, k_tiles, n_tiles, t_tiles, T,
                       n_blocks, t_blocks, e, splits > 1 ? part : nullptr, pm_h, std::min(pt_w, t_blocks), nb0);
    if (splits > 1) {
        // Several blocks per tile, each with a share of the tile's waves, where the epilogue is the wave's own business
        // -- as many as one round of blocks over the chip takes (a CU holds one of them): 4 up to 64 tiles, 2 up to 128.
        // Measured on 70B TP4 shards, one prompt of 256 rows (10 / 32 / 56 / 32 tiles): 43.1 / 35.0 / 82.0 / 58.2 ->
        // 38.2 / 32.8 / 81.0 / 54.9 us per projection, 221.6 -> 212.0 us per layer; 512 rows 282 -> 278; QKV at 2048 rows
        // (80 tiles) 94.2 -> 92.1, while four parts there (320 blocks, two rounds) took the pass from 25.6 to 38.2 us.
        constexpr bool wave_local = MODE != DEC_RESID || 32 * FM == GEMM_SSQ_COLS;
        int parts = 1;
        if (wave_local && (WM * WT) % 4 == 0) parts = total <= 64 ? 4 : (total <= 128 ? 2 : 1);
        hipLaunchKernelGGL((gemm_finish_kernel<FM, FT, WM, WT, MODE>), dim3(total * parts), dim3(64 * WM * WT), 0, s, part,
                           splits, N, n_tiles, T, total, t_blocks, e, pm_h, std::min(pt_w, t_blocks), nb0, parts);
    }
}

// tile configuration forced for every GEMM launch of the process (0 = choose by shape); a measurement and test hook
static std::atomic<int> g_force_tile{0};
bool set_gemm_tile(int code) {
    for (int ok : {0, 44, 48, 84, 88, 94, 49, 98, 72, 198, 194, 184, 1198, 2198, 3198})
        if (code == ok) { g_force_tile.store(code, std::memory_order_relaxed); return true; }
    return false;
}

// Estimated time in microseconds of one projection with block tiles of tm features x tt tokens (both multiples of 16),
// `step_us` per 32-deep k-step of a block; constants fitted to this chip (TP4-shaped projections at 128 .. 2048 rows):
//   * a block walks its k-steps and pays a fixed 11 us (pipeline fill, epilogue; 15 more when the epilogue is the
//     residual read-modify-write); the chip holds 256 such blocks at once (their LDS fills a CU), and a launch takes
//     whole rounds of them;
//   * launch_cfg splits the contraction when the tiles fill less than half of the chip: the partial sums are written
//     (about 5 TB/s) and a finishing pass reads them back (about 2.5 TB/s) behind a second launch.
static double gemm_estimate_us(int tm, int tt, double step_us, int n_tiles, int t_tiles, int k_tiles, bool resid, bool can_split) {
    const int resident = 256;
    const long total = (long)((n_tiles * 16 + tm - 1) / tm) * ((t_tiles * 16 + tt - 1) / tt);
    int splits = 1;
    if (can_split && 2 * total <= resident && k_tiles >= 32)
        splits = (int)std::max<long>(1, std::min<long>({8, resident / total, k_tiles / 16}));
    const long rounds = (total * splits + resident - 1) / resident;
    const double ksteps = (double)((k_tiles + splits - 1) / splits);
    double us = rounds * (ksteps * step_us + 11.0 + (resid && splits == 1 ? 15.0 : 0.0));
    if (splits > 1) {
        const double part_mb = (double)splits * total * tm * tt * 4.0 / 1e6;
        us += part_mb / 5.0 + 8.0 + part_mb / 2.5 + (resid ? 15.0 : 0.0);
    }
    return us;
}

// one 128-token tile, at least 32 k-tiles: skinny kernel + finishing pass; returns false when it does not apply
template <int MODE>
static bool launch_skinny(const h16_t *Wp, const h16_t *Xp, int N, int k_tiles, int n_tiles, int t_tiles, int T,
                          const GemmEpi &e, float *part, size_t part_floats, hipStream_t s) {
    if (part == nullptr || t_tiles > 8 || k_tiles < 32) return false;
    const int n_blocks = (n_tiles + 7) / 8;
    const size_t tile_floats = 4 * 4 * 1024;
    // two blocks fit a CU (registers): about 512 blocks in flight, at most 8 splits of at least 16 k-steps
    int splits = std::max(1, std::min({8, 512 / n_blocks, k_tiles / 16}));
    while (splits > 1 && (size_t)splits * n_blocks * tile_floats > part_floats) --splits;
    if ((size_t)splits * n_blocks * tile_floats > part_floats) return false;
    // An even number of splits over enough blocks runs as half as many splits of 8-wave blocks, the pairs of splits summed
    // inside the block: half the partial sums written, and read by the finishing pass.  Measured on the TP4 shard of the
    // 70B shape at 128 rows: W1/W3 (112 blocks x 4 -> x 2) 64.8 -> 59.4 us, W2 (64 x 8 -> x 4) 43.0 -> 38.5, 158.9 -> 149.8 us
    // per layer; with fewer than 160 blocks left the CUs that stay empty cost more (W_O 64 x 4 -> x 2: 22.1 -> 25.9,
    // QKV 20 x 8 -> x 4: 25.6 -> 32.4), and 8-wave blocks at an unchanged number of splits gain nothing there either.
    if (splits % 2 == 0 && n_blocks * (splits / 2) >= 160) {
        splits /= 2;
        hipLaunchKernelGGL(gemm_skinny_kernel<2>, dim3(n_blocks, splits), dim3(512), 0, s, Wp, Xp, k_tiles, n_tiles, t_tiles,
                           n_blocks, part);
    } else {
        hipLaunchKernelGGL(gemm_skinny_kernel<1>, dim3(n_blocks, splits), dim3(256), 0, s, Wp, Xp, k_tiles, n_tiles, t_tiles,
                           n_blocks, part);
    }
    hipLaunchKernelGGL((gemm_finish_kernel<1, 1, 4, 1, MODE>), dim3(n_blocks * 4), dim3(256), 0, s, part, splits, N, n_tiles,
                       T, n_blocks * 4, 4, e, 1, 4, 0, 1);
    return true;
}

template <int MODE>
static void launch_mode(const h16_t *Wp, const h16_t *Xp, int N, int K, int T, const GemmEpi &e, float *part,
                        size_t part_floats, hipStream_t s) {
    const int k_tiles = K / 32, n_tiles = N / 16, t_tiles = (T + 15) / 16;
    const int force = g_force_tile.load(std::memory_order_relaxed);
    // 198 = 256 x 256 on 8 waves with the two waves of a SIMD half a k-step out of phase; the smaller tile, on the same
    // loop, is 128 x 256 (194), or 256 x 128 (184) for the residual epilogue.  Which one: the shorter of two estimates
    // (gemm_estimate_us), i.e. rounds of blocks over the chip x a block's time, plus what a split contraction costs in
    // partial sums.
    const bool resid = MODE == DEC_RESID;
    const double t198 = gemm_estimate_us(256, 256, 0.55, n_tiles, t_tiles, k_tiles, resid, part != nullptr);
    const double tsml = gemm_estimate_us(resid ? 256 : 128, resid ? 128 : 256, 0.37, n_tiles, t_tiles, k_tiles, resid, part != nullptr);
    int cfg = t198 <= tsml ? 198 : 194;
    if (force) cfg = force;
    // the RESID epilogue emits one sum-of-squares partial per wave: its 32 FM features must be 128
    if (MODE == DEC_RESID && cfg != 88 && cfg != 84 && cfg != 184 && cfg != 98 && cfg % 1000 != 198) cfg = cfg == 72 ? 198 : (cfg == 194 ? 184 : 84);
    // one 128-token tile (a short prompt): 128-token block tiles; the split contraction then runs a short k-loop per
    // block with the weights coming from HBM, so the 256 x 128 tile of RESID keeps six stages in flight instead of four
    const bool short_prompt = !force && t_tiles <= 8;
    if (short_prompt && launch_skinny<MODE>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s)) return;
    if (short_prompt) cfg = MODE == DEC_RESID ? 846 : 44;
#define HX_G(FM, FT, WM, WT, S) launch_cfg<FM, FT, WM, WT, S, MODE>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s)
    if (cfg == 88) HX_G(4, 4, 2, 2, 4);
    else if (cfg == 98) HX_G(4, 2, 2, 4, 4);
    else if (cfg == 198) {
        // The chip holds 256 of these blocks; a launch of a few more than a multiple of 256 would run its last round
        // nearly empty (1280 rows x 14336 features: 280 tiles, two rounds for 1.09 rounds of work).  Then the feature
        // blocks whose tiles fill whole rounds go first, and the few that remain follow as a launch of their own, which
        // launch_cfg splits along the contraction so that it fills the chip as well.
        const int nb = (n_tiles + 15) / 16, tb = (t_tiles + 15) / 16, total = nb * tb, rem = total % 256;
        const int nA = (total - rem) / tb;
        if (!force && total > 256 && rem > 0 && rem <= 128 && part != nullptr && k_tiles >= 32 && nA >= 1 && nA < nb &&
            gemm_estimate_us(256, 256, 0.55, nA * 16, t_tiles, k_tiles, resid, true) +
                    gemm_estimate_us(256, 256, 0.55, (nb - nA) * 16, t_tiles, k_tiles, resid, true) <
                t198) {
            launch_cfg<4, 2, 2, 4, 4, MODE, true>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s, 0, nA);
            launch_cfg<4, 2, 2, 4, 4, MODE, true>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s, nA, nb - nA);
        } else {
            launch_cfg<4, 2, 2, 4, 4, MODE, true>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s);
        }
    }
    else if (cfg == 1198) launch_cfg<4, 2, 2, 4, 4, MODE, true, 1>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s);
    else if (cfg == 2198) launch_cfg<4, 2, 2, 4, 4, MODE, true, 2>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s);
    else if (cfg == 3198) launch_cfg<4, 2, 2, 4, 4, MODE, true, 3>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s);
    else if (cfg == 194) { if constexpr (MODE != DEC_RESID) launch_cfg<2, 2, 2, 4, 4, MODE, true>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s); }
    else if (cfg == 184) launch_cfg<4, 1, 2, 4, 4, MODE, true>(Wp, Xp, N, k_tiles, n_tiles, t_tiles, T, e, part, part_floats, s);
    else if (cfg == 94) { if constexpr (MODE != DEC_RESID) HX_G(2, 2, 2, 4, 4); }
    else if (cfg == 49) { if constexpr (MODE != DEC_RESID) HX_G(2, 2, 4, 2, 4); }
    else if (cfg == 84) HX_G(4, 2, 2, 2, 4);
    else if (cfg == 72) { if constexpr (MODE != DEC_RESID) HX_G(7, 2, 2, 2, 4); }
    else if (cfg == 846) { if constexpr (MODE == DEC_RESID) HX_G(4, 2, 2, 2, 6); }
    else if (cfg == 48) {
        if constexpr (MODE != DEC_RESID) HX_G(2, 4, 2, 2, 4);
    } else {
        if constexpr (MODE != DEC_RESID) HX_G(2, 2, 2, 2, 4);
    }
#undef HX_G
}

void launch_gemm_mfma(const h16_t *Wp, const h16_t *Xp, int N, int K, int T, const GemmEpi &e, float *part,
                      size_t part_floats, hipStream_t s) {
    switch (e.mode) {
        case DEC_RAW: launch_mode<DEC_RAW>(Wp, Xp, N, K, T, e, part, part_floats, s); break;
        case DEC_QKV: launch_mode<DEC_QKV>(Wp, Xp, N, K, T, e, part, part_floats, s); break;
        case DEC_RESID: launch_mode<DEC_RESID>(Wp, Xp, N, K, T, e, part, part_floats, s); break;
        case DEC_SWIGLU: launch_mode<DEC_SWIGLU>(Wp, Xp, N, K, T, e, part, part_floats, s); break;
    }
}

// -------------------------------------------------------------------------------------------------
// Prefill prologue: stage input rows (bf16, or fp32 for the validation surface) -> fp32 residual stream in its
// tiled order, (x * gain) in fragment tiles, sums of squares per 128-column group.  One wave owns 32 tokens x
// 128 columns and walks them as four 32 x 32 blocks in the lane layout of the MFMA result (lane = token % 32 +
// 32 * half, four consecutive features per lane and quad): every store of the residual stream is one contiguous
// 1 KB, every store of the operand two runs of 256 B, and the 64-byte row pieces it reads are fetched once.
// -------------------------------------------------------------------------------------------------
template <bool IN_H16>
__global__ __launch_bounds__(256) void prefill_prologue_kernel(const void *__restrict__ in, float *__restrict__ h_out,
                                                              const float *__restrict__ g, h16_t *__restrict__ hg,
                                                              float *__restrict__ ssq_out, int T, int H) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int token = blockIdx.x * 32 + (lane & 31), hl = lane >> 5;
    const int col0 = (blockIdx.y * 4 + wave) * GEMM_SSQ_COLS;
    if (col0 >= H) return;
    const bool tv = token < T;
    float ss = 0.f;
#pragma unroll
    for (int fb = 0; fb < GEMM_SSQ_COLS / 32; ++fb) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = col0 + fb * 32 + 8 * q + 4 * hl;
            float x[4] = {0.f, 0.f, 0.f, 0.f};
            if (tv) {
                if (IN_H16) {
                    const uint2 raw = *reinterpret_cast<const uint2 *>(reinterpret_cast<const h16_t *>(in) + (size_t)token * H + n);
                    h16x2_to_f32(raw.x, x[0], x[1]);
                    h16x2_to_f32(raw.y, x[2], x[3]);
                } else {
                    const float4 v = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(in) + (size_t)token * H + n);
                    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
                }
                if (h_out) *reinterpret_cast<float4 *>(h_out + h_tile_offset(token, n, H)) = make_float4(x[0], x[1], x[2], x[3]);
                const float4 g4 = *reinterpret_cast<const float4 *>(g + n);
                uint2 o;
                o.x = pack_h16x2(x[0] * g4.x, x[1] * g4.y);
                o.y = pack_h16x2(x[2] * g4.z, x[3] * g4.w);
                *reinterpret_cast<uint2 *>(hg + frag_offset(token, n, H >> 5)) = o;
            }
            ss += x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
        }
    }
    ss += __shfl_xor(ss, 32, 64);
    if (hl == 0 && tv) ssq_out[(size_t)(col0 / GEMM_SSQ_COLS) * T + token] = ss;
}

void launch_prefill_prologue(const void *in, int in_is_h16, float *h_out, const float *g, h16_t *hg, float *ssq_out,
                             int T, int H, hipStream_t s) {
    if (T <= 0) return;
    const dim3 grid((T + 31) / 32, (H / GEMM_SSQ_COLS + 3) / 4);
    if (in_is_h16)
        hipLaunchKernelGGL(prefill_prologue_kernel<true>, grid, dim3(256), 0, s, in, h_out, g, hg, ssq_out, T, H);
    else
        hipLaunchKernelGGL(prefill_prologue_kernel<false>, grid, dim3(256), 0, s, in, h_out, g, hg, ssq_out, T, H);
}

// tiled residual stream -> row-major fp32 (debug taps)
__global__ void untile_h_kernel(const float *__restrict__ h_tiled, float *__restrict__ out, int T, int H) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= (int64_t)T * H) return;
    const int t = (int)(i / H), n = (int)(i % H);
    *reinterpret_cast<float4 *>(out + i) = *reinterpret_cast<const float4 *>(h_tiled + h_tile_offset(t, n, H));
}
void launch_untile_h(const float *h_tiled, float *out, int T, int H, hipStream_t s) {
    const int64_t n4 = (int64_t)T * H / 4;
    if (n4 <= 0) return;
    hipLaunchKernelGGL(untile_h_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, h_tiled, out, T, H);
}

}  // namespace HX_NS
