// Host-side launchers of the stage kernels.  Every launcher only enqueues on `s`.
// Shapes are validated by the caller (stage.cpp) before any launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.h"

// Row bookkeeping of one call: token row i belongs to sequence row_seq[i] at absolute
// position row_pos[i] (device int32 arrays).  For decode they are derived on the device from the
// cache's committed lengths, so one step needs no host->device traffic.
struct RowMap {
    const int32_t *row_seq;   // [T]
    const int32_t *row_pos;   // [T]
};

// KV cache geometry of one (layer, sequence, kv head) slab; see kernels_bf16_attn.hip
struct KvGeom {
    int d;            // head dim (64 | 128)
    int hkv_l;        // local kv heads
    int smax;         // positions per sequence, multiple of 32
    int64_t seq_stride;   // elements between sequences  (= hkv_l * smax * d)
};

// ---- layout / utility (kernels_layout.hip) -------------------------------------------------
// Weights are packed k-tile-major: tile (kt, nt) of a matrix with dst_n_tiles feature tiles sits at
// ((kt * dst_n_tiles + nt) * 64 + lane) * 8 elements.  All blocks of a projection walk kt together, so at
// any moment the chip streams one contiguous window of HBM instead of hundreds of scattered slabs.
// dst tile (dst_tile0 + nt * dst_tile_stride) <- src[k0 + k][c0 + nt*16 + i], src row-major with
// leading dimension ld (elements), K % 32 == 0, N % 16 == 0.
// rope_d > 0 (fused QKV weight): columns are heads of width rope_d; each 16-row tile of a head holds 8
// rotary pairs (rows 0-7 = head columns 8*tl .. 8*tl+7, rows 8-15 = those + rope_d/2), so one MFMA tile is
// self-contained for RoPE.  The QKV projection output is in this permuted column order.
void launch_pack_weight(const h16_t *src, int64_t ld, int k0, int c0, int K, int N, h16_t *dst,
                        int dst_tile0, int dst_tile_stride, int dst_n_tiles, int rope_d, hipStream_t s);
void launch_accumulate_f32(float *dst, const float *src, int64_t n, hipStream_t s);
// decode row map: row i -> (seq i, pos lens[i])
void launch_decode_rowmap(const int32_t *lens, int32_t *row_seq, int32_t *row_pos, int b, hipStream_t s);
void launch_advance_lens(int32_t *lens, int b, hipStream_t s);

// plain streaming kernels of known size (HBM calibration for the benchmarks and profiler counters)
void launch_stream_copy(const void *src, void *dst, int64_t bytes, int blocks, hipStream_t s);
void launch_stream_read(const void *src, float *sink, int64_t bytes, int blocks, hipStream_t s);
// register-resident MFMA loops: 4 waves per block, per wave and iteration 2^20 flop (one 128 x 128 x 32 k-step)
void launch_mfma_probe(int variant, float *sink, int iters, int blocks, hipStream_t s);

// ---- 16-bit path (kernels_bf16_*.hip, compiled once per element type: namespaces bf16 and f16) --------------------

// ---- decode projections with fused epilogues (kernels_bf16_decode.hip) ---------------------------
enum { DEC_RAW = 0, DEC_QKV = 1, DEC_RESID = 2, DEC_SWIGLU = 3 };
#define DEC_SSQ_STRIDE 32      // tokens per unit row of the sum-of-squares scratch
struct DecodeEpi {
    int mode;                  // DEC_*
    // RMSNorm statistics of the rows feeding this projection: sums of squares per (16-column unit,
    // token); NULL when the input is not a normalised residual stream (W_O, W2)
    const float *ssq_in;
    int ssq_units, norm_dim;
    float eps;
    float *raw_out;            // RAW: [T][N] fp32
    // QKV
    int hq_l;
    KvGeom kg;
    const int32_t *row_pos;
    const float *cos_tab, *sin_tab;
    h16_t *q_hi, *q_lo, *kc, *vc;
    // RESID
    float *h;                  // residual stream [T][N] fp32, updated in place
    const float *g_next;       // gain of the next RMSNorm
    h16_t *hg;                // (h * g_next) as compact hi/lo decode operand (dec_act_offset)
    float *ssq_out;
    int last_layer;            // 1: write out_partial / out_resid (bf16 [T][N]) instead of updating h
    h16_t *out_partial, *out_resid;
    // SWIGLU
    h16_t *u;                 // compact hi/lo decode operand [T][F_l]
    int F_l;
};
// What the decode attention needs to finish a QKV projection whose contraction was split over blocks: it adds up the
// partial sums of its own heads, applies 1/rms and the rotary embedding, appends the new K / V row to the cache and
// goes on with q in registers -- the projection then needs no finishing launch (launch_decode_qkv, launch_attn_decode).
struct QkvTail {
    const float *part;         // [splits][T][N] partial sums; NULL: q and the cache rows are complete already
    int splits, T, N;
    const float *rstd;         // [T] 1/rms of the rows, left by the split kernel
    const float *cos_tab, *sin_tab;
};
// ---- prefill projections with fused epilogues (kernels_bf16_gemm.hip) ----------------------------
// Same epilogue roles as in decode (DEC_* modes), on packed operands: the input Xp is (h * gain) in
// fragment tiles, RMSNorm enters as the per-token scale rstd derived from `ssq_in`.
#define GEMM_SSQ_COLS 128      // features per sum-of-squares partial: ssq[H / 128][T]
struct GemmEpi {
    int mode;                  // DEC_RAW | DEC_QKV | DEC_RESID | DEC_SWIGLU
    const float *ssq_in;       // [norm_dim / 128][T] sums of squares of the input rows, NULL = not normalised
    int norm_dim;
    float eps;
    float *raw_out;            // RAW: [T][N] fp32
    // QKV
    int hq_l;
    KvGeom kg;
    RowMap rm;
    const float *cos_tab, *sin_tab;
    h16_t *q, *kc, *vc;       // q: fragment tiles [T/16][hq_l * d / 32]
    // RESID
    float *h;                  // residual stream, fp32, 32 x 32 tiled (h_tile_offset), updated in place
    const float *g_next;
    h16_t *hg;                // (h * g_next) in fragment tiles [T/16][N/32]
    float *ssq_out;            // [N / 128][T]
    int last_layer;
    h16_t *out_partial, *out_resid;
    // SWIGLU
    h16_t *u;                 // fragment tiles [T/16][F_l/32]
    int F_l;
};
// per row of logits [n][ld]: the largest of the first `valid` entries and its index + id0 (lowest index wins ties)
void launch_row_argmax(const float *logits, int64_t ld, int valid, int n, int id0, int32_t *token_out, float *logit_out,
                       hipStream_t s);
// rows_out[i] = table[clamp(tokens[i], 0, vocab - 1)], rows of row_bytes bytes (a multiple of 4)
void launch_embed_rows(const void *table, int64_t row_bytes, int vocab, const int32_t *tokens, int n, void *rows_out,
                       hipStream_t s);

// p[0 .. bytes) = 0 with a kernel; p 4-byte aligned, bytes a multiple of 4
void launch_fill_zero(void *p, size_t bytes, hipStream_t s);


// ---- fp32 path (kernels_f32.hip): plain layouts, vector ALU -----------------------------------
void f32_launch_rmsnorm(const float *in, const float *g, float *out, int T, int H, float eps, hipStream_t s);
void f32_launch_gemm(const float *X, const float *W, float *out, int T, int K, int N, hipStream_t s);
void f32_launch_rope_append(const float *qkv, int T, int hq_l, int hkv_l, int d, int smax, RowMap rm,
                            const float *cos_tab, const float *sin_tab, float *q_out, float *kc, float *vc,
                            hipStream_t s);
void f32_launch_attn(const float *q, const float *kc, const float *vc, int T, int hq_l, int hkv_l, int d,
                     int smax, RowMap rm, float *o, hipStream_t s);
void f32_launch_swiglu(const float *ab, float *u, int T, int F_l, hipStream_t s);
void f32_launch_kv_copy(float *kc, float *vc, float *k, float *v, int hkv_l, int d, int smax, int seq,
                        int pos0, int n, int to_cache, hipStream_t s);

// ---- launchers that depend on the 16-bit element type: the same declarations in namespace bf16 and in namespace f16 ----
#define HX_DECL_NS bf16
#include "kernels_h16.inc"
#undef HX_DECL_NS
#define HX_DECL_NS f16
#include "kernels_h16.inc"
#undef HX_DECL_NS
