// Layout and utility kernels: weight repacking, dtype conversion, row maps, cache staging.
#include "kernels.h"
#include "kvlayout.h"

// One thread builds one 16-byte lane slot of the packed matrix.
// rope_d > 0: the columns are heads of width rope_d and every 16-row tile of a head is filled with 8 rotary
// pairs: tile rows 0-7 = head columns 8*tl .. 8*tl+7, rows 8-15 = the same columns + rope_d/2.
__global__ void pack_weight_kernel(const h16_t *__restrict__ src, int64_t ld, int k0, int c0, int k_tiles,
                                   int n_tiles, h16_t *__restrict__ dst, int dst_tile0, int dst_tile_stride,
                                   int dst_n_tiles, int rope_d) {
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)n_tiles * k_tiles * 64;
    if (gid >= total) return;
    int lane = (int)(gid & 63);
    int64_t tile = gid >> 6;
    int kt = (int)(tile % k_tiles), nt = (int)(tile / k_tiles);
    int n = c0 + nt * 16 + (lane & 15);
    if (rope_d > 0) {
        const int tph = rope_d >> 4, head = nt / tph, tl = nt - head * tph, i = lane & 15;
        n = c0 + head * rope_d + tl * 8 + (i & 7) + (i >= 8 ? (rope_d >> 1) : 0);
    }
    int k = k0 + kt * 32 + 8 * (lane >> 4);
    union { h16_t e[8]; uint4 v; } u;
#pragma unroll
    for (int j = 0; j < 8; ++j) u.e[j] = src[(int64_t)(k + j) * ld + n];
    int64_t dt = (int64_t)dst_tile0 + (int64_t)nt * dst_tile_stride;
    *reinterpret_cast<uint4 *>(dst + (((int64_t)kt * dst_n_tiles + dt) * 64 + lane) * 8) = u.v;
}

void launch_pack_weight(const h16_t *src, int64_t ld, int k0, int c0, int K, int N, h16_t *dst,
                        int dst_tile0, int dst_tile_stride, int dst_n_tiles, int rope_d, hipStream_t s) {
    int k_tiles = K / 32, n_tiles = N / 16;
    int64_t total = (int64_t)n_tiles * k_tiles * 64;
    if (total == 0) return;
    int blocks = (int)((total + 255) / 256);
    hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks), dim3(256), 0, s, src, ld, k0, c0, k_tiles, n_tiles,
                       dst, dst_tile0, dst_tile_stride, dst_n_tiles, rope_d);
}

__global__ void accumulate_f32_kernel(float *__restrict__ dst, const float *__restrict__ src, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] += src[i];
}
void launch_accumulate_f32(float *dst, const float *src, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
    hipLaunchKernelGGL(accumulate_f32_kernel, dim3(blocks), dim3(256), 0, s, dst, src, n);
}

__global__ void decode_rowmap_kernel(const int32_t *lens, int32_t *row_seq, int32_t *row_pos, int b) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < b) { row_seq[i] = i; row_pos[i] = lens[i]; }
}
void launch_decode_rowmap(const int32_t *lens, int32_t *row_seq, int32_t *row_pos, int b, hipStream_t s) {
    hipLaunchKernelGGL(decode_rowmap_kernel, dim3((b + 63) / 64), dim3(64), 0, s, lens, row_seq, row_pos, b);
}
__global__ void advance_lens_kernel(int32_t *lens, int b) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < b) lens[i] += 1;
}
void launch_advance_lens(int32_t *lens, int b, hipStream_t s) {
    hipLaunchKernelGGL(advance_lens_kernel, dim3((b + 63) / 64), dim3(64), 0, s, lens, b);
}

// zero fill as a kernel (a memset node recorded into a captured graph is avoided on purpose)
__global__ void fill_zero_kernel(uint32_t *__restrict__ p, size_t n_words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n_words; i += stride) p[i] = 0u;
}
void launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
    const size_t n = bytes / 4;
    if (n == 0) return;
    const int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint32_t *>(p), n);
}

// ---- measurement utilities: plain streaming kernels of known size ---------------------------------
// copy: dst[i] = src[i] over n 16-byte words; read: sums every word into one float per thread block
// (so the loads cannot be dropped).  Both walk memory in 1 KB-per-wave chunks like the decode kernels.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                         int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n; i += stride) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *__restrict__ src, float *__restrict__ sink,
                                                         int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i + 7 * stride < n; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    for (; i < n; i += stride) { u32x4 v = src[i]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x9e3779b9u) sink[blockIdx.x] = 1.0f;     // practically never: keeps the loads alive
}
void launch_stream_copy(const void *src, void *dst, int64_t bytes, int blocks, hipStream_t s) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const u32x4 *>(src),
                       static_cast<u32x4 *>(dst), bytes / 16);
}
void launch_stream_read(const void *src, float *sink, int64_t bytes, int blocks, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const u32x4 *>(src), sink,
                       bytes / 16);
}

// ---- the model's ends: greedy argmax over a row of logits, embedding row gather --------------------------------
// One block of 1024 threads per row.  Each thread scans a strided slice (four entries per load when the row pitch
// allows it, several loads in flight) keeping (value, lowest index); the block reduces in LDS with the same rule, so
// the result is the first maximum of the row, as numpy / torch argmax define it.
template <bool VEC4>
__global__ __launch_bounds__(1024) void row_argmax_kernel(const float *__restrict__ logits, int64_t ld, int valid, int id0,
                                                         int32_t *__restrict__ token_out, float *__restrict__ logit_out) {
    __shared__ float sv[1024];
    __shared__ int si[1024];
    const float *row = logits + (int64_t)blockIdx.x * ld;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    auto take = [&](float v, int i) {
        if (i < valid && (v > bv || (v == bv && i < bi))) { bv = v; bi = i; }
    };
    if (VEC4) {
        const int n4 = (valid + 3) >> 2;          // the pitch is a multiple of 4: the last quad stays inside the row
#pragma unroll 4
        for (int q = threadIdx.x; q < n4; q += 1024) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(row + 4 * q);
            take(v[0], 4 * q); take(v[1], 4 * q + 1); take(v[2], 4 * q + 2); take(v[3], 4 * q + 3);
        }
    } else {
#pragma unroll 4
        for (int i = threadIdx.x; i < valid; i += 1024) take(row[i], i);
    }
    sv[threadIdx.x] = bv;
    si[threadIdx.x] = bi;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            const float v = sv[threadIdx.x + o];
            const int i = si[threadIdx.x + o];
            if (v > sv[threadIdx.x] || (v == sv[threadIdx.x] && i < si[threadIdx.x])) { sv[threadIdx.x] = v; si[threadIdx.x] = i; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        token_out[blockIdx.x] = id0 + (si[0] == 0x7fffffff ? 0 : si[0]);
        if (logit_out) logit_out[blockIdx.x] = sv[0];
    }
}
void launch_row_argmax(const float *logits, int64_t ld, int valid, int n, int id0, int32_t *token_out, float *logit_out,
                       hipStream_t s) {
    if (n <= 0) return;
    if (ld % 4 == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0)
        hipLaunchKernelGGL(row_argmax_kernel<true>, dim3(n), dim3(1024), 0, s, logits, ld, valid, id0, token_out, logit_out);
    else
        hipLaunchKernelGGL(row_argmax_kernel<false>, dim3(n), dim3(1024), 0, s, logits, ld, valid, id0, token_out, logit_out);
}

__global__ void embed_rows_kernel(const uint32_t *__restrict__ table, int64_t row_words, int vocab,
                                  const int32_t *__restrict__ tokens, uint32_t *__restrict__ out) {
    const int tok = min(max(tokens[blockIdx.x], 0), vocab - 1);
    const uint32_t *src = table + (int64_t)tok * row_words;
    uint32_t *dst = out + (int64_t)blockIdx.x * row_words;
    for (int64_t i = threadIdx.x; i < row_words; i += blockDim.x) dst[i] = src[i];
}
void launch_embed_rows(const void *table, int64_t row_bytes, int vocab, const int32_t *tokens, int n, void *rows_out,
                       hipStream_t s) {
    if (n <= 0) return;
    hipLaunchKernelGGL(embed_rows_kernel, dim3(n), dim3(256), 0, s, static_cast<const uint32_t *>(table), row_bytes / 4, vocab,
                       tokens, static_cast<uint32_t *>(rows_out));
}

// ---- measurement utility: register-resident MFMA loops (what the matrix cores sustain on this machine) ------
// variant 0: v_mfma_f32_16x16x32_bf16, 64 independent accumulators per wave; variant 1: v_mfma_f32_32x32x16_bf16,
// 16 accumulators; variants 2 / 3: the same with the LDS fragment reads of a 128 x 128 wave tile (16 reads per
// 32-deep k-step).  One 4-wave block per launch slot; every block runs `iters` k-steps of 2^20 flop per wave.
// RANDOM = false fills the operands with 1.0; RANDOM = true with random signs and mantissas (exponent fixed so that
// nothing overflows): the matrix cores draw far more power on operands whose bits toggle, and the chip then holds
// a lower clock, so the all-ones figure is an upper bound no real GEMM sees.
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
template <int VARIANT, bool RANDOM>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *sink, int iters) {
    __shared__ h16x8 sm[32][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 32 * 64; i += 256) {
        uint32_t h = (uint32_t)i * 2654435761u + blockIdx.x * 40503u;
        uint32_t w[4];
        for (int c = 0; c < 4; ++c) {
            h = h * 1664525u + 1013904223u;
            w[c] = RANDOM ? ((h & 0x807f807fu) | 0x3f003f00u) : 0x3f803f80u;      // +-[0.5, 1) or 1.0, twice
        }
        sm[i >> 6][i & 63] = *reinterpret_cast<const h16x8 *>(w);
    }
    __syncthreads();
    constexpr bool LDS = VARIANT >= 2;
    float total = 0.f;
    if (VARIANT == 0 || VARIANT == 2) {
        floatx4 acc[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        h16x8 a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { a[i] = sm[i][lane]; b[i] = sm[8 + i][lane]; }
        for (int it = 0; it < iters; ++it) {
            if (LDS) {
#pragma unroll
                for (int j = 0; j < 8; ++j) b[j] = sm[(16 + j + it) & 31][lane];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (LDS) a[i] = sm[(i + it + wave) & 31][lane];
#pragma unroll
                for (int j = 0; j < 8; ++j)      // written as asm: the builtin form makes the compiler shuffle accumulator registers in this loop
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[i]), "v"(b[j]));
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) total += acc[i][j][0] + acc[i][j][3];
    } else {
        floatx16 acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        h16x8 a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = sm[i][lane]; b[i] = sm[8 + i][lane]; }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                if (LDS) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) b[j] = sm[(16 + j + it + kh * 4) & 31][lane];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (LDS) a[i] = sm[(i + it + wave + kh * 4) & 31][lane];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[i]), "v"(b[j]));
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) total += acc[i][j][0] + acc[i][j][7];
    }
    if (total == 123.456f) sink[threadIdx.x] = total;      // practically never: keeps the math alive
}
// Variants 8..11: v_mfma_f32_16x16x32_bf16 on random operand bits with the 128 accumulator registers per wave that the
// two-phase GEMM loop holds (4 x 8 results), in accumulation registers (8, 10) or in ordinary vector registers (9, 11),
// issued row by row (8, 9) or in a serpentine that changes only one operand from one instruction to the next (10, 11):
// whether register class or operand order moves the energy per flop.
template <bool VACC, bool SNAKE>
__global__ __launch_bounds__(256) void mfma_probe2_kernel(float *sink, int iters) {
    __shared__ h16x8 sm[32][64];
    const int lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < 32 * 64; i += 256) {
        uint32_t h = (uint32_t)i * 2654435761u + blockIdx.x * 40503u;
        uint32_t w[4];
        for (int c = 0; c < 4; ++c) {
            h = h * 1664525u + 1013904223u;
            w[c] = (h & 0x807f807fu) | 0x3f003f00u;
        }
        sm[i >> 6][i & 63] = *reinterpret_cast<const h16x8 *>(w);
    }
    __syncthreads();
    floatx4 acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    h16x8 a[4], b[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = sm[i][lane];
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = sm[8 + j][lane];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 2; ++rep)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const int j = (SNAKE && (i & 1)) ? 7 - jj : jj;
                    if (VACC) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i][j]) : "v"(a[i]), "v"(b[j]));
                    else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[i]), "v"(b[j]));
                }
    }
    float total = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) total += acc[i][j][0] + acc[i][j][3];
    if (total == 123.456f) sink[threadIdx.x] = total;
}

void launch_mfma_probe(int variant, float *sink, int iters, int blocks, hipStream_t s) {
    if (variant >= 8 && variant <= 11) {       // per k-step: 64 MFMAs of 16384 flop = 2^20 flop per wave, as in the variants above
        switch (variant) {
            case 8: hipLaunchKernelGGL((mfma_probe2_kernel<false, false>), dim3(blocks), dim3(256), 0, s, sink, iters); break;
            case 9: hipLaunchKernelGGL((mfma_probe2_kernel<true, false>), dim3(blocks), dim3(256), 0, s, sink, iters); break;
            case 10: hipLaunchKernelGGL((mfma_probe2_kernel<false, true>), dim3(blocks), dim3(256), 0, s, sink, iters); break;
            default: hipLaunchKernelGGL((mfma_probe2_kernel<true, true>), dim3(blocks), dim3(256), 0, s, sink, iters); break;
        }
        return;
    }
#define HX_P(V, R) hipLaunchKernelGGL((mfma_probe_kernel<V, R>), dim3(blocks), dim3(256), 0, s, sink, iters)
    switch (variant) {
        case 0: HX_P(0, false); break;
        case 1: HX_P(1, false); break;
        case 2: HX_P(2, false); break;
        case 3: HX_P(3, false); break;
        case 4: HX_P(0, true); break;
        case 5: HX_P(1, true); break;
        case 6: HX_P(2, true); break;
        default: HX_P(3, true); break;
    }
#undef HX_P
}
