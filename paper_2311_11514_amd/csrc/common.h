// Shared device-side definitions for the gfx950 stage kernels.
//
// Operand layout ("fragment-major").  Every bf16 matrix that feeds the matrix cores -- weights and
// the activations this library produces for its own GEMMs -- is stored so that one
// v_mfma_f32_16x16x32_bf16 operand is a single contiguous 1 KB block: a matrix M[idx][k]
// (idx = output feature for weights, token row for activations; k = contraction index) is cut into
// tiles of 16 idx x 32 k; inside a tile lane l holds idx = l % 16, k = 8 * (l / 16) + j, j = 0..7.
// Activation tiles are ordered row-tile-major, ((it * k_tiles + kt) * 64 + lane) * 8 (frag_offset below);
// weight tiles k-tile-major, ((kt * n_tiles + it) * 64 + lane) * 8.  A wave fetches an operand with one
// coalesced 128-bit load per lane, from HBM or from LDS, with no transposition anywhere.
// Both MFMA inputs use this same mapping, so any k-ordering inside a tile cancels in the product.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef uint16_t bf16_t;   // raw storage

#define HX_WAVE 64

// Decode activations (at most 32 token rows) use a compact token-major layout instead: per token and
// k-tile one 128-byte line holding the 32 hi values then the 32 lo values of the hi + lo bf16 split.
// A decode projection then touches one cache line per (token, k-tile) instead of eight.
__host__ __device__ inline size_t dec_act_offset(int token, int k, int k_tiles, int plane) {
    return (((size_t)token * k_tiles + (k >> 5)) * 2 + plane) * 32 + (k & 31);
}

// Prefill keeps its fp32 residual stream in the order the 32x32 MFMA result leaves the registers: blocks of
// 32 tokens x 32 features, inside a block [quad q][lane][4] with lane = token % 32 + 32 * ((f % 8) / 4) and
// q = (f % 32) / 8.  A wave's read-modify-write of the stream is then one contiguous 1 KB access instead
// of 32 row-strided 32-byte pieces.  Returns the offset of 4 consecutive features n .. n+3 (n % 4 == 0).
__host__ __device__ inline size_t h_tile_offset(int token, int n, int N) {
    const size_t blk = (size_t)(token >> 5) * (N >> 5) + (n >> 5);
    const int f = n & 31;
    return ((blk * 4 + (f >> 3)) * 64 + (token & 31) + 32 * ((f & 7) >> 2)) * 4;
}

__host__ __device__ inline size_t frag_offset(int idx, int k, int k_tiles) {
    int it = idx >> 4, kt = k >> 5;
    int lane = (idx & 15) + 16 * ((k & 31) >> 3);
    return ((size_t)(it * (size_t)k_tiles + kt) * 64 + lane) * 8 + (k & 7);
}

__device__ inline float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// fp32 -> bf16, round-to-nearest-even, with the hardware's packed conversion (v_cvt_pk_bf16_f32: one instruction
// per pair instead of half a dozen integer operations per value; the epilogues and the softmax are full of these)
typedef __bf16 hx_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hx_floatx2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    const hx_floatx2 v = {lo, hi};
    const hx_bf16x2 h = __builtin_convertvector(v, hx_bf16x2);
    return *reinterpret_cast<const uint32_t *>(&h);
}
__device__ inline bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// x = hi + lo with both parts bf16: the pair carries ~16 mantissa bits of an fp32 activation.
// Decode kernels are HBM-bound, so feeding hi and lo through two MFMAs costs nothing and removes the
// bf16 rounding of activations from the error budget of deep stages.
__device__ inline void split_bf16(float x, bf16_t &hi, bf16_t &lo) {
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - bf16_to_f32(hi));
}
// packs hi parts of (a, b) into *phi and lo parts into *plo
__device__ inline void split_pack2(float a, float b, uint32_t &phi, uint32_t &plo) {
    bf16_t ah, al, bh, bl;
    split_bf16(a, ah, al);
    split_bf16(b, bh, bl);
    phi = (uint32_t)ah | ((uint32_t)bh << 16);
    plo = (uint32_t)al | ((uint32_t)bl << 16);
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// block-wide sum for blockDim.x = 256 (4 waves); `red` is >= 4 floats of LDS
__device__ inline float block_sum_256(float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}
__device__ inline float block_max_256(float v, float *red) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
