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

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float hx_floatx16;
typedef uint16_t h16_t;    // raw storage of one 16-bit element (bf16 or fp16)

// ---- the 16-bit element type of this translation unit -------------------------------------------------------------
// The bf16 and the fp16 stage share every kernel: layouts, indexing and schedules only know "16-bit element".  What
// differs -- the MFMA opcode, fp32 <-> element conversion -- sits in the few functions below, and each kernel source
// is compiled once per element type (HX_ELEM_F16 defined or not) into its own namespace HX_NS (bf16 / f16).
// h16x8 = the 8 elements one lane contributes to an MFMA operand.
#ifdef HX_ELEM_F16
#define HX_NS f16
typedef _Float16 hx_elem;
#else
#define HX_NS bf16
typedef __bf16 hx_elem;
#endif
typedef __attribute__((__vector_size__(8 * sizeof(hx_elem)))) hx_elem h16x8;

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

typedef hx_elem hx_elemx2 __attribute__((ext_vector_type(2)));
typedef float hx_floatx2 __attribute__((ext_vector_type(2)));
#ifdef HX_ELEM_F16
__device__ inline float h16_to_f32(h16_t v) {
    _Float16 h;
    __builtin_memcpy(&h, &v, 2);
    return (float)h;
}
#else
__device__ inline float h16_to_f32(h16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
#endif
// the two elements of a packed pair (low half first)
__device__ inline void h16x2_to_f32(uint32_t raw, float &a, float &b) {
#ifdef HX_ELEM_F16
    a = h16_to_f32((h16_t)(raw & 0xffffu));
    b = h16_to_f32((h16_t)(raw >> 16));
#else
    a = __uint_as_float(raw << 16);
    b = __uint_as_float(raw & 0xffff0000u);
#endif
}

// fp32 -> element, round-to-nearest-even, with the hardware's packed conversion (one instruction per pair instead of
// half a dozen integer operations per value; the epilogues and the softmax are full of these).  fp16: values beyond
// 65504 become infinite, as the format has it.
__device__ inline uint32_t pack_h16x2(float lo, float hi) {
    const hx_floatx2 v = {lo, hi};
    const hx_elemx2 h = __builtin_convertvector(v, hx_elemx2);
    return *reinterpret_cast<const uint32_t *>(&h);
}
__device__ inline h16_t f32_to_h16(float f) { return (h16_t)(pack_h16x2(f, 0.f) & 0xffffu); }

// the two MFMA forms of the kernels, on this translation unit's element type
__device__ __forceinline__ floatx4 hx_mfma16(h16x8 a, h16x8 b, floatx4 c) {
#ifdef HX_ELEM_F16
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
#endif
}
__device__ __forceinline__ hx_floatx16 hx_mfma32(h16x8 a, h16x8 b, hx_floatx16 c) {
#ifdef HX_ELEM_F16
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
}

// x = hi + lo with both parts 16-bit: the pair carries ~16 (bf16) / ~21 (fp16) mantissa bits of an fp32 activation.
// Decode kernels are HBM-bound, so feeding hi and lo through two MFMAs costs nothing and removes the
// bf16 rounding of activations from the error budget of deep stages.
__device__ inline void split_h16(float x, h16_t &hi, h16_t &lo) {
    hi = f32_to_h16(x);
    lo = f32_to_h16(x - h16_to_f32(hi));
}
// packs hi parts of (a, b) into *phi and lo parts into *plo
__device__ inline void split_pack2(float a, float b, uint32_t &phi, uint32_t &plo) {
    h16_t ah, al, bh, bl;
    split_h16(a, ah, al);
    split_h16(b, bh, bl);
    phi = (uint32_t)ah | ((uint32_t)bh << 16);
    plo = (uint32_t)al | ((uint32_t)bl << 16);
}

// Device-scope accesses for data that blocks of one launch hand to each other (the split attention's partials): stores
// that go through to where every compute die of the GPU sees them -- complete, for the issuing lane, once its store
// counter has drained -- and loads that read from there instead of a line the reader's own L2 may still hold.  Such
// data is a few KB per block, so nothing is lost by not caching it, and no block needs a device-wide fence, which
// writes the die's whole L2 back (about 0.8 us each, one after the other per die: more than the kernel itself once
// a launch has a few hundred blocks).
__device__ __forceinline__ void dev_store(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float dev_load(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
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
