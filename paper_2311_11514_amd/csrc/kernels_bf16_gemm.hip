// Prefill projection: LDS-staged MFMA GEMM, D^T[n][t] = sum_k Wp[n][k] * Xp[t][k].
//
// Block = 4 waves (2 x 2); each wave owns FM x FT tiles of 32 features x 32 tokens computed with
// v_mfma_f32_32x32x16_bf16 (measured on this chip: 85 % of the datasheet rate from registers against 64 % for
// the 16x16x32 form, which is issue-limited), so the block tile is (64 FM) features x (64 FT) tokens.  The
// large configuration (FM = FT = 4: 256 x 256 block, 128 x 128 per wave, 256 accumulator registers per
// lane) keeps LDS out of the way: per 32-deep k-step a wave issues 16 128-bit LDS reads for 32 MFMAs.
// Operands stay in the 16 x 32 fragment tiles shared with the decode kernels (see common.h): global -> LDS
// is a straight copy, and a 32x32x16 operand is gathered from two neighbouring 16-row tiles with per-lane
// LDS addresses (every 8 lanes still read 128 contiguous bytes: conflict-free).  Both MFMA inputs use the
// same gather, so the k-order inside a tile cancels.
// Weights are k-tile-major, so the weight tiles of a block's k-step are one contiguous run of HBM.
//
// blockIdx.x is remapped so that each XCD (blocks are dealt round-robin to the 8 XCDs) works on a
// contiguous range of tiles, token-block fastest: tiles resident on one XCD share weight panels in
// that XCD's L2.
#include <cstdlib>

#include "kernels.h"

#define HX_AS1(p) ((const __attribute__((address_space(1))) void *)(p))
#define HX_AS3(p) ((__attribute__((address_space(3))) void *)(p))
// s_waitcnt that only constrains vmcnt (gfx9 encoding: vmcnt[3:0] | expcnt<<4 | lgkmcnt<<8 | vmcnt[5:4]<<14)
#define HX_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
// Workgroup barrier WITHOUT the device-memory release a __syncthreads() carries: that release would make
// the compiler drain every outstanding direct-to-LDS load (vmcnt(0)) at each k-step and undo the
// pipelining.  LDS reads of the previous step have been consumed by MFMAs before this point; the loads
// of the step about to be read are covered by the explicit vmcnt wait issued just before.
#define HX_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// Operand tiles travel HBM -> LDS with direct-to-LDS loads (no registers in between): a wave copies one
// 1 KB fragment tile per instruction, lane l's 16 bytes landing at tile base + 16 l.  S stages of the k-loop
// are resident; loads run S - 1 steps ahead of the math and the wait before a step only covers that step's
// loads (vmcnt counts the rest).
template <int FM, int FT, int S>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const bf16_t *__restrict__ Wp, const bf16_t *__restrict__ Xp,
                                                       float *__restrict__ out, int N, int k_tiles, int n_tiles,
                                                       int t_tiles, int T, int n_blocks, int t_blocks) {
    constexpr int TA = 4 * FM, TB = 4 * FT;          // 16-row operand tiles per block and k-step
    constexpr int LPT = (TA + TB) / 4;               // direct-to-LDS loads per thread and stage
    constexpr int STAGE = (TA + TB) * 64;            // bf16x8 elements per stage
    extern __shared__ bf16x8 smem[];                 // [S][TA + TB][64]
    // XCD-aware remap of the linear block id
    const int total = n_blocks * t_blocks;
    int id = blockIdx.x;
    const int per_xcd = (total + 7) / 8;
    id = (id & 7) * per_xcd + (id >> 3);
    if (id >= total) return;                     // only when total is not a multiple of 8
    const int bm = id / t_blocks, bt = id - bm * t_blocks;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave & 1, wt = wave >> 1;

    floatx16 acc[FM][FT];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const bf16x8 *A = reinterpret_cast<const bf16x8 *>(Wp);
    const bf16x8 *B = reinterpret_cast<const bf16x8 *>(Xp);
    // this wave copies tiles wave, wave + 4, ... of both operands; out-of-range tiles are clamped to the last
    // valid tile (their products are never stored) so that every thread issues LPT loads per stage
    const bf16x8 *asrc[TA / 4], *bsrc[TB / 4];
#pragma unroll
    for (int i = 0; i < TA / 4; ++i) asrc[i] = A + (size_t)min(bm * TA + wave + 4 * i, n_tiles - 1) * 64 + lane;
#pragma unroll
    for (int i = 0; i < TB / 4; ++i) bsrc[i] = B + (size_t)min(bt * TB + wave + 4 * i, t_tiles - 1) * k_tiles * 64 + lane;
    const size_t astep = (size_t)n_tiles * 64;       // k-tile-major weights
    auto issue = [&](int kt) {
        bf16x8 *st = smem + (size_t)(kt % S) * STAGE;
#pragma unroll
        for (int i = 0; i < TA / 4; ++i)
            __builtin_amdgcn_global_load_lds(HX_AS1(asrc[i] + kt * astep), HX_AS3(st + (wave + 4 * i) * 64), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < TB / 4; ++i)
            __builtin_amdgcn_global_load_lds(HX_AS1(bsrc[i] + (size_t)kt * 64), HX_AS3(st + (TA + wave + 4 * i) * 64), 16, 0, 0);
    };
    // 32x32x16 operand for k-half kh of a pair of 16-row tiles: lane l takes row l % 32, k-group 2 kh + l / 32
    const int frag = ((lane & 31) >> 4) * 64 + (lane & 15) + 16 * (lane >> 5);
#pragma unroll
    for (int p = 0; p < S - 1; ++p)
        if (p < k_tiles) issue(p);
    for (int kt = 0; kt < k_tiles; ++kt) {
        // loads of the S - 2 later stages may stay in flight; near the end fewer were issued, so wait for all
        if (kt + S - 2 < k_tiles) HX_WAIT_VM((S - 2) * LPT);
        else HX_WAIT_VM(0);
        HX_LDS_BARRIER();         // stage kt is complete for every wave, and stage kt - 1 is no longer read
        if (kt + S - 1 < k_tiles) issue(kt + S - 1);
        const bf16x8 *sa = smem + (size_t)(kt % S) * STAGE + (wm * FM * 2) * 64 + frag;
        const bf16x8 *sb = smem + (size_t)(kt % S) * STAGE + (TA + wt * FT * 2) * 64 + frag;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            bf16x8 b[FT];
#pragma unroll
            for (int j = 0; j < FT; ++j) b[j] = sb[j * 128 + kh * 32];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const bf16x8 a = sa[i * 128 + kh * 32];
#pragma unroll
                for (int j = 0; j < FT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[j], acc[i][j], 0, 0, 0);
            }
        }
    }
    // 32 x 32 result: lane l holds token column l % 32 and, per register quad q, features 8 q + 4 (l / 32) .. + 3
#pragma unroll
    for (int j = 0; j < FT; ++j) {
        const int token = (bt * TB + (wt * FT + j) * 2) * 16 + (lane & 31);
        if (token >= T) continue;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = (bm * TA + (wm * FM + i) * 2) * 16 + 8 * q + 4 * (lane >> 5);
                if (n < N)
                    *reinterpret_cast<floatx4 *>(out + (size_t)token * N + n) =
                        floatx4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            }
    }
}

template <int FM, int FT, int S>
static void launch_cfg(const bf16_t *Wp, const bf16_t *Xp, float *out, int N, int k_tiles, int n_tiles, int t_tiles,
                       int T, hipStream_t s) {
    const int n_blocks = (n_tiles + 4 * FM - 1) / (4 * FM), t_blocks = (t_tiles + 4 * FT - 1) / (4 * FT);
    const int total = n_blocks * t_blocks;
    const int grid = (total + 7) / 8 * 8;
    auto kern = gemm_mfma_kernel<FM, FT, S>;
    const size_t dyn = (size_t)S * (4 * FM + 4 * FT) * 64 * sizeof(bf16x8);
    static bool raised = false;           // more than the default 64 KB of LDS per block
    if (!raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)dyn);
        raised = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), dyn, s, Wp, Xp, out, N, k_tiles, n_tiles, t_tiles, T, n_blocks,
                       t_blocks);
}

void launch_gemm_mfma(const bf16_t *Wp, const bf16_t *Xp, float *out, int N, int K, int T, hipStream_t s) {
    const int k_tiles = K / 32, n_tiles = N / 16, t_tiles = (T + 15) / 16;
    static const int force = std::getenv("HEXGEN_GEMM_TILE") ? std::atoi(std::getenv("HEXGEN_GEMM_TILE")) : 0;
    // tiles of 256 x 256 once they fill the chip; smaller tiles for small problems
    const long big = (long)((n_tiles + 15) / 16) * ((t_tiles + 15) / 16);
    int cfg = big >= 200 ? 88 : ((long)((n_tiles + 15) / 16) * ((t_tiles + 7) / 8) >= 200 ? 84 : 44);
    if (force) cfg = force;
#define HX_G(FM, FT, S) launch_cfg<FM, FT, S>(Wp, Xp, out, N, k_tiles, n_tiles, t_tiles, T, s)
    if (cfg == 88) HX_G(4, 4, 4);
    else if (cfg == 84) HX_G(4, 2, 4);
    else if (cfg == 48) HX_G(2, 4, 4);
    else HX_G(2, 2, 4);
#undef HX_G
}
