// bf16 KV-cache layout.  Per layer the cache is [seq][kv head] slabs of smax * d elements.
//
//  K slab: fragment tiles of 16 positions x 32 head-dim elements (the common operand layout with
//          idx = position, k = head-dim index): K is the A operand of S^T = K . Q^T.
//  V slab: tiles of 32 positions x 16 head-dim elements holding V^T (idx = head-dim index,
//          k-slot = position), the A operand of O^T = V^T . P^T.  The k-slots of a tile are
//          permuted so that they match what the S^T accumulators of two consecutive 16-position
//          tiles already hold per lane: lane group g = lane / 16 owns position offsets
//          4g..4g+3 (first tile) and 16+4g..16+4g+3 (second tile).  P therefore goes from the
//          score accumulators straight into the next MFMA with no cross-lane traffic.
#pragma once
#include "common.h"

__host__ __device__ inline size_t kv_k_offset(int pos, int dd, int d) {
    return frag_offset(pos, dd, d >> 5);
}
__host__ __device__ inline size_t kv_v_offset(int pos, int dd, int d) {
    int pt = pos >> 5, q = pos & 31, dt = dd >> 4;
    int g = (q & 15) >> 2, j = (q & 3) + 4 * (q >> 4);
    int lane = (dd & 15) + 16 * g;
    return ((size_t)(pt * (d >> 4) + dt) * 64 + lane) * 8 + j;
}
