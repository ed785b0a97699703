// Paged KV cache geometry and in-page element placement.
//
// Pool: [layer][K pages | V pages]; one page holds SEV_PAGE (16) tokens of every KV head;
// the block of one (page, head) is contiguous: 16 * head_dim elements.
//
// float32 caches keep a block as plain [token][head_dim].
//
// bfloat16 caches (head_dim 128) keep each block in the order the matrix-core attention kernel
// consumes it, so that one wave reads a block with four fully coalesced 1 KiB loads:
//   K block: [head_dim/8 chunks][16 tokens][8 elements]      — a 16x16x32 MFMA A-operand of
//            (16 keys x 32 dims) is 64 lanes x 16 B, contiguous.
//   V block: [4 tile pairs][64 lanes = 4 token groups x 16 dims][2 tiles][4 tokens] — lane
//            (dim d of a 16-dim tile, token group g) finds tokens 4g..4g+3 of two adjacent
//            dim tiles in one 16 B load.
#pragma once
#include <stdint.h>

struct KvGeom {
    char *pool;
    size_t layer_stride, v_offset;
    int L, Hkv, hd;
};

template <bool BF16>
__host__ __device__ inline int k_in_page(int t, int e, int hd) {
    if (BF16) return (((e >> 3) * 16 + t) << 3) + (e & 7);
    return t * hd + e;
}

template <bool BF16>
__host__ __device__ inline int v_in_page(int t, int e, int hd) {
    if (BF16) {
        const int tile = e >> 4, di = e & 15, pair = tile >> 1, tip = tile & 1, g = t >> 2, tt = t & 3;
        return ((((pair * 64) + g * 16 + di) * 2 + tip) << 2) + tt;
    }
    return t * hd + e;
}
