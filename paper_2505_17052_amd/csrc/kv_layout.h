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
//   V block: [4 dim tiles of 32][64 lanes = (half h, dim d)][8 tokens] — the A-operand of a
//            32x32x16 MFMA (32 dims x 16 tokens); lane (d, h) holds tokens 4h..4h+3 and 8+4h..8+4h+3,
//            which are exactly the keys whose scores that lane holds after the score MFMA.
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
        const int dt = e >> 5, d = e & 31, h = (t >> 2) & 1, slot = 4 * (t >> 3) + (t & 3);
        return (((dt * 64) + h * 32 + d) << 3) + slot;
    }
    return t * hd + e;
}
