// bfloat16 path for gfx950: matrix-core GEMMs that stream re-tiled bf16 weights once per step,
// paged-KV verification attention, and the fused element-wise stages between them.
//
// Precision recipe.  Weights and the KV cache are bf16.  Every activation that feeds a matrix
// core is carried as TWO bf16 planes, hi = bf16(x) and lo = bf16(x - hi), and multiplied in two
// MFMAs that accumulate into the same float32 registers; the residual stream, norms, rotary
// embedding, softmax and all accumulations are float32.  (A single bf16 plane per activation
// accumulates ~3 % relative error over 32 layers; the split keeps it near 1e-5.)
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <type_traits>

#include "sev_internal.h"
#include "kv_layout.h"

KvGeom sev_kv_geom(const sev_kv *kv);

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte vector (keeps staging arrays in registers)

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;          // round to nearest even (finite inputs)
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// hi/lo split of one float: hi = bf16(x), lo = bf16(x - hi)
__device__ __forceinline__ void split_bf16(float x, uint32_t &hi, uint32_t &lo) {
    hi = f32_to_bf16_bits(x);
    lo = f32_to_bf16_bits(x - bf16_bits_to_f32(hi));
}

// hi/lo split of two floats at once with the packed hardware conversion (round to nearest even):
// hi = {bf16(a), bf16(b)}, lo = {bf16(a - hi_a), bf16(b - hi_b)}, element 0 in the low half.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split_pack2(float a, float b, uint32_t &hi, uint32_t &lo) {
    const f32x2 v = {a, b};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    const bf16x2 l = __builtin_convertvector(v - __builtin_convertvector(h, f32x2), bf16x2);
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, l);
}

// Writes 8 consecutive-k activations of row m (k0 a multiple of 8) as hi and lo fragments.
__device__ __forceinline__ void store_split8(uint16_t *xp, int m, int k0, int m_tiles, const float *v) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) split_pack2(v[2 * i], v[2 * i + 1], h[i], l[i]);
    *(uint4 *)(xp + xpack_index(m, k0, 0, m_tiles)) = make_uint4(h[0], h[1], h[2], h[3]);
    *(uint4 *)(xp + xpack_index(m, k0, 1, m_tiles)) = make_uint4(l[0], l[1], l[2], l[3]);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float *red) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) s += red[w];
    __syncthreads();
    return s;
}

// ---------------------------------------------------------------------------
// weight re-tiling: canonical [rows][K] bf16 -> [tile][K/16][lane 64][8], where lane
// (n % 32) + 32*((k/8)%2) holds W[n][k..k+7]: exactly the A operand of a 32x32x16 MFMA.
//
// mode 0: source tile t lands at destination tile t + tile_add (plain, or a row range of a fused matrix).
// mode 1 / 2 (gate / up of the SwiGLU pair): destination tile t holds feed-forward columns
// [16t, 16t+16) of BOTH matrices, 4-row groups alternating so that an MFMA output lane owns the
// gate and the up value of the same 4 columns: tile row n = 8j + 4h + r (j = 0..3, h = 0..1, r = 0..3)
// is the gate (j even) or up (j odd) row 16t + 8(j/2) + 4h + r.
// mode 3 (q, k, v projections, head_dim 128): the same interleave inside every head, with the two
// halves of the head in the roles of gate and up: tile 4*head + t, row n holds the head's dim
// 16t + 8(j/2) + 4h + r (j even) or that dim + 64 (j odd), so that a lane owns both members of a
// rotary pair (i, i + 64).
// ---------------------------------------------------------------------------
__global__ void pack_bf16_kernel(uint4 *dst, const uint16_t *src, int K, int64_t n_chunks, int mode, int tile_add) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n_chunks) return;
    const int ksteps = K >> 4;
    const int lane = (int)(c & 63);
    const int64_t tk = c >> 6;
    const int kt = (int)(tk % ksteps);
    const int64_t t = tk / ksteps;                   // destination tile
    const int n = lane & 31;
    const int k = kt * 16 + 8 * (lane >> 5);
    int64_t row;
    if (mode == 0) {
        row = (t - tile_add) * 32 + n;
    } else if (mode == 3) {
        const int j = n >> 3;
        const int64_t tt = t - tile_add;
        row = (tt >> 2) * 128 + (j & 1) * 64 + (tt & 3) * 16 + 8 * (j >> 1) + (n & 7);
    } else {
        const int j = n >> 3;
        if ((j & 1) != mode - 1) return;             // this launch fills only its own 4-row groups
        row = t * 16 + 8 * (j >> 1) + (n & 7);
    }
    dst[(t * ksteps + kt) * 64 + lane] = *(const uint4 *)(src + row * K + k);
}

// n_rows source rows.  modes 0, 3: destination tiles tile_add .. tile_add + n_rows/32 - 1;
// modes 1, 2: destination tiles 0 .. n_rows/16 - 1.
void launch_pack_bf16(uint16_t *dst, const uint16_t *src, int n_rows, int K, int mode, int tile_add, hipStream_t st) {
    const bool whole = mode == 0 || mode == 3;
    const int64_t tiles = whole ? n_rows / 32 : n_rows / 16;
    const int64_t n_chunks = tiles * (K / 16) * 64;
    uint4 *d = (uint4 *)dst + (whole ? (int64_t)tile_add * (K / 16) * 64 : 0);
    hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st, d, src, K, n_chunks,
                       mode, 0);
}

// ---------------------------------------------------------------------------
// embedding gather.  One block per row: h = E[token] (float32), xa = split(h * g) for the first
// QKV GEMM (which applies the row's RMS scale in its epilogue), ssq = fixed-point sum of squares.
// ---------------------------------------------------------------------------
// Sums of squares of the residual rows are accumulated by many blocks; they are kept as 64-bit
// fixed point (2^-20 units) so that the atomic additions commute and the result is reproducible.
// One contribution (32 rows x <= 256 columns) is clamped to 1e10, so up to 1024 of them cannot wrap;
// what is lost below 2^-20 is far under the norm's epsilon once divided by the row width.
#define SSQ_SCALE 1048576.0f
__device__ __forceinline__ unsigned long long ssq_fix(float v) { return (unsigned long long)(fminf(v, 1.0e10f) * SSQ_SCALE); }
__device__ __forceinline__ float rms_scale(unsigned long long q, float inv_d, float eps) {
    return 1.0f / sqrtf((float)((double)q * (1.0 / 1048576.0)) * inv_d + eps);
}

__global__ __launch_bounds__(256) void embed_norm_kernel(const uint16_t *E, const int32_t *row_tok, const float *g,
                                                         float *h, uint16_t *xa, unsigned long long *ssq_out,
                                                         unsigned long long *ssq_clear, int d, int m_tiles) {
    __shared__ float red[4];
    const int m = blockIdx.x;
    const uint16_t *src = E + (size_t)row_tok[m] * d;
    float *hr = h + (size_t)m * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d / 8; c += 256) {
        const uint4 raw = *(const uint4 *)(src + c * 8);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
        float v[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = bf16_bits_to_f32(w[i] & 0xffffu);
            v[2 * i + 1] = bf16_bits_to_f32(w[i] >> 16);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += v[i] * v[i];
        *(float4 *)(hr + c * 8) = make_float4(v[0], v[1], v[2], v[3]);
        *(float4 *)(hr + c * 8 + 4) = make_float4(v[4], v[5], v[6], v[7]);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] *= g[c * 8 + i];
        store_split8(xa, m, c * 8, m_tiles, v);
    }
    ss = block_sum<256>(ss, red);
    if (threadIdx.x == 0) {
        ssq_out[m] = ssq_fix(ss);
        ssq_clear[m] = 0ull;
    }
}

// ---------------------------------------------------------------------------
// skinny-M GEMM on the matrix cores:  Y[M][N] = X[M][K] * W[N][K]^T, with the stage that follows
// the GEMM fused into its epilogue.
//
// A block of 4 waves covers up to 128 rows (MT tiles of 32) and 4*NT column tiles of 32 (NT = 1, 2, or 4
// with all 256 accumulator registers in use); wave w owns NT column tiles.  Weights go global -> registers, one fully coalesced 1 KiB fragment per
// load, PF stages ahead; each weight byte is read once per row block.  Activations (hi and lo
// planes, already in fragment order) go global -> LDS once per block and are shared by the 4 waves.
// MFMA 32x32x16: A = weight tile (32 n x 16 k), B = activation tile (16 k x 32 m), so a lane ends up
// with 4 consecutive output columns of one row per register quad.
// grid: 1-D over (column group, split-K slice, row block of MT tiles); see the block index decode.
//
// Split-K.  With S = 1 the block runs the epilogue itself.  With S > 1 it stores its accumulators
// in register order (coalesced 1 KiB stores, layout [slice][column tile][row tile]) and gemm_fixup_kernel,
// one wave per 32x32 output tile, adds the S slices in slice order and runs the same epilogue code.
//
// Normalisation.  RMSNorm scales row m by r[m] = 1/rms(h[m]) and column k by the gain g[k].  The
// producer of an activation matrix writes split(h * g) and the rows' sums of squares; the
// consuming GEMM multiplies its accumulators by r[m] (the scale commutes with the contraction).
//
// Epilogues (per 32x32 tile):
//   EPI_QKV    rotary embedding of q and k (weight rows of every head are interleaved so that a
//              lane holds both members of 4 rotary pairs), q -> hi/lo planes for the attention
//              kernel, k and v -> bf16 into the paged cache at position P + node
//   EPI_RESID  h += Y; xout = split(h * gain); adds the tile's sums of squares to ssq_out and
//              clears the buffer the next producer will add to
//   EPI_SWIGLU act = split(silu(gate) * up), gate and up rows interleaved in the weight tiles
//   EPI_ARGMAX per-wave arg-max of every row (+ optional float32 logits); never split
// ---------------------------------------------------------------------------
enum { EPI_QKV = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2, EPI_RESID = 3 };

struct GemmArgs {
    const uint4 *W;          // re-tiled weights
    const uint4 *X;          // xpack activations
    int n_tiles, k_steps, m_tiles_total, M, N;
    int col_groups, m_blocks, splits, mt, nt;   // grid decomposition (see the kernel's block index decode)
    float *part;             // split-K exchange: [S][column tile][row tile][4][64 lanes] float4
    const unsigned long long *ssq_in;   // [rows] sums of squares of the input rows, or null (input is not a normed stream)
    float inv_d, eps;
    // EPI_RESID
    float *h;                // residual stream [M][N]
    const float *gain;       // gains of the norm that follows
    uint16_t *xout;          // xpack (K = N) of h * gain
    unsigned long long *ssq_out, *ssq_clear;   // [rows]
    // EPI_SWIGLU
    uint16_t *act;           // xpack with K = N/2 (N counts gate and up rows)
    // EPI_QKV
    const float2 *row_cs;    // [rows][64] (cos, sin)
    const int32_t *row_kvloc; // [rows] physical page * 16 + token in page of the row's cache position
    int Hq, Hkv;
    char *k_layer;           // K pages of this layer; V pages follow at v_offset
    size_t v_offset;
    uint16_t *q_planes;      // [2][M][Hq*128]
    // EPI_ARGMAX
    float *lm_val;           // [col groups * 4][lm_stride]
    int32_t *lm_idx;
    int lm_stride;
    float *logits;           // optional: [M][N]
};

// Epilogue of one 32x32 output tile held in MFMA register order: lane (row = lane % 32, h = lane / 32)
// owns columns 8j + 4h + r (j = 0..3, r = 0..3) in acc[4j + r].  T = column tile, m = the lane's row.
// tile_pre issues every load the epilogue needs that does not depend on the accumulators (so that a
// caller can overlap them with its own loads); tile_epilogue consumes them and returns the lane's
// share of the tile's sum of squares (EPI_RESID).
struct TilePre {
    float rs;                // RMS scale of the row
    float4 hv[4], gn[4];     // EPI_RESID: residual values and gains of the lane's 16 columns
    float4 cs[4];            // EPI_QKV: (cos, sin) of the lane's 8 rotary pairs
    int kvloc;               // EPI_QKV: physical page * 16 + token in page of the row's cache position
};

template <int EPI, bool RS_KNOWN = false>
__device__ __forceinline__ TilePre tile_pre(const GemmArgs &g, int T, int m, int nsub, float rs_known = 1.0f) {
    TilePre p;
    p.rs = rs_known;
    p.kvloc = 0;
    if (m >= g.M) return p;
    if (!RS_KNOWN && g.ssq_in) p.rs = rms_scale(g.ssq_in[m], g.inv_d, g.eps);
    if constexpr (EPI == EPI_RESID) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int nn = T * 32 + 8 * j + nsub;
            p.hv[j] = *(const float4 *)(g.h + (size_t)m * g.N + nn);
            p.gn[j] = *(const float4 *)(g.gain + nn);
        }
    } else if constexpr (EPI == EPI_QKV) {
        const int hy = T >> 2, th = T & 3;
        if (hy >= g.Hq) p.kvloc = g.row_kvloc[m];
        if (hy < g.Hq + g.Hkv) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int i0 = 16 * th + 8 * jj + nsub;
                p.cs[2 * jj] = *(const float4 *)(g.row_cs + (size_t)m * 64 + i0);
                p.cs[2 * jj + 1] = *(const float4 *)(g.row_cs + (size_t)m * 64 + i0 + 2);
            }
        }
    }
    return p;
}

template <int EPI>
__device__ __forceinline__ float tile_epilogue(const GemmArgs &g, const f32x16 &acc, int T, int m, int nsub, const TilePre &p) {
    float ss = 0.f;
    if (m >= g.M) return ss;
    const float rs = p.rs;
    if constexpr (EPI == EPI_RESID) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int nn = T * 32 + 8 * j + nsub;
            float4 v = p.hv[j];
            v.x += acc[4 * j]; v.y += acc[4 * j + 1]; v.z += acc[4 * j + 2]; v.w += acc[4 * j + 3];
            *(float4 *)(g.h + (size_t)m * g.N + nn) = v;
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            const float4 gn = p.gn[j];
            uint32_t hi[2], lo[2];
            split_pack2(v.x * gn.x, v.y * gn.y, hi[0], lo[0]);
            split_pack2(v.z * gn.z, v.w * gn.w, hi[1], lo[1]);
            *(uint2 *)(g.xout + xpack_index(m, nn, 0, g.m_tiles_total)) = make_uint2(hi[0], hi[1]);
            *(uint2 *)(g.xout + xpack_index(m, nn, 1, g.m_tiles_total)) = make_uint2(lo[0], lo[1]);
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // the tile holds gate (register groups j = 0, 2) and up (j = 1, 3) of 16 feed-forward columns
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float gt = acc[8 * jj + r] * rs, up = acc[8 * jj + 4 + r] * rs;
                v[r] = gt / (1.0f + __expf(-gt)) * up;
            }
            uint32_t hi[2], lo[2];
            split_pack2(v[0], v[1], hi[0], lo[0]);
            split_pack2(v[2], v[3], hi[1], lo[1]);
            const int f0 = T * 16 + 8 * jj + nsub;
            *(uint2 *)(g.act + xpack_index(m, f0, 0, g.m_tiles_total)) = make_uint2(hi[0], hi[1]);
            *(uint2 *)(g.act + xpack_index(m, f0, 1, g.m_tiles_total)) = make_uint2(lo[0], lo[1]);
        }
    } else if constexpr (EPI == EPI_QKV) {
        // tile T = 4 * head + t: register groups j = 0, 2 hold dims 16t + 8(j/2) + 4h + r of the head,
        // groups j = 1, 3 the same dims + 64 (the rotary partners)
        const size_t qd = (size_t)g.Hq * 128;
        const int hy = T >> 2, th = T & 3;
        uint16_t *kc = nullptr, *vc = nullptr;
        int tk = 0;
        if (hy >= g.Hq) {
            const int kvh = hy < g.Hq + g.Hkv ? hy - g.Hq : hy - g.Hq - g.Hkv;
            const size_t pb = ((size_t)(p.kvloc >> 4) * g.Hkv + kvh) * (SEV_PAGE * 128);
            kc = (uint16_t *)g.k_layer + pb;
            vc = (uint16_t *)(g.k_layer + g.v_offset) + pb;
            tk = p.kvloc & 15;
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int i0 = 16 * th + 8 * jj + nsub;
            float va[4], vb[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                va[r] = acc[8 * jj + r] * rs;
                vb[r] = acc[8 * jj + 4 + r] * rs;
            }
            if (hy < g.Hq + g.Hkv) {
                const float4 c01 = p.cs[2 * jj], c23 = p.cs[2 * jj + 1];
                const float cs[4] = {c01.x, c01.z, c23.x, c23.z}, sn[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float x = va[r], y = vb[r];
                    va[r] = x * cs[r] - y * sn[r];
                    vb[r] = y * cs[r] + x * sn[r];
                }
            }
            if (hy < g.Hq) {
                uint32_t hi[2], lo[2];
                const size_t o = (size_t)m * qd + (size_t)hy * 128 + i0;
                split_pack2(va[0], va[1], hi[0], lo[0]);
                split_pack2(va[2], va[3], hi[1], lo[1]);
                *(uint2 *)(g.q_planes + o) = make_uint2(hi[0], hi[1]);
                *(uint2 *)(g.q_planes + (size_t)g.M * qd + o) = make_uint2(lo[0], lo[1]);
                split_pack2(vb[0], vb[1], hi[0], lo[0]);
                split_pack2(vb[2], vb[3], hi[1], lo[1]);
                *(uint2 *)(g.q_planes + o + 64) = make_uint2(hi[0], hi[1]);
                *(uint2 *)(g.q_planes + (size_t)g.M * qd + o + 64) = make_uint2(lo[0], lo[1]);
            } else if (hy < g.Hq + g.Hkv) {
                *(uint2 *)(kc + k_in_page<true>(tk, i0, 128)) =
                    make_uint2(f32_to_bf16_bits(va[0]) | (f32_to_bf16_bits(va[1]) << 16),
                               f32_to_bf16_bits(va[2]) | (f32_to_bf16_bits(va[3]) << 16));
                *(uint2 *)(kc + k_in_page<true>(tk, i0 + 64, 128)) =
                    make_uint2(f32_to_bf16_bits(vb[0]) | (f32_to_bf16_bits(vb[1]) << 16),
                               f32_to_bf16_bits(vb[2]) | (f32_to_bf16_bits(vb[3]) << 16));
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    vc[v_in_page<true>(tk, i0 + r, 128)] = (uint16_t)f32_to_bf16_bits(va[r]);
                    vc[v_in_page<true>(tk, i0 + 64 + r, 128)] = (uint16_t)f32_to_bf16_bits(vb[r]);
                }
            }
        }
    }
    return ss;
}

// Adds a block's per-row sums of squares (one value per lane < 32 and wave, in red[wave][row]) to
// ssq_out and clears ssq_clear; rows = number of rows covered, m0 = first row.
template <int STRIDE>
__device__ __forceinline__ void ssq_commit(const GemmArgs &g, float (*red)[STRIDE], int rows, int m0, bool clear) {
    __syncthreads();
    if ((int)threadIdx.x < rows) {
        const int t = threadIdx.x, m = m0 + t;
        if (m < g.M) {
            atomicAdd(g.ssq_out + m, ssq_fix((red[0][t] + red[1][t]) + (red[2][t] + red[3][t])));
            if (clear) g.ssq_clear[m] = 0ull;
        }
    }
}

// Kernel arguments live in memory and are fetched with scalar loads where the compiler first needs
// them; an argument block of several cache lines can then cost one memory latency per line, one after
// the other, in the middle of the kernel.  Naming one field of every line at the kernel's entry makes
// all of those fetches start together.
#define SEV_ARGS_NOW(...) asm volatile("" : : __VA_ARGS__)

// The arguments the prologue needs first (pointers and grid decomposition) are passed as leading
// scalars as well: the library is built with kernel-argument preloading, which hands the first 16
// dwords of the argument block to the wave in registers at launch, so the first loads can be issued
// without waiting for a scalar load of the argument block.
template <int MT, int NT, int EPI, int PF>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const uint4 *W_, const uint4 *X_, int n_tiles_, int k_steps_, int m_tiles_total_,
                                                        int col_groups_, int m_blocks_, int splits_, GemmArgs g) {
    g.W = W_; g.X = X_; g.n_tiles = n_tiles_; g.k_steps = k_steps_; g.m_tiles_total = m_tiles_total_;
    g.col_groups = col_groups_; g.m_blocks = m_blocks_; g.splits = splits_ & 0xffff;
    const int tpb = splits_ >> 16;                      // column tiles per block: 4 * NT, or fewer (the last wave then has fewer tiles)
    // a pipeline stage is KS k-steps of 16: two for the narrow tiles, one for NT = 4 (same 32 MFMAs per wave with MT = 4)
    constexpr int KS = NT == 4 ? 1 : 2;
    constexpr int XI = KS * MT / 2;                     // 16-byte activation loads per thread and stage
    static_assert(KS * MT % 2 == 0, "a stage of activations must be a whole number of 4 KiB");
    extern __shared__ u32x4 xs[];                       // [2 buffers][KS k-steps][MT][2 planes][64 lanes]
    __shared__ float red[4][MT * 32 < 128 ? 128 : MT * 32];
    constexpr int STAGE_U4 = KS * MT * 2 * 64;          // uint4 per stage
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // Block index decode, XCD-aware: consecutive block ids go round-robin to the 8 XCDs, each with its
    // own L2.  Blocks that share weight tiles (the row blocks of one column group) get ids 8 apart,
    // i.e. land on the same XCD back to back, so the second read can hit that L2.
    int q = blockIdx.x >> 3;
    const int mb = q % g.m_blocks;
    q /= g.m_blocks;
    const int split = q % g.splits;
    const int cg = (q / g.splits) * 8 + (blockIdx.x & 7);
    if (cg >= g.col_groups) return;                      // whole block leaves before any barrier
    const int tile0 = cg * tpb + wave * NT;
    const int my_tiles = min(NT, min(tpb - wave * NT, g.n_tiles - tile0));        // may be <= 0: the wave then only helps with the activations
    const int mt0 = mb * MT;
    const int n_stages = g.k_steps / KS;
    const int s_begin = (int)((unsigned)n_stages * (unsigned)split / (unsigned)g.splits);          // small numbers: 32-bit division
    const int s_end = (int)((unsigned)n_stages * (unsigned)(split + 1) / (unsigned)g.splits);
    const int n = s_end - s_begin;
    const int mrow = lane & 31, nsub = 4 * (lane >> 5);

    f32x16 acc[NT][MT];
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // weight fragment pointers of this lane (clamped to a valid tile so idle waves load harmlessly)
    const u32x4 *wp[NT];
#pragma unroll
    for (int a = 0; a < NT; ++a) {
        const int t = min(tile0 + a, g.n_tiles - 1);
        wp[a] = (const u32x4 *)g.W + ((size_t)t * g.k_steps) * 64 + lane;
    }
    // The gate/up GEMM reads its weights through a buffer descriptor that covers exactly the block's column tiles: a
    // tile the wave does not have (blocks of fewer than 4 * NT tiles, the matrix edge) lies past the descriptor's
    // end, where a load returns zeros and reads nothing, so the loop stays free of branches and the missing tile
    // costs no memory traffic.
    constexpr bool WBUF = EPI == EPI_SWIGLU && MT <= 2;      // the 128-row blocks never run narrower than 4 * NT tiles
    const int block_tiles = min(tpb, g.n_tiles - cg * tpb);
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const u32x4 *)g.W + (size_t)cg * tpb * g.k_steps * 64), 0, block_tiles * g.k_steps * 1024, 0x00020000);
    int woff[NT];
#pragma unroll
    for (int a = 0; a < NT; ++a) woff[a] = (((wave * NT + a) * g.k_steps) * 64 + lane) * 16;
    auto load_w = [&](int a, int step) -> u32x4 {      // 16 bytes per lane of k-step `step` of the wave's column tile a
        // The streaming hint keeps the weights from displacing the activations in the L2s (gate/up: 7 % faster with it).
        // The QKV projection streams the fewest weights per activation byte and is 4 % faster with plain loads.
        if constexpr (WBUF) return __builtin_amdgcn_raw_buffer_load_b128(wrs, woff[a] + step * 1024, 0, 2);      // 2: streaming hint
        else if constexpr (EPI == EPI_QKV) return wp[a][(size_t)step * 64];
        else return __builtin_nontemporal_load(&wp[a][(size_t)step * 64]);
    };
    // Software pipeline.  Loads return in issue order, so a wait on one load drains every older one:
    // to keep PF stages in flight, weights AND activations are fetched PF stages ahead into registers
    // and consumed in the order they were issued.  At the start of stage st (slot u = st % PF):
    //   xf holds the activation fragments of stage st;  LDS buffer (st+1)&1 holds X(st+1);
    //   wreg[u] holds W(st);  xreg[u] holds X(st+2).
    // During the stage each fragment register is refilled from LDS with its stage st+1 contents right
    // after its last MFMA, so the LDS reads of the next stage overlap the MFMAs of this one, and
    // X(st+2) goes from registers into the LDS buffer that stage st no longer reads (free since the
    // barrier that ended stage st-1).
    // The loop body is PF stages of straight-line code (no branches), which lets the compiler's
    // wait-count bookkeeping follow the loads across the back-edge.  The slice is padded to a multiple
    // of PF stages: padded stages re-load the last stage (cached) and feed zero activations.
    // Weights are read exactly once per row block: their loads carry the streaming (non-temporal) hint.
    static_assert(PF % 2 == 0, "LDS buffer parity must follow the slot index");
    u32x4 wreg[PF][NT][KS];
    u32x4 xreg[PF][XI];
    u32x4 xf[KS][MT][2];
    const u32x4 *xsrc[XI];
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        const int u = threadIdx.x + 256 * i;
        const int ksl = u / (MT * 128), within = u - ksl * (MT * 128);
        xsrc[i] = (const u32x4 *)g.X + ((size_t)ksl * g.m_tiles_total + mt0) * 128 + within;
    }
    const size_t x_stage = (size_t)KS * g.m_tiles_total * 128;      // 16-byte units per stage of all row tiles
    const int n_pad = (n + PF - 1) / PF * PF;
    // Every column group walks its K range from a different starting stage (and wraps around): the
    // blocks that run at the same time would otherwise all read the same few KiB of activations at the
    // same moment, i.e. hammer a few L2 channels while the others idle.  The row blocks of a column
    // group share the rotation, so they still read their common weight tiles together.  Short split-K
    // slices keep the common start: they are mostly pipeline fill, where sharing the first misses wins.
    const int rot = n >= 64 ? (int)((unsigned)cg * (unsigned)n / (unsigned)g.col_groups) : 0;
    auto phys = [&](int t) {                                        // logical stage -> stage index in K
        int i = min(t, n - 1) + rot;
        if (i >= n) i -= n;
        return s_begin + i;
    };
    const u32x4 zero4 = (u32x4){0u, 0u, 0u, 0u};

    {
        u32x4 x0[XI], x1[XI];
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            x0[i] = xsrc[i][(size_t)phys(0) * x_stage];
            x1[i] = xsrc[i][(size_t)phys(1) * x_stage];
        }
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int sx = phys(u + 2), sw = phys(u);
#pragma unroll
            for (int i = 0; i < XI; ++i) xreg[u][i] = xsrc[i][(size_t)sx * x_stage];
#pragma unroll
            for (int a = 0; a < NT; ++a)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) wreg[u][a][ks] = load_w(a, KS * sw + ks);
        }
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            xs[threadIdx.x + 256 * i] = x0[i];
            xs[STAGE_U4 + threadIdx.x + 256 * i] = (1 < n) ? x1[i] : zero4;
        }
    }
    // a block that runs the epilogue itself fetches its rows' sums of squares now, so that the row scales are
    // there when the loop ends
    unsigned long long sq_rows[MT];
#pragma unroll
    for (int b = 0; b < MT; ++b) {
        const int m = (mt0 + b) * 32 + mrow;
        sq_rows[b] = (g.splits == 1 && g.ssq_in && m < g.M) ? g.ssq_in[m] : 0ull;
    }
    // the rest of the argument block (epilogue pointers): fetched now, behind the first loads
    if constexpr (EPI == EPI_QKV) SEV_ARGS_NOW("s"(g.part), "s"(g.ssq_in), "s"(g.row_cs), "s"(g.q_planes));
    else if constexpr (EPI == EPI_ARGMAX) SEV_ARGS_NOW("s"(g.part), "s"(g.ssq_in), "s"(g.lm_val), "s"(g.logits));
    else SEV_ARGS_NOW("s"(g.part), "s"(g.ssq_in), "s"(g.act));
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int pl = 0; pl < 2; ++pl) xf[ks][b][pl] = xs[((ks * MT + b) * 2 + pl) * 64 + lane];
    __syncthreads();                                    // stage 0 overwrites buffer 0 early: every wave must have read its X(0) fragments

    // One group of PF stages.  The last group of a slice issues no global loads: what it would
    // prefetch lies beyond the slice, and the epilogue would have to wait for those loads to return
    // before it may reuse their registers.
    auto group = [&](int base, auto load_tag) {
        constexpr bool LOAD = decltype(load_tag)::value;
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int st = base + u;
            if constexpr (!LOAD) {
                if (st >= n) break;                     // padding of the slice (uniform): nothing left to multiply
            }
            const u32x4 *xnext = xs + ((u + 1) & 1) * STAGE_U4 + lane;      // X(st+1)
            // X(st+2): registers -> the LDS buffer whose fragments (stage st) were read during stage st-1
            const bool live = st + 2 < n;
            u32x4 *xd = xs + (u & 1) * STAGE_U4 + threadIdx.x;
            const int sx = phys(st + PF + 2), sw = phys(st + PF);
            // Everything else a stage has to do is spread between its MFMAs, so that the matrix pipe
            // never waits for a run of address arithmetic, loads and LDS traffic at the stage's end:
            // a weight fragment is refilled right after its last MFMA (column tiles are the outer loop),
            // the LDS write of X(st+2) and the loads that refill its registers follow the first group,
            // and every activation fragment is re-read from LDS (stage st+1) after its last use, which
            // falls into the last column tile's group.
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int a = 0; a < NT; ++a) {
                    const bf16x8 w = as_bf16x8(wreg[u][a][ks]);
#pragma unroll
                    for (int pl = 0; pl < 2; ++pl)
#pragma unroll
                        for (int b = 0; b < MT; ++b) {
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, as_bf16x8(xf[ks][b][pl]), acc[a][b], 0, 0, 0);
                            if (a == NT - 1) xf[ks][b][pl] = xnext[((ks * MT + b) * 2 + pl) * 64];
                        }
                    if constexpr (LOAD) wreg[u][a][ks] = load_w(a, KS * sw + ks);
                    if (ks == 0 && a == 0) {
#pragma unroll
                        for (int i = 0; i < XI; ++i) xd[256 * i] = live ? xreg[u][i] : zero4;
                        if constexpr (LOAD) {
#pragma unroll
                            for (int i = 0; i < XI; ++i) xreg[u][i] = xsrc[i][(size_t)sx * x_stage];
                        }
                    }
                }
            }
            // the same order for the instruction scheduler (0x008 MFMA, 0x100 DS read, 0x200 DS write, 0x020 VMEM read)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int a = 0; a < NT; ++a) {
                    if (a < NT - 1) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2 * MT, 0);
                    } else {
#pragma unroll
                        for (int i = 0; i < 2 * MT; ++i) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        }
                    }
                    if constexpr (LOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    if (ks == 0 && a == 0) {
                        __builtin_amdgcn_sched_group_barrier(0x200, XI, 0);
                        if constexpr (LOAD) __builtin_amdgcn_sched_group_barrier(0x020, XI, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
        }
    };
    for (int base = 0; base + PF < n_pad; base += PF) group(base, std::true_type{});
    group(n_pad - PF, std::false_type{});

    // ------------------------------------------------------------------ split-K: hand the slice to the fix-up kernel
    if (g.splits > 1) {
        // exchange layout [slice][column tile][row tile][4][64 lanes] float4: register order, 1 KiB per store instruction
#pragma unroll
        for (int a = 0; a < NT; ++a)
            if (a < my_tiles) {
#pragma unroll
                for (int b = 0; b < MT; ++b) {
                    float4 *mine = (float4 *)g.part + (((size_t)split * g.n_tiles + tile0 + a) * g.m_tiles_total + mt0 + b) * 256 + lane;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        mine[j * 64] = make_float4(acc[a][b][4 * j], acc[a][b][4 * j + 1], acc[a][b][4 * j + 2], acc[a][b][4 * j + 3]);
                }
            }
        return;
    }

    // ------------------------------------------------------------------ epilogues
    if constexpr (EPI != EPI_ARGMAX) {
        float ss[MT];
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            ss[b] = 0.f;
            const int m = (mt0 + b) * 32 + mrow;
            const float rs_b = g.ssq_in ? rms_scale(sq_rows[b], g.inv_d, g.eps) : 1.0f;
#pragma unroll
            for (int a = 0; a < NT; ++a)
                if (a < my_tiles) {
                    const TilePre pre = tile_pre<EPI, true>(g, tile0 + a, m, nsub, rs_b);
                    ss[b] += tile_epilogue<EPI>(g, acc[a][b], tile0 + a, m, nsub, pre);
                }
        }
        if constexpr (EPI == EPI_RESID) {
#pragma unroll
            for (int b = 0; b < MT; ++b) {
                ss[b] += __shfl_xor(ss[b], 32);
                if (lane < 32) red[wave][b * 32 + mrow] = ss[b];
            }
            ssq_commit(g, red, MT * 32, mt0 * 32, cg == 0);
        }
    } else {
        // arg-max over this wave's columns for every row (lowest index wins ties); the row scale is
        // positive, so it only matters for the logits that are written out
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            const int m = (mt0 + b) * 32 + mrow;
            const float rsb = (g.logits && g.ssq_in && m < g.M) ? rms_scale(sq_rows[b], g.inv_d, g.eps) : 1.0f;
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int a = 0; a < NT; ++a) {
                if (a >= my_tiles) continue;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int nn = (tile0 + a) * 32 + 8 * j + nsub;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float v = acc[a][b][4 * j + r];
                        if (v > bv) { bv = v; bi = nn + r; }       // indices ascend, so ">" keeps the lowest
                    }
                    if (g.logits && m < g.M)
                        *(float4 *)(g.logits + (size_t)m * g.N + nn) =
                            make_float4(acc[a][b][4 * j] * rsb, acc[a][b][4 * j + 1] * rsb, acc[a][b][4 * j + 2] * rsb,
                                        acc[a][b][4 * j + 3] * rsb);
                }
            }
            const float ov = __shfl_xor(bv, 32);
            const int oi = __shfl_xor(bi, 32);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            if (lane < 32 && m < g.M) {
                const size_t slot = (size_t)(cg * 4 + wave) * g.lm_stride + m;
                g.lm_val[slot] = bv;
                g.lm_idx[slot] = bi;
            }
        }
    }
}

// Split-K fix-up: block (group of 4 column tiles, row tile mt) of 4 waves; wave w sums the S slices of the
// 32x32 tile (column tile 4 * group + w, row tile mt) in slice order and runs its epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_fixup_kernel(const float *part_, const void *pa_, const void *pb_, const unsigned long long *ssq_in_,
                                                         int m_tiles_real_, int m_tiles_total_, int splits_, int n_tiles_, int M_, int N_, int heads_,
                                                         GemmArgs g) {
    __shared__ float red[4][128];
    // leading scalars (preloaded at wave launch): everything the first loads need; pa_ / pb_ are the residual stream and
    // the gains (EPI_RESID) or the rotary table and the rows' cache locations (EPI_QKV); heads_ = query heads | KV heads << 16
    g.part = const_cast<float *>(part_); g.ssq_in = ssq_in_; g.m_tiles_total = m_tiles_total_;
    g.splits = splits_; g.n_tiles = n_tiles_; g.M = M_; g.N = N_;
    g.Hq = heads_ & 0xffff; g.Hkv = heads_ >> 16;
    if constexpr (EPI == EPI_RESID) { g.h = (float *)const_cast<void *>(pa_); g.gain = (const float *)pb_; }
    if constexpr (EPI == EPI_QKV) { g.row_cs = (const float2 *)pa_; g.row_kvloc = (const int32_t *)pb_; }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int mt = blockIdx.x % m_tiles_real_, grp = blockIdx.x / m_tiles_real_;
    const int T = grp * 4 + wave;
    const int mrow = lane & 31, nsub = 4 * (lane >> 5);
    const int m = mt * 32 + mrow;
    const size_t slice_stride = (size_t)g.n_tiles * g.m_tiles_total * 256;
    const float4 *src = (const float4 *)g.part + ((size_t)min(T, g.n_tiles - 1) * g.m_tiles_total + mt) * 256 + lane;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const bool live = T < g.n_tiles;
    float ss = 0.f;
    if (live) {
        const TilePre pre = tile_pre<EPI>(g, T, m, nsub);       // issued ahead of the slice loads
        for (int s0 = 0; s0 < g.splits; s0 += 8) {
            float4 v[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    v[u][j] = src[(size_t)min(s0 + u, g.splits - 1) * slice_stride + j * 64];
            if (s0 == 0) {                                      // the rest of the argument block, behind the first loads
                if constexpr (EPI == EPI_QKV) SEV_ARGS_NOW("s"(g.q_planes), "s"(g.k_layer), "s"(g.inv_d));
                else SEV_ARGS_NOW("s"(g.xout), "s"(g.ssq_out), "s"(g.act), "s"(g.inv_d));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < g.splits) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc[4 * j] += v[u][j].x; acc[4 * j + 1] += v[u][j].y;
                        acc[4 * j + 2] += v[u][j].z; acc[4 * j + 3] += v[u][j].w;
                    }
                }
        }
        ss = tile_epilogue<EPI>(g, acc, T, m, nsub, pre);
    }
    if constexpr (EPI == EPI_RESID) {
        ss += __shfl_xor(ss, 32);
        if (lane < 32) red[wave][mrow] = ss;
        ssq_commit(g, red, 32, mt * 32, grp == 0);
    }
}

// ---------------------------------------------------------------------------
// final arg-max over the per-wave partial results of the LM-head GEMM; one block per row
__global__ __launch_bounds__(256) void lm_reduce_kernel(const float *val, const int32_t *idx, int n_part, int stride,
                                                        int32_t *out) {
    __shared__ float sv[256];
    __shared__ int si[256];
    const int m = blockIdx.x;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int p = threadIdx.x; p < n_part; p += 256) {
        const float v = val[(size_t)p * stride + m];
        const int i = idx[(size_t)p * stride + m];
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
    sv[threadIdx.x] = bv;
    si[threadIdx.x] = bi;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) {
            const float v = sv[threadIdx.x + s];
            const int i = si[threadIdx.x + s];
            if (v > sv[threadIdx.x] || (v == sv[threadIdx.x] && i < si[threadIdx.x])) { sv[threadIdx.x] = v; si[threadIdx.x] = i; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) out[m] = si[0];
}

// ---------------------------------------------------------------------------
// verification attention over the paged bf16 cache (head_dim 128, 16-token pages).
//
// Work item = (request, group of 32 query rows, KV chunk) x KV head.  The 32 rows are
// (query head in the GQA group) x (draft node), so every K/V byte is read once for the whole
// group.  The waves of a block (4, or 8 when a block takes a whole sequence) take alternate page pairs
// (32 keys) of the chunk; per pair a wave runs
//   S^T = K Q^T   : 8 k-steps of MFMA 32x32x16, A = keys (32 keys x 16 dims; the in-page K layout
//                   makes every 16-lane group read 256 contiguous bytes), B = q (hi and lo planes,
//                   kept in registers for the whole chunk)
//   O^T += V^T P^T: MFMA 32x32x16 per 32-dim tile and page; a lane of the S^T result holds 16 keys of
//                   ONE query, and the in-page V layout is chosen so that exactly those keys are the
//                   contraction slots of the lane's B operand: probabilities never leave registers
// with an online softmax per query row (one cross-lane exchange per pair: the other 16 keys of the
// row sit in lane ^ 32); then the waves' partial (max, sum, O) are merged through LDS.  A block that
// saw only a chunk writes its partial result for the cross-chunk merge; a block that saw the whole
// sequence (DIRECT) normalises and writes the O projection's operand itself.  Masking: keys < P are visible to every row; key P + j is visible
// to a row iff bit j of the row's ancestor mask is set.
// ---------------------------------------------------------------------------
// ONCE: every K/V byte is read by exactly one block (each request has a single row group); its loads then carry the
// streaming hint.
template <int WAVES, bool DIRECT, bool ONCE>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 2 : 1) void attn_bf16_kernel(const int4 *it_a_, const int4 *it_b_, const int32_t *it_pages_,
                                                                                    const uint16_t *q_planes, char *pool_, size_t layer_off_, size_t v_off_,
                                                                                    int M, int heads_,
                                                                                    DevPlan p, KvGeom g, int n_items_sib,
                                                                                    float *att_o, float2 *att_ml, float scale_log2e,
                                                                                    uint16_t *o_pack, int m_tiles) {
    // (leading scalars: preloaded at wave launch; layer_off_ = layer * layer stride of the pool, v_off_ = offset of the
    // V pages, heads_ = query heads | KV heads << 16)
    p.it_a = const_cast<int4 *>(it_a_); p.it_b = const_cast<int4 *>(it_b_); p.it_pages = const_cast<int32_t *>(it_pages_);
    const int Hq = heads_ & 0xffff;
    g.Hkv = heads_ >> 16;
    g.v_offset = v_off_;
    extern __shared__ float lds[];                    // WAVES merge slots: 64 accumulator registers + max + sum per lane
    // Block index -> (work item, KV head).  Consecutive block ids go round-robin to the 8 XCDs, each with its own L2;
    // the blocks of one XCD (ids 8 apart) walk, in this order: the KV heads, the `sib` row groups of one (request, chunk)
    // - items that read the same K/V, side by side in the work list - and then the next set of row groups.  The blocks
    // that share a chunk so run on one XCD at about the same time and the chunk comes from memory once (trees of 64
    // nodes, 8 row groups: 45 ns per page against 78 ns when the groups are spread over the XCDs).  sib = 1 when the
    // requests differ in their number of row groups.  The grid is padded to whole groups of 8 sets; the padding leaves
    // before the barrier.
    const int n_items = n_items_sib & 0xffffff, sib = n_items_sib >> 24;
    const int jb = (int)(blockIdx.x >> 3), kvh = jb % g.Hkv, tb = jb / g.Hkv;
    const int item = ((tb / sib) * 8 + (int)(blockIdx.x & 7)) * sib + tb % sib;
    if (item >= n_items) return;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index as a scalar: loop bounds stay uniform
    // everything the block needs to know comes from two 16-byte loads and one page-id load, all independent
    const int4 ia = p.it_a[item], ib = p.it_b[item];
    const int rg = ia.x, page0 = ia.y, npages = ia.z, P = ia.w, n = ib.x, row0 = ib.y;
    const int npairs = (npages + 1) >> 1;
    const int my_pairs = npairs > wave ? (npairs - wave + WAVES - 1) / WAVES : 0;   // this wave takes pairs wave, wave+WAVES, ...
    int pt_val;                                         // lane j < 32: page (j&1) of this wave's pair j/2
    {
        const int pidx = 2 * (wave + WAVES * ((lane & 31) >> 1)) + (lane & 1);
        pt_val = p.it_pages[(size_t)item * SEV_ATT_MAX_CP + pidx];    // the list is padded with the last page
    }
    const int G = Hq / g.Hkv;
    const int qrow = lane & 31, half = lane >> 5;
    const size_t page_stride = (size_t)g.Hkv * 4096;
    const size_t qd = (size_t)Hq * 128;
    // K fragment of k-step ks: lane (key = lane % 32 -> page (key / 16), token key % 16; dims 16 ks + 8 half .. +7)
    //   byte offset in the page block: ((2 ks + half) * 16 + token) * 16
    // V fragment of (dim tile dt, page): lane (dim = lane % 32, half) -> 16 bytes at ((dt * 64 + lane) * 16)
    const char *Kl = pool_ + layer_off_ + (size_t)kvh * 4096 + (half * 16 + (lane & 15)) * 16;
    const char *Vl = pool_ + layer_off_ + g.v_offset + (size_t)kvh * 4096 + lane * 16;
    const int kpage_sel = (lane >> 4) & 1;             // which page of the pair this lane's key belongs to

    // K and V fragments of one page pair live in registers; the keys of the next pair are requested as
    // soon as the score MFMAs have consumed the current ones, the values right after the PV MFMAs.  Two
    // blocks share a compute unit, so the other block's waves fill the time a wave waits for its loads.
    // Where the cache is read once, its loads carry the streaming hint, which keeps q, the page lists and the partial
    // results in the L2s (8-12 % faster on workloads of 0.3-0.5 GB of K/V per layer).  Requests with several row groups
    // (trees, wide GQA groups) re-read their K/V through the L2s, which the hint would defeat (measured: 60 % slower
    // with 8 groups, 20 % with 2).
    auto ld = [](const char *p_) -> u32x4 {
        if constexpr (ONCE) return __builtin_nontemporal_load((const u32x4 *)p_);
        else return *(const u32x4 *)p_;
    };
    u32x4 kf[8], vf[2][4];
    auto load_k = [&](int i) {
        const int pg = __shfl(pt_val, 2 * i + kpage_sel);
        const char *a = Kl + (size_t)pg * page_stride;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kf[ks] = ld(a + ks * 512);
    };
    auto load_v = [&](int i) {
        const char *a0 = Vl + (size_t)__shfl(pt_val, 2 * i) * page_stride, *a1 = Vl + (size_t)__shfl(pt_val, 2 * i + 1) * page_stride;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            vf[0][dt] = ld(a0 + dt * 1024);
            vf[1][dt] = ld(a1 + dt * 1024);
        }
    };
    load_k(0);                                             // padded page list: always a valid page, even for an idle wave
    load_v(0);
    SEV_ARGS_NOW("s"(p.row_anc), "s"(p.causal), "s"(att_o), "s"(att_ml), "s"(o_pack));   // the rest of the argument block, behind the first loads

    // query fragments of this lane's row (hi and lo planes, 8 k-steps): 64 registers for the whole chunk
    const int R = rg * 32 + qrow;
    const bool row_live = R < G * n;
    u32x4 qf[2][8];
    unsigned long long anc = 0ull;
    const int hg = row_live ? R / n : 0, node = row_live ? R - hg * n : 0;
    {
        const uint16_t *qp = q_planes + (size_t)(row0 + node) * qd + (size_t)(kvh * G + hg) * 128 + 8 * half;
#pragma unroll
        for (int pl = 0; pl < 2; ++pl)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                qf[pl][ks] = *(const u32x4 *)(qp + (size_t)pl * M * qd + 16 * ks);     // dead rows read row (row0, head 0): harmless, never stored
        anc = p.row_anc[row0 + node];
        if (!row_live) anc = 0ull;
    }
    // Everything loaded so far (the first K and V fragments, q, the ancestor mask) is awaited HERE, once: the loop's
    // first MFMA needs most of it anyway.  Left to the loop, the compiler's wait-count bookkeeping has to assume at
    // every iteration that the q loads of the prologue may still be pending behind the K and V loads, and makes each
    // iteration's score MFMAs wait for the V fragments requested just before, i.e. for a whole memory latency.
#pragma unroll
    for (int pl = 0; pl < 2; ++pl)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) asm volatile("" : : "v"(qf[pl][ks]));
    asm volatile("" : : "v"(anc));

    f32x16 oacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[t][r] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;

    // MASKED = false: a pair whose 32 keys all lie in the committed prefix (every row sees every key); most pairs are.
    auto pair_step = [&](int i, auto prefetch_tag, auto masked_tag) {
        constexpr bool PREFETCH = decltype(prefetch_tag)::value;
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int lp0 = 2 * (wave + WAVES * i);             // chunk-local pages of the pair
        const bool has1 = (lp0 + 1) < npages;
        // scores of this lane's query against keys 8j + 4*half + r of the pair (j = 0..3 -> register 4j + r)
        f32x16 sh;
#pragma unroll
        for (int r = 0; r < 16; ++r) sh[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            sh = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), as_bf16x8(qf[0][ks]), sh, 0, 0, 0);
            sh = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), as_bf16x8(qf[1][ks]), sh, 0, 0, 0);
        }
        if (PREFETCH) load_k(i + 1);
        const int jbase = (page0 + lp0) * 16 + 4 * half - P;    // draft-node index of key register 0 (negative: prefix)
        // (no memory access sits under control flow inside a pair step: the compiler's wait counts then stay exact)
        float sc[16];
        float mx = -INFINITY;
        // sc holds the raw scores (masked ones: -inf); the softmax scale goes into the one multiply-add in front of
        // each exponential
        if constexpr (!MASKED) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sc[r] = sh[r];
                mx = fmaxf(mx, sc[r]);
            }
        }
#pragma unroll
        for (int j4 = 0; MASKED && j4 < 4; ++j4) {
            // 4-bit visibility of keys j..j+3: prefix keys (index < 0) always, draft key i iff ancestor bit i
            // (the mask has no bits at or above n); plain shifts and selects
            const int j = jbase + 8 * j4;
            const unsigned up = j < 64 ? (unsigned)(anc >> max(j, 0)) : 0u;             // j >= 0 (the tail of the last page can reach past 63)
            const unsigned dn = (unsigned)((anc << (-max(j, -3))) | ((1ull << (-max(j, -3))) - 1ull));   // -3 <= j < 0
            unsigned vis4 = j >= 0 ? up : (j <= -4 ? 0xFu : dn);
            // chains (any length): key j is visible iff j <= the row's own node index
            const int dcs = node - j;
            const unsigned visc = dcs >= 3 ? 0xFu : (dcs < 0 ? 0u : (2u << dcs) - 1u);
            vis4 = p.causal ? (row_live ? visc : 0xFu) : vis4;
            if (j4 >= 2) vis4 = has1 ? vis4 : 0u;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float v = ((vis4 >> r) & 1u) ? sh[4 * j4 + r] : -INFINITY;
                sc[4 * j4 + r] = v;
                mx = fmaxf(mx, v);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2e;      // (the scale is positive)
        const float mnew = fmaxf(mrun, mx);
        const float muse = (mnew == -INFINITY) ? 0.f : mnew;
        const float alpha = __builtin_amdgcn_exp2f(mrun - muse);
        mrun = mnew;
        float ps = 0.f;
        uint32_t ph[8], pl_[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale_log2e, -muse));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r + 1], scale_log2e, -muse));
            ps += p0 + p1;
            split_pack2(p0, p1, ph[r / 2], pl_[r / 2]);
        }
        lrun = lrun * alpha + ps;
        // the running maximum rarely moves after the first pairs: the 64 accumulator registers are rescaled only when
        // some row's maximum did (alpha is exactly 1 otherwise, so skipping changes nothing)
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[t][r] *= alpha;
        }
        // page kk of the pair is contraction step kk: its 8 slots of this lane are score registers 8kk .. 8kk+7
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const bf16x8 pH = as_bf16x8((u32x4){ph[4 * kk], ph[4 * kk + 1], ph[4 * kk + 2], ph[4 * kk + 3]});
            const bf16x8 pL = as_bf16x8((u32x4){pl_[4 * kk], pl_[4 * kk + 1], pl_[4 * kk + 2], pl_[4 * kk + 3]});
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vf[kk][dt]), pH, oacc[dt], 0, 0, 0);
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vf[kk][dt]), pL, oacc[dt], 0, 0, 0);
            }
        }
        if (PREFETCH) load_v(i + 1);
    };
    // pairs in key order: first those that lie wholly inside the prefix, then the few that hold draft nodes, the end of
    // the last page or padding
    // pair i covers keys [(page0 + lp0) * 16, (page0 + lp0 + 2) * 16), lp0 = 2 (wave + WAVES i): inside the prefix iff
    // 2 (wave + WAVES i) <= P / 16 - page0 - 2
    const int room = P / 16 - page0 - 2;
    const int n_plain = (room >= 0 && (room >> 1) >= wave) ? min(my_pairs - 1, ((room >> 1) - wave + WAVES) / WAVES) : 0;     // (the last pair always takes the general path)
    int i = 0;
    for (; i < n_plain; ++i) pair_step(i, std::true_type{}, std::false_type{});
    for (; i + 1 < my_pairs; ++i) pair_step(i, std::true_type{}, std::true_type{});
    if (my_pairs > 0) pair_step(my_pairs - 1, std::false_type{}, std::true_type{});

    // ---- merge the waves through LDS in one step: every wave publishes its (max, sum, O) in the
    // accumulators' own register layout; then wave w reduces register quads [w * QW, (w + 1) * QW) of all
    // waves (a quad = 4 consecutive dims of the lane's query) and stores them, so that the reduction and
    // the stores are spread over the whole block.
    f32x4 *slotO = (f32x4 *)lds;                        // [WAVES][16 register quads][64 lanes]
    float *slotM = lds + WAVES * 16 * 64 * 4;           // [WAVES][64 lanes] (max), then the same for sums
    float *slotL = slotM + WAVES * 64;
    slotM[wave * 64 + lane] = mrun;
    slotL[wave * 64 + lane] = lrun;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            slotO[(wave * 16 + t * 4 + j) * 64 + lane] = (f32x4){oacc[t][4 * j], oacc[t][4 * j + 1], oacc[t][4 * j + 2], oacc[t][4 * j + 3]};
    __syncthreads();
    float mall = -INFINITY;
#pragma unroll
    for (int v = 0; v < WAVES; ++v) mall = fmaxf(mall, slotM[v * 64 + lane]);
    const float mfin = (mall == -INFINITY) ? 0.f : mall;
    float wsc[WAVES];
    float l = 0.f;
#pragma unroll
    for (int v = 0; v < WAVES; ++v) {
        wsc[v] = __builtin_amdgcn_exp2f(slotM[v * 64 + lane] - mfin);
        l += slotL[v * 64 + lane] * wsc[v];
    }
    l += __shfl_xor(l, 32);                             // the other half of the row's keys
    constexpr int QW = 16 / WAVES;
    const float inv = DIRECT ? 1.0f / l : 1.0f;
    const size_t base = ((size_t)item * g.Hkv + kvh) * 32;
    if (!DIRECT && wave == 0 && half == 0) att_ml[base + qrow] = make_float2(mall, l);
#pragma unroll
    for (int qi = 0; qi < QW; ++qi) {
        const int q = wave * QW + qi;                   // register quad: dims 32 (q / 4) + 8 (q % 4) + 4 half .. +3 of this lane's query
        f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < WAVES; ++v) {
            const f32x4 x = slotO[(v * 16 + q) * 64 + lane];
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] += x[r] * wsc[v];
        }
        const int dim = 32 * (q >> 2) + 8 * (q & 3) + 4 * half;
        if constexpr (DIRECT) {
            // the block saw the whole sequence: normalise and write hi/lo fragments for the O projection
            if (row_live) {
                uint32_t hi[2], lo[2];
                split_pack2(o[0] * inv, o[1] * inv, hi[0], lo[0]);
                split_pack2(o[2] * inv, o[3] * inv, hi[1], lo[1]);
                const int m = row0 + node, kk = (kvh * G + hg) * 128 + dim;
                *(uint2 *)(o_pack + xpack_index(m, kk, 0, m_tiles)) = make_uint2(hi[0], hi[1]);
                *(uint2 *)(o_pack + xpack_index(m, kk, 1, m_tiles)) = make_uint2(lo[0], lo[1]);
            }
        } else {
            *(float4 *)(att_o + (base + qrow) * 128 + dim) = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
}

// cross-chunk merge + normalisation; writes the attention output as hi/lo fragments for the O projection.
// grid (merge groups, Hkv), 256 threads: thread owns (row q = t/8, 16 dims).
__global__ __launch_bounds__(256) void attn_merge_kernel(const int4 *mg_rec, const float *att_o, const float2 *att_ml, uint16_t *o_pack,
                                                         int Hq, int Hkv, int m_tiles) {
    // (all arguments are scalars: preloaded at wave launch; one 16-byte record describes the group)
    const int grpi = blockIdx.x, kvh = blockIdx.y;
    const int4 rec = mg_rec[grpi];
    const int rg = rec.x & 0xffff, cnt = rec.x >> 16, item0 = rec.y, n = rec.z & 0xffff, stride = rec.z >> 16, row0 = rec.w, G = Hq / Hkv;
    const int q = threadIdx.x >> 3, d0 = (threadIdx.x & 7) * 16;
    const int R = rg * 32 + q;
    if (R >= G * n) return;
    const int hg = R / n, node = R - hg * n;
    // chunks are combined four at a time with a running maximum: all loads of a batch are issued together
    // (a group rarely has more than four chunks, so the kernel is one round of loads deep)
    float mg = -INFINITY, l = 0.f, acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    for (int c0 = 0; c0 < cnt; c0 += 4) {
        float2 ml[4];
        float4 o[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t base = ((size_t)(item0 + min(c0 + u, cnt - 1) * stride) * Hkv + kvh) * 32 + q;
            ml[u] = att_ml[base];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[u][e] = *(const float4 *)(att_o + base * 128 + d0 + 4 * e);
        }
        float mb = mg;
#pragma unroll
        for (int u = 0; u < 4; ++u) mb = (c0 + u < cnt) ? fmaxf(mb, ml[u].x) : mb;
        const float muse = (mb == -INFINITY) ? 0.f : mb;
        const float keep = exp2f(mg - muse);
        l *= keep;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] *= keep;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float sc = (c0 + u < cnt) ? exp2f(ml[u].x - muse) : 0.f;
            l += sc * ml[u].y;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[4 * e] += sc * o[u][e].x; acc[4 * e + 1] += sc * o[u][e].y;
                acc[4 * e + 2] += sc * o[u][e].z; acc[4 * e + 3] += sc * o[u][e].w;
            }
        }
        mg = mb;
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] *= inv;
    const int m = row0 + node, k0 = (kvh * G + hg) * 128 + d0;
    store_split8(o_pack, m, k0, m_tiles, acc);
    store_split8(o_pack, m, k0 + 8, m_tiles, acc + 8);
}

// ---------------------------------------------------------------------------
// host orchestration of one forward pass
// ---------------------------------------------------------------------------
struct GemmCfg {
    int MT, NT, S, PF;
    int T;                  // column tiles per block (4 * NT unless a narrower block fills the chip better)
};

enum { G_QKV = 0, G_O, G_GU, G_DOWN, G_LM };

// Tile configuration of one GEMM.  Row tiles per block MT (weights are re-read through L2 by each row
// block), column tiles per wave NT, split-K slices S, prefetch depth PF.  The handle's tuning overrides
// (struct Tune: read from the environment when the handle was created) replace the choice in experiments.
static GemmCfg choose_cfg(int which, int m_tiles, int n_tiles, int k_steps, size_t part_elems, const Tune &tune) {
    GemmCfg c;
    c.MT = (which == G_LM && m_tiles >= 3) ? 4 : (m_tiles >= 2 ? 2 : 1);
    c.NT = (n_tiles % 2 == 0) ? 2 : 1;
    if (which == G_LM && c.MT == 4) c.NT = 4;            // never split: the widest tile halves the activation re-reads
    if (which == G_GU && m_tiles == 4 && ((n_tiles + 15) / 16) >= 200) {
        c.MT = 4;                                        // enough rows to fill the chip with 128 x 512 blocks, no split needed
        c.NT = 4;
    }
    c.PF = 4;
    c.S = 1;
    const bool splittable = which != G_LM;
    auto blocks_of = [&](const GemmCfg &x) {
        return ((n_tiles + 4 * x.NT - 1) / (4 * x.NT)) * ((m_tiles + x.MT - 1) / x.MT);
    };
    auto pick_s = [&]() {
        c.S = 1;
        if (!splittable) return;
        const int blocks = blocks_of(c);
        c.S = std::min(16, std::max(1, 256 / blocks));
        c.S = std::min(c.S, std::max(1, (k_steps / 2) / 8));          // at least 8 stages per slice
    };
    pick_s();
    // From 5 row tiles on (more than 128 rows) the matrix pipe starts to bind and the shape of the row blocks decides
    // how many rounds of blocks the chip needs: rows in as few blocks as 5 row tiles per block allow (5 -> 5, 6 -> 3 + 3,
    // 7 -> 4 + 4, 9 -> 5 + 5, ... 16 -> 4 x 4), because every row block re-reads the weights through the L2s and issues
    // its own barriers.  Measured on the 8B and 70B shapes at 160 ... 512 rows (per GEMM, fix-up included): gate/up
    // -17 ... -25 % at 160, 192, 288 and 320 rows, down -5 ... -32 %, QKV -17 ... -25 % where it applies.
    const int m_total = (m_tiles + 3) / 4 * 4;           // row tiles of the operand buffers (blocks must stay inside)
    int few = (m_tiles + 4) / 5, mt_few = (m_tiles + few - 1) / few;
    if (few * mt_few > m_total) { few = (m_tiles + 3) / 4; mt_few = 4; }      // (4 always fits the padding)
    if (which != G_LM && m_tiles >= 5 && n_tiles % 2 == 0) {
        const GemmCfg narrow = c;
        c.MT = mt_few;
        c.NT = 2;
        pick_s();
        if (which == G_GU) {
            // never split: compare with the 128 x 512 blocks by rounds of blocks x tiles per block (the wide block's
            // tiles are 14 % cheaper: one weight fragment feeds four row tiles and the stage has one barrier)
            GemmCfg wide = c;
            wide.MT = 4; wide.NT = 4;
            const double cost_few = (double)((blocks_of(c) + 255) / 256) * c.MT * c.NT;
            const double cost_wide = (double)((blocks_of(wide) + 255) / 256) * 16 * 0.86;
            if (cost_wide < cost_few) c = wide;
        } else {
            // split GEMMs: the slices must stay long (64 k-steps).  O and down (light epilogues) may also take the
            // 128 x 512 block with more slices; the two are compared by rounds x tiles x (k-steps + pipeline fill) plus
            // the fix-up's launch and exchange traffic, in units of one tile x k-step (0.055 us)
            auto cost = [&](const GemmCfg &x) {
                const double e = x.NT == 4 ? 0.86 : 1.0;
                double u = (double)((blocks_of(x) * x.S + 255) / 256) * x.MT * x.NT * e * ((double)k_steps / x.S + 24.0);
                if (x.S > 1) u += (5.0 + (double)x.S * m_tiles * n_tiles * 8192.0 / 6.5e6) / 0.0547;
                return u;
            };
            const GemmCfg few_cfg = c;
            const bool few_ok = c.S == 1 || k_steps / c.S >= 64;
            bool wide_ok = false;
            GemmCfg wide = c;
            if (which == G_O || which == G_DOWN) {
                c.MT = 4; c.NT = 4;
                pick_s();
                wide = c;
                wide_ok = (wide.S == 1 || k_steps / wide.S >= 64) && (size_t)wide.S * n_tiles * m_total * 1024 <= part_elems;
            }
            if (few_ok && wide_ok) c = cost(wide) < cost(few_cfg) ? wide : few_cfg;
            else if (few_ok) c = few_cfg;
            else if (wide_ok) c = wide;
            else c = narrow;
            // a GEMM that runs unsplit in one round of 64-row blocks keeps them, rather than gain a fix-up kernel, when
            // they occupy more units than the split blocks would (as many, if K is short: the fix-up then costs more
            // than the larger tiles save)
            const int wide_blocks = blocks_of(c) * c.S, narrow_blocks = blocks_of(narrow);
            if (narrow.S == 1 && c.S > 1 && narrow_blocks <= 256 &&
                (narrow_blocks > wide_blocks || (narrow_blocks == wide_blocks && k_steps < 512))) c = narrow;
        }
    }
    // short slices are mostly pipeline fill: halve the block width instead of splitting that deep
    if (splittable && c.NT == 2 && c.S > 1 && (k_steps / 2) / c.S < 24) {
        c.NT = 1;
        pick_s();
    }
    if (tune.has_gemm[which]) {                          // "MT,NT,S,PF"; S = 0 keeps the automatic split
        const int mt = tune.gemm[which][0], nt = tune.gemm[which][1], sp = tune.gemm[which][2], pf = tune.gemm[which][3];
        if (mt >= 1 && mt <= 5 && (nt == 1 || nt == 2 || (nt == 4 && mt == 4 && pf == 4)) &&
            sp >= 0 && sp <= 32 && (pf == 4 || (pf == 6 && mt <= 2)) &&
            (m_tiles + mt - 1) / mt * mt <= (m_tiles + 3) / 4 * 4) {     // the row blocks must stay inside the padded row tiles
            c.MT = mt;
            c.NT = (nt == 4 && c.MT != 4) ? 2 : nt;
            c.PF = pf;
            pick_s();
            if (splittable && sp > 0) c.S = sp;
        }
    }
    c.S = std::min(c.S, std::max(1, k_steps / 2));
    // The unsplit gate/up GEMM, when it leaves compute units idle: blocks one or two column tiles narrower (the last
    // wave of a block then has fewer tiles than the others) if that brings the block count closer to the number of
    // compute units.  With few rows the kernel is bound by the requests a compute unit can keep in flight, so every
    // unit counts: the 8B shape has 896 column tiles, 112 x 2 = 224 blocks of 8 or 128 x 2 = 256 blocks of 7.
    c.T = 4 * c.NT;
    if (c.S == 1 && which == G_GU && c.MT <= 2) {
        const int m_blocks = (m_tiles + c.MT - 1) / c.MT;
        auto blocks_t = [&](int t) { return ((n_tiles + t - 1) / t) * m_blocks; };
        for (int t = 4 * c.NT - 1; t >= 3 * c.NT + 1; --t)
            if (blocks_t(4 * c.NT) < 256 && blocks_t(t) <= 256 && blocks_t(t) > blocks_t(c.T)) c.T = t;
    }
    if (tune.tpb) {                                      // tuning experiments: tiles per block of the gate/up GEMM
        const int t = tune.tpb;
        if (which == G_GU && c.S == 1 && t >= 3 * c.NT + 1 && t <= 4 * c.NT) c.T = t;
    }
    // the exchange buffer holds S slices of (padded columns) x (padded rows)
    const size_t slice = (size_t)n_tiles * ((m_tiles + 3) / 4 * 4) * 1024;
    while (c.S > 1 && (size_t)c.S * slice > part_elems) --c.S;
    return c;
}

// one wave per 32x32 output tile; ga.splits slices in the exchange buffer
template <int EPI>
static void launch_fixup(const GemmArgs &ga, int m_tiles, hipStream_t st) {
    hipLaunchKernelGGL((gemm_fixup_kernel<EPI>), dim3((unsigned)((ga.n_tiles + 3) / 4 * m_tiles)), dim3(256), 0, st, (const float *)ga.part,
                       EPI == EPI_QKV ? (const void *)ga.row_cs : (const void *)ga.h, EPI == EPI_QKV ? (const void *)ga.row_kvloc : (const void *)ga.gain,
                       ga.ssq_in, m_tiles, ga.m_tiles_total, ga.splits, ga.n_tiles, ga.M, ga.N, ga.Hq | (ga.Hkv << 16), ga);
}

template <int EPI>
static void launch_gemm(GemmArgs ga, const GemmCfg &c, int m_tiles, hipStream_t st) {
    ga.col_groups = (ga.n_tiles + c.T - 1) / c.T;
    ga.m_blocks = (m_tiles + c.MT - 1) / c.MT;
    ga.splits = c.S;
    ga.mt = c.MT;
    ga.nt = c.NT;
    const int g8 = (ga.col_groups + 7) / 8 * 8;
    dim3 grid((unsigned)(g8 * ga.m_blocks * ga.splits));
    const size_t lds = (size_t)2 * (c.NT == 4 ? 1 : 2) * c.MT * 2 * 64 * 16;
#define SEV_LAUNCH(MT_, NT_, PF_)                                                                                     \
    hipLaunchKernelGGL((gemm_bf16_kernel<MT_, NT_, EPI, PF_>), grid, dim3(256), lds, st, ga.W, ga.X, ga.n_tiles, ga.k_steps,         \
                       ga.m_tiles_total, ga.col_groups, ga.m_blocks, ga.splits | (c.T << 16), ga)
#define SEV_BY_NT(MT_, PF_)                                                                                           \
    do {                                                                                                              \
        if (c.NT == 2) SEV_LAUNCH(MT_, 2, PF_); else SEV_LAUNCH(MT_, 1, PF_);                                         \
    } while (0)
    if (c.MT == 4 && c.NT == 4) SEV_LAUNCH(4, 4, 4);
    else if (c.MT == 5) SEV_BY_NT(5, 4);
    else if (c.MT == 4) SEV_BY_NT(4, 4);
    else if (c.MT == 3) SEV_BY_NT(3, 4);
    else if (c.MT == 2) { if (c.PF == 6) SEV_BY_NT(2, 6); else SEV_BY_NT(2, 4); }
    else { if (c.PF == 6) SEV_BY_NT(1, 6); else SEV_BY_NT(1, 4); }
#undef SEV_BY_NT
#undef SEV_LAUNCH
    if constexpr (EPI != EPI_ARGMAX) {
        if (c.S > 1) launch_fixup<EPI>(ga, m_tiles, st);
    }
}

void bf16_forward(const sev_model *m, sev_kv *kv, int rows, int B, int n_items, int n_groups, int sib, bool att_direct,
                  float *logits_out, hipStream_t st) {
    const sev_model_desc &d = m->d;
    KvGeom g = sev_kv_geom(kv);
    const int m_tiles_real = (rows + 31) / 32;
    const int m_tiles = (m_tiles_real + 3) / 4 * 4;
    auto Wp = [&](size_t off) { return (const uint4 *)(m->arena + off); };
    auto Gp = [&](size_t off) { return (const float *)(m->arena + off); };
    uint16_t *xa = (uint16_t *)kv->xa, *qp = (uint16_t *)kv->q_buf, *op = (uint16_t *)kv->o_buf, *act = (uint16_t *)kv->act;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)d.head_dim);

    {
        Prof p(kv, st, PROF_OTHER);
        hipLaunchKernelGGL(embed_norm_kernel, dim3(rows), dim3(256), 0, st, (const uint16_t *)(m->arena + m->off_embed),
                           kv->plan.row_tok, Gp(m->layers[0].g_attn), kv->h, xa, kv->ssq[1], kv->ssq[0], d.d_model, m_tiles);
    }
    const GemmCfg pq = choose_cfg(G_QKV, m_tiles_real, m->n_qkv / 32, d.d_model / 16, kv->part_elems, kv->tune);
    const GemmCfg po = choose_cfg(G_O, m_tiles_real, d.d_model / 32, m->q_dim / 16, kv->part_elems, kv->tune);
    const GemmCfg pg = choose_cfg(G_GU, m_tiles_real, d.d_ffn / 16, d.d_model / 16, kv->part_elems, kv->tune);
    const GemmCfg pd = choose_cfg(G_DOWN, m_tiles_real, d.d_model / 32, d.d_ffn / 16, kv->part_elems, kv->tune);
    const GemmCfg pl = choose_cfg(G_LM, m_tiles_real, d.vocab / 32, d.d_model / 16, kv->part_elems, kv->tune);
    GemmArgs base;
    memset(&base, 0, sizeof(base));
    base.m_tiles_total = m_tiles;
    base.M = rows;
    base.part = kv->part;
    base.inv_d = 1.0f / (float)d.d_model;
    base.eps = d.rms_eps;
    base.h = kv->h;
    for (int l = 0; l < d.n_layers; ++l) {
        const LayerOffsets &lo = m->layers[l];
        {   // QKV projection; rotary embedding, q planes and the cache append in its epilogue
            Prof p(kv, st, PROF_GEMM_QKV);
            GemmArgs ga = base;
            ga.W = Wp(lo.wqkv); ga.X = (const uint4 *)xa; ga.n_tiles = m->n_qkv / 32; ga.k_steps = d.d_model / 16;
            ga.N = m->n_qkv; ga.ssq_in = kv->ssq[1];
            ga.row_cs = kv->plan.row_cs; ga.row_kvloc = kv->plan.row_kvloc; ga.Hq = d.n_q_heads; ga.Hkv = d.n_kv_heads;
            ga.k_layer = g.pool + (size_t)l * g.layer_stride; ga.v_offset = g.v_offset; ga.q_planes = qp;
            launch_gemm<EPI_QKV>(ga, pq, m_tiles_real, st);
        }
        {
            Prof p(kv, st, PROF_ATTN);
            const bool once = n_groups == B;             // one row group per request: every K/V byte is read by one block
#define SEV_ATTN(WAVES_, DIRECT_, ONCE_, THREADS_, LDS_)                                                                                   \
    hipLaunchKernelGGL((attn_bf16_kernel<WAVES_, DIRECT_, ONCE_>), dim3((unsigned)((n_items / sib + 7) / 8 * 8 * sib * d.n_kv_heads)), dim3(THREADS_), LDS_, st, \
                       kv->plan.it_a, kv->plan.it_b, kv->plan.it_pages, qp, g.pool, (size_t)l * g.layer_stride, g.v_offset, rows,           \
                       d.n_q_heads | (d.n_kv_heads << 16), kv->plan, g, n_items | (sib << 24), kv->att_o, kv->att_ml, scale_log2e, op, m_tiles)
            if (att_direct) {                            // one block of 8 waves per (request, row group, KV head): no chunks, no merge
                const size_t lds = (size_t)(8 * 64 * 64 + 2 * 8 * 64) * 4;      // 8 merge slots
                if (once) SEV_ATTN(8, true, true, 512, lds); else SEV_ATTN(8, true, false, 512, lds);
            } else {
                const size_t lds = (size_t)(4 * 64 * 64 + 2 * 4 * 64) * 4;   // 4 merge slots
                if (once) SEV_ATTN(4, false, true, 256, lds); else SEV_ATTN(4, false, false, 256, lds);
                hipLaunchKernelGGL(attn_merge_kernel, dim3(n_groups, d.n_kv_heads), dim3(256), 0, st, (const int4 *)kv->plan.mg_rec,
                                   (const float *)kv->att_o, (const float2 *)kv->att_ml, op, d.n_q_heads, d.n_kv_heads, m_tiles);
            }
#undef SEV_ATTN
        }
        {   // output projection; residual add, FFN-norm operand and scale in its epilogue
            Prof p(kv, st, PROF_GEMM_O);
            GemmArgs ga = base;
            ga.W = Wp(lo.wo); ga.X = (const uint4 *)op; ga.n_tiles = d.d_model / 32; ga.k_steps = m->q_dim / 16;
            ga.N = d.d_model; ga.gain = Gp(lo.g_ffn); ga.xout = xa; ga.ssq_out = kv->ssq[0]; ga.ssq_clear = kv->ssq[1];
            launch_gemm<EPI_RESID>(ga, po, m_tiles_real, st);
        }
        {   // gate/up projection with fused SwiGLU
            Prof p(kv, st, PROF_GEMM_GU);
            GemmArgs ga = base;
            ga.W = Wp(lo.wgu); ga.X = (const uint4 *)xa; ga.n_tiles = d.d_ffn / 16; ga.k_steps = d.d_model / 16;
            ga.N = 2 * d.d_ffn; ga.act = act; ga.ssq_in = kv->ssq[0];
            launch_gemm<EPI_SWIGLU>(ga, pg, m_tiles_real, st);
        }
        {   // down projection; residual add, next norm's operand and scale in its epilogue
            Prof p(kv, st, PROF_GEMM_DOWN);
            GemmArgs ga = base;
            ga.W = Wp(lo.wd); ga.X = (const uint4 *)act; ga.n_tiles = d.d_model / 32; ga.k_steps = d.d_ffn / 16;
            ga.N = d.d_model; ga.gain = (l + 1 < d.n_layers) ? Gp(m->layers[l + 1].g_attn) : Gp(m->off_gfinal); ga.xout = xa;
            ga.ssq_out = kv->ssq[1]; ga.ssq_clear = kv->ssq[0];
            launch_gemm<EPI_RESID>(ga, pd, m_tiles_real, st);
        }
    }
    {   // LM head with fused arg-max
        Prof p(kv, st, PROF_GEMM_LM);
        GemmArgs ga = base;
        ga.W = Wp(m->off_lm); ga.X = (const uint4 *)xa; ga.n_tiles = d.vocab / 32; ga.k_steps = d.d_model / 16; ga.N = d.vocab;
        ga.ssq_in = kv->ssq[1];
        ga.lm_val = kv->lm_val; ga.lm_idx = kv->lm_idx; ga.lm_stride = m_tiles * 32; ga.logits = logits_out;
        launch_gemm<EPI_ARGMAX>(ga, pl, m_tiles_real, st);
        const int n_part = ((ga.n_tiles + 4 * pl.NT - 1) / (4 * pl.NT)) * 4;
        hipLaunchKernelGGL(lm_reduce_kernel, dim3(rows), dim3(256), 0, st, kv->lm_val, kv->lm_idx, n_part, ga.lm_stride,
                           kv->row_argmax);
    }
}
