// float32 path: straightforward kernels for float32 models.  Every step of the forward pass
// (embedding, RMSNorm, projections, rotary embedding + cache append, masked attention over the
// paged cache, SwiGLU, output head) is computed here in float32 with plain FMA arithmetic.
#include "sev_internal.h"
#include "kv_layout.h"

KvGeom sev_kv_geom(const sev_kv *kv);

__global__ void copy_f32_kernel(float *dst, const float *src, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}
void launch_pack_f32(float *dst, const float *src, int64_t n, hipStream_t st) {
    if (n > 0) hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dst, src, n);
}

// h[m][:] = E[tok[m]][:]
__global__ void embed_f32_kernel(const float *E, const int32_t *row_tok, float *h, int d) {
    const float *src = E + (size_t)row_tok[blockIdx.x] * d;
    float *dst = h + (size_t)blockIdx.x * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = src[i];
}

// y = x * rsqrt(mean(x^2) + eps) * g, one block per row
__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float *h, const float *g, float *y, int d, float eps) {
    __shared__ float red[256];
    const float *x = h + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) ss += x[i] * x[i];
    red[threadIdx.x] = ss;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const float r = 1.0f / sqrtf(red[0] / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) y[(size_t)blockIdx.x * d + i] = x[i] * r * g[i];
}

// Y[m][n] (+)= sum_k X[m][k] * W[n][k].  Block: 64 columns x 16 rows, K tiled by 32 through LDS.
template <bool ACC>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *X, const float *W, float *Y, int M, int N, int K) {
    __shared__ float Ws[64][33];
    __shared__ float Xs[16][33];
    const int tn = threadIdx.x & 63, tm = threadIdx.x >> 6;
    const int n0 = blockIdx.x * 64, m0 = blockIdx.y * 16;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int i = threadIdx.x; i < 64 * 32; i += 256) {
            const int r = i >> 5, c = i & 31;
            Ws[r][c] = (n0 + r < N && k0 + c < K) ? W[(size_t)(n0 + r) * K + k0 + c] : 0.f;
        }
        for (int i = threadIdx.x; i < 16 * 32; i += 256) {
            const int r = i >> 5, c = i & 31;
            Xs[r][c] = (m0 + r < M && k0 + c < K) ? X[(size_t)(m0 + r) * K + k0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const float w = Ws[tn][k];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += Xs[tm + 4 * j][k] * w;
        }
        __syncthreads();
    }
    if (n0 + tn < N) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + tm + 4 * j;
            if (m < M) {
                float *y = Y + (size_t)m * N + n0 + tn;
                *y = ACC ? *y + acc[j] : acc[j];
            }
        }
    }
}

static void gemm_f32(const float *X, const float *W, float *Y, int M, int N, int K, bool acc, hipStream_t st) {
    dim3 grid((N + 63) / 64, (M + 15) / 16);
    if (acc) hipLaunchKernelGGL(gemm_f32_kernel<true>, grid, dim3(256), 0, st, X, W, Y, M, N, K);
    else hipLaunchKernelGGL(gemm_f32_kernel<false>, grid, dim3(256), 0, st, X, W, Y, M, N, K);
}

// Rotary embedding of q (in place) and k, and append of k, v to the paged cache at position P + node.
// grid (rows, Hq + Hkv): blocks y < Hq rotate a query head, the others handle a KV head.
__global__ void rope_kv_f32_kernel(float *qkv, DevPlan p, KvGeom g, const int32_t *page_table, int max_pages, int layer,
                                   int Hq, int n_qkv) {
    const int m = blockIdx.x, hy = blockIdx.y, hd = g.hd, half = hd / 2;
    const float2 *cs = p.row_cs + (size_t)m * half;
    float *row = qkv + (size_t)m * n_qkv;
    if (hy < Hq) {
        float *q = row + hy * hd;
        for (int i = threadIdx.x; i < half; i += blockDim.x) {
            const float a = q[i], b = q[i + half], c = cs[i].x, s = cs[i].y;
            q[i] = a * c - b * s;
            q[i + half] = b * c + a * s;
        }
        return;
    }
    const int h = hy - Hq, b = p.row_req[m];
    const int tok = p.req_P[b] + p.row_node[m];
    const int slot = p.req_slot[b];
    const size_t blk = (size_t)SEV_PAGE * hd;
    const size_t pb = ((size_t)page_table[(size_t)slot * max_pages + tok / SEV_PAGE] * g.Hkv + h) * blk;
    float *kc = (float *)(g.pool + (size_t)layer * g.layer_stride) + pb + (size_t)(tok % SEV_PAGE) * hd;
    float *vc = (float *)(g.pool + (size_t)layer * g.layer_stride + g.v_offset) + pb + (size_t)(tok % SEV_PAGE) * hd;
    const float *k = row + Hq * hd + h * hd;
    const float *v = row + (Hq + g.Hkv) * hd + h * hd;
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        const float a = k[i], bb = k[i + half], c = cs[i].x, s = cs[i].y;
        kc[i] = a * c - bb * s;
        kc[i + half] = bb * c + a * s;
        vc[i] = v[i];
        vc[i + half] = v[i + half];
    }
}

// Masked attention of one (row, query head) per wave over the request's paged cache:
// all prefix positions, plus the block's nodes that are ancestors-or-self of the row's node (chains:
// the nodes up to the row's own, whatever the block length).
__global__ __launch_bounds__(64) void attn_f32_kernel(const float *qkv, float *out, DevPlan p, KvGeom g,
                                                      const int32_t *page_table, int max_pages, int layer, int Hq,
                                                      int n_qkv, float scale) {
    const int m = blockIdx.x, j = blockIdx.y, lane = threadIdx.x, hd = g.hd;
    const int b = p.row_req[m], P = p.req_P[b], n = p.req_n[b], slot = p.req_slot[b];
    const unsigned long long anc = p.row_anc[m];
    const int node = p.row_node[m];
    const int h = (j * g.Hkv) / Hq;
    const float *q = qkv + (size_t)m * n_qkv + j * hd;
    const int32_t *pt = page_table + (size_t)slot * max_pages;
    const size_t blk = (size_t)SEV_PAGE * hd;
    const float *Kl = (const float *)(g.pool + (size_t)layer * g.layer_stride);
    const float *Vl = (const float *)(g.pool + (size_t)layer * g.layer_stride + g.v_offset);
    float qv[4], acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) qv[r] = (lane + 64 * r < hd) ? q[lane + 64 * r] : 0.f;
    float mx = -INFINITY, den = 0.f;
    for (int t = 0; t < P + n; ++t) {
        if (t >= P && (p.causal ? (t - P > node) : !((anc >> (t - P)) & 1ull))) continue;
        const size_t pb = ((size_t)pt[t / SEV_PAGE] * g.Hkv + h) * blk + (size_t)(t % SEV_PAGE) * hd;
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (lane + 64 * r < hd) s += qv[r] * Kl[pb + lane + 64 * r];
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        s *= scale;
        const float mn = fmaxf(mx, s);
        const float corr = expf(mx - mn), pe = expf(s - mn);
        den = den * corr + pe;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (lane + 64 * r < hd) acc[r] = acc[r] * corr + pe * Vl[pb + lane + 64 * r];
        mx = mn;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (lane + 64 * r < hd) out[(size_t)m * (Hq * hd) + j * hd + lane + 64 * r] = acc[r] / den;
}

__global__ void swiglu_f32_kernel(const float *gu, float *act, int F, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int64_t m = i / F;
    const int f = (int)(i - m * F);
    const float gt = gu[m * 2 * F + f], up = gu[m * 2 * F + F + f];
    act[i] = gt / (1.0f + expf(-gt)) * up;
}

void f32_forward(const sev_model *m, sev_kv *kv, int rows, int B, float *logits_out, hipStream_t st) {
    (void)B;
    const sev_model_desc &d = m->d;
    KvGeom g = sev_kv_geom(kv);
    const float *arena = nullptr;
    auto W = [&](size_t off) { return (const float *)(m->arena + off); };
    (void)arena;
    float *h = kv->h, *xa = (float *)kv->xa, *qkv = (float *)kv->q_buf, *ob = (float *)kv->o_buf,
          *act = (float *)kv->act, *gu = kv->part;
    hipLaunchKernelGGL(embed_f32_kernel, dim3(rows), dim3(256), 0, st, W(m->off_embed), kv->plan.row_tok, h, d.d_model);
    const float scale = 1.0f / sqrtf((float)d.head_dim);
    for (int l = 0; l < d.n_layers; ++l) {
        const LayerOffsets &lo = m->layers[l];
        hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3(rows), dim3(256), 0, st, h, W(lo.g_attn), xa, d.d_model, d.rms_eps);
        gemm_f32(xa, W(lo.wqkv), qkv, rows, m->n_qkv, d.d_model, false, st);
        hipLaunchKernelGGL(rope_kv_f32_kernel, dim3(rows, d.n_q_heads + d.n_kv_heads), dim3(64), 0, st, qkv, kv->plan, g,
                           kv->page_table, kv->max_pages_per_req, l, d.n_q_heads, m->n_qkv);
        hipLaunchKernelGGL(attn_f32_kernel, dim3(rows, d.n_q_heads), dim3(64), 0, st, qkv, ob, kv->plan, g,
                           kv->page_table, kv->max_pages_per_req, l, d.n_q_heads, m->n_qkv, scale);
        gemm_f32(ob, W(lo.wo), h, rows, d.d_model, m->q_dim, true, st);
        hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3(rows), dim3(256), 0, st, h, W(lo.g_ffn), xa, d.d_model, d.rms_eps);
        gemm_f32(xa, W(lo.wgu), gu, rows, 2 * d.d_ffn, d.d_model, false, st);
        const int64_t tot = (int64_t)rows * d.d_ffn;
        hipLaunchKernelGGL(swiglu_f32_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, gu, act, d.d_ffn, tot);
        gemm_f32(act, W(lo.wd), h, rows, d.d_model, d.d_ffn, true, st);
    }
    hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3(rows), dim3(256), 0, st, h, W(m->off_gfinal), xa, d.d_model, d.rms_eps);
    float *lg = logits_out ? logits_out : kv->logits_f32;
    gemm_f32(xa, W(m->off_lm), lg, rows, d.vocab, d.d_model, false, st);
    launch_argmax_rows_f32(lg, rows, d.vocab, kv->row_argmax, st);
}
