// Kernels shared by both precisions: call plan, acceptance, KV commit, cache import/export.
#include <algorithm>

#include "sev_internal.h"
#include "kv_layout.h"

// ---------------------------------------------------------------------------
// fills
// ---------------------------------------------------------------------------
__global__ void fill_f32_kernel(float *p, float v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
__global__ void fill_i32_kernel(int32_t *p, int32_t v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
void launch_fill_f32(float *p, float v, int64_t n, hipStream_t st) {
    if (n > 0) hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
}
void launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t st) {
    if (n > 0) hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
}

// ---------------------------------------------------------------------------
// call plan: everything the forward pass needs to know about the batch,
// derived on the device from the lengths passed by value.
//
// Per request: row range, prefix length, slot.  Per draft node (row): request,
// node index, rotary position P + depth, ancestor-or-self bit mask, token.
// Per row and rotary frequency: (cos, sin) of pos * base^(-2i/hd), evaluated in
// double so that positions in the thousands keep full float accuracy.
// For the matrix-core attention: the list of (request, row group, KV chunk)
// work items and the per (request, row group) merge groups.
// ---------------------------------------------------------------------------
struct PlanDev {
    DevPlan p;
    int32_t *seq_len, *pend_n, *pend_P;
    uint32_t *err;
    int vocab, hd, G;          // G = query heads per KV head
    double rope_base;
    int chunk_pages;
    const int32_t *tokens, *parents;
    const int32_t *page_table;
    int max_pages;
};

__global__ __launch_bounds__(256) void plan_kernel(PlanArgs a, PlanDev d) {
    __shared__ int s_row0[SEV_MAX_BATCH + 1];
    __shared__ int s_item0[SEV_MAX_BATCH + 1];
    __shared__ int s_grp0[SEV_MAX_BATCH + 1];
    const int t = threadIdx.x;
    const int B = a.B;
    int my_items = 0, my_groups = 0, my_chunks = 0;
    if (t < B) {
        const int slot = a.slot[t], P = a.prefix[t], n = a.nd[t];
        if (d.seq_len[slot] != P) atomicOr(d.err, 1u);
        d.pend_n[slot] = 0;                      // a new verify drops whatever was pending
        d.pend_P[slot] = P;
        my_groups = (d.G * n + 31) / 32;
        const int pages = (max(P + n, a.pad_tokens) + SEV_PAGE - 1) / SEV_PAGE;
        my_chunks = (pages + d.chunk_pages - 1) / d.chunk_pages;
        my_items = my_groups * my_chunks;
        s_row0[t + 1] = n;
        s_item0[t + 1] = my_items;
        s_grp0[t + 1] = my_groups;
    }
    __syncthreads();
    if (t == 0) {
        s_row0[0] = s_item0[0] = s_grp0[0] = 0;
        for (int b = 0; b < B; ++b) {
            s_row0[b + 1] += s_row0[b];
            s_item0[b + 1] += s_item0[b];
            s_grp0[b + 1] += s_grp0[b];
        }
    }
    __syncthreads();
    if (t < B) {
        const int slot = a.slot[t], P = a.prefix[t], n = a.nd[t], row0 = s_row0[t];
        d.p.req_slot[t] = slot;
        d.p.req_P[t] = P;
        d.p.req_n[t] = n;
        d.p.req_row0[t] = row0;
        if (t == B - 1) d.p.req_row0[B] = s_row0[B];
        // trees: parents precede children, so one forward sweep gives depth and ancestor set
        // (the rows of chains are filled in parallel by plan_fill_kernel)
        unsigned long long anc_prev = 0;
        int depth_prev = -1;
        for (int i = 0; d.parents && i < n; ++i) {
            int par = d.parents[t * a.k_max + i];
            if (par < -1 || par >= i) { atomicOr(d.err, 2u); par = -1; }
            unsigned long long anc;
            int depth;
            if (par < 0) { anc = 0; depth = 0; }
            else if (par == i - 1) { anc = anc_prev; depth = depth_prev + 1; }
            else { anc = d.p.row_anc[row0 + par]; depth = d.p.row_pos[row0 + par] - P + 1; }
            anc |= 1ull << i;
            int tok = d.tokens[t * a.tok_stride + a.tok_off + i];
            if (tok < 0 || tok >= d.vocab) { atomicOr(d.err, 4u); tok = 0; }
            d.p.row_req[row0 + i] = t;
            d.p.row_node[row0 + i] = i;
            d.p.row_pos[row0 + i] = P + depth;
            d.p.row_anc[row0 + i] = anc;
            d.p.row_tok[row0 + i] = tok;
            d.p.row_kvloc[row0 + i] = d.page_table[(size_t)slot * d.max_pages + (P + i) / SEV_PAGE] * SEV_PAGE + (P + i) % SEV_PAGE;
            anc_prev = anc;
            depth_prev = depth;
        }
        // attention work items of this request: its pages are split evenly over my_chunks chunks
        const int pages = (max(P + n, a.pad_tokens) + SEV_PAGE - 1) / SEV_PAGE;
        const int cpp = (pages + my_chunks - 1) / my_chunks;
        // item order: chunk by chunk, the row groups of one chunk side by side (the attention kernel puts them on
        // one XCD, where the chunk is then fetched from memory once for all of them)
        const int it0 = s_item0[t], g0 = s_grp0[t];
        for (int rg = 0; rg < my_groups; ++rg) {
            d.p.mg_rec[g0 + rg] = make_int4(rg | (my_chunks << 16), it0 + rg, n | (my_groups << 16), row0);
            for (int c = 0; c < my_chunks; ++c) {
                const int p0 = c * cpp, it = it0 + c * my_groups + rg;
                d.p.it_a[it] = make_int4(rg, p0, min(cpp, pages - p0), P);
                d.p.it_b[it] = make_int4(n, row0, t, slot);
            }
        }
    }
}

// Second half of the plan, one thread per entry: the rows of chain blocks (request, node, position,
// token, cache location), the physical page ids of every attention work item (padded with the
// chunk's last page, so that the attention kernel can load its page ids without knowing the chunk
// length) and the rotary table (cos, sin)(pos * theta_i), computed in double.
__device__ __forceinline__ int find_request(const int32_t *row0, int B, int m) {
    int lo = 0, hi = B - 1;                                   // largest b with row0[b] <= m
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (row0[mid] <= m) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__global__ __launch_bounds__(256) void plan_fill_kernel(PlanArgs a, PlanDev d, int n_items, int rows) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (!d.parents && idx < rows) {
        const int b = find_request(d.p.req_row0, a.B, idx), i = idx - d.p.req_row0[b];
        const int P = d.p.req_P[b], slot = d.p.req_slot[b];
        int tok = d.tokens[b * a.tok_stride + a.tok_off + i];
        if (tok < 0 || tok >= d.vocab) { atomicOr(d.err, 4u); tok = 0; }
        d.p.row_req[idx] = b;
        d.p.row_node[idx] = i;
        d.p.row_pos[idx] = P + i;
        d.p.row_anc[idx] = i < 63 ? (2ull << i) - 1ull : ~0ull;
        d.p.row_tok[idx] = tok;
        d.p.row_kvloc[idx] = d.page_table[(size_t)slot * d.max_pages + (P + i) / SEV_PAGE] * SEV_PAGE + (P + i) % SEV_PAGE;
    }
    if (idx < n_items * SEV_ATT_MAX_CP) {
        const int it = idx / SEV_ATT_MAX_CP, i = idx - it * SEV_ATT_MAX_CP;
        const int4 ia = d.p.it_a[it], ib = d.p.it_b[it];
        d.p.it_pages[idx] = d.page_table[(size_t)ib.w * d.max_pages + ia.y + min(i, ia.z - 1)];
    }
    const int half = d.hd / 2;
    if (idx < rows * half) {
        const int r = idx / half, i = idx - r * half;
        int pos;
        if (d.parents) pos = d.p.row_pos[r];                  // written by plan_kernel
        else {
            const int b = find_request(d.p.req_row0, a.B, r);
            pos = d.p.req_P[b] + r - d.p.req_row0[b];
        }
        const double theta = pow(d.rope_base, -2.0 * (double)i / (double)d.hd);
        double s, c;
        sincos((double)pos * theta, &s, &c);
        d.p.row_cs[idx] = make_float2((float)c, (float)s);
    }
}

void launch_plan(const sev_kv *kv, const PlanArgs &pa, const int32_t *draft_tokens, const int32_t *parents, int rows,
                 int chunk_pages, int n_items, hipStream_t st) {
    PlanDev d;
    d.p = kv->plan;
    d.seq_len = kv->seq_len;
    d.pend_n = kv->pend_n;
    d.pend_P = kv->pend_P;
    d.err = kv->err_flags;
    d.vocab = kv->model->d.vocab;
    d.hd = kv->model->d.head_dim;
    d.G = kv->model->d.n_q_heads / kv->model->d.n_kv_heads;
    d.rope_base = (double)kv->model->d.rope_base;
    d.chunk_pages = chunk_pages;
    d.tokens = draft_tokens;
    d.parents = parents;
    d.page_table = kv->page_table;
    d.max_pages = kv->max_pages_per_req;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, st, pa, d);
    const int64_t entries = std::max<int64_t>((int64_t)n_items * SEV_ATT_MAX_CP, (int64_t)rows * std::max(1, d.hd / 2));
    hipLaunchKernelGGL(plan_fill_kernel, dim3((unsigned)((entries + 255) / 256)), dim3(256), 0, st, pa, d, n_items, rows);
}

// ---------------------------------------------------------------------------
// greedy acceptance (paper section 4.1: accepted candidates plus one additional
// token from the server's own forward pass).  One thread per request.
// ---------------------------------------------------------------------------
__global__ void accept_kernel(DevPlan p, int B, int k_max, int mode, const int32_t *tokens, const int32_t *parents,
                              const int32_t *row_argmax, const int32_t *next_tok, int32_t *pend_n, int32_t *pend_a,
                              int32_t *pend_bonus, int32_t *pend_path, int32_t *accept_len, int32_t *bonus_out,
                              int32_t *path_out) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int slot = p.req_slot[b], n = p.req_n[b], row0 = p.req_row0[b];
    int32_t *path = pend_path + (size_t)slot * SEV_MAX_DRAFT;
    int a = 0, want;
    if (mode == 1) {                       // append: keep the whole chain
        for (int i = 0; i < n && i < SEV_MAX_DRAFT; ++i) path[i] = i;     // (longer appended blocks are never re-ordered)
        a = n;
        want = row_argmax[row0 + n - 1];
    } else {
        want = next_tok[slot];
        int cur = -1;
        while (true) {
            int nxt = -1;
            // children of `cur` come after it; the lowest matching index wins
            for (int c = cur + 1; c < n; ++c) {
                const int par = parents ? parents[b * k_max + c] : c - 1;
                const int par_ok = (par < -1 || par >= c) ? -1 : par;
                if (par_ok == cur && tokens[b * k_max + c] == want) { nxt = c; break; }
            }
            if (nxt < 0) break;
            path[a++] = nxt;
            cur = nxt;
            want = row_argmax[row0 + nxt];
        }
    }
    for (int i = a; i < SEV_MAX_DRAFT; ++i) path[i] = -1;
    pend_n[slot] = n;
    pend_a[slot] = a;
    pend_bonus[slot] = want;
    accept_len[b] = a;
    bonus_out[b] = want;
    if (path_out)
        for (int i = 0; i < k_max; ++i) path_out[b * k_max + i] = i < a ? path[i] : -1;
}

void launch_accept(const sev_kv *kv, int B, int k_max, int mode, const int32_t *draft_tokens, const int32_t *parents,
                   int32_t *accept_len, int32_t *bonus, int32_t *accept_path, hipStream_t st) {
    hipLaunchKernelGGL(accept_kernel, dim3((B + 63) / 64), dim3(64), 0, st, kv->plan, B, k_max, mode, draft_tokens,
                       parents, kv->row_argmax, kv->next_tok, kv->pend_n, kv->pend_a, kv->pend_bonus, kv->pend_path,
                       accept_len, bonus, accept_path);
}

// ---------------------------------------------------------------------------
// commit / rollback (paper section 4.2: the cache follows the accepted tokens)
// ---------------------------------------------------------------------------
struct SlotList {
    int32_t s[SEV_MAX_BATCH];
};

// grid (ceil(L*Hkv*hd/256), B).  Each thread owns one (layer, kv head, element) and moves it for the
// accepted nodes in ascending order; destinations never lie ahead of a source still to be read
// because an accepted node's index is at least its depth.
template <typename T, bool BF16>
__global__ void commit_copy_kernel(SlotList sl, KvGeom g, const int32_t *page_table, int max_pages,
                                   const int32_t *pend_n, const int32_t *pend_a, const int32_t *pend_P,
                                   const int32_t *pend_path) {
    const int slot = sl.s[blockIdx.y];
    if (pend_n[slot] == 0) return;
    const int a = pend_a[slot], P = pend_P[slot];
    if (a > SEV_MAX_DRAFT) return;                       // an appended block longer than any draft: already in place
    const int32_t *path = pend_path + (size_t)slot * SEV_MAX_DRAFT;
    bool moved = false;
    for (int j = 0; j < a; ++j) moved |= (path[j] != j);
    if (!moved) return;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int per_layer = g.Hkv * g.hd;
    if (idx >= g.L * per_layer) return;
    const int layer = idx / per_layer, rem = idx - layer * per_layer, h = rem / g.hd, e = rem - h * g.hd;
    const int32_t *pt = page_table + (size_t)slot * max_pages;
    T *base = (T *)(g.pool + (size_t)layer * g.layer_stride);
    T *vbase = (T *)(g.pool + (size_t)layer * g.layer_stride + g.v_offset);
    for (int j = 0; j < a; ++j) {
        const int src = P + path[j], dst = P + j;
        if (src == dst) continue;
        const size_t so = (size_t)pt[src / SEV_PAGE] * g.Hkv + h, dofs = (size_t)pt[dst / SEV_PAGE] * g.Hkv + h;
        const int blk = SEV_PAGE * g.hd;
        base[dofs * blk + k_in_page<BF16>(dst % SEV_PAGE, e, g.hd)] = base[so * blk + k_in_page<BF16>(src % SEV_PAGE, e, g.hd)];
        vbase[dofs * blk + v_in_page<BF16>(dst % SEV_PAGE, e, g.hd)] = vbase[so * blk + v_in_page<BF16>(src % SEV_PAGE, e, g.hd)];
    }
}

__global__ void commit_state_kernel(SlotList sl, int B, int rollback, int32_t *seq_len, int32_t *next_tok,
                                    int32_t *pend_n, const int32_t *pend_a, const int32_t *pend_bonus) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int slot = sl.s[b];
    if (pend_n[slot] == 0) return;
    if (!rollback) {
        seq_len[slot] += pend_a[slot];
        next_tok[slot] = pend_bonus[slot];
    }
    pend_n[slot] = 0;
}

// ---------------------------------------------------------------------------
// stochastic verification (paper section 4.1: the draft/verify cycle preserves the server
// model's output distribution, by the accept / resample rule of speculative sampling, in its
// multi-step form for trees; section 5: temperature 0.7).  All random numbers are inputs.
//
// softmax_stats_kernel: one block per row: the row's largest logit and the sum of
//   exp((logit - max) / T).
// sample_walk_kernel: one block per request.  The block's root must be the server's own previous
//   token.  At the current node, with p = the server distribution computed there, the children
//   are tried in index order: child c (token x, edge distribution q_c) is accepted iff
//   u_acc[c] * q_c(x) < p(x); a rejection replaces p by the normalised residual max(0, p - q_c)
//   (the normaliser is a block-wide sum over the vocabulary, in a fixed order); an acceptance
//   moves to c.  When no child is left the emitted token is drawn from the current p by inverse
//   CDF in token-id order: sums of groups of 64 consecutive ids, a scan over the groups, then a
//   scan inside the group that holds u_emit * total.  Chains are trees whose node i has parent
//   i - 1.
// ---------------------------------------------------------------------------
#define SEV_MAX_REJ 16   // rejected siblings remembered at one node

__global__ __launch_bounds__(1024) void softmax_stats_kernel(const float *logits, int vocab, float inv_t, float2 *stats) {
    // one pass with a running maximum (the sum is rescaled whenever the maximum grows); 16-byte loads where the
    // row allows it; the partial (max, sum) pairs are combined in a fixed order
    __shared__ float red_m[16], red_s[16];
    const float *row = logits + (size_t)blockIdx.x * vocab;
    float m = -INFINITY, sum = 0.f;
    auto take = [&](float x) {
        if (x > m) { sum *= expf((m - x) * inv_t); m = x; }       // exp(-inf) = 0 covers the first element
        sum += expf((x - m) * inv_t);
    };
    const bool vec = ((vocab & 3) == 0) && ((((size_t)blockIdx.x * vocab) & 3) == 0) && ((((uintptr_t)logits) & 15) == 0);
    if (vec) {
        const float4 *r4 = (const float4 *)row;
        for (int i = threadIdx.x; i < (vocab >> 2); i += 1024) {
            const float4 x = r4[i];
            const float mx4 = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
            if (mx4 > m) { sum *= expf((m - mx4) * inv_t); m = mx4; }
            sum += expf((x.x - m) * inv_t) + expf((x.y - m) * inv_t) + expf((x.z - m) * inv_t) + expf((x.w - m) * inv_t);
        }
    } else {
        for (int v = threadIdx.x; v < vocab; v += 1024) take(row[v]);
    }
    // wave, then block: (m, s) pairs merge as s = s_a * exp((m_a - m) / T) + s_b * exp((m_b - m) / T)
    auto merge = [&](float mo, float so) {
        const float mn = fmaxf(m, mo);
        const float a = (m == -INFINITY) ? 0.f : expf((m - mn) * inv_t), b = (mo == -INFINITY) ? 0.f : expf((mo - mn) * inv_t);
        sum = sum * a + so * b;
        m = mn;
    };
    for (int o = 32; o > 0; o >>= 1) merge(__shfl_xor(m, o), __shfl_xor(sum, o));
    if ((threadIdx.x & 63) == 0) { red_m[threadIdx.x >> 6] = m; red_s[threadIdx.x >> 6] = sum; }
    __syncthreads();
    if (threadIdx.x == 0) {
        m = red_m[0]; sum = red_s[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) merge(red_m[w], red_s[w]);
        stats[blockIdx.x] = make_float2(m, sum);
    }
}

struct WalkState {
    int cur, a, nrej, child, action;       // action: 0 accepted a child, 1 rejected one (in rej[nrej]), 2 no child left
    int rej[SEV_MAX_REJ + 1];
    float R[SEV_MAX_REJ + 1];
    int path[SEV_MAX_DRAFT];
};

__global__ __launch_bounds__(1024) void sample_walk_kernel(DevPlan p, int k_max, const int32_t *tokens, const int32_t *parents,
                                                           const float *logits, const float *draft_probs, const float2 *stats, int vocab,
                                                           float inv_t, const float *u_acc, const float *u_emit, const int32_t *next_tok,
                                                           uint32_t *err, int32_t *pend_n, int32_t *pend_a, int32_t *pend_bonus,
                                                           int32_t *pend_path, int32_t *accept_len, int32_t *emitted, int32_t *path_out) {
    __shared__ WalkState s;
    __shared__ float s_part[16];
    __shared__ int s_pick;
    extern __shared__ float s_grp[];                    // [ceil(vocab / 64)] sums of 64 consecutive ids (draw pass)
    const int b = blockIdx.x, t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int n_groups = (vocab + 63) >> 6;
    const int slot = p.req_slot[b], n = p.req_n[b], row0 = p.req_row0[b];
    // the block's tokens and (sanitised) parents in LDS, and for every node the outcome of its acceptance test
    // against the plain softmax at its parent: the test the walk needs as long as no sibling was rejected at that
    // parent, taken for all nodes at once instead of one after the other along the path
    __shared__ int s_tk[SEV_MAX_DRAFT], s_par[SEV_MAX_DRAFT], s_acc0[SEV_MAX_DRAFT];
    if (t < n) {
        const int c = t;
        const int q0 = parents ? parents[(size_t)b * k_max + c] : c - 1;
        const int q = (q0 < -1 || q0 >= c) ? -1 : q0;
        int x = tokens[(size_t)b * k_max + c];
        if (x < 0 || x >= vocab) x = 0;                 // the embedding step has flagged it and used id 0 as well
        s_tk[c] = x;
        s_par[c] = q;
        int ok = 0;
        if (q >= 0) {
            const float2 st = stats[row0 + q];
            const float px = expf((logits[(size_t)(row0 + q) * vocab + x] - st.x) * inv_t) / st.y;
            ok = u_acc[(size_t)b * k_max + c] * draft_probs[(size_t)(row0 + c) * vocab + x] < px;
        }
        s_acc0[c] = ok;
    }
    __syncthreads();
    const int *tk = s_tk;
    auto parent_of = [&](int c) { return s_par[c]; };
    // value at token v of the current distribution: the node's softmax, then one residual step per rejected sibling
    auto current = [&](int v) {
        const float2 st = stats[row0 + s.cur];
        float r = expf((logits[(size_t)(row0 + s.cur) * vocab + v] - st.x) * inv_t) / st.y;
        for (int j = 0; j < s.nrej; ++j) r = fmaxf(r - draft_probs[(size_t)(row0 + s.rej[j]) * vocab + v], 0.f) / s.R[j];
        return r;
    };
    // the same for four consecutive ids (16-byte loads: a block has one compute unit's worth of loads in flight, so the
    // passes over the vocabulary are bound by how many bytes each load carries)
    auto current4 = [&](int i) {
        const float2 st = stats[row0 + s.cur];
        const float4 l = ((const float4 *)(logits + (size_t)(row0 + s.cur) * vocab))[i];
        float4 r = make_float4(expf((l.x - st.x) * inv_t) / st.y, expf((l.y - st.x) * inv_t) / st.y, expf((l.z - st.x) * inv_t) / st.y,
                               expf((l.w - st.x) * inv_t) / st.y);
        for (int j = 0; j < s.nrej; ++j) {
            const float4 q = ((const float4 *)(draft_probs + (size_t)(row0 + s.rej[j]) * vocab))[i];
            const float R = s.R[j];
            r = make_float4(fmaxf(r.x - q.x, 0.f) / R, fmaxf(r.y - q.y, 0.f) / R, fmaxf(r.z - q.z, 0.f) / R, fmaxf(r.w - q.w, 0.f) / R);
        }
        return r;
    };
    const bool vec = ((vocab & 3) == 0) && ((((uintptr_t)logits | (uintptr_t)draft_probs) & 15) == 0);
    if (t == 0) {
        s.cur = -1;
        s.a = 0;
        s.nrej = 0;
        for (int c = 0; c < n; ++c)
            if (parent_of(c) == -1 && tk[c] == next_tok[slot]) { s.cur = c; break; }
        if (s.cur >= 0) { s.path[0] = s.cur; s.a = 1; s.child = s.cur + 1; }
    }
    __syncthreads();
    int tok = next_tok[slot];
    if (s.cur >= 0) {
        for (int guard = 0; guard <= 2 * SEV_MAX_DRAFT; ++guard) {          // every round consumes a child or ends the walk
            if (t == 0) {
                s.action = 2;
                for (int c = s.child; c < n; ++c) {
                    if (parent_of(c) != s.cur) continue;
                    const int x = tk[c];
                    s.child = c + 1;
                    const bool ok = s.nrej == 0 ? s_acc0[c] != 0
                                                : u_acc[(size_t)b * k_max + c] * draft_probs[(size_t)(row0 + c) * vocab + x] < current(x);
                    if (ok) {
                        s.cur = c;
                        s.path[s.a++] = c;
                        s.nrej = 0;
                        s.action = 0;
                    } else {
                        s.rej[s.nrej] = c;
                        s.action = 1;
                    }
                    break;
                }
            }
            __syncthreads();
            const int action = s.action;
            if (action == 0) {
                __syncthreads();                                              // everyone has read the action before thread 0 writes the next one
                continue;
            }
            // a block-wide pass over the vocabulary, thread t at ids t, t + 1024, ... (coalesced)
            if (action == 1) {
                // normaliser of the residual against the rejected child; wave sums, then the 16 wave totals in order
                const float *qrow = draft_probs + (size_t)(row0 + s.rej[s.nrej]) * vocab;
                float sum = 0.f;
                if (vec) {
#pragma unroll 2
                    for (int i = t; i < (vocab >> 2); i += 1024) {
                        const float4 r = current4(i), q = ((const float4 *)qrow)[i];
                        sum += (fmaxf(r.x - q.x, 0.f) + fmaxf(r.y - q.y, 0.f)) + (fmaxf(r.z - q.z, 0.f) + fmaxf(r.w - q.w, 0.f));
                    }
                } else {
                    for (int v = t; v < vocab; v += 1024) sum += fmaxf(current(v) - qrow[v], 0.f);
                }
                for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
                if (lane == 0) s_part[wave] = sum;
                __syncthreads();
                if (t == 0) {
                    float tot = 0.f;
                    for (int i = 0; i < 16; ++i) tot += s_part[i];
                    if (s.nrej >= SEV_MAX_REJ) atomicOr(err, 8u);           // more rejected siblings than the walk remembers
                    else if (tot > 0.f) { s.R[s.nrej] = tot; ++s.nrej; }    // an empty residual leaves the distribution as it is
                }
                __syncthreads();
                continue;
            }
            // the draw: inverse CDF of the current distribution in token-id order.  Sums of groups of 64 consecutive ids
            // go to LDS (a wave per group, lanes = ids); wave 0 then finds the group that holds u_emit * total (every
            // lane sums a run of groups, a scan over the lanes, then that lane's groups in order) and the id inside it.
            if (vec) {
                // a wave takes 256 ids = four groups at a time, a lane four consecutive ids, 16 lanes a group
#pragma unroll 2
                for (int sg = wave; sg * 256 < vocab; sg += 16) {
                    const int i = sg * 64 + lane;
                    float x = 0.f;
                    if (4 * i < vocab) {
                        const float4 r = current4(i);
                        x = (r.x + r.y) + (r.z + r.w);
                    }
                    for (int o = 8; o > 0; o >>= 1) x += __shfl_xor(x, o);
                    const int g = sg * 4 + (lane >> 4);
                    if ((lane & 15) == 0 && g < n_groups) s_grp[g] = x;
                }
            } else {
                for (int g = wave; g < n_groups; g += 16) {
                    const int v = g * 64 + lane;
                    float r = v < vocab ? current(v) : 0.f;
                    for (int o = 32; o > 0; o >>= 1) r += __shfl_xor(r, o);
                    if (lane == 0) s_grp[g] = r;
                }
            }
            __syncthreads();
            if (wave == 0) {
                const int gpl = (n_groups + 63) >> 6;                        // groups per lane
                float ls = 0.f;
                for (int i = 0; i < gpl; ++i) {
                    const int g = lane * gpl + i;
                    ls += g < n_groups ? s_grp[g] : 0.f;
                }
                float inc = ls;                                              // inclusive scan over the lanes
                for (int o = 1; o < 64; o <<= 1) {
                    const float y = __shfl_up(inc, o);
                    if (lane >= o) inc += y;
                }
                const float target = u_emit[b] * __shfl(inc, 63);
                const unsigned long long hit = __ballot(target < inc);
                const int L = hit ? __ffsll((long long)hit) - 1 : 63;
                float cum = __shfl(inc - ls, L);                             // weight before lane L's groups
                int gsel = min((L + 1) * gpl, n_groups) - 1;
                for (int i = 0; i < gpl; ++i) {                              // uniform: every lane walks lane L's groups
                    const int g = L * gpl + i;
                    if (g >= n_groups) break;
                    const float gs = s_grp[g];
                    if (target < cum + gs) { gsel = g; break; }
                    cum += gs;
                }
                const int v = gsel * 64 + lane;
                const float w = v < vocab ? current(v) : 0.f;
                float winc = w;
                for (int o = 1; o < 64; o <<= 1) {
                    const float y = __shfl_up(winc, o);
                    if (lane >= o) winc += y;
                }
                const unsigned long long first = __ballot(target < cum + winc && w > 0.f), any = __ballot(w > 0.f);
                int pick;
                if (first) pick = gsel * 64 + __ffsll((long long)first) - 1;
                else if (any) pick = gsel * 64 + 63 - __clzll((long long)any);       // rounding at the very end: the last id with weight
                else pick = min(gsel * 64, vocab - 1);
                if (lane == 0) s_pick = pick;
            }
            __syncthreads();
            tok = s_pick;
            break;
        }
    }
    __syncthreads();
    if (t < SEV_MAX_DRAFT) pend_path[(size_t)slot * SEV_MAX_DRAFT + t] = t < s.a ? s.path[t] : -1;
    if (path_out && t < k_max) path_out[(size_t)b * k_max + t] = t < s.a ? s.path[t] : -1;
    if (t == 0) {
        const int a = s.a;
        pend_n[slot] = n;
        pend_a[slot] = a;
        pend_bonus[slot] = tok;
        accept_len[b] = a;
        emitted[b] = tok;
    }
}

void launch_sample(const sev_kv *kv, int B, int k_max, int rows, const int32_t *tokens, const int32_t *parents, const float *logits,
                   const float *draft_probs, float2 *stats, float temperature, const float *u_acc, const float *u_emit,
                   int32_t *accept_len, int32_t *emitted, int32_t *accept_path, hipStream_t st) {
    const int vocab = kv->model->d.vocab;
    const float inv_t = 1.0f / temperature;
    hipLaunchKernelGGL(softmax_stats_kernel, dim3(rows), dim3(1024), 0, st, logits, vocab, inv_t, stats);
    hipLaunchKernelGGL(sample_walk_kernel, dim3(B), dim3(1024), (size_t)((vocab + 63) / 64) * 4, st, kv->plan, k_max, tokens, parents, logits, draft_probs, stats, vocab,
                       inv_t, u_acc, u_emit, kv->next_tok, kv->err_flags, kv->pend_n, kv->pend_a, kv->pend_bonus, kv->pend_path, accept_len,
                       emitted, accept_path);
}

KvGeom sev_kv_geom(const sev_kv *kv);

void launch_commit(const sev_kv *kv, const int32_t *slots, int B, bool rollback, hipStream_t st) {
    SlotList sl;
    for (int b = 0; b < B; ++b) sl.s[b] = slots ? slots[b] : b;
    KvGeom g = sev_kv_geom(kv);
    if (!rollback) {
        const int n = g.L * g.Hkv * g.hd;
        dim3 grid((n + 255) / 256, B);
        if (kv->model->d.dtype == SEV_BF16)
            hipLaunchKernelGGL((commit_copy_kernel<uint16_t, true>), grid, dim3(256), 0, st, sl, g, kv->page_table,
                               kv->max_pages_per_req, kv->pend_n, kv->pend_a, kv->pend_P, kv->pend_path);
        else
            hipLaunchKernelGGL((commit_copy_kernel<float, false>), grid, dim3(256), 0, st, sl, g, kv->page_table,
                               kv->max_pages_per_req, kv->pend_n, kv->pend_a, kv->pend_P, kv->pend_path);
    }
    hipLaunchKernelGGL(commit_state_kernel, dim3((B + 63) / 64), dim3(64), 0, st, sl, B, rollback ? 1 : 0, kv->seq_len,
                       kv->next_tok, kv->pend_n, kv->pend_a, kv->pend_bonus);
}

// ---------------------------------------------------------------------------
// cache import / export: plain [n][Hkv][hd] <-> paged layout
// ---------------------------------------------------------------------------
template <typename T, bool BF16>
__global__ void kv_copy_kernel(KvGeom g, const int32_t *pt, int layer, int start, int n, T *k, T *v, int to_cache) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)n * g.Hkv * g.hd;
    if (idx >= total) return;
    const int e = (int)(idx % g.hd), h = (int)((idx / g.hd) % g.Hkv), t = (int)(idx / ((int64_t)g.hd * g.Hkv));
    const int tok = start + t;
    const size_t blk = (size_t)SEV_PAGE * g.hd;
    const size_t pb = ((size_t)pt[tok / SEV_PAGE] * g.Hkv + h) * blk;
    T *kp = (T *)(g.pool + (size_t)layer * g.layer_stride) + pb + k_in_page<BF16>(tok % SEV_PAGE, e, g.hd);
    T *vp = (T *)(g.pool + (size_t)layer * g.layer_stride + g.v_offset) + pb + v_in_page<BF16>(tok % SEV_PAGE, e, g.hd);
    if (to_cache) { *kp = k[idx]; *vp = v[idx]; }
    else { k[idx] = *kp; v[idx] = *vp; }
}

void launch_kv_copy(const sev_kv *kv, int slot, int layer, int start, int n, void *k, void *v, int to_cache,
                    hipStream_t st) {
    KvGeom g = sev_kv_geom(kv);
    const int64_t total = (int64_t)n * g.Hkv * g.hd;
    if (total == 0) return;
    const int32_t *pt = kv->page_table + (size_t)slot * kv->max_pages_per_req;
    dim3 grid((unsigned)((total + 255) / 256));
    if (kv->model->d.dtype == SEV_BF16)
        hipLaunchKernelGGL((kv_copy_kernel<uint16_t, true>), grid, dim3(256), 0, st, g, pt, layer, start, n,
                           (uint16_t *)k, (uint16_t *)v, to_cache);
    else
        hipLaunchKernelGGL((kv_copy_kernel<float, false>), grid, dim3(256), 0, st, g, pt, layer, start, n, (float *)k,
                           (float *)v, to_cache);
}

// ---------------------------------------------------------------------------
// row-wise arg-max over materialised logits (lowest index wins ties)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float *logits, int vocab, int32_t *out) {
    __shared__ float sv[256];
    __shared__ int si[256];
    const float *row = logits + (size_t)blockIdx.x * vocab;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < vocab; i += 256) {
        const float v = row[i];
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
    if (threadIdx.x == 0) out[blockIdx.x] = si[0];
}

void launch_argmax_rows_f32(const float *logits, int rows, int vocab, int32_t *out, hipStream_t st) {
    hipLaunchKernelGGL(argmax_rows_kernel, dim3(rows), dim3(256), 0, st, logits, vocab, out);
}
