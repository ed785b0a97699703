// Host side of libsev: handles, argument validation, weight arena and workspace layout, and the
// launch sequence of one verification step.  All arithmetic of the method runs in the kernels.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "sev_internal.h"
#include "kv_layout.h"

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int sev_fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char *sev_last_error(void) { return g_err; }

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int static_scratch(void **out);      // device address of the static scratch array on the current device

// ---------------------------------------------------------------------------
// model
// ---------------------------------------------------------------------------
static int check_desc(const sev_model_desc *d) {
    if (!d) return sev_fail(SEV_EINVAL, "null model description");
    if (d->n_layers < 1 || d->d_model < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 2 ||
        d->d_ffn < 1 || d->vocab < 1)
        return sev_fail(SEV_EINVAL, "model dimensions must be positive");
    if (d->n_q_heads % d->n_kv_heads) return sev_fail(SEV_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    if (d->head_dim % 2) return sev_fail(SEV_EINVAL, "head_dim must be even");
    if (!(d->rope_base > 1.0f) || !(d->rms_eps >= 0.0f)) return sev_fail(SEV_EINVAL, "bad rope_base / rms_eps");
    if (d->dtype == SEV_F32) {
        if (d->head_dim > 256) return sev_fail(SEV_EINVAL, "float32 path supports head_dim <= 256");
    } else if (d->dtype == SEV_BF16) {
        if (d->head_dim != 128) return sev_fail(SEV_EINVAL, "bfloat16 path requires head_dim 128");
        if (d->d_model % 64 || d->d_ffn % 64 || (d->n_q_heads * d->head_dim) % 64)
            return sev_fail(SEV_EINVAL, "bfloat16 path requires d_model, d_ffn and n_q_heads*head_dim to be multiples of 64");
        if (d->vocab % 32) return sev_fail(SEV_EINVAL, "bfloat16 path requires vocab to be a multiple of 32");
        if ((d->n_q_heads / d->n_kv_heads) > 16) return sev_fail(SEV_EINVAL, "at most 16 query heads per KV head");
    } else {
        return sev_fail(SEV_EINVAL, "dtype must be SEV_F32 or SEV_BF16");
    }
    return SEV_OK;
}

static size_t layout_model(const sev_model_desc &d, sev_model *m) {
    const size_t esz = d.dtype == SEV_F32 ? 4 : 2;
    const size_t q_dim = (size_t)d.n_q_heads * d.head_dim, kv_dim = (size_t)d.n_kv_heads * d.head_dim;
    const size_t n_qkv = q_dim + 2 * kv_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    size_t off_embed = take((size_t)d.vocab * d.d_model * esz);
    size_t off_lm = take((size_t)d.vocab * d.d_model * esz);
    size_t off_gfinal = take((size_t)d.d_model * 4);
    if (m) {
        m->off_embed = off_embed;
        m->off_lm = off_lm;
        m->off_gfinal = off_gfinal;
        m->layers.resize(d.n_layers);
        m->n_qkv = (int)n_qkv;
        m->q_dim = (int)q_dim;
        m->kv_dim = (int)kv_dim;
    }
    for (int l = 0; l < d.n_layers; ++l) {
        LayerOffsets lo;
        lo.wqkv = take(n_qkv * d.d_model * esz);
        lo.wo = take((size_t)d.d_model * q_dim * esz);
        lo.wgu = take((size_t)2 * d.d_ffn * d.d_model * esz);
        lo.wd = take((size_t)d.d_model * d.d_ffn * esz);
        lo.g_attn = take((size_t)d.d_model * 4);
        lo.g_ffn = take((size_t)d.d_model * 4);
        if (m) m->layers[l] = lo;
    }
    return off;
}

extern "C" size_t sev_model_arena_bytes(const sev_model_desc *desc) {
    if (check_desc(desc) != SEV_OK) return 0;
    return layout_model(*desc, nullptr);
}

extern "C" int sev_model_create(const sev_model_desc *desc, void *arena, size_t arena_bytes, sev_model **out) {
    if (!out) return sev_fail(SEV_EINVAL, "null output handle");
    *out = nullptr;
    int rc = check_desc(desc);
    if (rc) return rc;
    if (!arena || ((uintptr_t)arena & 255)) return sev_fail(SEV_EINVAL, "arena must be a 256-byte aligned device pointer");
    sev_model *m = new (std::nothrow) sev_model();
    if (!m) return sev_fail(SEV_ENOSPACE, "host allocation failed");
    m->d = *desc;
    m->arena = (char *)arena;
    m->arena_bytes = arena_bytes;
    const size_t need = layout_model(*desc, m);
    if (arena_bytes < need) {
        delete m;
        return sev_fail(SEV_ENOSPACE, "arena too small: %zu < %zu bytes", arena_bytes, need);
    }
    launch_fill_f32((float *)(m->arena + m->off_gfinal), 1.0f, desc->d_model, 0);
    for (int l = 0; l < desc->n_layers; ++l) {
        launch_fill_f32((float *)(m->arena + m->layers[l].g_attn), 1.0f, desc->d_model, 0);
        launch_fill_f32((float *)(m->arena + m->layers[l].g_ffn), 1.0f, desc->d_model, 0);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        delete m;
        return sev_fail(SEV_EHIP, "initialising norm gains: %s", hipGetErrorString(e));
    }
    *out = m;
    return SEV_OK;
}

extern "C" int sev_model_destroy(sev_model *m) {
    delete m;
    return SEV_OK;
}

extern "C" int sev_model_load_tensor(sev_model *m, int kind, int layer, const void *src, void *stream) {
    if (!m || !src) return sev_fail(SEV_EINVAL, "null model or source");
    const sev_model_desc &d = m->d;
    hipStream_t st = (hipStream_t)stream;
    const bool per_layer = !(kind == SEV_W_EMBED || kind == SEV_W_LM_HEAD || kind == SEV_W_NORM_FINAL);
    if (per_layer && (layer < 0 || layer >= d.n_layers)) return sev_fail(SEV_EINVAL, "layer %d out of range", layer);
    const LayerOffsets *lo = per_layer ? &m->layers[layer] : nullptr;
    // norm gains: float32 vectors in both precisions
    if (kind == SEV_W_NORM_ATTN || kind == SEV_W_NORM_FFN || kind == SEV_W_NORM_FINAL) {
        size_t off = kind == SEV_W_NORM_FINAL ? m->off_gfinal : (kind == SEV_W_NORM_ATTN ? lo->g_attn : lo->g_ffn);
        launch_pack_f32((float *)(m->arena + off), (const float *)src, d.d_model, st);
        return SEV_OK;
    }
    // destination matrix (possibly a row range of a fused matrix): rows, K, row offset
    size_t off;
    int rows, K, row0 = 0, mode = 0;
    switch (kind) {
    case SEV_W_EMBED: off = m->off_embed; rows = d.vocab; K = d.d_model; break;
    case SEV_W_LM_HEAD: off = m->off_lm; rows = d.vocab; K = d.d_model; break;
    // q, k, v rows: rotary partners interleaved inside each head's tiles of the bf16 layout
    case SEV_W_WQ: off = lo->wqkv; rows = m->q_dim; K = d.d_model; mode = 3; break;
    case SEV_W_WK: off = lo->wqkv; rows = m->kv_dim; K = d.d_model; row0 = m->q_dim; mode = 3; break;
    case SEV_W_WV: off = lo->wqkv; rows = m->kv_dim; K = d.d_model; row0 = m->q_dim + m->kv_dim; mode = 3; break;
    case SEV_W_WO: off = lo->wo; rows = d.d_model; K = m->q_dim; break;
    // gate and up rows are interleaved in 4-row groups inside each 32-row tile of the bf16 layout
    case SEV_W_WG: off = lo->wgu; rows = d.d_ffn; K = d.d_model; mode = 1; break;
    case SEV_W_WU: off = lo->wgu; rows = d.d_ffn; K = d.d_model; mode = 2; row0 = d.d_ffn; break;
    case SEV_W_WD: off = lo->wd; rows = d.d_model; K = d.d_ffn; break;
    default: return sev_fail(SEV_EINVAL, "unknown tensor kind %d", kind);
    }
    if (d.dtype == SEV_F32) {
        launch_pack_f32((float *)(m->arena + off) + (size_t)row0 * K, (const float *)src, (int64_t)rows * K, st);
    } else if (kind == SEV_W_EMBED) {
        SEV_HIP(hipMemcpyAsync(m->arena + off, src, (size_t)rows * K * 2, hipMemcpyDeviceToDevice, st));
    } else {
        // bf16 matrices are re-tiled into 32x16 MFMA operand fragments; a row offset inside a fused
        // matrix is a tile offset (all offsets are multiples of 32 by construction of the shapes)
        if (rows % 32 || row0 % 32 || K % 16) return sev_fail(SEV_EINVAL, "tensor %d: rows/K not tileable", kind);
        launch_pack_bf16((uint16_t *)(m->arena + off), (const uint16_t *)src, rows, K, mode, (mode == 0 || mode == 3) ? row0 / 32 : 0, st);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return sev_fail(SEV_EHIP, "load_tensor: %s", hipGetErrorString(e));
    return SEV_OK;
}

// ---------------------------------------------------------------------------
// KV cache
// ---------------------------------------------------------------------------
static size_t kv_block_bytes(const sev_model_desc &d) {
    return (size_t)SEV_PAGE * d.head_dim * (d.dtype == SEV_F32 ? 4 : 2);
}

extern "C" size_t sev_kv_pool_bytes(const sev_model *m, int64_t n_pages, int page_size) {
    if (!m || n_pages < 1 || page_size != SEV_PAGE) return 0;
    return (size_t)m->d.n_layers * 2 * (size_t)n_pages * m->d.n_kv_heads * kv_block_bytes(m->d);
}

KvGeom sev_kv_geom(const sev_kv *kv) {
    KvGeom g;
    g.pool = kv->pool;
    g.layer_stride = kv->layer_stride;
    g.v_offset = kv->v_offset;
    g.L = kv->model->d.n_layers;
    g.Hkv = kv->model->d.n_kv_heads;
    g.hd = kv->model->d.head_dim;
    return g;
}

#define ATT_ITEMS_CAP 4096

static void read_tune(Tune *t) {
    static const char *names[5] = {"SEV_TUNE_QKV", "SEV_TUNE_O", "SEV_TUNE_GU", "SEV_TUNE_DOWN", "SEV_TUNE_LM"};
    memset(t, 0, sizeof(*t));
    for (int i = 0; i < 5; ++i)
        if (const char *e = getenv(names[i]))
            t->has_gemm[i] = sscanf(e, "%d,%d,%d,%d", &t->gemm[i][0], &t->gemm[i][1], &t->gemm[i][2], &t->gemm[i][3]) == 4;
    if (const char *e = getenv("SEV_TUNE_TPB")) t->tpb = atoi(e);
    if (const char *e = getenv("SEV_TUNE_CP")) t->cp = atoi(e);
}

extern "C" int sev_kv_create(const sev_model *m, int max_requests, int max_rows, int64_t n_pages, int page_size,
                             void *pool, size_t pool_bytes, sev_kv **out) {
    if (!out) return sev_fail(SEV_EINVAL, "null output handle");
    *out = nullptr;
    if (!m) return sev_fail(SEV_EINVAL, "null model");
    if (page_size != SEV_PAGE) return sev_fail(SEV_EINVAL, "page_size must be %d", SEV_PAGE);
    if (max_requests < 1 || max_requests > 65536 || max_rows < 1 || max_rows > (1 << 20) || n_pages < 1 ||
        n_pages > (1 << 26))
        return sev_fail(SEV_EINVAL, "max_requests / max_rows / n_pages out of range");
    if (!pool || ((uintptr_t)pool & 255)) return sev_fail(SEV_EINVAL, "pool must be a 256-byte aligned device pointer");
    const size_t need = sev_kv_pool_bytes(m, n_pages, page_size);
    if (pool_bytes < need) return sev_fail(SEV_ENOSPACE, "pool too small: %zu < %zu bytes", pool_bytes, need);
    sev_kv *kv = new (std::nothrow) sev_kv();
    if (!kv) return sev_fail(SEV_ENOSPACE, "host allocation failed");
    const sev_model_desc &d = m->d;
    kv->model = m;
    kv->max_req = max_requests;
    kv->max_rows = max_rows;
    kv->page_size = page_size;
    kv->n_pages = n_pages;
    kv->pool = (char *)pool;
    kv->pool_bytes = pool_bytes;
    kv->v_offset = (size_t)n_pages * d.n_kv_heads * kv_block_bytes(d);
    kv->layer_stride = 2 * kv->v_offset;
    kv->max_pages_per_req = (int)n_pages;
    read_tune(&kv->tune);
    kv->prof_on = 0;
    memset(kv->prof_ms, 0, sizeof(kv->prof_ms));
    memset(kv->prof_n, 0, sizeof(kv->prof_n));
    kv->host_pages.assign(max_requests, 0);

    const bool bf = d.dtype == SEV_BF16;
    const size_t rows_pad = align_up((size_t)max_rows, 128);
    const int G = d.n_q_heads / d.n_kv_heads;
    kv->max_items = bf ? ATT_ITEMS_CAP : 1;
    kv->max_groups = bf ? (int)(rows_pad * G / 32 + SEV_MAX_BATCH) : 1;
    const size_t n_qkv = m->n_qkv;
    kv->part_elems = rows_pad * std::max<size_t>(16 * std::max<size_t>(n_qkv, d.d_model), 4 * (size_t)d.d_ffn);

    // carve the workspace
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    const size_t o_pt = take((size_t)max_requests * kv->max_pages_per_req * 4);
    const size_t o_seq = take((size_t)max_requests * 4), o_nt = take((size_t)max_requests * 4);
    const size_t o_pn = take((size_t)max_requests * 4), o_pa = take((size_t)max_requests * 4);
    const size_t o_pb = take((size_t)max_requests * 4), o_pP = take((size_t)max_requests * 4);
    const size_t o_pp = take((size_t)max_requests * SEV_MAX_DRAFT * 4);
    const size_t o_err = take(4);
    const size_t o_rq = take(4 * (size_t)(SEV_MAX_BATCH + 1) * 4);
    const size_t o_row = take(5 * rows_pad * 4);
    const size_t o_anc = take(rows_pad * 8);
    const size_t o_cs = take(rows_pad * (d.head_dim / 2) * 8);
    const size_t o_it = take((size_t)kv->max_items * (32 + SEV_ATT_MAX_CP * 4));
    const size_t o_mg = take(4 * (size_t)kv->max_groups * 4);
    const size_t o_h = take(rows_pad * d.d_model * 4);
    const size_t o_part = take(kv->part_elems * 4);
    const size_t o_xa = take(rows_pad * d.d_model * 4);
    const size_t o_q = take(rows_pad * n_qkv * 4);
    const size_t o_o = take(rows_pad * m->q_dim * 4);
    const size_t o_act = take(rows_pad * d.d_ffn * 4);
    const size_t o_ao = take(bf ? (size_t)kv->max_items * d.n_kv_heads * 32 * d.head_dim * 4 : 4);
    const size_t o_ml = take(bf ? (size_t)kv->max_items * d.n_kv_heads * 32 * 8 : 4);
    const size_t o_lv = take(bf ? (size_t)(d.vocab / 32 + 4) * rows_pad * 4 : 4);
    const size_t o_li = take(bf ? (size_t)(d.vocab / 32 + 4) * rows_pad * 4 : 4);
    const size_t o_am = take(rows_pad * 4);
    const size_t o_lg = take(bf ? 4 : rows_pad * (size_t)d.vocab * 4);
    const size_t o_ssq = take(2 * rows_pad * 8);
    const size_t o_tmp = take(2 * SEV_MAX_BATCH * 4);
    const size_t o_rst = take(rows_pad * 8);
    kv->ws_bytes = off;
    hipError_t e = hipMalloc((void **)&kv->ws, kv->ws_bytes);
    if (e != hipSuccess) {
        delete kv;
        return sev_fail(SEV_EHIP, "workspace allocation of %zu bytes failed: %s", off, hipGetErrorString(e));
    }
    e = hipMemset(kv->ws, 0, kv->ws_bytes);
    if (e != hipSuccess) {
        hipFree(kv->ws);
        delete kv;
        return sev_fail(SEV_EHIP, "workspace clear failed: %s", hipGetErrorString(e));
    }
    char *w = kv->ws;
    kv->page_table = (int32_t *)(w + o_pt);
    kv->seq_len = (int32_t *)(w + o_seq);
    kv->next_tok = (int32_t *)(w + o_nt);
    kv->pend_n = (int32_t *)(w + o_pn);
    kv->pend_a = (int32_t *)(w + o_pa);
    kv->pend_bonus = (int32_t *)(w + o_pb);
    kv->pend_P = (int32_t *)(w + o_pP);
    kv->pend_path = (int32_t *)(w + o_pp);
    kv->err_flags = (uint32_t *)(w + o_err);
    int32_t *rq = (int32_t *)(w + o_rq);
    kv->plan.req_slot = rq;
    kv->plan.req_P = rq + (SEV_MAX_BATCH + 1);
    kv->plan.req_n = rq + 2 * (SEV_MAX_BATCH + 1);
    kv->plan.req_row0 = rq + 3 * (SEV_MAX_BATCH + 1);
    int32_t *rw = (int32_t *)(w + o_row);
    kv->plan.row_req = rw;
    kv->plan.row_node = rw + rows_pad;
    kv->plan.row_pos = rw + 2 * rows_pad;
    kv->plan.row_tok = rw + 3 * rows_pad;
    kv->plan.row_kvloc = rw + 4 * rows_pad;
    kv->plan.row_anc = (unsigned long long *)(w + o_anc);
    kv->plan.row_cs = (float2 *)(w + o_cs);
    kv->plan.it_a = (int4 *)(w + o_it);
    kv->plan.it_b = kv->plan.it_a + kv->max_items;
    kv->plan.it_pages = (int32_t *)(kv->plan.it_b + kv->max_items);
    kv->plan.mg_rec = (int4 *)(w + o_mg);
    kv->h = (float *)(w + o_h);
    kv->part = (float *)(w + o_part);
    kv->xa = w + o_xa;
    kv->q_buf = w + o_q;
    kv->o_buf = w + o_o;
    kv->act = w + o_act;
    kv->att_o = (float *)(w + o_ao);
    kv->att_ml = (float2 *)(w + o_ml);
    kv->lm_val = (float *)(w + o_lv);
    kv->lm_idx = (int32_t *)(w + o_li);
    kv->row_argmax = (int32_t *)(w + o_am);
    kv->logits_f32 = (float *)(w + o_lg);
    kv->row_stats = (float2 *)(w + o_rst);
    kv->tmp_accept = (int32_t *)(w + o_tmp);
    kv->tmp_bonus = kv->tmp_accept + SEV_MAX_BATCH;
    kv->ssq[0] = (unsigned long long *)(w + o_ssq);
    kv->ssq[1] = kv->ssq[0] + rows_pad;
    launch_fill_i32(kv->next_tok, -1, max_requests, 0);
    {   // set-up for sev_verify_sample_static: look the static scratch up for this device now (a failure only
        // matters to that entry point, which reports it)
        void *unused = nullptr;
        (void)static_scratch(&unused);
    }
    e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        hipFree(kv->ws);
        delete kv;
        return sev_fail(SEV_EHIP, "workspace initialisation failed: %s", hipGetErrorString(e));
    }
    *out = kv;
    return SEV_OK;
}

extern "C" int sev_kv_destroy(sev_kv *kv) {
    if (!kv) return SEV_OK;
    for (auto &s : kv->spans) {
        hipEventDestroy(s.a);
        hipEventDestroy(s.b);
    }
    hipFree(kv->ws);
    delete kv;
    return SEV_OK;
}

extern "C" int sev_kv_set_pages(sev_kv *kv, int slot, const int32_t *page_ids, int n_pages, void *stream) {
    if (!kv) return sev_fail(SEV_EINVAL, "null cache");
    if (slot < 0 || slot >= kv->max_req) return sev_fail(SEV_EINVAL, "slot %d out of range", slot);
    if (n_pages < 0 || n_pages > kv->max_pages_per_req || (n_pages && !page_ids))
        return sev_fail(SEV_EINVAL, "bad page list");
    for (int i = 0; i < n_pages; ++i)
        if (page_ids[i] < 0 || page_ids[i] >= kv->n_pages)
            return sev_fail(SEV_EINVAL, "page id %d out of range at index %d", page_ids[i], i);
    if (n_pages)
        SEV_HIP(hipMemcpyAsync(kv->page_table + (size_t)slot * kv->max_pages_per_req, page_ids, (size_t)n_pages * 4,
                               hipMemcpyHostToDevice, (hipStream_t)stream));
    kv->host_pages[slot] = n_pages;
    return SEV_OK;
}

struct StateArgs {
    int32_t slot[SEV_MAX_BATCH], len[SEV_MAX_BATCH], nt[SEV_MAX_BATCH];
};

__global__ void set_state_kernel(StateArgs a, int B, int32_t *seq_len, int32_t *next_tok, int32_t *pend_n) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    seq_len[a.slot[b]] = a.len[b];
    next_tok[a.slot[b]] = a.nt[b];
    pend_n[a.slot[b]] = 0;
}

extern "C" int sev_kv_set_state(sev_kv *kv, const int32_t *slots, const int32_t *seq_lens, const int32_t *next_toks,
                                int B, void *stream) {
    if (!kv || !seq_lens || !next_toks) return sev_fail(SEV_EINVAL, "null argument");
    if (B < 1 || B > SEV_MAX_BATCH) return sev_fail(SEV_EINVAL, "B=%d outside 1..%d", B, SEV_MAX_BATCH);
    StateArgs a;
    for (int b = 0; b < B; ++b) {
        const int slot = slots ? slots[b] : b;
        if (slot < 0 || slot >= kv->max_req) return sev_fail(SEV_EINVAL, "slot %d out of range", slot);
        if (seq_lens[b] < 0 || (int64_t)seq_lens[b] > (int64_t)kv->host_pages[slot] * SEV_PAGE)
            return sev_fail(SEV_ENOSPACE, "length %d exceeds the %d pages of slot %d", seq_lens[b], kv->host_pages[slot], slot);
        if (next_toks[b] < -1 || next_toks[b] >= kv->model->d.vocab) return sev_fail(SEV_EINVAL, "next_tok out of range");
        a.slot[b] = slot;
        a.len[b] = seq_lens[b];
        a.nt[b] = next_toks[b];
    }
    hipLaunchKernelGGL(set_state_kernel, dim3((B + 63) / 64), dim3(64), 0, (hipStream_t)stream, a, B, kv->seq_len,
                       kv->next_tok, kv->pend_n);
    SEV_HIP(hipGetLastError());
    return SEV_OK;
}

extern "C" int sev_kv_get_state(sev_kv *kv, int slot, int32_t *seq_len, int32_t *next_tok, uint32_t *error_flags,
                                void *stream) {
    if (!kv) return sev_fail(SEV_EINVAL, "null cache");
    if (slot < 0 || slot >= kv->max_req) return sev_fail(SEV_EINVAL, "slot %d out of range", slot);
    hipStream_t st = (hipStream_t)stream;
    int32_t a = 0, b = 0;
    uint32_t f = 0;
    SEV_HIP(hipMemcpyAsync(&a, kv->seq_len + slot, 4, hipMemcpyDeviceToHost, st));
    SEV_HIP(hipMemcpyAsync(&b, kv->next_tok + slot, 4, hipMemcpyDeviceToHost, st));
    SEV_HIP(hipMemcpyAsync(&f, kv->err_flags, 4, hipMemcpyDeviceToHost, st));
    SEV_HIP(hipStreamSynchronize(st));
    if (seq_len) *seq_len = a;
    if (next_tok) *next_tok = b;
    if (error_flags) *error_flags = f;
    return SEV_OK;
}

extern "C" int sev_kv_copy_tokens(sev_kv *kv, int slot, int layer, int start, int n_tokens, void *k, void *v,
                                  int to_cache, void *stream) {
    if (!kv || !k || !v) return sev_fail(SEV_EINVAL, "null argument");
    if (slot < 0 || slot >= kv->max_req) return sev_fail(SEV_EINVAL, "slot %d out of range", slot);
    if (layer < 0 || layer >= kv->model->d.n_layers) return sev_fail(SEV_EINVAL, "layer %d out of range", layer);
    if (start < 0 || n_tokens < 0) return sev_fail(SEV_EINVAL, "negative range");
    if ((int64_t)start + n_tokens > (int64_t)kv->host_pages[slot] * SEV_PAGE)
        return sev_fail(SEV_ENOSPACE, "tokens %d..%d exceed the %d pages of slot %d", start, start + n_tokens,
                        kv->host_pages[slot], slot);
    launch_kv_copy(kv, slot, layer, start, n_tokens, k, v, to_cache, (hipStream_t)stream);
    SEV_HIP(hipGetLastError());
    return SEV_OK;
}

// ---------------------------------------------------------------------------
// profiling spans
// ---------------------------------------------------------------------------
Prof::Prof(sev_kv *kv_, hipStream_t st_, int cls_) : kv(kv_), st(st_), cls(cls_), a(nullptr), b(nullptr), on(false) {
    if (!((kv->prof_on >> cls_) & 1)) return;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
    on = true;
    hipEventRecord(a, st);
}
Prof::~Prof() {
    if (!on) return;
    hipEventRecord(b, st);
    kv->spans.push_back({a, b, cls});
}

static void prof_collect(sev_kv *kv) {
    for (auto &s : kv->spans) {
        hipEventSynchronize(s.b);
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, s.a, s.b) == hipSuccess) {
            kv->prof_ms[s.cls] += ms;
            kv->prof_n[s.cls] += 1;
        }
        hipEventDestroy(s.a);
        hipEventDestroy(s.b);
    }
    kv->spans.clear();
}

extern "C" int sev_profile_enable(sev_kv *kv, unsigned class_mask) {
    if (!kv) return sev_fail(SEV_EINVAL, "null cache");
    prof_collect(kv);
    kv->prof_on = (int)(class_mask & ((1u << PROF_N) - 1));
    memset(kv->prof_ms, 0, sizeof(kv->prof_ms));
    memset(kv->prof_n, 0, sizeof(kv->prof_n));
    return SEV_OK;
}

extern "C" int sev_profile_read(sev_kv *kv, int which, double *total_ms, int64_t *launches) {
    if (!kv || which < 0 || which >= PROF_N) return sev_fail(SEV_EINVAL, "bad profile class");
    prof_collect(kv);
    if (total_ms) *total_ms = kv->prof_ms[which];
    if (launches) *launches = kv->prof_n[which];
    return SEV_OK;
}

extern "C" const char *sev_profile_name(int which) {
    static const char *names[PROF_N] = {"gemm_qkv", "gemm_o", "gemm_gate_up_swiglu", "gemm_down", "gemm_lm_head_argmax",
                                        "attention", "other"};
    return (which >= 0 && which < PROF_N) ? names[which] : nullptr;
}

// ---------------------------------------------------------------------------
// verify
// ---------------------------------------------------------------------------
// Pages per attention chunk.  Every (request, row group, chunk, KV head) is one block with a fixed cost
// of several microseconds (work item and page list, query fragments, wave merge, partial result) on
// top of its page pairs, and all blocks start together: the shortest kernel is the one whose blocks
// all run at once, one per compute unit, with chunks as small as that allows (measured on the
// 8B-shape workloads).  Work lists that do not fit even with the largest chunks fall back to 64-page
// chunks.  The pages of a request are then split evenly over its chunks.
static int pick_chunk_pages(const sev_kv *kv, const PlanArgs &pa, int *n_items, int *n_groups, int *sib, bool *direct) {
    const sev_model_desc &d = kv->model->d;
    const int G = d.n_q_heads / d.n_kv_heads;
    static int n_cu = 0;
    if (!n_cu) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
            v = 256;
        n_cu = v;
    }
    int64_t total_groups = 0;
    for (int b = 0; b < pa.B; ++b) total_groups += (G * pa.nd[b] + 31) / 32;
    // row groups per request when all requests have the same number (the attention kernel then keeps the groups that
    // share a KV chunk on one XCD), else 1
    *sib = (G * pa.nd[0] + 31) / 32;
    for (int b = 1; b < pa.B; ++b)
        if ((G * pa.nd[b] + 31) / 32 != *sib) *sib = 1;
    if (*sib > 127) *sib = 1;
    auto items_for = [&](int64_t cp) {
        int64_t items = 0;
        for (int b = 0; b < pa.B; ++b) {
            const int64_t pages = (std::max(pa.prefix[b] + pa.nd[b], pa.pad_tokens) + SEV_PAGE - 1) / SEV_PAGE;
            items += ((G * pa.nd[b] + 31) / 32) * ((pages + cp - 1) / cp);
        }
        return items;
    };
    // Whole sequences: when every request is short (64 pages: at most 4 page pairs per wave) and there are
    // enough (request, row group, KV head) blocks for half the chip, a block of 8 waves takes the whole
    // sequence and writes the attention output itself: no partial results, no merge kernel.  Longer
    // sequences are faster split over several compute units (measured on the 8B-shape workloads: one
    // compute unit needs about 0.75 us per page pair and SIMD).
    *direct = false;
    int64_t max_pages = 0;
    for (int b = 0; b < pa.B; ++b)
        max_pages = std::max<int64_t>(max_pages, (std::max(pa.prefix[b] + pa.nd[b], pa.pad_tokens) + SEV_PAGE - 1) / SEV_PAGE);
    if (!kv->tune.cp && max_pages <= 64 && total_groups * d.n_kv_heads * 2 >= n_cu &&
        total_groups <= kv->max_items) {
        *direct = true;
        *n_items = (int)total_groups;
        *n_groups = (int)total_groups;
        return SEV_ATT_MAX_CP;
    }
    int64_t cp = 0;
    for (int64_t c = 8; c <= SEV_ATT_MAX_CHUNK; c += 8)
        if (items_for(c) * d.n_kv_heads <= (int64_t)n_cu) { cp = c; break; }
    if (!cp) cp = 64;
    if (kv->tune.cp >= 2 && kv->tune.cp <= SEV_ATT_MAX_CHUNK) cp = kv->tune.cp;      // tuning experiments: pages per attention chunk
    for (;; cp = std::min<int64_t>(cp * 2, SEV_ATT_MAX_CHUNK)) {
        const int64_t items = items_for(cp);
        if (items <= kv->max_items) {
            *n_items = (int)items;
            *n_groups = (int)total_groups;
            return (int)cp;
        }
        if (cp >= SEV_ATT_MAX_CHUNK) return -1;
    }
}

// One block forward: the shared body of sev_verify_ex and sev_prefill.  The caller has checked the
// public limits; here: slots, capacity, row budget.
struct BlockCall {
    const int32_t *slots, *prefix_lens, *lens;   // host; lens == nullptr: every request has n_all nodes
    int n_all;
    const int32_t *tokens;                       // device: node i of request b at tokens[b * tok_stride + tok_off + i]
    int tok_stride, tok_off;
    const int32_t *parents;                      // device [B][tok_stride] or nullptr (chains)
    int B, mode;
    int32_t *accept_len, *bonus_token, *accept_path, *row_argmax;
    float *logits;
    // stochastic rule (chains): set draft_probs to switch from greedy acceptance to accept / resample
    const float *draft_probs, *u_accept, *u_emit;
    float temperature;
};

static int run_block(const sev_model *m, sev_kv *kv, const BlockCall &c, hipStream_t st) {
    PlanArgs pa;
    pa.B = c.B;
    pa.k_max = c.tok_stride;
    pa.mode = c.mode & 1;
    pa.pad_tokens = 0;
    pa.tok_stride = c.tok_stride;
    pa.tok_off = c.tok_off;
    int64_t rows = 0;
    for (int b = 0; b < c.B; ++b) {
        const int slot = c.slots ? c.slots[b] : b;
        if (slot < 0 || slot >= kv->max_req) return sev_fail(SEV_EINVAL, "request %d: slot %d out of range", b, slot);
        for (int e = 0; e < b; ++e)
            if (pa.slot[e] == slot) return sev_fail(SEV_EINVAL, "slot %d listed twice", slot);
        const int n = c.lens ? c.lens[b] : c.n_all;
        const int P = c.prefix_lens[b];
        if (P < 0) return sev_fail(SEV_EINVAL, "request %d: negative prefix length", b);
        if ((int64_t)P + n > (int64_t)kv->host_pages[slot] * SEV_PAGE)
            return sev_fail(SEV_ENOSPACE, "request %d: %d+%d tokens exceed the %d pages of slot %d", b, P, n,
                            kv->host_pages[slot], slot);
        pa.slot[b] = slot;
        pa.prefix[b] = P;
        pa.nd[b] = n;
        rows += n;
    }
    if (rows > kv->max_rows) return sev_fail(SEV_ENOSPACE, "%lld tokens exceed max_rows=%d", (long long)rows, kv->max_rows);
    if (c.mode & 2) {
        // the paper's formulation of a heterogeneous batch: every sequence padded to the longest one,
        // a dense mask hiding the padding; here: every request's attention walks that many cache slots
        if (m->d.dtype != SEV_BF16) return sev_fail(SEV_EINVAL, "the padded-KV variant exists for the bfloat16 path only");
        for (int b = 0; b < c.B; ++b) pa.pad_tokens = std::max(pa.pad_tokens, pa.prefix[b] + pa.nd[b]);
        for (int b = 0; b < c.B; ++b)
            if ((int64_t)pa.pad_tokens > (int64_t)kv->host_pages[pa.slot[b]] * SEV_PAGE)
                return sev_fail(SEV_ENOSPACE, "request %d: padding to %d tokens exceeds the %d pages of slot %d", b, pa.pad_tokens,
                                kv->host_pages[pa.slot[b]], pa.slot[b]);
    }
    int n_items = 0, n_groups = 0, sib = 1, cp = 64;
    bool att_direct = false;
    if (m->d.dtype == SEV_BF16) {
        cp = pick_chunk_pages(kv, pa, &n_items, &n_groups, &sib, &att_direct);
        if (cp < 0) return sev_fail(SEV_ENOSPACE, "attention work list does not fit");
    }
    kv->plan.causal = c.parents ? 0 : 1;
    {
        Prof p(kv, st, PROF_OTHER);
        launch_plan(kv, pa, c.tokens, c.parents, (int)rows, cp, n_items, st);
    }
    if (m->d.dtype == SEV_F32) f32_forward(m, kv, (int)rows, c.B, c.logits, st);
    else bf16_forward(m, kv, (int)rows, c.B, n_items, n_groups, sib, att_direct, c.logits, st);
    {
        Prof p(kv, st, PROF_OTHER);
        if (c.draft_probs)
            launch_sample(kv, c.B, c.tok_stride, (int)rows, c.tokens, c.parents, c.logits, c.draft_probs, kv->row_stats, c.temperature,
                          c.u_accept, c.u_emit, c.accept_len, c.bonus_token, c.accept_path, st);
        else
            launch_accept(kv, c.B, c.tok_stride, c.mode & 1, c.tokens, c.parents, c.accept_len, c.bonus_token, c.accept_path, st);
        if (c.row_argmax)
            SEV_HIP(hipMemcpyAsync(c.row_argmax, kv->row_argmax, (size_t)rows * 4, hipMemcpyDeviceToDevice, st));
    }
    SEV_HIP(hipGetLastError());
    return SEV_OK;
}

extern "C" int sev_verify_ex(const sev_model *m, sev_kv *kv, const sev_verify_args *a, void *stream) {
    if (!m || !kv || !a) return sev_fail(SEV_EINVAL, "null argument");
    if (kv->model != m) return sev_fail(SEV_EINVAL, "cache was created for another model");
    if (a->B < 1 || a->B > SEV_MAX_BATCH) return sev_fail(SEV_EINVAL, "B=%d outside 1..%d", a->B, SEV_MAX_BATCH);
    if (a->k_max < 1 || a->k_max > SEV_MAX_DRAFT) return sev_fail(SEV_EINVAL, "k=%d outside 1..%d", a->k_max, SEV_MAX_DRAFT);
    if (!a->prefix_lens || !a->draft_tokens || !a->accept_len || !a->bonus_token)
        return sev_fail(SEV_EINVAL, "prefix_lens, draft_tokens, accept_len and bonus_token are required");
    if (a->mode < 0 || a->mode > 3) return sev_fail(SEV_EINVAL, "mode must be 0 (verify) or 1 (append), optionally | 2 (padded KV)");
    if ((a->mode & 1) && a->parents) return sev_fail(SEV_EINVAL, "append mode takes chains only");
    if (a->draft_lens)
        for (int b = 0; b < a->B; ++b)
            if (a->draft_lens[b] < 1 || a->draft_lens[b] > a->k_max)
                return sev_fail(SEV_EINVAL, "request %d: draft length %d outside 1..%d", b, a->draft_lens[b], a->k_max);
    BlockCall c;
    memset(&c, 0, sizeof(c));
    c.slots = a->slots; c.prefix_lens = a->prefix_lens; c.lens = a->draft_lens; c.n_all = a->k_max;
    c.tokens = a->draft_tokens; c.tok_stride = a->k_max; c.tok_off = 0; c.parents = a->parents;
    c.B = a->B; c.mode = a->mode;
    c.accept_len = a->accept_len; c.bonus_token = a->bonus_token; c.accept_path = a->accept_path;
    c.row_argmax = a->row_argmax; c.logits = a->logits;
    return run_block(m, kv, c, (hipStream_t)stream);
}

extern "C" int sev_verify_sample(const sev_model *m, sev_kv *kv, const sev_sample_args *a, void *stream) {
    if (!m || !kv || !a) return sev_fail(SEV_EINVAL, "null argument");
    if (kv->model != m) return sev_fail(SEV_EINVAL, "cache was created for another model");
    if (a->B < 1 || a->B > SEV_MAX_BATCH) return sev_fail(SEV_EINVAL, "B=%d outside 1..%d", a->B, SEV_MAX_BATCH);
    if (a->k_max < 1 || a->k_max > SEV_MAX_DRAFT) return sev_fail(SEV_EINVAL, "k=%d outside 1..%d", a->k_max, SEV_MAX_DRAFT);
    if (!a->prefix_lens || !a->draft_tokens || !a->draft_probs || !a->u_accept || !a->u_emit || !a->logits_ws || !a->accept_len ||
        !a->emitted_token)
        return sev_fail(SEV_EINVAL, "prefix_lens, draft_tokens, draft_probs, u_accept, u_emit, logits_ws, accept_len and emitted_token are required");
    if (!(a->temperature > 0.0f) || !(a->temperature < 1e4f)) return sev_fail(SEV_EINVAL, "temperature must be positive");
    if (a->draft_lens)
        for (int b = 0; b < a->B; ++b)
            if (a->draft_lens[b] < 1 || a->draft_lens[b] > a->k_max)
                return sev_fail(SEV_EINVAL, "request %d: draft length %d outside 1..%d", b, a->draft_lens[b], a->k_max);
    BlockCall c;
    memset(&c, 0, sizeof(c));
    c.slots = a->slots; c.prefix_lens = a->prefix_lens; c.lens = a->draft_lens; c.n_all = a->k_max;
    c.tokens = a->draft_tokens; c.tok_stride = a->k_max; c.tok_off = 0; c.parents = a->parents;
    c.B = a->B; c.mode = 0;
    c.accept_len = a->accept_len; c.bonus_token = a->emitted_token; c.accept_path = a->accept_path; c.logits = a->logits_ws;
    c.draft_probs = a->draft_probs; c.u_accept = a->u_accept; c.u_emit = a->u_emit; c.temperature = a->temperature;
    return run_block(m, kv, c, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------
// stochastic verification without a caller workspace: the block's logits live in a static device array
// ---------------------------------------------------------------------------
// File-scope device memory, one copy per GPU, held until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: the device address is looked up once per device (with that device current) and every
// kernel argument below uses the looked-up pointer.
static __device__ __align__(256) unsigned char sev_static_scratch[SEV_STATIC_SCRATCH_BYTES];

#define SEV_MAX_DEVICES 64
static void *g_scratch_ptr[SEV_MAX_DEVICES];     // per device; written once (same value from any thread)

static int static_scratch(void **out) {
    int dev = -1;
    SEV_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= SEV_MAX_DEVICES) return sev_fail(SEV_EINVAL, "device %d beyond the %d the static scratch table covers", dev, SEV_MAX_DEVICES);
    void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        SEV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(sev_static_scratch)));
        if (!p || ((uintptr_t)p & 255)) return sev_fail(SEV_EHIP, "static scratch: bad device address %p", p);
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return SEV_OK;
}

extern "C" int sev_verify_sample_static(const sev_model *m, sev_kv *kv, const sev_sample_args *a, void *stream) {
    if (!m || !kv || !a) return sev_fail(SEV_EINVAL, "null argument");
    if (a->B < 1 || a->B > SEV_MAX_BATCH) return sev_fail(SEV_EINVAL, "B=%d outside 1..%d", a->B, SEV_MAX_BATCH);
    if (a->k_max < 1 || a->k_max > SEV_MAX_DRAFT) return sev_fail(SEV_EINVAL, "k=%d outside 1..%d", a->k_max, SEV_MAX_DRAFT);
    if (a->logits_ws) return sev_fail(SEV_EINVAL, "logits_ws must be NULL: this entry point keeps the logits in the library's static scratch");
    if (kv->prof_on) return sev_fail(SEV_ESTATE, "per-kernel profiling creates events; switch it off for the entry point that allocates nothing");
    int64_t rows = 0;
    for (int b = 0; b < a->B; ++b) {
        const int n = a->draft_lens ? a->draft_lens[b] : a->k_max;
        if (n < 1 || n > a->k_max) return sev_fail(SEV_EINVAL, "request %d: draft length %d outside 1..%d", b, n, a->k_max);
        rows += n;
    }
    const size_t need = (size_t)rows * (size_t)m->d.vocab * sizeof(float);
    if (need > (size_t)SEV_STATIC_SCRATCH_BYTES)
        return sev_fail(SEV_ENOSPACE, "%lld rows x %d logits need %zu bytes; the static scratch holds %zu", (long long)rows, m->d.vocab, need,
                        (size_t)SEV_STATIC_SCRATCH_BYTES);
    void *scratch = nullptr;
    const int rc = static_scratch(&scratch);
    if (rc != SEV_OK) return rc;
    sev_sample_args b = *a;
    b.logits_ws = (float *)scratch;            // every row the sampling kernels read is written by this call's LM head first
    return sev_verify_sample(m, kv, &b, stream);
}

// Prefill: long chains are fed through the same forward pass in chunks that fit the row budget, each
// chunk appended (all tokens kept) and committed before the next one starts.
extern "C" int sev_prefill(const sev_model *m, sev_kv *kv, const int32_t *slots, const int32_t *start_lens,
                           const int32_t *n_tokens, const int32_t *tokens, int B, int t_max, void *stream) {
    if (!m || !kv) return sev_fail(SEV_EINVAL, "null argument");
    if (kv->model != m) return sev_fail(SEV_EINVAL, "cache was created for another model");
    if (B < 1 || B > SEV_MAX_BATCH) return sev_fail(SEV_EINVAL, "B=%d outside 1..%d", B, SEV_MAX_BATCH);
    if (!start_lens || !n_tokens || !tokens || t_max < 1) return sev_fail(SEV_EINVAL, "start_lens, n_tokens and tokens are required");
    int64_t longest = 0;
    for (int b = 0; b < B; ++b) {
        if (n_tokens[b] < 1 || n_tokens[b] > t_max) return sev_fail(SEV_EINVAL, "request %d: %d tokens outside 1..%d", b, n_tokens[b], t_max);
        const int slot = slots ? slots[b] : b;
        if (slot < 0 || slot >= kv->max_req) return sev_fail(SEV_EINVAL, "request %d: slot %d out of range", b, slot);
        if (start_lens[b] < 0 || (int64_t)start_lens[b] + n_tokens[b] > (int64_t)kv->host_pages[slot] * SEV_PAGE)
            return sev_fail(SEV_ENOSPACE, "request %d: %d+%d tokens exceed the %d pages of slot %d", b, start_lens[b], n_tokens[b],
                            kv->host_pages[slot], slot);
        longest = std::max<int64_t>(longest, n_tokens[b]);
    }
    hipStream_t st = (hipStream_t)stream;
    // chunk length: all still-active requests advance together; rows of a chunk fit max_rows, and a request's
    // rows per chunk stay moderate so that the attention work list fits
    int32_t sl[SEV_MAX_BATCH], pre[SEV_MAX_BATCH], len[SEV_MAX_BATCH], idx[SEV_MAX_BATCH];
    for (int64_t done = 0; done < longest;) {
        int act = 0;
        for (int b = 0; b < B; ++b)
            if (n_tokens[b] > done) idx[act++] = b;
        const int64_t ch = std::max<int64_t>(1, std::min<int64_t>(512, kv->max_rows / act));
        for (int r = 0; r < act; ++r) {
            const int b = idx[r];
            sl[r] = slots ? slots[b] : b;
            pre[r] = start_lens[b] + (int32_t)done;
            len[r] = (int32_t)std::min<int64_t>(ch, n_tokens[b] - done);
        }
        // the chunk's rows must be contiguous per request in the token array: request r reads row idx[r] of tokens.
        // Requests that have finished leave holes in the batch, so each active request is issued with its own row.
        // (B is small on this path; one block call per chunk covers all requests when none has finished.)
        bool dense = (act == B);
        if (dense) {
            BlockCall c;
            memset(&c, 0, sizeof(c));
            c.slots = sl; c.prefix_lens = pre; c.lens = len; c.tokens = tokens; c.tok_stride = t_max; c.tok_off = (int)done;
            c.B = act; c.mode = 1; c.accept_len = kv->tmp_accept; c.bonus_token = kv->tmp_bonus;
            const int rc = run_block(m, kv, c, st);
            if (rc != SEV_OK) return rc;
            launch_commit(kv, sl, act, false, st);
        } else {
            for (int r = 0; r < act; ++r) {
                BlockCall c;
                memset(&c, 0, sizeof(c));
                c.slots = sl + r; c.prefix_lens = pre + r; c.lens = len + r;
                c.tokens = tokens + (size_t)idx[r] * t_max; c.tok_stride = t_max; c.tok_off = (int)done;
                c.B = 1; c.mode = 1; c.accept_len = kv->tmp_accept; c.bonus_token = kv->tmp_bonus;
                const int rc = run_block(m, kv, c, st);
                if (rc != SEV_OK) return rc;
                launch_commit(kv, sl + r, 1, false, st);
            }
        }
        done += ch;
    }
    SEV_HIP(hipGetLastError());
    return SEV_OK;
}

extern "C" int sev_verify(const sev_model *weights, sev_kv *kv_cache, const int32_t *prefix_lens,
                          const int32_t *draft_tokens, const int32_t *draft_mask, int B, int k, int32_t *accept_len,
                          int32_t *bonus_token, void *stream) {
    sev_verify_args a;
    memset(&a, 0, sizeof(a));
    a.B = B;
    a.k_max = k;
    a.prefix_lens = prefix_lens;
    a.draft_tokens = draft_tokens;
    a.parents = draft_mask;
    a.accept_len = accept_len;
    a.bonus_token = bonus_token;
    return sev_verify_ex(weights, kv_cache, &a, stream);
}

static int check_slots(sev_kv *kv, const int32_t *slots, int B) {
    if (!kv) return sev_fail(SEV_EINVAL, "null cache");
    if (B < 1 || B > SEV_MAX_BATCH) return sev_fail(SEV_EINVAL, "B=%d outside 1..%d", B, SEV_MAX_BATCH);
    for (int b = 0; b < B; ++b) {
        const int s = slots ? slots[b] : b;
        if (s < 0 || s >= kv->max_req) return sev_fail(SEV_EINVAL, "slot %d out of range", s);
    }
    return SEV_OK;
}

extern "C" int sev_kv_commit(sev_kv *kv, const int32_t *slots, int B, void *stream) {
    int rc = check_slots(kv, slots, B);
    if (rc) return rc;
    Prof p(kv, (hipStream_t)stream, PROF_OTHER);
    launch_commit(kv, slots, B, false, (hipStream_t)stream);
    SEV_HIP(hipGetLastError());
    return SEV_OK;
}

extern "C" int sev_kv_rollback(sev_kv *kv, const int32_t *slots, int B, void *stream) {
    int rc = check_slots(kv, slots, B);
    if (rc) return rc;
    launch_commit(kv, slots, B, true, (hipStream_t)stream);
    SEV_HIP(hipGetLastError());
    return SEV_OK;
}
