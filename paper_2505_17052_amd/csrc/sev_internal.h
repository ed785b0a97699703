// Internal declarations shared by the translation units of libsev.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

#include "../../include/sev.h"

#define SEV_PAGE 16
#define SEV_ATT_MAX_CP 256   // pages per attention work item, upper bound (a block of 8 waves x 16 pairs)
#define SEV_ATT_MAX_CHUNK 128   // pages per chunk when sequences are split over several blocks of 4 waves

// ---------------------------------------------------------------------------
// error plumbing (host)
// ---------------------------------------------------------------------------
int sev_fail(int code, const char *fmt, ...);
#define SEV_HIP(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess)                                                              \
            return sev_fail(SEV_EHIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

// ---------------------------------------------------------------------------
// packed activation layout for the matrix-core GEMMs ("xpack")
//
// A [M][K] activation matrix is carried as two bf16 planes (hi = bf16(x),
// lo = bf16(x - hi)), already arranged as MFMA 32x32x16 operand fragments:
//   [K/16 k-steps][m_tiles][plane 2][lane 64][8 bf16]
// lane = (m % 32) + 32 * ((k / 8) % 2), element = k % 8.  One fragment is 1 KiB.
// m_tiles is ceil(M/32) rounded up to a multiple of 4.
// ---------------------------------------------------------------------------
__host__ __device__ inline int64_t xpack_index(int m, int k, int plane, int m_tiles) {
    return ((((int64_t)(k >> 4) * m_tiles + (m >> 5)) * 2 + plane) << 9) + (((m & 31) + (((k >> 3) & 1) << 5)) << 3) +
           (k & 7);
}

struct LayerOffsets {
    size_t wqkv, wo, wgu, wd, g_attn, g_ffn;
};

struct sev_model {
    sev_model_desc d;
    char *arena;
    size_t arena_bytes;
    size_t off_embed, off_lm, off_gfinal;
    std::vector<LayerOffsets> layers;
    int n_qkv;   // (Hq + 2 Hkv) * hd
    int q_dim;   // Hq * hd
    int kv_dim;  // Hkv * hd
};

// Per-call description handed to the plan kernel by value.
struct PlanArgs {
    int B, k_max, mode;
    int pad_tokens;           // > 0: attention walks every request's pages up to this many tokens (padded-KV comparison variant)
    int tok_stride, tok_off;  // token of node i of request b: tokens[b * tok_stride + tok_off + i]
    int32_t slot[SEV_MAX_BATCH];
    int32_t prefix[SEV_MAX_BATCH];
    int32_t nd[SEV_MAX_BATCH];
};

// Device-side call plan (one per sev_kv; rebuilt by every verify).
struct DevPlan {
    // per request
    int32_t *req_slot, *req_P, *req_n, *req_row0;
    // per row (draft node)
    int32_t *row_req, *row_node, *row_pos, *row_tok;
    int32_t *row_kvloc;       // physical page * 16 + token in page of the cache position P + node the row is written to
    unsigned long long *row_anc;
    float2 *row_cs;           // [rows][hd/2] (cos, sin) of pos * theta_i
    // attention work items (bf16 path): a = {row group, first page, pages, prefix length},
    // b = {draft nodes, first row, request, 0}; pages = physical page ids of the chunk, SEV_ATT_MAX_CP per item
    int4 *it_a, *it_b;
    int32_t *it_pages;
    int4 *mg_rec;             // [merge groups] {row group | chunks << 16, first work item, draft nodes | item stride << 16, first row}
    int causal;               // 1: blocks are chains (node i sees nodes <= i; any length), 0: trees (ancestor masks, <= 64 nodes)
};

enum ProfClass { PROF_GEMM_QKV = 0, PROF_GEMM_O, PROF_GEMM_GU, PROF_GEMM_DOWN, PROF_GEMM_LM, PROF_ATTN, PROF_OTHER, PROF_N };

struct ProfSpan {
    hipEvent_t a, b;
    int cls;
};

// Tile-shape overrides for tuning experiments, read from the environment ONCE, when the handle is created:
// SEV_TUNE_QKV / _O / _GU / _DOWN / _LM = "MT,NT,S,PF" (S = 0 keeps the automatic split), SEV_TUNE_TPB = column tiles
// per block of the gate/up GEMM, SEV_TUNE_CP = pages per attention chunk.  Unset (the normal case): all zero.
struct Tune {
    int gemm[5][4];
    bool has_gemm[5];
    int tpb, cp;
};

struct sev_kv {
    const sev_model *model;
    Tune tune;
    int max_req, max_rows, page_size;
    int64_t n_pages;
    char *pool;
    size_t pool_bytes;
    size_t layer_stride;      // bytes between layers in the pool
    size_t v_offset;          // bytes from a layer's K pages to its V pages
    int max_pages_per_req;

    // device state (one allocation: `ws`)
    char *ws;
    size_t ws_bytes;
    int32_t *page_table;      // [max_req][max_pages_per_req]
    int32_t *seq_len, *next_tok;             // [max_req]
    int32_t *pend_n, *pend_a, *pend_bonus, *pend_P;   // [max_req] pending block: size, accepted, bonus, prefix length at verify
    int32_t *pend_path;       // [max_req][SEV_MAX_DRAFT]
    uint32_t *err_flags;      // [1]
    DevPlan plan;
    int max_items, max_groups;

    // activations
    float *h;                 // [rows][d] residual stream
    float *part;              // split-K exchange buffer / f32 scratch
    size_t part_elems;
    unsigned long long *ssq[2];   // bf16: fixed-point sums of squares of the residual rows (two buffers, used alternately)
    void *xa;                 // normed activations (xpack for bf16, [rows][d] f32 otherwise)
    void *q_buf;              // bf16: q hi/lo planes [2][rows][Hq*hd]; f32: qkv [rows][n_qkv]
    void *o_buf;              // attention output (xpack K=q_dim, or f32 [rows][q_dim])
    void *act;                // SwiGLU output (xpack K=d_ffn, or f32 [rows][d_ffn])
    float *att_o;             // attention partials [items*Hkv][32][hd]
    float2 *att_ml;           // [items*Hkv][32] (running max, sum)
    float *lm_val;            // [tiles][rows] partial arg-max values
    int32_t *lm_idx;
    int32_t *row_argmax;      // [rows]
    int32_t *tmp_accept, *tmp_bonus;         // [SEV_MAX_BATCH] outputs of internal block runs (prefill)
    float2 *row_stats;        // [rows] (largest logit, sum of exp((logit - max) / T)) of the stochastic rule
    float *logits_f32;        // f32 path only: [rows][vocab]

    // host mirrors
    std::vector<int> host_pages;   // pages assigned per slot
    // profiling
    int prof_on;
    std::vector<ProfSpan> spans;
    double prof_ms[PROF_N];
    int64_t prof_n[PROF_N];
};

struct Prof {
    sev_kv *kv;
    hipStream_t st;
    int cls;
    hipEvent_t a, b;
    bool on;
    Prof(sev_kv *kv_, hipStream_t st_, int cls_);
    ~Prof();
};

// ---------------------------------------------------------------------------
// launchers (defined in the kernel translation units)
// ---------------------------------------------------------------------------
// common
void launch_fill_f32(float *p, float v, int64_t n, hipStream_t st);
void launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t st);
void launch_plan(const sev_kv *kv, const PlanArgs &pa, const int32_t *draft_tokens, const int32_t *parents, int rows,
                 int chunk_pages, int n_items, hipStream_t st);
void launch_accept(const sev_kv *kv, int B, int k_max, int mode, const int32_t *draft_tokens, const int32_t *parents,
                   int32_t *accept_len, int32_t *bonus, int32_t *accept_path, hipStream_t st);
void launch_sample(const sev_kv *kv, int B, int k_max, int rows, const int32_t *tokens, const int32_t *parents, const float *logits,
                   const float *draft_probs, float2 *stats, float temperature, const float *u_acc, const float *u_emit,
                   int32_t *accept_len, int32_t *emitted, int32_t *accept_path, hipStream_t st);
void launch_commit(const sev_kv *kv, const int32_t *slots_dev_by_value, int B, bool rollback, hipStream_t st);
void launch_kv_copy(const sev_kv *kv, int slot, int layer, int start, int n, void *k, void *v, int to_cache, hipStream_t st);
void launch_argmax_rows_f32(const float *logits, int rows, int vocab, int32_t *out, hipStream_t st);

// f32 path
void launch_pack_f32(float *dst, const float *src, int64_t n, hipStream_t st);
void f32_forward(const sev_model *m, sev_kv *kv, int rows, int B, float *logits_out, hipStream_t st);

// bf16 path
void launch_pack_bf16(uint16_t *dst, const uint16_t *src, int n_rows, int K, int mode, int tile_add, hipStream_t st);
void bf16_forward(const sev_model *m, sev_kv *kv, int rows, int B, int n_items, int n_groups, int sib, bool att_direct,
                  float *logits_out, hipStream_t st);
