// Host-side sanitizer driver: exercises, without a GPU, every path of libsev's host code that ends before a
// launch (argument validation of the C ABI), the whole batch former / depth calibration / alignment check (pure
// host code) and the seeded generators of synth/rng.c, in a build with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code.  Exit status 0 and no sanitizer report = pass.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/sev.h"
#include "../../include/sev_sched.h"

extern "C" {
void synth_normal_f32(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, double scale, void *out);
void synth_normal_bf16(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, double scale, void *out);
void synth_uniform_i32(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, int32_t lo, int32_t hi, void *out);
void synth_uniform_f64(uint64_t seed, uint64_t stream, uint64_t offset, uint64_t n, void *out);
}

static int fails = 0;
#define EXPECT(cond)                                                             \
    do {                                                                         \
        if (!(cond)) { ++fails; fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); } \
    } while (0)

static uint64_t lcg(uint64_t &s) { s = s * 6364136223846793005ull + 1442695040888963407ull; return s >> 33; }

static void abi_validation() {
    sev_model_desc ok = {2, 256, 4, 4, 64, 688, 1024, 10000.0f, 1e-5f, SEV_F32};
    EXPECT(sev_model_arena_bytes(&ok) > 0);
    EXPECT(sev_model_arena_bytes(nullptr) == 0);
    sev_model_desc bad = ok;
    bad.n_kv_heads = 3;
    EXPECT(sev_model_arena_bytes(&bad) == 0 && strstr(sev_last_error(), "multiple"));
    bad = ok; bad.head_dim = 63;
    EXPECT(sev_model_arena_bytes(&bad) == 0);
    bad = ok; bad.dtype = 7;
    EXPECT(sev_model_arena_bytes(&bad) == 0);
    bad = ok; bad.dtype = SEV_BF16;                       // bf16 path: head_dim 128 only
    EXPECT(sev_model_arena_bytes(&bad) == 0);
    bad = ok; bad.vocab = 0;
    EXPECT(sev_model_arena_bytes(&bad) == 0);
    bad = ok; bad.rope_base = 1.0f;
    EXPECT(sev_model_arena_bytes(&bad) == 0);
    sev_model_desc big = {80, 8192, 64, 8, 128, 28672, 128256, 500000.0f, 1e-5f, SEV_BF16};
    EXPECT(sev_model_arena_bytes(&big) > (size_t)139e9);  // 64-bit sizes throughout
    sev_model *m = nullptr;
    EXPECT(sev_model_create(&ok, nullptr, 0, &m) == SEV_EINVAL && m == nullptr);
    EXPECT(sev_model_create(&ok, (void *)0x1001, 1 << 20, &m) == SEV_EINVAL);      // misaligned arena
    EXPECT(sev_model_create(&ok, (void *)0x1000, 16, nullptr) == SEV_EINVAL);
    EXPECT(sev_model_destroy(nullptr) == SEV_OK);
    EXPECT(sev_model_load_tensor(nullptr, SEV_W_WQ, 0, nullptr, nullptr) == SEV_EINVAL);
    EXPECT(sev_kv_pool_bytes(nullptr, 4, 16) == 0);
    sev_kv *kv = nullptr;
    EXPECT(sev_kv_create(nullptr, 1, 1, 1, 16, nullptr, 0, &kv) == SEV_EINVAL && kv == nullptr);
    EXPECT(sev_kv_destroy(nullptr) == SEV_OK);
    int32_t pages[4] = {0, 1, 2, 3}, one[1] = {0};
    EXPECT(sev_kv_set_pages(nullptr, 0, pages, 4, nullptr) == SEV_EINVAL);
    EXPECT(sev_kv_set_state(nullptr, one, one, one, 1, nullptr) == SEV_EINVAL);
    EXPECT(sev_kv_get_state(nullptr, 0, nullptr, nullptr, nullptr, nullptr) == SEV_EINVAL);
    EXPECT(sev_kv_copy_tokens(nullptr, 0, 0, 0, 1, pages, pages, 0, nullptr) == SEV_EINVAL);
    EXPECT(sev_verify(nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == SEV_EINVAL);
    sev_verify_args va;
    memset(&va, 0, sizeof(va));
    EXPECT(sev_verify_ex(nullptr, nullptr, &va, nullptr) == SEV_EINVAL);
    EXPECT(sev_verify_ex(nullptr, nullptr, nullptr, nullptr) == SEV_EINVAL);
    sev_sample_args sa;
    memset(&sa, 0, sizeof(sa));
    EXPECT(sev_verify_sample(nullptr, nullptr, &sa, nullptr) == SEV_EINVAL);
    EXPECT(sev_verify_sample_static(nullptr, nullptr, &sa, nullptr) == SEV_EINVAL);
    EXPECT(sev_prefill(nullptr, nullptr, nullptr, one, one, one, 1, 1, nullptr) == SEV_EINVAL);
    EXPECT(sev_kv_commit(nullptr, nullptr, 1, nullptr) == SEV_EINVAL);
    EXPECT(sev_kv_rollback(nullptr, nullptr, 1, nullptr) == SEV_EINVAL);
    EXPECT(sev_profile_enable(nullptr, 1) == SEV_EINVAL);
    EXPECT(sev_profile_read(nullptr, 0, nullptr, nullptr) == SEV_EINVAL);
    int n_cls = 0;
    while (sev_profile_name(n_cls)) ++n_cls;
    EXPECT(n_cls >= 6 && sev_profile_name(-1) == nullptr && sev_profile_name(1000) == nullptr);
    EXPECT(strlen(sev_last_error()) > 0);
}

static void scheduler() {
    sev_sched *s = nullptr;
    sev_sched_desc d = {0, 64, 1, 0};
    EXPECT(sev_sched_create(&d, &s) == SEV_EINVAL && s == nullptr);
    d = {4, 0, 1, 0};
    EXPECT(sev_sched_create(&d, &s) == SEV_EINVAL);
    d = {4, 64, 5, 0};
    EXPECT(sev_sched_create(&d, &s) == SEV_EINVAL);
    EXPECT(sev_sched_create(nullptr, &s) == SEV_EINVAL);
    EXPECT(sev_sched_destroy(nullptr) == SEV_OK);
    // random traffic: invariants of every batch (sizes, row budget, arrival order, nothing lost or served twice)
    for (int trial = 0; trial < 40; ++trial) {
        uint64_t rs = 1000 + trial;
        d.max_batch = 1 + (int)(lcg(rs) % 16);
        d.max_rows = 8 + (int)(lcg(rs) % 120);
        d.min_batch = 1 + (int)(lcg(rs) % d.max_batch);
        d.max_wait_us = (int64_t)(lcg(rs) % 3000);
        EXPECT(sev_sched_create(&d, &s) == SEV_OK && s);
        if (!s) return;
        const int R = 40;
        std::vector<int64_t> arr(R);
        std::vector<int> rows(R), served(R, 0);
        int64_t t = 0;
        for (int r = 0; r < R; ++r) {
            t += (int64_t)(lcg(rs) % 700);
            arr[r] = t;
            rows[r] = 1 + (int)(lcg(rs) % 8);
            EXPECT(sev_sched_submit(s, r, rows[r], arr[r]) == SEV_OK);
        }
        EXPECT(sev_sched_submit(s, 3, 2, 5) == SEV_ESTATE);           // request 3 already waits
        EXPECT(sev_sched_submit(s, R, 0, 5) == SEV_EINVAL);
        EXPECT(sev_sched_submit(s, R, d.max_rows + 1, 5) == SEV_EINVAL);
        EXPECT(sev_sched_submit(s, -1, 1, 5) == SEV_EINVAL);
        EXPECT(sev_sched_pending(s) == R);
        std::vector<int32_t> req(d.max_batch), rw(d.max_batch);
        int64_t now = 0, last_arrival = -1;
        int guard = 0, total = 0;
        while (sev_sched_pending(s) > 0 && ++guard < 10000) {
            int32_t n = -1;
            int64_t wake = -7;
            EXPECT(sev_sched_next_batch(s, now, req.data(), (guard & 1) ? rw.data() : nullptr, &n, &wake) == SEV_OK);
            if (n == 0) {
                EXPECT(wake > now);
                if (wake <= now) break;
                now = wake;
                continue;
            }
            EXPECT(n >= 1 && n <= d.max_batch && wake == now);
            int sum = 0;
            for (int i = 0; i < n; ++i) {
                const int r = req[i];
                EXPECT(r >= 0 && r < R);
                if (r < 0 || r >= R) continue;
                EXPECT(served[r] == 0 && arr[r] <= now && arr[r] >= last_arrival);
                last_arrival = arr[r];
                served[r] = 1;
                sum += rows[r];
                if (guard & 1) EXPECT(rw[i] == rows[r]);
            }
            EXPECT(sum <= d.max_rows);
            total += n;
            EXPECT(sev_sched_record_verify(s, 900 + (int64_t)(lcg(rs) % 400)) == SEV_OK);
            now += 1000;
        }
        EXPECT(total == R && sev_sched_pending(s) == 0);
        const int64_t est = sev_sched_verify_estimate(s);
        EXPECT(est >= 900 && est <= 1300);
        int32_t n = -1;
        int64_t wake = 0;
        EXPECT(sev_sched_next_batch(s, now, req.data(), nullptr, &n, &wake) == SEV_OK && n == 0 && wake == -1);
        EXPECT(sev_sched_next_batch(s, now, nullptr, nullptr, &n, &wake) == SEV_EINVAL);
        EXPECT(sev_sched_record_verify(s, -5) == SEV_EINVAL);
        EXPECT(sev_sched_destroy(s) == SEV_OK);
        s = nullptr;
    }
    EXPECT(sev_sched_calibrate_depth(94200, 11000, 15000, 1, 64) == 7);
    EXPECT(sev_sched_calibrate_depth(94200, 11000, 40000, 1, 64) == 5);
    EXPECT(sev_sched_calibrate_depth(94200, 11000, 50000, 1, 64) == 4);
    EXPECT(sev_sched_calibrate_depth(10, 11000, 50000, 2, 64) == 2);
    EXPECT(sev_sched_calibrate_depth(INT64_MAX, 1, 0, 1, 64) == 64);
    EXPECT(sev_sched_calibrate_depth(INT64_MAX, INT64_MAX, 0, 1, 64) == 1);
    EXPECT(sev_sched_calibrate_depth(INT64_MAX, INT64_MAX - 1, 0, 1, 64) == 1);
    EXPECT(sev_sched_calibrate_depth(INT64_MAX, 1, INT64_MIN + 1, 1, 64) < 0);
    EXPECT(sev_sched_calibrate_depth(-1, 1, 0, 1, 64) < 0);
    EXPECT(sev_sched_calibrate_depth(1, 0, 0, 1, 4) < 0);
    EXPECT(sev_sched_calibrate_depth(1, 1, 0, 0, 4) < 0);
    EXPECT(sev_sched_calibrate_depth(1, 1, 0, 5, 4) < 0);
}

static void alignment() {
    // random trees, random root-to-node paths: the kept set is the subtree of the matching child
    for (int trial = 0; trial < 200; ++trial) {
        uint64_t rs = 77 + trial;
        const int n = 1 + (int)(lcg(rs) % 48);
        std::vector<int32_t> par(n), tok(n), kept(n), newp(n);
        for (int i = 0; i < n; ++i) {
            par[i] = (int32_t)(lcg(rs) % (uint64_t)(i + 1)) - 1;
            tok[i] = (int32_t)(lcg(rs) % 5);
        }
        std::vector<int32_t> path;
        int cur = -1;
        for (int step = 0; step < 6; ++step) {
            int pick = -1;
            for (int c = cur + 1; c < n; ++c)
                if (par[c] == cur && (lcg(rs) & 1)) { pick = c; break; }
            if (pick < 0) break;
            path.push_back(pick);
            cur = pick;
        }
        int32_t nk = -1;
        const int32_t bonus = (int32_t)(lcg(rs) % 5);
        EXPECT(sev_edge_align(par.data(), tok.data(), n, path.data(), (int32_t)path.size(), bonus, kept.data(), newp.data(), &nk) == SEV_OK);
        int want = -1;
        for (int c = 0; c < n; ++c)
            if (par[c] == cur && tok[c] == bonus) { want = c; break; }
        if (want < 0) {
            EXPECT(nk == 0);
            continue;
        }
        EXPECT(nk >= 1 && kept[0] == want && newp[0] == -1);
        for (int i = 1; i < nk; ++i) {
            EXPECT(kept[i] > kept[i - 1] && newp[i] >= 0 && newp[i] < i);
            if (newp[i] >= 0 && newp[i] < i) EXPECT(kept[newp[i]] == par[kept[i]]);
        }
    }
    int32_t par[3] = {-1, 0, 5}, tok[3] = {1, 2, 3}, path[1] = {0}, kept[3], newp[3], nk;
    EXPECT(sev_edge_align(par, tok, 3, path, 1, 2, kept, newp, &nk) == SEV_EINVAL);        // parent index not below the child's
    par[2] = 1;
    int32_t badpath[2] = {1, 0};
    EXPECT(sev_edge_align(par, tok, 3, badpath, 2, 2, kept, newp, &nk) == SEV_EINVAL);     // not a root-to-node path
    EXPECT(sev_edge_align(nullptr, tok, 3, path, 1, 2, kept, newp, &nk) == SEV_EINVAL);
    EXPECT(sev_edge_align(par, tok, 3, path, 1, 2, kept, newp, &nk) == SEV_OK && nk == 2 && kept[0] == 1 && kept[1] == 2);
}

static void generators() {
    for (uint64_t n : {0ull, 1ull, 2ull, 3ull, 7ull, 8ull, 1023ull, 4099ull}) {
        std::vector<float> f(n + 1, -1.0f);
        std::vector<uint16_t> h(n + 1, 0xdead);
        std::vector<int32_t> iv(n + 1, -1);
        std::vector<double> dv(n + 1, -1.0);
        synth_normal_f32(5, 9, 3, n, 0.02, f.data());
        synth_normal_bf16(5, 9, 3, n, 0.02, h.data());
        synth_uniform_i32(5, 10, 0, n, -4, 9, iv.data());
        synth_uniform_f64(5, 11, UINT64_MAX - 2, n, dv.data());        // counter wrap-around
        EXPECT(f[n] == -1.0f && h[n] == 0xdead && iv[n] == -1 && dv[n] == -1.0);      // nothing written past n
        for (uint64_t i = 0; i < n; ++i) {
            EXPECT(f[i] == f[i] && f[i] > -0.2f && f[i] < 0.2f);
            EXPECT(iv[i] >= -4 && iv[i] < 9);
            EXPECT(dv[i] >= 0.0 && dv[i] < 1.0);
            uint32_t w = (uint32_t)h[i] << 16;
            float hv;
            memcpy(&hv, &w, 4);
            EXPECT(hv > f[i] - 2e-3f && hv < f[i] + 2e-3f);            // bf16 of the same draw
        }
    }
    // value i depends on (seed, stream, offset + i) only
    float a[16], b[8];
    synth_normal_f32(1, 2, 0, 16, 1.0, a);
    synth_normal_f32(1, 2, 8, 8, 1.0, b);
    EXPECT(memcmp(a + 8, b, sizeof(b)) == 0);
    int32_t e[4];
    synth_uniform_i32(1, 2, 0, 4, INT32_MIN, INT32_MAX, e);             // widest range: no signed overflow
}

int main() {
    abi_validation();
    scheduler();
    alignment();
    generators();
    if (fails) {
        fprintf(stderr, "%d checks failed\n", fails);
        return 1;
    }
    printf("host sanitizer driver: all checks passed\n");
    return 0;
}
