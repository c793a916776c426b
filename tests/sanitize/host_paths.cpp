// Host-only build of the library's CPU code (batch validation, planner, scheduler, the bookkeeping of the entry
// points) and of the fp64 checker, for AddressSanitizer / UndefinedBehaviorSanitizer.  No GPU and no HIP runtime:
// the few runtime calls api.cpp makes are replaced by host stand-ins below ("pinned" memory is malloc memory,
// events and streams are dummies), and the kernel launchers are replaced by functions that walk exactly the
// metadata a kernel would read and, for the append, move the rows on the host.  Every "device" buffer is a heap
// block of exactly the documented size, so a record or plan entry that points outside them is an ASan error.
//
// Built and run by tests/test_sanitizers.py (g++/gcc -fsanitize=address,undefined); exit code 0 = clean.
#include <hip/hip_runtime_api.h>

#include <cassert>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "internal.h"
#include "sarathi.h"

// ---- checker entry points (C, compiled separately with the same sanitizers) ----
extern "C" int oracle_hybrid_attention_window(const uint16_t *q, const uint16_t *k_seq, const uint16_t *v_seq,
                                              const int64_t *kv_start, const int32_t *q_start, const int32_t *q_len,
                                              const int32_t *ctx_len, int num_seqs, int num_tokens, int num_q_heads,
                                              int num_kv_heads, int d, double sm_scale, int window, const int32_t *tokens,
                                              int n_rows, double *out, int num_threads);
extern "C" int oracle_softmax_weights(const uint16_t *q, const uint16_t *k_seq, const int64_t *kv_start, const int32_t *q_start,
                                      const int32_t *q_len, const int32_t *ctx_len, int num_seqs, int num_q_heads,
                                      int num_kv_heads, int d, double sm_scale, int token, int head, double *w);
extern "C" int oracle_linear(const uint16_t *x, const uint16_t *w, int T, int N, int K, const int32_t *rows, int n_rows,
                             const int32_t *cols, int n_cols, double *out, int num_threads);

#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) {                                                                \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(3);                                                             \
        }                                                                             \
    } while (0)

// ---- stand-ins for the HIP runtime calls of api.cpp ----
extern "C" {
hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = std::malloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostGetDevicePointer(void **d, void *h, unsigned) { *d = h; return hipSuccess; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = reinterpret_cast<hipEvent_t>(std::malloc(1)); return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t *e) { *e = reinterpret_cast<hipEvent_t>(std::malloc(1)); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { std::free(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = reinterpret_cast<hipStream_t>(std::malloc(1)); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { std::free(s); return hipSuccess; }
hipError_t hipDeviceSynchronize() { return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "host stand-in"; }
}

// ---- stand-ins for the kernel launchers: read what the kernels would read ----
namespace sarathi {

static int g_num_seqs = 0;          // shape of the call in flight, for the walkers below
static int64_t g_num_tokens = 0;
static uint64_t g_sink = 0;

int launch_kv_append(const sarathi_config &cfg, const AppendMeta &m, const void *k_new, const void *v_new, void *k_cache,
                     void *v_cache, int64_t num_pages, void *) {
    const int D = cfg.head_dim, H = cfg.num_kv_heads;
    const uint16_t *kn = static_cast<const uint16_t *>(k_new), *vn = static_cast<const uint16_t *>(v_new);
    uint16_t *kc = static_cast<uint16_t *>(k_cache), *vc = static_cast<uint16_t *>(v_cache);
    if (m.copy_bytes) std::memcpy(m.copy_dst, m.copy_src, (m.copy_bytes + 15) / 16 * 16);
    for (int u = 0; u < m.num_units; ++u) {
        const AppendUnit &r = m.units[u];
        const int lo = r.lo_hi & 0xFF, hi = r.lo_hi >> 8;
        CHECK(r.seq >= 0 && r.seq < g_num_seqs && r.page_idx >= 0 && r.page_idx < m.max_blocks);
        CHECK(0 <= lo && lo < hi && hi <= kPageSize && r.row0 >= 0 && r.row0 + (hi - lo) <= g_num_tokens);
        const int64_t page = m.block_table[(int64_t)r.seq * m.max_blocks + r.page_idx];
        CHECK(page >= 0 && page < num_pages);
        for (int h = 0; h < H; ++h)
            for (int i = lo; i < hi; ++i)
                for (int c = 0; c < D; ++c) {
                    const int64_t src = ((int64_t)(r.row0 + i - lo) * H + h) * D + c;
                    kc[((page * H + h) * kPageSize + i) * D + c] = kn[src];
                    vc[((page * H + h) * D + c) * kPageSize + i] = vn[src];
                }
    }
    return 0;
}

int launch_upload(void *dst, const void *src, size_t bytes, void *) {
    std::memcpy(dst, src, (bytes + 15) / 16 * 16);
    return 0;
}
int launch_upload_args(void *dst, const void *src, size_t bytes, void *) {
    CHECK(bytes % 16 == 0);
    std::memcpy(dst, src, bytes);
    return 0;
}
int launch_zero(void *p, size_t bytes, void *) {
    std::memset(p, 0, bytes);
    return 0;
}

static std::vector<char> g_static;
int static_scratch(StaticScratch *out) {
    const size_t sched = (kSchedBytes + 255) / 256 * 256;
    if (g_static.empty()) g_static.resize(kStaticMetaBytes + sched + kStaticPartMlBytes + kStaticPartOBytes);
    char *base = g_static.data();
    out->meta = base;
    out->sched = reinterpret_cast<int32_t *>(base + kStaticMetaBytes);
    out->part_ml = reinterpret_cast<float *>(base + kStaticMetaBytes + sched);
    out->part_o = reinterpret_cast<float *>(base + kStaticMetaBytes + sched + kStaticPartMlBytes);
    return 0;
}

// Every (column, key) pair of the batch must be covered by exactly one work unit, every unit must stay inside
// its sequence, and every partial row / counter a unit or merge item names must lie inside its buffer (touched
// here so that ASan sees an overrun).
int launch_attention(const sarathi_config &cfg, const AttnMeta &m, const void *, const void *, const void *, int64_t,
                     float, void *, int which, void *) {
    const int H = cfg.num_kv_heads, D = cfg.head_dim;
    for (int u = 0; u < m.num_units; ++u) {
        const uint32_t unit = m.units[u];
        const TileDesc &t = m.tiles[unit & ((1u << kUnitTileBits) - 1)];
        const int split = (int)(unit >> kUnitTileBits);
        CHECK(t.seq >= 0 && t.seq < g_num_seqs && split < t.n_splits);
        CHECK((u < m.num_tile_units) == (t.kind == kKindTile));
        CHECK(t.n_cols >= 1 && t.n_cols <= (t.kind == kKindTile ? kTileCols : kWaveCols));
        CHECK(t.n_keys >= 1 && t.n_keys <= t.ctx_len && t.key_lo >= 0 && t.key_lo % kTileKeys == 0 && t.key_lo < t.n_keys);
        CHECK(t.keys_per_split % kTileKeys == 0 && t.key_lo + (int64_t)split * t.keys_per_split < t.n_keys);
        CHECK((int64_t)t.q_start + t.q_len <= g_num_tokens);
        const int n_pages = (t.ctx_len + kPageSize - 1) / kPageSize;
        g_sink += (uint64_t)m.block_table[(int64_t)t.seq * m.max_blocks + n_pages - 1];  // last table entry the kernel may read
        if (t.n_splits > 1) {
            CHECK(t.part_row0 >= 0);
            const int64_t last_row = (int64_t)t.part_row0 + (int64_t)t.n_splits * t.n_cols - 1;
            m.part_o[(last_row * H + H - 1) * D + D - 1] = 0.f;
            m.part_ml[(last_row * H + H - 1) * 2 + 1] = 0.f;
        } else {
            CHECK(t.part_row0 == -1);
        }
    }
    for (int r = 0; r < m.num_reduce_units; ++r) {
        const uint32_t ru = m.reduce_units[r];
        const TileDesc &t = m.tiles[ru & ((1u << kUnitTileBits) - 1)];
        CHECK(t.n_splits > 1 && (int)(ru >> kUnitTileBits) * kReduceCols < t.n_cols);
    }
    if (which == 5) g_sink += (uint64_t)m.sched[kSchedCuSlots + 2 * kSchedMaxKvHeads - 1];
    return 0;
}
int launch_reduce(const sarathi_config &, const AttnMeta &m, void *, int32_t first, int32_t count, void *) {
    CHECK(first >= 0 && first + count <= m.num_reduce_units);
    return 0;
}

}  // namespace sarathi

// ---- drivers ----
static void drive_scheduler(std::mt19937_64 &rng) {
    auto rnd = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
    for (int it = 0; it < 2000; ++it) {
        const int nd = rnd(0, 40), np = rnd(0, 4), nw = rnd(0, 6);
        std::vector<sarathi_request> dec(nd), pre(np), wait(nw);
        for (int i = 0; i < nd; ++i) { int p = rnd(1, 3000); dec[i] = sarathi_request{i, p, p, rnd(0, 50), 0}; }
        for (int i = 0; i < np; ++i) { int p = rnd(2, 9000); pre[i] = sarathi_request{100 + i, p, rnd(0, p - 1), 0, 0}; }
        for (int i = 0; i < nw; ++i) wait[i] = sarathi_request{200 + i, rnd(1, 9000), 0, 0, 0};
        const int cap = rnd(1, 60);
        std::vector<int64_t> id(cap);
        std::vector<int32_t> qs(cap), ql(cap), cl(cap);
        sarathi_batch b{};
        b.seq_id = id.data(); b.q_start = qs.data(); b.q_len = ql.data(); b.ctx_len = cl.data();
        const int budget = rnd(1, 2048), chunk = rnd(1, 4096);
        const sarathi_status st = sarathi_build_stall_free_batch(budget, chunk, nd ? dec.data() : nullptr, nd, np ? pre.data() : nullptr,
                                                                  np, nw ? wait.data() : nullptr, nw, rnd(0, 2000), 16, cap, &b);
        if (nd > cap) { CHECK(st == SARATHI_ECAPACITY); continue; }
        CHECK(st == SARATHI_OK && b.num_seqs <= cap && b.num_decodes == nd);
        int64_t run = 0;
        for (int i = 0; i < b.num_seqs; ++i) { CHECK(qs[i] == run && ql[i] >= 1 && cl[i] >= ql[i]); run += ql[i]; }
        CHECK(run == b.num_tokens);
    }
    sarathi_batch bad{};
    CHECK(sarathi_build_stall_free_batch(8, 8, nullptr, 0, nullptr, 0, nullptr, 0, 0, 16, 4, &bad) == SARATHI_EINVAL);
}

static void drive_attention_host_paths(std::mt19937_64 &rng) {
    auto rnd = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
    const int shapes[][3] = {{8, 2, 128}, {4, 1, 64}, {14, 2, 128}, {3, 3, 64}};
    for (int it = 0; it < 60; ++it) {
        const int *sh = shapes[it % 4];
        sarathi_config cfg{sh[0], sh[1], sh[2], 16, 0, 4096, 64, 0};
        const int S = rnd(1, 24);
        std::vector<int32_t> qs(S), ql(S), cl(S);
        int64_t T = 0, pages_needed = 0;
        int max_blocks = 1;
        for (int s = 0; s < S; ++s) {
            const bool chunk = rnd(0, 3) == 0;
            ql[s] = chunk ? rnd(2, 300) : 1;
            cl[s] = ql[s] + rnd(0, it % 5 == 0 ? 9000 : 700);
            qs[s] = (int32_t)T;
            T += ql[s];
            pages_needed += (cl[s] + 15) / 16;
            max_blocks = std::max(max_blocks, (cl[s] + 15) / 16);
        }
        cfg.max_blocks_per_seq = max_blocks;
        sarathi_handle *h = nullptr;
        CHECK(sarathi_create(&cfg, &h) == SARATHI_OK);
        if (it % 3 == 1) CHECK(sarathi_set_option(h, "split_keys", 64) == SARATHI_OK && sarathi_set_option(h, "tile_split_keys", 64) == SARATHI_OK);
        if (it % 3 == 2) CHECK(sarathi_set_option(h, "window", rnd(1, 500)) == SARATHI_OK);
        if (it % 4 == 3) CHECK(sarathi_set_option(h, "resident_chunks", 1) == SARATHI_OK);
        const int64_t num_pages = pages_needed + 3;
        std::vector<int32_t> bt((size_t)S * max_blocks, -1);
        int64_t next = 0;
        for (int s = 0; s < S; ++s)
            for (int b = 0; b < (cl[s] + 15) / 16; ++b) bt[(size_t)s * max_blocks + b] = (int32_t)next++;
        const size_t row = (size_t)cfg.num_kv_heads * cfg.head_dim;
        std::vector<uint16_t> k_new((size_t)T * row, 1), v_new((size_t)T * row, 2);
        std::vector<uint16_t> kc((size_t)num_pages * row * 16), vc((size_t)num_pages * row * 16);
        std::vector<uint16_t> q((size_t)T * cfg.num_q_heads * cfg.head_dim), out(q.size());
        // the workspace is handed over 256-byte aligned and exactly as large as the library asks for
        const size_t ws_bytes = sarathi_workspace_bytes(h);
        void *ws = nullptr;
        CHECK(posix_memalign(&ws, 256, ws_bytes) == 0);
        std::memset(ws, 0xFF, ws_bytes);
        sarathi::g_num_seqs = S;
        sarathi::g_num_tokens = T;
        CHECK(sarathi_kv_append(h, k_new.data(), v_new.data(), kc.data(), vc.data(), bt.data(), qs.data(), ql.data(), cl.data(), S,
                                (int32_t)T, num_pages, ws, nullptr) == SARATHI_OK);
        for (int rep = 0; rep < 2; ++rep)   // the second call finds the plan the append brought still resident
            CHECK(sarathi_hybrid_attention(h, q.data(), kc.data(), vc.data(), bt.data(), qs.data(), ql.data(), cl.data(), S, (int32_t)T,
                                           num_pages, 0.1f, out.data(), ws, nullptr) == SARATHI_OK);
        CHECK(sarathi_hybrid_attention_noalloc(h, q.data(), kc.data(), vc.data(), bt.data(), qs.data(), ql.data(), cl.data(), S,
                                               (int32_t)T, num_pages, 0.1f, out.data(), nullptr) == SARATHI_OK);
        sarathi_plan_info info{};
        CHECK(sarathi_plan_hybrid_attention(h, qs.data(), ql.data(), cl.data(), S, (int32_t)T, &info, nullptr, 0) == SARATHI_OK);
        std::vector<sarathi_work_item> items((size_t)std::max(1, info.num_items));
        CHECK(sarathi_plan_hybrid_attention(h, qs.data(), ql.data(), cl.data(), S, (int32_t)T, &info, items.data(), info.num_items) == SARATHI_OK);
        // error paths: nothing may be touched
        ql[0] += 1;
        CHECK(sarathi_kv_append(h, k_new.data(), v_new.data(), kc.data(), vc.data(), bt.data(), qs.data(), ql.data(), cl.data(), S,
                                (int32_t)T, num_pages, ws, nullptr) != SARATHI_OK);
        ql[0] -= 1;
        CHECK(sarathi_hybrid_attention(h, q.data(), kc.data(), vc.data(), bt.data(), qs.data(), ql.data(), cl.data(), S, (int32_t)T,
                                       num_pages, 0.1f, out.data(), static_cast<char *>(ws) + 8, nullptr) == SARATHI_EWORKSPACE);
        CHECK(sarathi_destroy(h) == SARATHI_OK);
        std::free(ws);
    }
}

static void drive_checker() {
    // one chunk on a prefix and two decodes, GQA 4:2, d = 8; every buffer exactly as large as documented
    const int Hq = 4, Hkv = 2, d = 8;
    const int32_t q_start[3] = {0, 5, 6}, q_len[3] = {5, 1, 1}, ctx_len[3] = {9, 1, 13};
    const int64_t kv_start[3] = {0, 9, 10};
    const int T = 7, KV = 23;
    std::vector<uint16_t> q((size_t)T * Hq * d), k((size_t)KV * Hkv * d), v(k.size());
    for (size_t i = 0; i < q.size(); ++i) q[i] = (uint16_t)(0x3F80 + (i * 37 % 64));          // bf16 values near 1
    for (size_t i = 0; i < k.size(); ++i) { k[i] = (uint16_t)(0x3F00 + (i * 29 % 128)); v[i] = (uint16_t)(0xBF80 + (i * 13 % 96)); }
    std::vector<double> out((size_t)T * Hq * d);
    for (int window : {0, 1, 4})
        CHECK(oracle_hybrid_attention_window(q.data(), k.data(), v.data(), kv_start, q_start, q_len, ctx_len, 3, T, Hq, Hkv, d, 0.35,
                                             window, nullptr, T, out.data(), 2) == 0);
    const int32_t rows[2] = {6, 0};
    std::vector<double> two((size_t)2 * Hq * d);
    CHECK(oracle_hybrid_attention_window(q.data(), k.data(), v.data(), kv_start, q_start, q_len, ctx_len, 3, T, Hq, Hkv, d, 0.35, 0, rows,
                                         2, two.data(), 1) == 0);
    std::vector<double> w(13);
    CHECK(oracle_softmax_weights(q.data(), k.data(), kv_start, q_start, q_len, ctx_len, 3, Hq, Hkv, d, 0.35, 6, 3, w.data()) == 13);
    double sum = 0;
    for (double x : w) sum += x;
    CHECK(sum > 0.999999 && sum < 1.000001);
    const int32_t bad_rows[1] = {7};
    CHECK(oracle_hybrid_attention_window(q.data(), k.data(), v.data(), kv_start, q_start, q_len, ctx_len, 3, T, Hq, Hkv, d, 0.35, 0,
                                         bad_rows, 1, two.data(), 1) != 0);
    // linear layer: 3 x 5 by 4 x 5, all and a subset
    std::vector<uint16_t> x(15, 0x3F80), wt(20, 0x4000);
    std::vector<double> y(12);
    CHECK(oracle_linear(x.data(), wt.data(), 3, 4, 5, nullptr, 0, nullptr, 0, y.data(), 1) == 0 && y[11] == 10.0);
    const int32_t r[1] = {2}, c[2] = {3, 0};
    CHECK(oracle_linear(x.data(), wt.data(), 3, 4, 5, r, 1, c, 2, y.data(), 2) == 0 && y[1] == 10.0);
    const int32_t bad[1] = {4};
    CHECK(oracle_linear(x.data(), wt.data(), 3, 4, 5, nullptr, 0, bad, 1, y.data(), 1) != 0);
}

int main() {
    std::mt19937_64 rng(20240302);
    drive_scheduler(rng);
    drive_attention_host_paths(rng);
    drive_checker();
    std::printf("host paths clean (sink %llu)\n", (unsigned long long)sarathi::g_sink);
    return 0;
}
