// Host side of sarathi_hybrid_attention: validation of the batch description, workspace
// layout, and the decomposition of one iteration's attention into independent work items.
//
// Decomposition.  For a KV head, the query side of sequence s is a list of COLUMNS,
// col = row*G + head_in_group (G = Hq/Hkv query heads share the KV head, paper section 2.2),
// so a decode has G columns and a chunk of c rows has c*G.  Columns are cut into tiles of 16
// (the N dimension of the 16x16x32 matrix-core instruction); a tile needs keys
// 0 .. position of its last row.  Long key ranges are cut into splits of about `split_keys`
// keys so that (a) a decode with a long context (paper section 3.3: decode cost grows with
// the accumulated context and differs across requests) does not become the tail of the
// launch and (b) there are enough items to fill 256 compute units.  Splits are merged by a
// second kernel in a fixed order.
#include <algorithm>
#include <cstdio>

#include "internal.h"

namespace sarathi {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

constexpr int32_t kMaxSplitItems = 8192;
constexpr int32_t kMaxPartRows = 32768;
constexpr int32_t kMinSplitKeys = 256;
constexpr int32_t kMinTileSplitKeys = 1024;

WorkspaceLayout make_workspace_layout(const sarathi_config &cfg) {
    WorkspaceLayout w{};
    const int64_t G = cfg.num_q_heads / cfg.num_kv_heads;
    // wave tiles only exist for sequences below tile_min_cols columns; bounding every sequence by
    // 16-column tiles covers both kinds
    const int64_t max_tiles = ceil_div((int64_t)cfg.max_tokens * G, kWaveCols) + cfg.max_seqs;
    w.max_items = (int32_t)std::min<int64_t>(max_tiles + kMaxSplitItems, INT32_MAX / 64);
    w.max_reduce_items = (int32_t)std::min<int64_t>(max_tiles, INT32_MAX / 64);
    w.max_part_rows = kMaxPartRows;
    size_t off = 0;
    w.seq_meta = off;      off = align_up(off + sizeof(int32_t) * 3 * (size_t)cfg.max_seqs, 256);
    w.items = off;         off = align_up(off + sizeof(WorkItem) * (size_t)w.max_items, 256);
    w.reduce_items = off;  off = align_up(off + sizeof(ReduceItem) * (size_t)w.max_reduce_items, 256);
    w.part_ml = off;       off = align_up(off + sizeof(float) * 2 * (size_t)w.max_part_rows * cfg.num_kv_heads, 256);
    w.part_o = off;        off = align_up(off + sizeof(float) * (size_t)w.max_part_rows * cfg.num_kv_heads * cfg.head_dim, 256);
    w.total = off;
    return w;
}

sarathi_status validate_batch(const sarathi_config &cfg, const int32_t *q_start, const int32_t *q_len,
                              const int32_t *ctx_len, int32_t num_seqs, int32_t num_tokens,
                              int64_t num_pages, std::string &err) {
    char buf[160];
    if (num_seqs < 0 || num_tokens < 0) { err = "negative num_seqs or num_tokens"; return SARATHI_EINVAL; }
    if (num_seqs == 0) {
        if (num_tokens != 0) { err = "num_tokens != 0 with num_seqs == 0"; return SARATHI_EINVAL; }
        return SARATHI_OK;
    }
    if (!q_start || !q_len || !ctx_len) { err = "null length array"; return SARATHI_EINVAL; }
    if (num_seqs > cfg.max_seqs) { err = "num_seqs exceeds max_seqs"; return SARATHI_ECAPACITY; }
    if (num_tokens > cfg.max_tokens) { err = "num_tokens exceeds max_tokens"; return SARATHI_ECAPACITY; }
    if (num_pages < 1) { err = "num_pages < 1"; return SARATHI_EINVAL; }
    int64_t run = 0;
    for (int32_t s = 0; s < num_seqs; ++s) {
        if (q_len[s] < 1 || ctx_len[s] < q_len[s]) {
            snprintf(buf, sizeof buf, "sequence %d: need 1 <= q_len <= ctx_len (q_len %d, ctx_len %d)", s, q_len[s], ctx_len[s]);
            err = buf;
            return SARATHI_EINVAL;
        }
        if (q_start[s] != run) {
            snprintf(buf, sizeof buf, "sequence %d: q_start %d is not the prefix sum of q_len (%lld)", s, q_start[s], (long long)run);
            err = buf;
            return SARATHI_EINVAL;
        }
        if (ceil_div(ctx_len[s], cfg.page_size) > cfg.max_blocks_per_seq) {
            snprintf(buf, sizeof buf, "sequence %d: ctx_len %d needs more than max_blocks_per_seq pages", s, ctx_len[s]);
            err = buf;
            return SARATHI_ECAPACITY;
        }
        run += q_len[s];
    }
    if (run != num_tokens) { err = "sum of q_len != num_tokens"; return SARATHI_EINVAL; }
    return SARATHI_OK;
}

namespace {

struct Tile {
    int32_t seq, col_begin, n_cols, n_keys;
};

inline int32_t steps_of(const WorkItem &w) { return (int32_t)ceil_div(w.key_end - w.key_begin, kTileKeys); }

// Emits the items of one kind for `tiles`, splitting key ranges longer than ~1.5 * split_keys,
// and appends them to `out` sorted longest first (counting sort on 32-key steps).
void emit_items(const std::vector<Tile> &tiles, int64_t split_keys, int32_t kind, Plan &plan,
                std::vector<WorkItem> &scratch, std::vector<int32_t> &bucket) {
    scratch.clear();
    int32_t max_steps = 0;
    for (const Tile &t : tiles) {
        int32_t ns = (t.n_keys <= split_keys + split_keys / 2) ? 1 : (int32_t)ceil_div(t.n_keys, split_keys);
        const int32_t per = (int32_t)(ceil_div(ceil_div(t.n_keys, ns), kTileKeys) * kTileKeys);
        ns = (int32_t)ceil_div(t.n_keys, per);
        int32_t part_row = -1;
        if (ns > 1) {
            part_row = plan.num_part_rows;
            plan.num_part_rows += ns * t.n_cols;
            plan.reduce_items.push_back({t.seq, t.col_begin, t.n_cols, part_row, ns, {0, 0, 0}});
        }
        for (int32_t i = 0; i < ns; ++i) {
            WorkItem w{};
            w.seq = t.seq;
            w.col_begin = t.col_begin;
            w.n_cols = t.n_cols;
            w.key_begin = i * per;
            w.key_end = std::min(t.n_keys, (i + 1) * per);
            w.part_row = ns > 1 ? part_row + i * t.n_cols : -1;
            w.kind = kind;
            scratch.push_back(w);
            max_steps = std::max(max_steps, steps_of(w));
        }
    }
    bucket.assign((size_t)max_steps + 2, 0);
    for (const WorkItem &w : scratch) bucket[(size_t)(max_steps - steps_of(w)) + 1]++;
    for (size_t i = 1; i < bucket.size(); ++i) bucket[i] += bucket[i - 1];
    const size_t base = plan.items.size();
    plan.items.resize(base + scratch.size());
    for (const WorkItem &w : scratch) plan.items[base + (size_t)bucket[(size_t)(max_steps - steps_of(w))]++] = w;
}

// Split items and partial rows a choice of split_keys would need.
void count_splits(const std::vector<Tile> &tiles, int64_t split_keys, int64_t &n_split_items, int64_t &rows) {
    for (const Tile &t : tiles) {
        if (t.n_keys <= split_keys + split_keys / 2) continue;
        const int64_t ns = ceil_div(t.n_keys, split_keys);
        n_split_items += ns;
        rows += ns * t.n_cols;
    }
}

}  // namespace

void plan_attention(const sarathi_config &cfg, const Options &opt, const WorkspaceLayout &ws,
                    const int32_t *q_len, const int32_t *ctx_len, int32_t num_seqs, Plan &plan) {
    plan.items.clear();
    plan.reduce_items.clear();
    plan.num_part_rows = 0;
    plan.num_tile_items = 0;
    const int32_t G = cfg.num_q_heads / cfg.num_kv_heads;

    static thread_local std::vector<Tile> wave_tiles, chunk_tiles;
    static thread_local std::vector<WorkItem> scratch;
    static thread_local std::vector<int32_t> bucket;
    wave_tiles.clear();
    chunk_tiles.clear();
    int64_t wave_keys = 0, chunk_keys = 0;
    for (int32_t s = 0; s < num_seqs; ++s) {
        const int32_t prefix = ctx_len[s] - q_len[s];
        const int64_t n_cols = (int64_t)q_len[s] * G;
        const bool chunk = n_cols >= opt.tile_min_cols;   // prefill chunk: 128-column LDS-staged tiles
        const int32_t width = chunk ? kTileCols : kWaveCols;
        for (int64_t c0 = 0; c0 < n_cols; c0 += width) {
            const int32_t nc = (int32_t)std::min<int64_t>(width, n_cols - c0);
            const int32_t last_row = (int32_t)((c0 + nc - 1) / G);
            const int32_t n_keys = prefix + last_row + 1;   // keys 0 .. position of the tile's last row
            if (chunk) { chunk_tiles.push_back({s, (int32_t)c0, nc, n_keys}); chunk_keys += n_keys; }
            else       { wave_tiles.push_back({s, (int32_t)c0, nc, n_keys});  wave_keys += n_keys; }
        }
    }

    // Keys per split: the automatic choice aims at ~target items per KV head, never below a
    // floor, and both are coarsened together until the partial buffers suffice.
    auto pick = [](int64_t forced, int64_t total, int64_t target, int64_t floor_keys) {
        int64_t k = forced > 0 ? forced : std::max<int64_t>(floor_keys, ceil_div(total, std::max<int64_t>(1, target)));
        return ceil_div(k, kTileKeys) * kTileKeys;
    };
    int64_t wave_split = pick(opt.split_keys, wave_keys, opt.target_items, kMinSplitKeys);
    int64_t tile_split = pick(opt.tile_split_keys, chunk_keys, opt.tile_target_items, kMinTileSplitKeys);
    for (;;) {
        int64_t n_split_items = 0, rows = 0;
        count_splits(wave_tiles, wave_split, n_split_items, rows);
        count_splits(chunk_tiles, tile_split, n_split_items, rows);
        if (n_split_items <= kMaxSplitItems && rows <= ws.max_part_rows &&
            (int64_t)wave_tiles.size() + (int64_t)chunk_tiles.size() + n_split_items <= ws.max_items)
            break;
        wave_split *= 2;
        tile_split *= 2;
    }
    plan.split_keys = (int32_t)std::min<int64_t>(wave_split, INT32_MAX);
    plan.tile_split_keys = (int32_t)std::min<int64_t>(tile_split, INT32_MAX);

    emit_items(chunk_tiles, tile_split, kKindTile, plan, scratch, bucket);
    plan.num_tile_items = (int32_t)plan.items.size();
    emit_items(wave_tiles, wave_split, kKindWave, plan, scratch, bucket);
}

}  // namespace sarathi
