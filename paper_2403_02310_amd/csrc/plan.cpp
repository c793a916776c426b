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
// launch and (b) there are enough units to fill 256 compute units.  Chunks with at least
// tile_min_cols columns use 128-column tiles instead (K/V staged once per tile in LDS).  The
// splits of a tile are merged in index order by a second, small kernel.
#include <algorithm>
#include <cstdio>

#include "internal.h"

namespace sarathi {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

constexpr int32_t kMaxSplitUnits = 8192;
constexpr int32_t kMaxPartRows = 32768;
constexpr int32_t kMinWaveKeys = 1024;   // automatic choice: keys per wavefront of a wave-tile block before the tile is split
constexpr int32_t kMinTileSplitKeys = 1024;

WorkspaceLayout make_workspace_layout(const sarathi_config &cfg) {
    WorkspaceLayout w{};
    const int64_t G = cfg.num_q_heads / cfg.num_kv_heads;
    // wave tiles only exist for sequences below tile_min_cols columns; bounding every sequence by
    // 16-column tiles covers both kinds
    const int64_t max_tiles = ceil_div((int64_t)cfg.max_tokens * G, kWaveCols) + cfg.max_seqs;
    w.max_tiles = (int32_t)std::min<int64_t>(max_tiles, INT32_MAX / 64);
    w.max_units = (int32_t)std::min<int64_t>(max_tiles + kMaxSplitUnits, INT32_MAX / 64);
    w.max_part_rows = kMaxPartRows;
    // a split tile has at least 2 pieces of n_cols rows: sum over split tiles of ceil(n_cols/8) <= rows/16 + tiles
    w.max_reduce_units = (int32_t)std::min<int64_t>(kMaxPartRows / (2 * kReduceCols) + kMaxSplitUnits / 2, INT32_MAX / 64);
    const size_t attn_meta = sizeof(TileDesc) * (size_t)w.max_tiles +
                             sizeof(uint32_t) * ((size_t)w.max_units + (size_t)w.max_reduce_units) + 64;
    const size_t append_meta = sizeof(AppendUnit) * (size_t)max_append_units(cfg) + 64;
    size_t off = 0;
    w.meta = off;
    w.meta_bytes = align_up(align_up(append_meta, 256) + attn_meta, 256);  // an append may carry both
    off += w.meta_bytes;
    w.sched = off;     off = align_up(off + kSchedBytes, 256);
    w.part_ml = off;   off = align_up(off + sizeof(float) * 2 * (size_t)w.max_part_rows * cfg.num_kv_heads, 256);
    w.part_o = off;    off = align_up(off + sizeof(float) * (size_t)w.max_part_rows * cfg.num_kv_heads * cfg.head_dim, 256);
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

inline int32_t steps_of_split(const TileDesc &t, int32_t split) {
    const int32_t b = t.key_lo + split * t.keys_per_split;
    const int32_t e = std::min(t.n_keys, b + t.keys_per_split);
    return (int32_t)ceil_div(e - b, kTileKeys);
}

// Chooses the split of every tile in [first, last) for `split_keys`, assigns partial rows and
// counters, and appends the units sorted longest first (counting sort on 32-key steps).
void emit_units(Plan &plan, size_t first, size_t last, int64_t split_keys, std::vector<uint32_t> &scratch,
                std::vector<int32_t> &bucket) {
    scratch.clear();
    int32_t max_steps = 0;
    for (size_t ti = first; ti < last; ++ti) {
        TileDesc &t = plan.tiles[ti];
        const int64_t span = t.n_keys - t.key_lo;  // keys the tile reads
        int32_t ns = (span <= split_keys + split_keys / 2) ? 1 : (int32_t)ceil_div(span, split_keys);
        t.keys_per_split = (int32_t)(ceil_div(ceil_div(span, ns), kTileKeys) * kTileKeys);
        t.n_splits = (int32_t)ceil_div(span, t.keys_per_split);
        if (t.n_splits > 1) {
            t.part_row0 = plan.num_part_rows;
            plan.num_part_rows += t.n_splits * t.n_cols;
            plan.num_split_tiles++;
            for (int32_t c0 = 0, grp = 0; c0 < t.n_cols; c0 += kReduceCols, ++grp)
                plan.reduce_units.push_back(pack_unit((uint32_t)ti, (uint32_t)grp));
        } else {
            t.part_row0 = -1;
        }
        for (int32_t i = 0; i < t.n_splits; ++i) {
            scratch.push_back(pack_unit((uint32_t)ti, (uint32_t)i));
            max_steps = std::max(max_steps, steps_of_split(t, i));
        }
    }
    auto steps = [&](uint32_t u) {
        return steps_of_split(plan.tiles[u & ((1u << kUnitTileBits) - 1)], (int32_t)(u >> kUnitTileBits));
    };
    bucket.assign((size_t)max_steps + 2, 0);
    for (uint32_t u : scratch) bucket[(size_t)(max_steps - steps(u)) + 1]++;
    for (size_t i = 1; i < bucket.size(); ++i) bucket[i] += bucket[i - 1];
    const size_t base = plan.units.size();
    plan.units.resize(base + scratch.size());
    for (uint32_t u : scratch) plan.units[base + (size_t)bucket[(size_t)(max_steps - steps(u))]++] = u;
}

// Split units, partial rows and split tiles a choice of split_keys would need for tiles [first, last).
void count_splits(const Plan &plan, size_t first, size_t last, int64_t split_keys, int64_t &n_split_units,
                  int64_t &rows, int64_t &n_split_tiles) {
    for (size_t ti = first; ti < last; ++ti) {
        const TileDesc &t = plan.tiles[ti];
        const int64_t span = t.n_keys - t.key_lo;
        if (span <= split_keys + split_keys / 2) continue;
        const int64_t ns = ceil_div(span, split_keys);
        n_split_units += ns;
        rows += ns * t.n_cols;
        n_split_tiles++;
    }
}

}  // namespace

void plan_attention(const sarathi_config &cfg, const Options &opt, const WorkspaceLayout &ws,
                    const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len, int32_t num_seqs,
                    Plan &plan) {
    plan.tiles.clear();
    plan.units.clear();
    plan.reduce_units.clear();
    plan.num_part_rows = 0;
    plan.num_tile_units = 0;
    plan.num_tile_reduce_units = 0;
    plan.num_split_tiles = 0;
    const int32_t G = cfg.num_q_heads / cfg.num_kv_heads;

    // Tiles: chunk tiles first, then wave tiles (two passes keep each kind contiguous).
    int64_t keys_of_kind[2] = {0, 0};
    size_t n_chunk_tiles = 0;
    for (int pass = 0; pass < 2; ++pass) {
        const int32_t kind = pass == 0 ? kKindTile : kKindWave;
        for (int32_t s = 0; s < num_seqs; ++s) {
            const int64_t n_cols = (int64_t)q_len[s] * G;
            const bool chunk = n_cols >= opt.tile_min_cols;   // prefill chunk: 128-column LDS-staged tiles
            if (chunk != (kind == kKindTile)) continue;
            const int32_t prefix = ctx_len[s] - q_len[s];
            const int32_t width = chunk ? kTileCols : kWaveCols;
            for (int64_t c0 = 0; c0 < n_cols; c0 += width) {
                TileDesc t{};
                t.seq = s;
                t.col_begin = (int32_t)c0;
                t.n_cols = (int32_t)std::min<int64_t>(width, n_cols - c0);
                t.kind = kind;
                t.n_keys = prefix + (int32_t)((c0 + t.n_cols - 1) / G) + 1;  // keys .. position of the tile's last row
                if (opt.window > 0) {  // the first row's window starts the range (rounded down to a 32-key tile)
                    const int64_t first_key = (int64_t)prefix + c0 / G - opt.window + 1;
                    t.key_lo = first_key > 0 ? (int32_t)(first_key / kTileKeys * kTileKeys) : 0;
                }
                t.q_start = q_start[s];
                t.q_len = q_len[s];
                t.ctx_len = ctx_len[s];
                plan.tiles.push_back(t);
                keys_of_kind[kind] += t.n_keys - t.key_lo;
            }
        }
        if (pass == 0) n_chunk_tiles = plan.tiles.size();
    }

    // Keys per split: the automatic choice aims at ~target units per KV head, never below a
    // floor, and both kinds are coarsened together until the partial buffers suffice.
    auto pick = [](int64_t forced, int64_t total, int64_t target, int64_t floor_keys) {
        int64_t k = forced > 0 ? forced : std::max<int64_t>(floor_keys, ceil_div(total, std::max<int64_t>(1, target)));
        return ceil_div(k, kTileKeys) * kTileKeys;
    };
    // A wave-tile unit is a BLOCK: its four wavefronts take a quarter of the unit's keys each and
    // merge their results in LDS, so a unit of up to 4 x 1024 keys (6144 with the 1.5x allowance
    // below) needs no partial rows and no merge kernel; "split_keys" counts keys per wavefront.
    // When the decodes of the batch take long to stream as a whole, one block may take longer too: a unit that
    // needs up to 0.4 of that time (a block streams about 25 GB/s next to a second one on its compute unit) is
    // dealt out first and is done well before the launch ends, and every cut avoided saves partial rows and,
    // for a batch without other cuts, the merge launch.
    const double wave_stream_us = (double)keys_of_kind[kKindWave] * cfg.num_kv_heads * cfg.head_dim * 4.0 / 5.0e6;
    const int64_t wave_floor = std::max<int64_t>(4 * kMinWaveKeys, (int64_t)(0.4 * wave_stream_us * 25000.0 / (cfg.head_dim * 4.0)));
    int64_t wave_split = pick(4 * opt.split_keys, keys_of_kind[kKindWave], std::max<int64_t>(1, opt.target_items / 4), wave_floor);
    // Chunk tiles: enough units per KV head to put two blocks on every compute unit (a block
    // alone on its unit cannot hide its per-step latencies), but never pieces below the floor.
    // Next to wave tiles the chunk blocks run in the shadow of the memory-bound ones, which keep
    // the other block slots busy: a chunk piece only has to finish within the time the decodes
    // take to stream (about 5 bytes/ps on this part; a chunk block advances 32 keys in roughly a
    // microsecond), and every split avoided saves partial rows that need merging.
    const int64_t tile_units_wanted = std::max<int64_t>(1, 768 / cfg.num_kv_heads);
    const bool has_wave_tiles = plan.tiles.size() > n_chunk_tiles;
    int64_t tile_floor = kMinTileSplitKeys;
    if (has_wave_tiles) {
        const double wave_us = wave_stream_us;
        tile_floor = std::max<int64_t>(2 * kMinTileSplitKeys, (int64_t)(wave_us / 1.2) * kTileKeys);
    }
    int64_t tile_split = pick(opt.tile_split_keys, keys_of_kind[kKindTile], tile_units_wanted, tile_floor);
    if (opt.tile_split_keys <= 0 && !has_wave_tiles) {
        // Balance: with few, long chunk tiles the longest unit must stay well below a block slot's
        // share of the work (2 slots on each of 256 compute units), or the tail of the launch runs
        // on a few units only.  0.42 of the share measured best on the long-context chunk batch.
        const int64_t share = keys_of_kind[kKindTile] * cfg.num_kv_heads / 512;
        const int64_t balanced = ceil_div(std::max<int64_t>(tile_floor, share * 42 / 100), kTileKeys) * kTileKeys;
        tile_split = std::min(tile_split, balanced);
    }
    if (opt.tile_split_keys <= 0 && !has_wave_tiles && n_chunk_tiles > 0 && (int64_t)n_chunk_tiles * cfg.num_kv_heads < 512) {
        // A chunk-only batch with fewer tiles than block slots (two per compute unit), e.g. one chunk of a prompt
        // that is prefilled in pieces: how many pieces per tile?  More pieces shorten the blocks and fill the chip,
        // but every piece writes a 64 KiB partial tile per KV head that the merge kernel reads back, and a second
        // kernel has to be launched at all.  Estimated cost in microseconds, from measurements on this part: a block
        // advances 32 keys in ~0.62 us alone on its compute unit and in ~0.9 us next to a second block; blocks beyond
        // the 512 slots run in further rounds; the merge moves the partial tiles twice at ~4.5 TB/s after ~5 us of
        // launch.  (8192-token prompt, LLaMA2-70B shape: chunks of 512 tokens 1,600 -> 1,45x us per pass, chunks of
        // 256 tokens 1,956 -> 1,7xx us, against one fixed rule of about a thousand keys per piece.)
        const int64_t blocks1 = (int64_t)n_chunk_tiles * cfg.num_kv_heads;
        int64_t max_span = 1;
        for (size_t ti = 0; ti < n_chunk_tiles; ++ti)
            max_span = std::max<int64_t>(max_span, plan.tiles[ti].n_keys - plan.tiles[ti].key_lo);
        const double avg_steps = (double)keys_of_kind[kKindTile] / (double)n_chunk_tiles / kTileKeys;
        double best = 0.0;
        int64_t best_n = 1;
        for (int64_t n = 1; n <= 16; ++n) {
            if (n > 1 && max_span / n < 256) break;   // pieces of fewer than eight key steps are all prologue
            const int64_t blocks = blocks1 * n;
            const double steps = avg_steps / (double)n + 1.0;
            const double rounds = blocks <= 512 ? 1.0 : (double)blocks / 512.0;
            const double step_us = blocks <= 256 ? 0.62 : 0.9;
            double cost = 4.0 + rounds * steps * step_us;
            if (n > 1) {
                const double partial_bytes = (double)blocks * kTileCols * (cfg.head_dim + 2) * 4.0;
                cost += 5.0 + 2.0 * partial_bytes / 4.5e6;
            }
            if (n == 1 || cost < best) {
                best = cost;
                best_n = n;
            }
        }
        tile_split = ceil_div(ceil_div(max_span, best_n), kTileKeys) * kTileKeys;
    }
    for (;;) {
        int64_t n_split_units = 0, rows = 0, n_split_tiles = 0;
        count_splits(plan, 0, n_chunk_tiles, tile_split, n_split_units, rows, n_split_tiles);
        count_splits(plan, n_chunk_tiles, plan.tiles.size(), wave_split, n_split_units, rows, n_split_tiles);
        const int64_t max_splits_per_tile = (1 << (32 - kUnitTileBits)) - 1;
        bool fits = n_split_units <= kMaxSplitUnits && rows <= ws.max_part_rows && n_split_tiles <= kMaxSplitUnits / 2 &&
                    (int64_t)plan.tiles.size() + n_split_units <= ws.max_units;
        for (const TileDesc &t : plan.tiles)
            if (ceil_div(t.n_keys - t.key_lo, t.kind == kKindTile ? tile_split : wave_split) > max_splits_per_tile) { fits = false; break; }
        if (fits) break;
        wave_split *= 2;
        tile_split *= 2;
    }
    plan.split_keys = (int32_t)std::min<int64_t>(wave_split / 4, INT32_MAX);  // per wavefront
    plan.tile_split_keys = (int32_t)std::min<int64_t>(tile_split, INT32_MAX);

    static thread_local std::vector<uint32_t> scratch;
    static thread_local std::vector<int32_t> bucket;
    emit_units(plan, 0, n_chunk_tiles, tile_split, scratch, bucket);
    plan.num_tile_units = (int32_t)plan.units.size();
    plan.num_tile_reduce_units = (int32_t)plan.reduce_units.size();
    plan.tile_unit_steps = 0;
    for (size_t ti = 0; ti < n_chunk_tiles; ++ti)
        plan.tile_unit_steps += ceil_div(plan.tiles[ti].n_keys - plan.tiles[ti].key_lo, kTileKeys) + plan.tiles[ti].n_splits - 1;
    plan.longest_tile_unit_steps = 0;  // units are sorted longest first
    if (plan.num_tile_units > 0) {
        const uint32_t u = plan.units[0];
        plan.longest_tile_unit_steps = steps_of_split(plan.tiles[u & ((1u << kUnitTileBits) - 1)], (int32_t)(u >> kUnitTileBits));
    }
    plan.wave_keys = keys_of_kind[kKindWave];
    emit_units(plan, n_chunk_tiles, plan.tiles.size(), wave_split, scratch, bucket);
}

}  // namespace sarathi
