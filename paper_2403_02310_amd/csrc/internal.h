// Internal declarations shared by the host planner and the HIP launchers of libsarathi.
// Not part of the ABI (the ABI is include/sarathi.h).
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "sarathi.h"

namespace sarathi {

constexpr int kPageSize = 16;     // tokens per page (the only supported value)
constexpr int kTileKeys = 32;     // keys per inner-loop tile = two pages = one MFMA contraction depth
constexpr int kWaveCols = 16;     // query columns a wave tile carries (16x16x32 MFMA N dimension)
constexpr int kTileCols = 128;    // query columns a chunk tile carries (4 waves x 32x32x16 MFMA N dimension)
constexpr int kKindWave = 0;      // WorkItem::kind
constexpr int kKindTile = 1;

// One unit of attention work: a tile of query columns of one sequence against a key range.
// A "column" is one (query row, query head inside a KV group) pair: col = row*G + head_in_group.
// The same item runs once per KV head (the KV head is taken from the block index).
struct WorkItem {
    int32_t seq;
    int32_t col_begin;
    int32_t n_cols;
    int32_t key_begin;   // multiple of kTileKeys
    int32_t key_end;     // exclusive
    int32_t part_row;    // first partial row, or -1: normalise and write `out` directly
    int32_t kind;
    int32_t reserved;
};
static_assert(sizeof(WorkItem) == 32, "WorkItem is copied to the device as raw bytes");
static_assert(sizeof(WorkItem) == sizeof(sarathi_work_item), "debug view must mirror WorkItem");

// Merge of the splits of one tile: partial rows part_row + split*n_cols + col.
struct ReduceItem {
    int32_t seq;
    int32_t col_begin;
    int32_t n_cols;
    int32_t part_row;
    int32_t n_splits;
    int32_t reserved[3];
};
static_assert(sizeof(ReduceItem) == 32, "ReduceItem is copied to the device as raw bytes");

struct Plan {
    std::vector<WorkItem> items;          // chunk tiles first (num_tile_items of them), then wave tiles
    int32_t num_tile_items = 0;
    std::vector<ReduceItem> reduce_items;
    int32_t num_part_rows = 0;
    int32_t split_keys = 0;
    int32_t tile_split_keys = 0;
};

// Byte offsets of the regions inside the caller's workspace (all 256-byte aligned).
struct WorkspaceLayout {
    size_t seq_meta;      // int32 [3][max_seqs]: q_start, q_len, ctx_len
    size_t items;         // WorkItem [max_items]
    size_t reduce_items;  // ReduceItem [max_reduce_items]
    size_t part_ml;       // float [max_part_rows][Hkv][2]
    size_t part_o;        // float [max_part_rows][Hkv][head_dim]
    size_t total;
    int32_t max_items;
    int32_t max_reduce_items;
    int32_t max_part_rows;
};

struct Options {
    int64_t split_keys = 0;      // 0 = automatic
    int64_t target_items = 1536; // automatic choice aims for about this many wave items per KV head
    int64_t tile_split_keys = 0;  // the same two knobs for the 128-column chunk tiles
    int64_t tile_target_items = 96;
    int64_t tile_min_cols = 64;   // sequences with fewer columns (q_len*G) use wave tiles only
};

WorkspaceLayout make_workspace_layout(const sarathi_config &cfg);

// Validation of a batch description; returns SARATHI_OK or an error with `err` set.
sarathi_status validate_batch(const sarathi_config &cfg, const int32_t *q_start, const int32_t *q_len,
                              const int32_t *ctx_len, int32_t num_seqs, int32_t num_tokens,
                              int64_t num_pages, std::string &err);

// Work decomposition for sarathi_hybrid_attention.
void plan_attention(const sarathi_config &cfg, const Options &opt, const WorkspaceLayout &ws,
                    const int32_t *q_len, const int32_t *ctx_len, int32_t num_seqs, Plan &plan);

// ---- device launchers (attn_kernels.hip); each returns a hipError_t cast to int ----
struct DeviceBatch {
    const int32_t *q_start;      // dev [S]
    const int32_t *q_len;        // dev [S]
    const int32_t *ctx_len;      // dev [S]
    const int32_t *block_table;  // dev [S][max_blocks]
    int32_t max_blocks;
    int32_t num_seqs;
    int32_t num_tokens;
};

int launch_kv_append(const sarathi_config &cfg, const DeviceBatch &b, const void *k_new, const void *v_new,
                     void *k_cache, void *v_cache, int64_t num_pages, void *stream);

int launch_attention(const sarathi_config &cfg, const DeviceBatch &b, const void *q, const void *k_cache,
                     const void *v_cache, int64_t num_pages, float sm_scale, void *out, const WorkItem *items,
                     int32_t num_tile_items, int32_t num_items, float *part_ml, float *part_o, void *stream);

int launch_reduce(const sarathi_config &cfg, const DeviceBatch &b, const ReduceItem *items, int32_t num_items,
                  const float *part_ml, const float *part_o, void *out, void *stream);

}  // namespace sarathi
