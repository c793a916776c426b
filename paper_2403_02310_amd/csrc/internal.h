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
constexpr int kReduceCols = 8;    // columns one block of the merge kernel handles
constexpr int kKindWave = 0;
constexpr int kKindTile = 1;
// Scheduling words of the one-launch hybrid kernel when blocks pick their role at run time:
// one "a chunk block lives here" flag per compute unit (indexed by hardware ids), then per-KV-head
// queue heads [kind][kv head].  The host zeroes them (fill kernel) in front of every launch that uses them.
constexpr int kSchedCuSlots = 4096;
constexpr int kSchedMaxKvHeads = 128;
constexpr size_t kSchedBytes = sizeof(int32_t) * (kSchedCuSlots + 2 * kSchedMaxKvHeads);
constexpr int kChunkBlocksForRoles = 256;   // one per compute unit
// Dynamic LDS that, added to a wave-tile block's own 17-34 KiB, leaves room for one such block per compute unit (160 KiB).
constexpr int kOneBlockPerUnitLdsPad = 64 * 1024;

// One tile of query columns of one sequence.  A "column" is one (query row, query head inside
// a KV group) pair: col = row*G + head_in_group.  Its key range key_lo..n_keys-1 (key_lo = 0
// without a sliding window, else a multiple of 32 at or below the first key its first row sees) is
// cut into n_splits pieces of keys_per_split keys (a multiple of 32; the last piece is shorter);
// every piece is one work unit, run once per KV head.  The descriptor carries the sequence's lengths
// so that a unit needs no further lookups.
struct TileDesc {
    int32_t seq;
    int32_t col_begin;
    int32_t n_cols;
    int32_t kind;
    int32_t n_keys;
    int32_t keys_per_split;
    int32_t n_splits;
    int32_t part_row0;    // first partial row of split 0 (split i uses part_row0 + i*n_cols ..), -1 if n_splits == 1
    int32_t key_lo;
    int32_t q_start;
    int32_t q_len;
    int32_t ctx_len;
};
static_assert(sizeof(TileDesc) == 48, "TileDesc is copied to the device as raw bytes");

// A work unit = (tile index, split index) packed into 32 bits.
constexpr int kUnitTileBits = 22;
inline uint32_t pack_unit(uint32_t tile, uint32_t split) { return (split << kUnitTileBits) | tile; }

struct Plan {
    std::vector<TileDesc> tiles;
    std::vector<uint32_t> units;      // chunk-tile units first (num_tile_units), then wave-tile units; longest first in each group;
                                      // every unit is one block per KV head (a wave-tile block quarters its keys among its wavefronts)
    int32_t num_tile_units = 0;
    std::vector<uint32_t> reduce_units;  // (8-column group, tile) of every split tile, for the merge kernel; chunk tiles first
    int32_t num_tile_reduce_units = 0;   // how many of them belong to chunk tiles
    int32_t num_split_tiles = 0;      // tiles with n_splits > 1
    int32_t num_part_rows = 0;
    int32_t split_keys = 0;
    int32_t tile_split_keys = 0;
    int64_t tile_unit_steps = 0;      // 32-key steps summed over the chunk-tile units
    int32_t longest_tile_unit_steps = 0;  // 32-key steps of the longest chunk-tile unit
    int64_t wave_keys = 0;            // keys summed over the wave tiles
};

// Byte offsets of the regions inside the caller's workspace (all 256-byte aligned).
struct WorkspaceLayout {
    size_t meta;          // per-call metadata, packed: sequence arrays + hints (append) or tile descriptors + units (attention)
    size_t meta_bytes;
    size_t sched;         // int32 [kSchedCuSlots + 2*kSchedMaxKvHeads], zeroed by the host before each launch that uses it
    size_t part_ml;       // float [max_part_rows][Hkv][2]
    size_t part_o;        // float [max_part_rows][Hkv][head_dim]
    size_t total;
    int32_t max_tiles;
    int32_t max_units;
    int32_t max_reduce_units;
    int32_t max_part_rows;
};

struct Options {
    int64_t split_keys = 0;         // keys per wavefront of a wave-tile block (a block covers four times as many); 0 = automatic
    int64_t target_items = 1536;    // automatic choice aims for about this many wavefronts of wave-tile work per KV head
    int64_t tile_split_keys = 0;    // keys per split of the 128-column chunk tiles, 0 = automatic
    int64_t tile_min_cols = 64;     // sequences with fewer columns (q_len*G) use wave tiles only
    int64_t plan_at_append = 1;     // sarathi_kv_append also plans and uploads the attention metadata of its batch
    int64_t interleave = 2;         // batches with both kinds of tile: 0 = two launches in sequence, 1 = chunk kernel on a
                                    // second stream next to the wave kernel, 2 = one launch holding both kinds of block
    int64_t window = 0;             // sliding-window attention: a query sees its last `window` keys (itself included); 0 = all
    int64_t stream_kv = -1;         // decode K/V loads carry the streaming (non-temporal) hint: -1 = when the batch's chunk
                                    // work is absent or small next to its decode streams, or its longest chunk unit
                                    // runs about as long as they do; 0 = never, 1 = always
    int64_t decode_blocks_per_cu = -1;  // launches of wave tiles only: 2 = as many blocks per compute unit as fit, 1 = one (unused LDS
                                    // keeps a second one out, so blocks start longest first as units fall free instead of
                                    // all at once); -1 = one for up to 1024 blocks, two beyond
    int64_t inline_append = 1;      // KV append: up to 224 page records travel in the kernel's arguments (else all are read from the pinned buffer)
    int64_t lds_pad_kb = 0;         // diagnostic only: KiB of unused LDS added to every attention block
    int64_t resident_chunks = -1;   // one-launch mode: blocks take their role (chunk or wave tiles) when they start, so that
                                    // a compute unit holds at most one chunk block while decode work remains
                                    // (-1 = when there are more chunk blocks than compute units, 0 = never, 1 = always)
};

WorkspaceLayout make_workspace_layout(const sarathi_config &cfg);

// Validation of a batch description; returns SARATHI_OK or an error with `err` set.
sarathi_status validate_batch(const sarathi_config &cfg, const int32_t *q_start, const int32_t *q_len,
                              const int32_t *ctx_len, int32_t num_seqs, int32_t num_tokens,
                              int64_t num_pages, std::string &err);

// Work decomposition for sarathi_hybrid_attention.
void plan_attention(const sarathi_config &cfg, const Options &opt, const WorkspaceLayout &ws,
                    const int32_t *q_start, const int32_t *q_len, const int32_t *ctx_len, int32_t num_seqs,
                    Plan &plan);

// ---- device launchers (attn_kernels.hip); each returns a hipError_t cast to int ----
// The append kernel's work item is a page unit: the slots [lo, hi) of ONE cache page that this
// iteration fills for one sequence (a decode has one unit, a chunk one per page it touches).
struct AppendUnit {
    int32_t seq;        // sequence index (row of the block table)
    int32_t page_idx;   // logical page of the sequence (column of the block table)
    int32_t row0;       // batch row of the token that goes to slot `lo`
    int32_t lo_hi;      // lo | hi << 8, 0 <= lo < hi <= 16
};
static_assert(sizeof(AppendUnit) == 16, "AppendUnit is uploaded as is and read as one 16-byte word");
// every sequence touches at most q_len/16 + 2 pages
inline int64_t max_append_units(const sarathi_config &cfg) {
    return (int64_t)cfg.max_tokens / kPageSize + 2 * (int64_t)cfg.max_seqs;
}

struct AppendMeta {
    const AppendUnit *units;     // [num_units]; device memory, or pinned host memory by the address the device uses for it
    const AppendUnit *units_host = nullptr;  // the same records as the host addresses them (null: not host-readable);
                                             // few enough of them travel in the kernel's arguments instead
    const int32_t *block_table;  // dev [S][max_blocks]
    int32_t max_blocks;
    int32_t num_units;
    // bytes the launch also moves from copy_src (pinned host memory, device-side address) to copy_dst (device):
    // rounded up to 16, both 16-byte aligned; 0 = nothing
    void *copy_dst = nullptr;
    const void *copy_src = nullptr;
    size_t copy_bytes = 0;
};

int launch_kv_append(const sarathi_config &cfg, const AppendMeta &m, const void *k_new, const void *v_new,
                     void *k_cache, void *v_cache, int64_t num_pages, void *stream);

struct AttnMeta {
    const TileDesc *tiles;       // dev
    const uint32_t *units;       // dev
    int32_t num_tile_units;
    int32_t num_units;
    const int32_t *block_table;  // dev [S][max_blocks]
    int32_t max_blocks;
    const uint32_t *reduce_units;  // dev
    int32_t num_reduce_units;
    int32_t num_tile_reduce_units;   // leading entries of reduce_units that belong to chunk tiles
    float *part_ml;              // dev
    float *part_o;               // dev
    int32_t *sched;              // dev, kSchedBytes
    int32_t window;              // sliding window in keys, 0 = none
    int32_t stream_kv;           // 1: the wave tiles' K/V loads carry the streaming hint
    int32_t lds_pad_bytes = 0;   // diagnostic: dynamic LDS added to the attention launches (fewer blocks per compute unit)
};

// which: bit 0 = the chunk-tile kernel, bit 1 = the wave-tile kernel, 4 = both kinds in one launch,
// 5 = one launch whose blocks take their role at run time (needs m.sched zeroed, see launch_zero)
int launch_attention(const sarathi_config &cfg, const AttnMeta &m, const void *q, const void *k_cache,
                     const void *v_cache, int64_t num_pages, float sm_scale, void *out, int which, void *stream);

// Merges the split tiles named by reduce_units[first .. first+count).
// Fills `bytes` (a multiple of 4) at `ptr` with zeros by a small kernel (no memset node: callers may capture).
int launch_zero(void *ptr, size_t bytes, void *stream);
// Copies `bytes` (rounded up to 16; both buffers hold the rounded size and are 16-byte aligned) from pinned
// host memory, given by the address the device uses for it, to device memory by a small kernel.
int launch_upload(void *dst, const void *pinned_src, size_t bytes, void *stream);

int launch_reduce(const sarathi_config &cfg, const AttnMeta &m, void *out, int32_t first, int32_t count, void *stream);

// ---- scratch memory inside the library's device image (allocation-free entry point) ----
// One array per GPU, laid out as the regions of a caller's workspace are: metadata, scheduling words, split-KV
// partials.  The sizes are fixed at build time; a batch whose plan does not fit is refused.
constexpr size_t kStaticMetaBytes = (size_t)96 << 10;     // packed plan of one call
constexpr size_t kStaticPartMlBytes = (size_t)512 << 10;  // (maximum, sum) of the partial rows: part_o bytes * 2 / head_dim at most
constexpr size_t kStaticPartOBytes = (size_t)16 << 20;    // unnormalised outputs of the partial rows
struct StaticScratch {
    char *meta;
    int32_t *sched;
    float *part_ml;
    float *part_o;
};
// Device addresses of the regions on the CURRENT device (looked up once per device, then remembered).
int static_scratch(StaticScratch *out);
// Copies `bytes` (a multiple of 16, dst 16-byte aligned) from ordinary host memory to device memory by kernels that
// carry the data in their arguments: no pinned buffer, no runtime copy, the host buffer is free on return.
int launch_upload_args(void *dst, const void *host_src, size_t bytes, void *stream);

// ---- linear layer (linear_kernels.hip) ----
struct LinearPlan {
    int32_t feature_tile; // output features per workgroup tile: 256 or 128
    int32_t token_tile;   // tokens per workgroup tile: 256, 128, 64 or 32
    int32_t n_tiles;      // feature tiles
    int32_t t_tiles;      // token tiles
    int32_t splits;       // pieces of the k range (1 = none); pieces write fp32 partial tiles
    int32_t k_per_split;  // multiple of 64
};
// Tiling of y[T, N] = x[T, K] w[N, K]^T; the k range is cut only as far as `workspace_bytes` holds the partial tiles.
LinearPlan plan_linear(int32_t T, int32_t N, int32_t K, size_t workspace_bytes);
int launch_linear(const LinearPlan &pl, const void *x, const void *w, void *y, int32_t T, int32_t N, int32_t K,
                  void *workspace, void *stream);

}  // namespace sarathi
