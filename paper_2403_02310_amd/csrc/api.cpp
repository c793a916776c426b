// Entry points of libsarathi that touch the HIP runtime: handle life cycle, metadata staging,
// and the enqueue of the kernels.  Everything here is argument checking, planning and
// bookkeeping; every step of the attention path itself runs in the kernels.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "internal.h"

using namespace sarathi;

namespace {
constexpr int kStagingSlots = 16;
constexpr int kStagingHalf = kStagingSlots / 2;
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
}  // namespace

struct sarathi_handle {
    sarathi_config cfg;
    Options opt;
    WorkspaceLayout ws;
    std::string err;
    Plan plan;
    // Ring of pinned host buffers for the per-call metadata, in two halves.  An event is recorded behind the
    // upload (a kernel that reads the pinned buffer) out of a half's LAST slot only, and waited for before the half's first slot is written again,
    // half a ring of calls later: calls may be enqueued back to back without the host ever waiting in the
    // steady state, and the stream carries one event per kStagingHalf calls instead of one per call (an
    // event record between two kernels keeps the second from starting for ~6 us: kernel trace of the
    // hybrid batch).  All copies out of a half go through one stream, so that its event covers them.
    void *staging[kStagingSlots] = {};
    void *staging_dev[kStagingSlots] = {};  // the same buffers as the device addresses them
    hipEvent_t half_done[2] = {};
    bool half_pending[2] = {};
    hipStream_t half_stream[2] = {};
    bool staging_used = false;
    size_t staging_bytes = 0;
    int next_slot = 0;
    bool staging_ready = false;
    // Attention metadata uploaded ahead of time by sarathi_kv_append: the iteration's attention
    // call gets the same description, so its plan rides along in the append's copy.  Valid while
    // `resident_*` describe what the metadata region of `resident_ws` holds.
    void *resident_ws = nullptr;
    void *resident_stream = nullptr;
    std::vector<int32_t> resident_desc;  // q_len | ctx_len of the planned batch
    uint64_t resident_opt_version = 0;
    uint64_t opt_version = 1;
    size_t resident_attn_off = 0;        // byte offset of the attention metadata inside the region
    // Second stream (default priority) on which the chunk-tile kernel runs next to the wave-tile
    // kernel, and the events that fork it from / join it into the caller's stream.
    hipStream_t side_stream = nullptr;
    hipEvent_t fork_event = nullptr, join_event = nullptr;
    // Optional per-kernel timing: event pairs recorded around each launch.
    int time_kernels = 0;  // 0 off, 1 attention launches only, 2 also the append and merge kernels
    int64_t time_every = 1;  // bracket every n-th launch of a kind only
    uint64_t timing_seen[3] = {0, 0, 0};
    std::vector<std::pair<hipEvent_t, hipEvent_t>> timing_pool[3];  // append, attention, merge
    size_t timing_used[3] = {0, 0, 0};
    // host image of the packed plan for the allocation-free entry point (sized once, at creation)
    std::vector<char> noalloc_meta;
};

namespace {

sarathi_status fail(sarathi_handle *h, sarathi_status st, const std::string &msg) {
    if (h) h->err = msg;
    return st;
}

sarathi_status hip_fail(sarathi_handle *h, const char *what, hipError_t e) {
    return fail(h, SARATHI_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

sarathi_status ensure_staging(sarathi_handle *h) {
    if (h->staging_ready) return SARATHI_OK;
    h->staging_bytes = h->ws.meta_bytes;  // mirrors the metadata region of the workspace
    for (int i = 0; i < kStagingSlots; ++i) {
        hipError_t e = hipHostMalloc(&h->staging[i], h->staging_bytes, hipHostMallocDefault);
        if (e != hipSuccess) return hip_fail(h, "hipHostMalloc(staging)", e);
        e = hipHostGetDevicePointer(&h->staging_dev[i], h->staging[i], 0);
        if (e != hipSuccess) return hip_fail(h, "hipHostGetDevicePointer(staging)", e);
    }
    for (int i = 0; i < 2; ++i) {
        hipError_t e = hipEventCreateWithFlags(&h->half_done[i], hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(h, "hipEventCreate", e);
    }
    h->staging_ready = true;
    return SARATHI_OK;
}

sarathi_status acquire_slot(sarathi_handle *h, hipStream_t stream, int *slot) {
    const int s = h->next_slot;
    const int half = s / kStagingHalf;
    if (s % kStagingHalf == 0) {
        if (h->half_pending[half]) {  // recorded half a ring of calls ago
            hipError_t e = hipEventSynchronize(h->half_done[half]);
            if (e != hipSuccess) return hip_fail(h, "hipEventSynchronize(staging half)", e);
            h->half_pending[half] = false;
        }
        h->half_stream[half] = stream;
    } else if (stream != h->half_stream[half]) {
        // another stream inside a half: the half's event would not cover the copies already enqueued
        hipError_t e = hipStreamSynchronize(h->half_stream[half]);
        if (e != hipSuccess) return hip_fail(h, "hipStreamSynchronize(staging half)", e);
        h->half_stream[half] = stream;
    }
    h->next_slot = (s + 1) % kStagingSlots;
    h->staging_used = true;
    *slot = s;
    return SARATHI_OK;
}

// After the launch that reads `slot` has been enqueued on `stream` (or was given up: a half's last slot
// records the half's event either way, so that the launches out of its other slots stay covered).
sarathi_status release_slot(sarathi_handle *h, int slot, hipStream_t stream) {
    if (slot % kStagingHalf != kStagingHalf - 1) return SARATHI_OK;
    const int half = slot / kStagingHalf;
    hipError_t e = hipEventRecord(h->half_done[half], stream);
    if (e != hipSuccess) return hip_fail(h, "hipEventRecord(staging half)", e);
    h->half_pending[half] = true;
    return SARATHI_OK;
}

// Releases an acquired slot on every path out of the call that holds it.
struct SlotGuard {
    sarathi_handle *h;
    int slot;
    hipStream_t stream;
    bool released = false;
    sarathi_status release() {
        released = true;
        return release_slot(h, slot, stream);
    }
    ~SlotGuard() {
        if (!released) (void)release_slot(h, slot, stream);
    }
};

constexpr size_t kMaxTimedLaunches = 8192;

// Records the start event of a timed launch; returns the pair index or -1 when timing is off/full.
int timing_begin(sarathi_handle *h, int kind, hipStream_t s) {
    if (h->time_kernels < (kind == 1 ? 1 : 2) || h->timing_used[kind] >= kMaxTimedLaunches) return -1;
    if (h->timing_seen[kind]++ % (uint64_t)h->time_every != 0) return -1;
    auto &pool = h->timing_pool[kind];
    if (h->timing_used[kind] == pool.size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return -1;
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return -1; }
        pool.emplace_back(a, b);
    }
    const int idx = (int)h->timing_used[kind];
    if (hipEventRecord(pool[idx].first, s) != hipSuccess) return -1;
    return idx;
}

void timing_end(sarathi_handle *h, int kind, int idx, hipStream_t s) {
    if (idx < 0) return;
    if (hipEventRecord(h->timing_pool[kind][idx].second, s) == hipSuccess) h->timing_used[kind] = (size_t)idx + 1;
}

// Attention metadata, packed back to back at `dst`: tile descriptors, work units, merge units.
struct AttnMetaOffsets {
    size_t units, reduce, total;
};
AttnMetaOffsets attn_meta_offsets(const Plan &pl) {
    AttnMetaOffsets o;
    o.units = align_up(sizeof(TileDesc) * pl.tiles.size(), 16);
    o.reduce = o.units + sizeof(uint32_t) * pl.units.size();
    o.total = align_up(o.reduce + sizeof(uint32_t) * pl.reduce_units.size(), 16);
    return o;
}
template <typename T>
void copy_vector(char *dst, const std::vector<T> &v) {   // an empty vector may have no storage at all
    if (!v.empty()) std::memcpy(dst, v.data(), sizeof(T) * v.size());
}
void pack_attn_meta(char *dst, const Plan &pl, const AttnMetaOffsets &o) {
    copy_vector(dst, pl.tiles);
    copy_vector(dst + o.units, pl.units);
    copy_vector(dst + o.reduce, pl.reduce_units);
}

bool resident_plan_matches(const sarathi_handle *h, const int32_t *q_len, const int32_t *ctx_len, int32_t n,
                           const void *workspace, const void *stream) {
    if (h->resident_ws != workspace || h->resident_stream != stream || h->resident_opt_version != h->opt_version) return false;
    if (h->resident_desc.size() != 2 * (size_t)n) return false;
    return std::memcmp(h->resident_desc.data(), q_len, sizeof(int32_t) * (size_t)n) == 0 &&
           std::memcmp(h->resident_desc.data() + n, ctx_len, sizeof(int32_t) * (size_t)n) == 0;
}

// Enqueues the attention launch (and the merge of split tiles) for h->plan, whose packed metadata is at `dev`.
// `instrumented` = false: the allocation-free entry point, which records no timing events and never forks a
// second stream (both create runtime objects on first use).
sarathi_status enqueue_attention(sarathi_handle *h, char *dev, float *part_ml, float *part_o, int32_t *sched,
                                 const int32_t *block_table, const void *q, const void *k_cache, const void *v_cache,
                                 int64_t num_pages, float sm_scale, void *out, hipStream_t s, bool instrumented) {
    const Plan &pl = h->plan;
    const AttnMetaOffsets mo = attn_meta_offsets(pl);
    const size_t units_off = mo.units, reduce_off = mo.reduce;
    void *stream = static_cast<void *>(s);
    hipError_t e;

    AttnMeta m;
    m.tiles = reinterpret_cast<const TileDesc *>(dev);
    m.units = reinterpret_cast<const uint32_t *>(dev + units_off);
    m.num_tile_units = pl.num_tile_units;
    m.num_units = (int32_t)pl.units.size();
    m.block_table = block_table;
    m.max_blocks = h->cfg.max_blocks_per_seq;
    m.reduce_units = reinterpret_cast<const uint32_t *>(dev + reduce_off);
    m.num_reduce_units = (int32_t)pl.reduce_units.size();
    m.num_tile_reduce_units = pl.num_tile_reduce_units;
    m.part_ml = part_ml;
    m.part_o = part_o;
    m.sched = sched;
    m.window = (int32_t)h->opt.window;
    m.lds_pad_bytes = (int32_t)h->opt.lds_pad_kb * 1024;
    {
        // A small decode-only batch whose blocks are all resident at once shares the memory system evenly among
        // them, so the longest decode runs at a 512th of the bandwidth for most of its life and then alone at what
        // one block can pull (~36 GB/s): a tail of 15-20 us on 64 decodes.  With one block per compute unit the blocks
        // start longest first as units fall free and each streams at twice the share; one block per unit already
        // reaches the chip's streaming rate (256 blocks x 25.5 GB/s).  Measured on 48 ... 128 decodes: -12 to -20 %;
        // from ~192 decodes on the launch is long enough for two per unit to win by 2-4 %.
        const int64_t wave_blocks = (int64_t)((int32_t)pl.units.size() - pl.num_tile_units) * h->cfg.num_kv_heads;
        const bool wave_only = pl.num_tile_units == 0;
        const bool one = h->opt.decode_blocks_per_cu == 1 || (h->opt.decode_blocks_per_cu < 0 && wave_blocks <= 1024);
        if (wave_only && one && m.lds_pad_bytes == 0) m.lds_pad_bytes = kOneBlockPerUnitLdsPad;
    }
    // Rough durations: chunk work with one block per compute unit (~0.65 us per 32-key step), and the time
    // the decodes need to stream their keys and values (~5 bytes/ps).
    const double chunk_us = (double)pl.tile_unit_steps * h->cfg.num_kv_heads * 0.65 / kChunkBlocksForRoles;
    const double wave_us = (double)pl.wave_keys * h->cfg.num_kv_heads * h->cfg.head_dim * 4.0 / 5.0e6;
    // The streaming hint pays on decode streams (+2 to +7 % without chunk work) and where the batch's longest
    // chunk unit runs about as long as the decodes stream, because the chunk blocks, whose K/V tiles then stay in
    // L2, are what the launch waits for (+1 to +3 % on a 512-token chunk behind a 3000-token prefix next to 64
    // decodes); it costs 2 to 3 % where the decodes are the last to finish next to chunk work that matters (the
    // same batch with a 1400-token prefix; the long-context batch).  A chunk block's 32-key step takes ~0.9 us
    // next to streaming decodes.
    const double chunk_tail_us = (double)pl.longest_tile_unit_steps * 0.9;
    const bool stream_auto = chunk_us < 0.1 * wave_us || chunk_tail_us > 0.7 * wave_us;
    m.stream_kv = h->opt.stream_kv >= 0 ? (int32_t)h->opt.stream_kv : (stream_auto ? 1 : 0);
    // Chunk tiles (compute-bound) and wave tiles (memory-bound) are two kernels; when the batch
    // has both they run side by side: the chunk kernel is forked onto a second stream, where the
    // merge of its own split tiles follows it (hidden behind the longer wave kernel).
    const bool both = pl.num_tile_units > 0 && (int32_t)pl.units.size() > pl.num_tile_units;
    const bool fork = both && h->opt.interleave == 1 && instrumented;
    if (fork && !h->side_stream) {
        e = hipStreamCreateWithFlags(&h->side_stream, hipStreamNonBlocking);
        if (e != hipSuccess) return hip_fail(h, "hipStreamCreate(side)", e);
        e = hipEventCreateWithFlags(&h->fork_event, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&h->join_event, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(h, "hipEventCreate(fork/join)", e);
    }
    int32_t merged_on_side = 0;
    const int t1 = instrumented ? timing_begin(h, 1, s) : -1;
    if (fork) {
        e = hipEventRecord(h->fork_event, s);
        if (e == hipSuccess) e = hipStreamWaitEvent(h->side_stream, h->fork_event, 0);
        if (e != hipSuccess) return hip_fail(h, "fork to side stream", e);
        e = (hipError_t)launch_attention(h->cfg, m, q, k_cache, v_cache, num_pages, sm_scale, out, 1, h->side_stream);
        if (e == hipSuccess) e = (hipError_t)launch_reduce(h->cfg, m, out, 0, m.num_tile_reduce_units, h->side_stream);
        merged_on_side = m.num_tile_reduce_units;
        if (e == hipSuccess) e = hipEventRecord(h->join_event, h->side_stream);
        if (e == hipSuccess) e = (hipError_t)launch_attention(h->cfg, m, q, k_cache, v_cache, num_pages, sm_scale, out, 2, stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(s, h->join_event, 0);
    } else if (both && h->opt.interleave != 0) {  // one launch (also where the second stream is not to be used)
        // Run-time roles pay (a few atomics per block) when chunk blocks would otherwise pile up two
        // to a compute unit for a good part of the launch: more chunk blocks than units, and chunk
        // work that is not small next to the time the decodes need to stream.
        const bool many_chunk_blocks = (int64_t)pl.num_tile_units * h->cfg.num_kv_heads > kChunkBlocksForRoles &&
                                       chunk_us > 0.25 * wave_us;
        const bool roles = h->cfg.num_kv_heads <= kSchedMaxKvHeads &&
                           (h->opt.resident_chunks == 1 || (h->opt.resident_chunks < 0 && many_chunk_blocks));
        if (roles) {  // the scheduling words start at zero, whatever the last user of the memory left there
            e = (hipError_t)launch_zero(m.sched, kSchedBytes, stream);
            if (e != hipSuccess) return hip_fail(h, "launch zero fill", e);
        }
        e = (hipError_t)launch_attention(h->cfg, m, q, k_cache, v_cache, num_pages, sm_scale, out, roles ? 5 : 4, stream);
    } else {
        e = (hipError_t)launch_attention(h->cfg, m, q, k_cache, v_cache, num_pages, sm_scale, out, 3, stream);
    }
    timing_end(h, 1, t1, s);
    if (e != hipSuccess) return hip_fail(h, "launch attention", e);
    if (m.num_reduce_units > merged_on_side) {
        const int t2 = instrumented ? timing_begin(h, 2, s) : -1;
        e = (hipError_t)launch_reduce(h->cfg, m, out, merged_on_side, m.num_reduce_units - merged_on_side, stream);
        timing_end(h, 2, t2, s);
        if (e != hipSuccess) return hip_fail(h, "launch split-KV merge", e);
    }
    return SARATHI_OK;
}

}  // namespace

extern "C" sarathi_status sarathi_create(const sarathi_config *config, sarathi_handle **out) {
    if (!config || !out) return SARATHI_EINVAL;
    *out = nullptr;
    const sarathi_config &c = *config;
    if (c.num_q_heads < 1 || c.num_kv_heads < 1 || c.max_tokens < 1 || c.max_seqs < 1 || c.max_blocks_per_seq < 1)
        return SARATHI_EINVAL;
    if (c.num_q_heads % c.num_kv_heads != 0) return SARATHI_ESHAPE;
    if (c.head_dim != 64 && c.head_dim != 128) return SARATHI_ESHAPE;
    if (c.page_size != kPageSize) return SARATHI_ESHAPE;
    if (c.dtype != 0) return SARATHI_ESHAPE;
    sarathi_handle *h = new (std::nothrow) sarathi_handle();
    if (!h) return SARATHI_EINVAL;
    h->cfg = c;
    h->ws = make_workspace_layout(c);
    if (h->ws.max_tiles >= (1 << kUnitTileBits)) {  // tile indices are packed into 22 bits
        delete h;
        return SARATHI_ECAPACITY;
    }
    h->noalloc_meta.resize(kStaticMetaBytes);
    *out = h;
    return SARATHI_OK;
}

extern "C" sarathi_status sarathi_destroy(sarathi_handle *h) {
    if (!h) return SARATHI_EINVAL;
    if (h->staging_ready || h->staging[0]) {
        // copies out of the pinned buffers may still be queued (on streams this handle does not own)
        if (h->staging_used) (void)hipDeviceSynchronize();
        for (int i = 0; i < 2; ++i)
            if (h->half_done[i]) (void)hipEventDestroy(h->half_done[i]);
        for (int i = 0; i < kStagingSlots; ++i)
            if (h->staging[i]) (void)hipHostFree(h->staging[i]);
    }
    for (auto &pool : h->timing_pool)
        for (auto &pr : pool) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
    if (h->side_stream) {
        (void)hipStreamSynchronize(h->side_stream);
        (void)hipStreamDestroy(h->side_stream);
    }
    if (h->fork_event) (void)hipEventDestroy(h->fork_event);
    if (h->join_event) (void)hipEventDestroy(h->join_event);
    delete h;
    return SARATHI_OK;
}

extern "C" size_t sarathi_workspace_bytes(const sarathi_handle *h) { return h ? h->ws.total : 0; }

extern "C" const char *sarathi_last_error(const sarathi_handle *h) { return h ? h->err.c_str() : "null handle"; }

extern "C" sarathi_status sarathi_set_option(sarathi_handle *h, const char *name, int64_t value) {
    if (!h || !name) return SARATHI_EINVAL;
    h->opt_version++;  // a resident plan made under the old options is not reused
    if (std::strcmp(name, "split_keys") == 0) {
        if (value < 0 || value > (1 << 24)) return fail(h, SARATHI_EINVAL, "split_keys out of range");
        h->opt.split_keys = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "target_items") == 0) {
        if (value < 1 || value > (1 << 24)) return fail(h, SARATHI_EINVAL, "target_items out of range");
        h->opt.target_items = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "tile_split_keys") == 0) {
        if (value < 0 || value > (1 << 24)) return fail(h, SARATHI_EINVAL, "tile_split_keys out of range");
        h->opt.tile_split_keys = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "window") == 0) {
        if (value < 0 || value > INT32_MAX) return fail(h, SARATHI_EINVAL, "window must be >= 0 (0 = no sliding window)");
        h->opt.window = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "stream_kv") == 0) {
        if (value < -1 || value > 1) return fail(h, SARATHI_EINVAL, "stream_kv must be -1, 0 or 1");
        h->opt.stream_kv = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "decode_blocks_per_cu") == 0) {
        if (value != -1 && value != 1 && value != 2) return fail(h, SARATHI_EINVAL, "decode_blocks_per_cu must be -1, 1 or 2");
        h->opt.decode_blocks_per_cu = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "inline_append") == 0) {
        h->opt.inline_append = value != 0;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "lds_pad_kb") == 0) {
        if (value < 0 || value > 96) return fail(h, SARATHI_EINVAL, "lds_pad_kb must be 0 .. 96");
        h->opt.lds_pad_kb = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "resident_chunks") == 0) {
        if (value < -1 || value > 1) return fail(h, SARATHI_EINVAL, "resident_chunks must be -1, 0 or 1");
        h->opt.resident_chunks = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "tile_min_cols") == 0) {
        if (value < 1 || value > (1 << 30)) return fail(h, SARATHI_EINVAL, "tile_min_cols out of range");
        h->opt.tile_min_cols = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "plan_at_append") == 0) {
        h->opt.plan_at_append = value != 0;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "interleave") == 0) {
        if (value < 0 || value > 2) return SARATHI_EINVAL;
        h->opt.interleave = value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "time_kernels") == 0) {
        if (value < 0 || value > 2) return SARATHI_EINVAL;
        h->time_kernels = (int)value;
        return SARATHI_OK;
    }
    if (std::strcmp(name, "time_every") == 0) {
        if (value < 1 || value > (1 << 20)) return fail(h, SARATHI_EINVAL, "time_every must be >= 1");
        h->time_every = value;
        for (auto &n : h->timing_seen) n = 0;
        return SARATHI_OK;
    }
    return fail(h, SARATHI_EINVAL, std::string("unknown option: ") + name);
}

extern "C" sarathi_status sarathi_get_kernel_times(sarathi_handle *h, sarathi_kernel_times *out) {
    if (!h || !out) return SARATHI_EINVAL;
    double ms[3] = {0, 0, 0};
    int64_t n[3] = {0, 0, 0};
    for (int kind = 0; kind < 3; ++kind) {
        for (size_t i = 0; i < h->timing_used[kind]; ++i) {
            auto &pr = h->timing_pool[kind][i];
            hipError_t e = hipEventSynchronize(pr.second);
            if (e != hipSuccess) return hip_fail(h, "hipEventSynchronize(timing)", e);
            float t = 0.f;
            e = hipEventElapsedTime(&t, pr.first, pr.second);
            if (e != hipSuccess) return hip_fail(h, "hipEventElapsedTime", e);
            ms[kind] += t;
            n[kind]++;
        }
        h->timing_used[kind] = 0;
    }
    out->append_ms = ms[0]; out->attention_ms = ms[1]; out->merge_ms = ms[2];
    out->append_launches = n[0]; out->attention_launches = n[1]; out->merge_launches = n[2];
    return SARATHI_OK;
}

extern "C" sarathi_status sarathi_plan_hybrid_attention(sarathi_handle *h, const int32_t *q_start, const int32_t *q_len,
                                                        const int32_t *ctx_len, int32_t num_seqs, int32_t num_tokens,
                                                        sarathi_plan_info *info, sarathi_work_item *items_out,
                                                        int32_t items_capacity) {
    if (!h) return SARATHI_EINVAL;
    if (!info) return fail(h, SARATHI_EINVAL, "null info");
    sarathi_status st = validate_batch(h->cfg, q_start, q_len, ctx_len, num_seqs, num_tokens, 1, h->err);
    if (st != SARATHI_OK) return st;
    h->resident_ws = nullptr;  // h->plan is about to be overwritten
    plan_attention(h->cfg, h->opt, h->ws, q_start, q_len, ctx_len, num_seqs, h->plan);
    const Plan &pl = h->plan;
    info->num_items = (int32_t)pl.units.size();
    info->num_reduce_items = pl.num_split_tiles;
    info->num_part_rows = pl.num_part_rows;
    info->split_keys = pl.split_keys;
    info->num_tile_items = pl.num_tile_units;
    info->tile_split_keys = pl.tile_split_keys;
    if (items_out) {
        if (items_capacity < info->num_items) return fail(h, SARATHI_ECAPACITY, "items_capacity too small");
        for (size_t i = 0; i < pl.units.size(); ++i) {
            const uint32_t u = pl.units[i];
            const TileDesc &t = pl.tiles[u & ((1u << kUnitTileBits) - 1)];
            const int32_t split = (int32_t)(u >> kUnitTileBits);
            sarathi_work_item &w = items_out[i];
            w.seq = t.seq;
            w.col_begin = t.col_begin;
            w.n_cols = t.n_cols;
            w.key_begin = t.key_lo + split * t.keys_per_split;
            w.key_end = std::min(t.n_keys, w.key_begin + t.keys_per_split);
            w.part_row = t.n_splits > 1 ? t.part_row0 + split * t.n_cols : -1;
            w.kind = t.kind;
            w.reserved = 0;
        }
    }
    return SARATHI_OK;
}

extern "C" sarathi_status sarathi_kv_append(sarathi_handle *h, const void *k_new, const void *v_new, void *k_cache,
                                            void *v_cache, const int32_t *block_table, const int32_t *q_start,
                                            const int32_t *q_len, const int32_t *ctx_len, int32_t num_seqs,
                                            int32_t num_tokens, int64_t num_pages, void *workspace, void *stream) {
    if (!h) return SARATHI_EINVAL;
    sarathi_status st = validate_batch(h->cfg, q_start, q_len, ctx_len, num_seqs, num_tokens, num_pages, h->err);
    if (st != SARATHI_OK) return st;
    if (num_seqs == 0) return SARATHI_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_table) return fail(h, SARATHI_EINVAL, "null tensor pointer");
    if (!workspace) return fail(h, SARATHI_EWORKSPACE, "null workspace");
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return fail(h, SARATHI_EWORKSPACE, "workspace is not 256-byte aligned");
    if ((st = ensure_staging(h)) != SARATHI_OK) return st;
    int slot;
    if ((st = acquire_slot(h, static_cast<hipStream_t>(stream), &slot)) != SARATHI_OK) return st;
    SlotGuard guard{h, slot, static_cast<hipStream_t>(stream)};

    // Metadata: one record per cache page that this iteration writes into.
    AppendUnit *units = static_cast<AppendUnit *>(h->staging[slot]);
    const size_t n = (size_t)num_seqs;
    size_t n_units = 0;
    for (int32_t i = 0; i < num_seqs; ++i) {
        const int32_t prefix = ctx_len[i] - q_len[i];
        for (int32_t pg = prefix / kPageSize; pg <= (ctx_len[i] - 1) / kPageSize; ++pg) {
            const int32_t first = std::max(prefix, pg * kPageSize), end = std::min(ctx_len[i], (pg + 1) * kPageSize);
            units[n_units++] = AppendUnit{i, pg, q_start[i] + (first - prefix), (first - pg * kPageSize) | ((end - pg * kPageSize) << 8)};
        }
    }
    size_t used = sizeof(AppendUnit) * n_units;
    if (used > h->staging_bytes) return fail(h, SARATHI_ECAPACITY, "internal: metadata exceeds staging buffer");
    // The attention call of this iteration will get the same description: plan it now and let
    // its metadata ride along in the append launch (no host-to-device copy of its own).
    h->resident_ws = nullptr;
    if (h->opt.plan_at_append) {
        plan_attention(h->cfg, h->opt, h->ws, q_start, q_len, ctx_len, num_seqs, h->plan);
        const AttnMetaOffsets o = attn_meta_offsets(h->plan);
        const size_t attn_off = align_up(used, 256);
        if (attn_off + o.total <= h->staging_bytes) {
            pack_attn_meta(reinterpret_cast<char *>(units) + attn_off, h->plan, o);
            used = attn_off + o.total;
            h->resident_attn_off = attn_off;
            h->resident_desc.resize(2 * n);
            std::memcpy(h->resident_desc.data(), q_len, sizeof(int32_t) * n);
            std::memcpy(h->resident_desc.data() + n, ctx_len, sizeof(int32_t) * n);
            h->resident_opt_version = h->opt_version;
            h->resident_stream = stream;
            h->resident_ws = workspace;
        }
    }

    // One launch: the append blocks read their records straight from the pinned buffer, and a few more blocks of
    // the same launch move the attention metadata into the workspace (no copy in front of the append kernel).
    char *dev = static_cast<char *>(workspace) + h->ws.meta;
    hipStream_t s = static_cast<hipStream_t>(stream);
    AppendMeta m;
    m.units = static_cast<const AppendUnit *>(h->staging_dev[slot]);
    if (h->opt.inline_append) m.units_host = units;
    m.block_table = block_table;
    m.max_blocks = h->cfg.max_blocks_per_seq;
    m.num_units = (int32_t)n_units;
    if (h->resident_ws) {
        m.copy_dst = dev + h->resident_attn_off;
        m.copy_src = static_cast<const char *>(h->staging_dev[slot]) + h->resident_attn_off;
        m.copy_bytes = used - h->resident_attn_off;
    }
    const int t0 = timing_begin(h, 0, s);
    hipError_t e = (hipError_t)launch_kv_append(h->cfg, m, k_new, v_new, k_cache, v_cache, num_pages, stream);
    timing_end(h, 0, t0, s);
    if (e != hipSuccess) { h->resident_ws = nullptr; return hip_fail(h, "launch kv_append", e); }
    if ((st = guard.release()) != SARATHI_OK) return st;
    return SARATHI_OK;
}

extern "C" sarathi_status sarathi_hybrid_attention(sarathi_handle *h, const void *q, const void *k_cache,
                                                   const void *v_cache, const int32_t *block_table,
                                                   const int32_t *q_start, const int32_t *q_len,
                                                   const int32_t *ctx_len, int32_t num_seqs, int32_t num_tokens,
                                                   int64_t num_pages, float sm_scale, void *out, void *workspace,
                                                   void *stream) {
    if (!h) return SARATHI_EINVAL;
    sarathi_status st = validate_batch(h->cfg, q_start, q_len, ctx_len, num_seqs, num_tokens, num_pages, h->err);
    if (st != SARATHI_OK) return st;
    if (num_seqs == 0) return SARATHI_OK;
    if (!q || !k_cache || !v_cache || !block_table || !out) return fail(h, SARATHI_EINVAL, "null tensor pointer");
    if (!(sm_scale > 0.0f) || sm_scale - sm_scale != 0.0f) return fail(h, SARATHI_EINVAL, "sm_scale must be positive and finite");
    if (!workspace) return fail(h, SARATHI_EWORKSPACE, "null workspace");
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return fail(h, SARATHI_EWORKSPACE, "workspace is not 256-byte aligned");
    char *ws = static_cast<char *>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    char *dev;
    if (resident_plan_matches(h, q_len, ctx_len, num_seqs, workspace, stream)) {
        // planned and uploaded by the sarathi_kv_append of this iteration (h->plan is that plan)
        dev = ws + h->ws.meta + h->resident_attn_off;
    } else {
        plan_attention(h->cfg, h->opt, h->ws, q_start, q_len, ctx_len, num_seqs, h->plan);
        if ((st = ensure_staging(h)) != SARATHI_OK) return st;
        int slot;
        if ((st = acquire_slot(h, s, &slot)) != SARATHI_OK) return st;
        SlotGuard guard{h, slot, s};
        const AttnMetaOffsets o = attn_meta_offsets(h->plan);
        if (o.total > h->staging_bytes) return fail(h, SARATHI_ECAPACITY, "internal: metadata exceeds staging buffer");
        char *host = static_cast<char *>(h->staging[slot]);
        pack_attn_meta(host, h->plan, o);
        dev = ws + h->ws.meta;
        h->resident_ws = nullptr;  // the region no longer holds what an earlier append put there
        e = (hipError_t)launch_upload(dev, h->staging_dev[slot], o.total, stream);
        if (e != hipSuccess) return hip_fail(h, "launch upload(metadata)", e);
        if ((st = guard.release()) != SARATHI_OK) return st;
    }
    return enqueue_attention(h, dev, reinterpret_cast<float *>(ws + h->ws.part_ml), reinterpret_cast<float *>(ws + h->ws.part_o),
                             reinterpret_cast<int32_t *>(ws + h->ws.sched), block_table, q, k_cache, v_cache, num_pages, sm_scale,
                             out, s, /*instrumented=*/true);
}

extern "C" sarathi_status sarathi_hybrid_attention_noalloc(sarathi_handle *h, const void *q, const void *k_cache,
                                                           const void *v_cache, const int32_t *block_table,
                                                           const int32_t *q_start, const int32_t *q_len,
                                                           const int32_t *ctx_len, int32_t num_seqs, int32_t num_tokens,
                                                           int64_t num_pages, float sm_scale, void *out, void *stream) {
    if (!h) return SARATHI_EINVAL;
    sarathi_status st = validate_batch(h->cfg, q_start, q_len, ctx_len, num_seqs, num_tokens, num_pages, h->err);
    if (st != SARATHI_OK) return st;
    if (num_seqs == 0) return SARATHI_OK;
    if (!q || !k_cache || !v_cache || !block_table || !out) return fail(h, SARATHI_EINVAL, "null tensor pointer");
    if (!(sm_scale > 0.0f) || sm_scale - sm_scale != 0.0f) return fail(h, SARATHI_EINVAL, "sm_scale must be positive and finite");
    // Partial rows the built-in scratch holds for this shape; the planner coarsens its splits until they fit.
    const size_t row_bytes = sizeof(float) * (size_t)h->cfg.num_kv_heads * h->cfg.head_dim;
    WorkspaceLayout lay = h->ws;
    lay.max_part_rows = (int32_t)std::min<size_t>((size_t)lay.max_part_rows, kStaticPartOBytes / row_bytes);
    if (lay.max_part_rows < 2 * kTileCols || sizeof(float) * 2 * (size_t)lay.max_part_rows * h->cfg.num_kv_heads > kStaticPartMlBytes)
        return fail(h, SARATHI_ECAPACITY, "allocation-free entry point: num_kv_heads * head_dim is too large for the built-in scratch");
    h->resident_ws = nullptr;  // h->plan is about to be overwritten
    plan_attention(h->cfg, h->opt, lay, q_start, q_len, ctx_len, num_seqs, h->plan);
    const AttnMetaOffsets o = attn_meta_offsets(h->plan);
    if (o.total > kStaticMetaBytes || o.total > h->noalloc_meta.size()) {
        char buf[200];
        snprintf(buf, sizeof buf, "allocation-free entry point: the batch's plan needs %zu bytes of metadata, the built-in "
                 "scratch holds %zu (about %zu sequences or 128-column tiles)", o.total, kStaticMetaBytes, kStaticMetaBytes / 52);
        return fail(h, SARATHI_ECAPACITY, buf);
    }
    StaticScratch sc;
    hipError_t e = (hipError_t)static_scratch(&sc);
    if (e != hipSuccess) return hip_fail(h, "hipGetSymbolAddress(scratch)", e);
    std::memset(h->noalloc_meta.data(), 0, o.total);
    pack_attn_meta(h->noalloc_meta.data(), h->plan, o);
    e = (hipError_t)launch_upload_args(sc.meta, h->noalloc_meta.data(), o.total, stream);
    if (e != hipSuccess) return hip_fail(h, "launch upload(metadata in kernel arguments)", e);
    return enqueue_attention(h, sc.meta, sc.part_ml, sc.part_o, sc.sched, block_table, q, k_cache, v_cache, num_pages, sm_scale,
                             out, static_cast<hipStream_t>(stream), /*instrumented=*/false);
}
