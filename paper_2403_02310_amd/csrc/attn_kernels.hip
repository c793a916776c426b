// gfx950 kernels of libsarathi: KV append, hybrid-batch attention over the paged cache,
// and the split-KV merge.
//
// Attention kernel (16-column wave tile).  A work item is 16 query COLUMNS (col = row*G +
// head_in_group, all sharing one KV head) against a key range; a workgroup of four wavefronts owns
// it, each wavefront walks a quarter of the keys in tiles of 32 (two pages), and the four results
// are merged in LDS (a decode has four memory streams from its first cycle and ends four times
// sooner than on one wavefront).  Both contractions run on v_mfma_f32_16x16x32_bf16 in the
// TRANSPOSED form so that the score accumulators already are the operand of the second one:
//
//   S^T[key, col] = sum_c K[key, c] * Q[col, c]      A = K tile (16 keys x 32 ch), B = Q^T
//   O^T[c,  col] += sum_key V^T[c, key] * P^T[key, col]   A = V^T tile (16 ch x 32 keys), B = P^T
//
// Operand layout of the instruction (64 lanes; g = lane/16, n = lane%16): A lane holds row n,
// contraction indices 8g..8g+7; B lane holds column n, contraction indices 8g..8g+7; the
// accumulator lane holds column n, rows 4g..4g+3.  With the K rows of the two score MFMAs of a
// tile assigned as  row 4g'+i of MFMA b  <->  key 8g'+4b+i,  lane (g, n) ends up with the eight
// scores of column n for keys 8g..8g+7 of the tile: exactly the B operand (P^T) of the second
// contraction, and V^T for those eight keys is one 16-byte run of the channel-major V page.
// So K, V and Q go from global memory straight into MFMA operands: no LDS, no transposes, no
// barriers in the key loop; the softmax is per-lane work plus two cross-lane steps (lanes n, n+16,
// n+32, n+48).
//
// Chunk-tile path (prefill chunks).  A workgroup of four wavefronts owns 128 columns of one
// sequence (32 per wave) and walks the key range in 32-key tiles staged once per workgroup in
// LDS (rings of four K tiles and four V tiles filled by direct global -> LDS loads, K three tiles
// ahead of the step and V two; one barrier per tile), so K/V are fetched from L2/HBM once per 128
// columns instead of once per 16.  The contractions use v_mfma_f32_32x32x16_bf16, again in
// transposed form with the K rows of a tile permuted (MFMA row 16u+8a+4h+b <-> key 16u+8h+4a+b)
// so that accumulator lane (h, n) holds, for column n, keys 8h..8h+7 of page u in registers
// 8u..8u+7: the B operand of the second contraction without any data movement.  K rows are
// XOR-swizzled in LDS and the two 16-byte halves of a V^T row are swapped on every other group
// of eight channels, which makes both the staging writes and the operand reads bank-conflict free.
//
// Both paths share one launch: a block is either one chunk tile or one wave tile, so the
// memory-bound decodes fill the machine next to the MFMA-bound chunk tiles (the paper's reason
// for hybrid batches, section 4.1).
//
// The running maximum is only raised when a tile exceeds it by more than 2^8 (the softmax is
// invariant to the reference point as long as sum and output use the same one), which removes
// the accumulator rescale from almost every tile.
//
// Split-KV.  A tile whose key range was cut into pieces has every piece write its partial
// (reference maximum, sum, unnormalised output) triple; a second, small kernel merges the
// pieces of each tile in index order, so the result is bitwise reproducible.  (Merging inside
// the attention kernel by the last piece to finish was built twice and dropped on its timings.
// With device-scope release/acquire fences every block writes back and invalidates a whole L2 of
// this multi-die part: several times slower.  Without fences, the partial rows themselves written and
// read with device-scope accesses, whole 512-byte rows at a time, and a piece that finds the others
// done merging without publishing: correct, and still slower than the second kernel in every case
// measured (a 512-token chunk alone 57 us against 40 + 13, chunks of 256 tokens 1,866 us per prompt
// against 1,717), because such accesses bypass the L2 that serves the second kernel's reads, and
// ONE block per tile reads what 16 blocks of the merge kernel read in parallel.)
//
// Masking is by select: keys beyond a column's position (causal mask inside a chunk, section
// 4.1 of the paper) or beyond the item's key range get score -inf; V of slots at or beyond
// ctx_len is zeroed so that stale cache contents (possibly NaN) cannot reach an accumulator.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "internal.h"

namespace sarathi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct AttnParams {
    const uint16_t *q;
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    uint16_t *out;
    const int32_t *block_table;
    const TileDesc *tiles;
    const uint32_t *units;
    float *part_ml;
    float *part_o;
    int64_t num_pages;
    int32_t max_blocks;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t group;
    int32_t num_tile_units;  // units [0, num_tile_units) are 128-column chunk tiles (one block each)
    int32_t num_units;       // the rest are 16-column wave tiles (one block each as well)
    float scale_log2;        // sm_scale * log2(e): the softmax runs in base 2
    int32_t *sched;          // scheduling words of the run-time role assignment (else unused)
    int32_t window;          // sliding window: a query at position p sees keys p-window+1 .. p; 0 = all keys up to p
};

// What one work unit (tile, split) covers.
struct UnitRange {
    int32_t key_begin;
    int32_t key_end;   // exclusive
    int32_t part_row;  // first partial row of this split, or -1: write `out` directly
};
__device__ __forceinline__ UnitRange unit_range(const TileDesc &t, int split) {
    UnitRange r;
    r.key_begin = t.key_lo + split * t.keys_per_split;
    r.key_end = min(t.n_keys, r.key_begin + t.keys_per_split);
    r.part_row = t.n_splits > 1 ? t.part_row0 + split * t.n_cols : -1;
    return r;
}

constexpr float kNegSentinel = -1.0e30f;  // finite "no key seen yet" running maximum
constexpr float kRescaleSlack = 8.0f;     // raise the softmax reference only when exceeded by 2^8
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16x8 load_bf16x8(const uint16_t *p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p));
}
__device__ __forceinline__ bf16x8 load_bf16x8_stream(const uint16_t *p) {
    return __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)));
}

template <int D>
struct TileRegs {
    bf16x8 k[2][D / 32];  // A operands of the two score MFMAs, per 32-channel step
    bf16x8 v[D / 16];     // A operands of the output MFMAs, per 16-channel tile
};

// Read-only int32 data fetched with scalar loads (the block table: wave-uniform indices).
typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;

template <int D>
struct LaneGeom {
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    const_i32_ptr bt;      // this sequence's block-table row (scalar loads)
    int64_t page_stride;   // elements per page (all KV heads)
    int64_t k_lane_off;    // element offset of this lane's K row start inside a page
    int64_t v_lane_off;    // element offset of this lane's V^T run inside a page
    int64_t last_page_id;  // num_pages - 1 (page ids are clamped: a corrupt table cannot fault)
    int32_t n_pages_seq;   // pages that hold positions < ctx_len
    int32_t k_pg_sel;      // which of the tile's two pages this lane's K rows come from
    int32_t v_pg_sel;
};

// The two block-table entries of a 32-key tile.  They are wave-uniform and come by scalar loads, which the
// vector-memory counter does not see.  (As vector loads they were the youngest loads in flight when their
// values were needed, and loads return in order: waiting for them meant waiting for the previous tile's K/V
// too, so only one tile was ever in flight.)
struct TilePages {
    int32_t e0, e1;
};
template <int D>
__device__ __forceinline__ TilePages tile_pages(const LaneGeom<D> &ge, int tile) {
    // Pages at or beyond ceil(ctx_len/16) are never dereferenced: the index is clamped to the
    // sequence's last page and whatever is loaded for such keys is masked in compute_tile.
    return TilePages{ge.bt[min(tile * 2, ge.n_pages_seq - 1)], ge.bt[min(tile * 2 + 1, ge.n_pages_seq - 1)]};
}

// Requests the K/V of `tile`, whose table entries arrive in `pages` (fetched a tile earlier), and fetches the
// entries of the tile after it into `pages`.  The page bases are formed on the scalar unit; a lane only picks
// one of the two.  STREAM: the loads carry the non-temporal hint (K/V read once, far more than the caches hold).
template <int D, bool STREAM>
__device__ __forceinline__ void load_tile(const LaneGeom<D> &ge, int tile, TileRegs<D> &r, TilePages &pages) {
    const int64_t p0 = pages.e0 < 0 ? 0 : (pages.e0 > ge.last_page_id ? ge.last_page_id : (int64_t)pages.e0);
    const int64_t p1 = pages.e1 < 0 ? 0 : (pages.e1 > ge.last_page_id ? ge.last_page_id : (int64_t)pages.e1);
    pages = tile_pages(ge, tile + 1);
    const int64_t o0 = p0 * ge.page_stride, o1 = p1 * ge.page_stride;
    const uint16_t *kp = ge.k_cache + (ge.k_pg_sel ? o1 : o0) + ge.k_lane_off;
    const uint16_t *vp = ge.v_cache + (ge.v_pg_sel ? o1 : o0) + ge.v_lane_off;
    if (STREAM) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int s = 0; s < D / 32; ++s) r.k[b][s] = load_bf16x8_stream(kp + b * 4 * D + s * 32);
#pragma unroll
        for (int t = 0; t < D / 16; ++t) r.v[t] = load_bf16x8_stream(vp + t * 16 * kPageSize);
    } else {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int s = 0; s < D / 32; ++s) r.k[b][s] = load_bf16x8(kp + b * 4 * D + s * 32);
#pragma unroll
        for (int t = 0; t < D / 16; ++t) r.v[t] = load_bf16x8(vp + t * 16 * kPageSize);
    }
}

template <int D>
struct SoftmaxState {
    f32x4 o[D / 16];  // O^T accumulators: channel 16t + 4g + i, column n
    float m;          // running maximum (base-2 scaled scores), identical in the 4 lanes of a column
    float l;          // this lane's share of the running sum (summed over g at the end)
};

template <int D>
__device__ __forceinline__ void compute_tile(TileRegs<D> &r, const bf16x8 (&qreg)[D / 32], SoftmaxState<D> &st,
                                             int tile, int g, int pos_eff, int min_pos_eff, int lo, int max_lo, int ctx,
                                             float scale_log2) {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.k[0][s], qreg[s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.k[1][s], qreg[s], s1, 0, 0, 0);
    }
    const int key0 = tile * kTileKeys + g * 8;  // this lane's eight keys: key0 .. key0+7
    float t[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        t[j] = s0[j] * scale_log2;
        t[4 + j] = s1[j] * scale_log2;
    }
    if (tile * kTileKeys + (kTileKeys - 1) > min_pos_eff) {  // wave-uniform: some lane must mask
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = (key0 + j <= pos_eff) ? t[j] : -INFINITY;
    }
    if (tile * kTileKeys < max_lo) {  // wave-uniform: some lane's sliding window starts inside or after this tile
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = (key0 + j >= lo) ? t[j] : -INFINITY;
    }
    if (tile * kTileKeys + kTileKeys > ctx) {  // wave-uniform: tile holds slots at or beyond ctx_len
        u32x4 keep;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            keep[w] = ((key0 + 2 * w < ctx) ? 0x0000FFFFu : 0u) | ((key0 + 2 * w + 1 < ctx) ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int c = 0; c < D / 16; ++c) r.v[c] = __builtin_bit_cast(bf16x8, __builtin_bit_cast(u32x4, r.v[c]) & keep);
    }
    float tmax = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    if (__any(tmax > st.m + kRescaleSlack)) {  // wave-uniform; rare after the first tiles
        const float m_new = fmaxf(st.m, tmax);
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
        st.l *= alpha;
        st.m = m_new;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) st.o[c] *= alpha;
    }
    f32x8 p;
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = __builtin_amdgcn_exp2f(t[j] - st.m);
        psum += p[j];
    }
    st.l += psum;
    const bf16x8 pT = __builtin_convertvector(p, bf16x8);
#pragma unroll
    for (int c = 0; c < D / 16; ++c)
        st.o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.v[c], pT, st.o[c], 0, 0, 0);
}

// LDS a wave-tile block needs to merge its four wavefronts: per wave 16 columns x (D + 4) floats of
// unnormalised output (the pad spreads the columns over the banks) and 16 x (maximum, sum).
template <int D>
struct WaveMergeSmem {
    static constexpr int kColStride = D + 4;
    static constexpr int kOutFloats = 4 * kWaveCols * kColStride;
    static constexpr int kTotalFloats = kOutFloats + 4 * kWaveCols * 2;
};

// One wave-tile unit = one block.  The unit's key range is quartered (in multiples of 32 keys) among
// the block's four wavefronts, which run the same loop as independent split-KV pieces and then merge
// their (maximum, sum, unnormalised output) through LDS in wavefront order: the block writes the final
// rows, or one set of partial rows if the tile is split further across blocks.
template <int D, bool STREAM>
__device__ __forceinline__ void wave16_path(const AttnParams &p, const TileDesc &it, int split, int kvh, float *merge_lds) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;
    const int g = lane >> 4;
    const int seq = it.seq;
    const int ctx = it.ctx_len;
    const int q_start = it.q_start;
    const int prefix = ctx - it.q_len;
    const int G = p.group;
    UnitRange ur = unit_range(it, split);
    {   // this wavefront's quarter of the unit (possibly empty: then it contributes weight zero)
        const int quarter = ((ur.key_end - ur.key_begin + 3) / 4 + kTileKeys - 1) / kTileKeys * kTileKeys;
        const int b = ur.key_begin + wave * quarter;   // a multiple of 32, as every piece start
        ur.key_end = min(ur.key_end, b + quarter);
        ur.key_begin = min(b, ur.key_end);
    }
    const bool piece_empty = ur.key_begin >= ur.key_end;

    // Lanes beyond the tile's valid columns shadow column 0 of the tile and store nothing.
    const bool col_valid = n < it.n_cols;
    const int col = it.col_begin + (col_valid ? n : 0);
    const int row = col / G;
    const int head = kvh * G + (col - row * G);
    const int pos_eff = min(prefix + row, ur.key_end - 1);                 // last key this column may see here
    const int min_pos_eff = min(prefix + it.col_begin / G, ur.key_end - 1);  // the same for the tile's first column
    // first key inside this column's sliding window, and the largest such key over the tile's columns
    const int lo = p.window > 0 ? max(0, prefix + row - p.window + 1) : 0;
    const int max_lo = p.window > 0 ? max(0, prefix + (it.col_begin + it.n_cols - 1) / G - p.window + 1) : 0;

    bf16x8 qreg[D / 32];
    {
        const uint16_t *qp = p.q + ((int64_t)(q_start + row) * p.num_q_heads + head) * D + g * 8;
#pragma unroll
        for (int s = 0; s < D / 32; ++s) qreg[s] = load_bf16x8(qp + s * 32);
    }

    LaneGeom<D> ge;
    ge.k_cache = p.k_cache;
    ge.v_cache = p.v_cache;
    ge.bt = (const_i32_ptr)(p.block_table + (int64_t)seq * p.max_blocks);
    ge.page_stride = (int64_t)p.num_kv_heads * kPageSize * D;
    ge.last_page_id = p.num_pages - 1;
    ge.n_pages_seq = (ctx + kPageSize - 1) / kPageSize;
    ge.k_pg_sel = n >> 3;
    ge.v_pg_sel = g >> 1;
    // K row of MFMA b, A-row n:  page n/8, slot ((n/4)&1)*8 + 4b + n%4 ; this lane reads channels 8g.. of each 32-step
    ge.k_lane_off = (int64_t)kvh * kPageSize * D + (((n >> 2) & 1) * 8 + (n & 3)) * D + g * 8;
    // V^T run of output tile t, A-row n: channel 16t+n, slots 8*(g&1) .. +7 of page g/2
    ge.v_lane_off = (int64_t)kvh * D * kPageSize + n * kPageSize + (g & 1) * 8;

    SoftmaxState<D> st;
#pragma unroll
    for (int c = 0; c < D / 16; ++c) st.o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m = kNegSentinel;
    st.l = 0.f;

    const int tile_begin = ur.key_begin / kTileKeys;
    const int tile_end = piece_empty ? tile_begin : (ur.key_end + kTileKeys - 1) / kTileKeys;

    // Two register sets, ping-pong: the loads of tile i+1 are in flight while tile i computes.
    TileRegs<D> ra, rb;
    TilePages pages = tile_pages(ge, tile_begin);
    load_tile<D, STREAM>(ge, tile_begin, ra, pages);
    int tile = tile_begin;
    for (; tile + 1 < tile_end; tile += 2) {
        load_tile<D, STREAM>(ge, tile + 1, rb, pages);
        compute_tile<D>(ra, qreg, st, tile, g, pos_eff, min_pos_eff, lo, max_lo, ctx, p.scale_log2);
        if (tile + 2 < tile_end) load_tile<D, STREAM>(ge, tile + 2, ra, pages);
        compute_tile<D>(rb, qreg, st, tile + 1, g, pos_eff, min_pos_eff, lo, max_lo, ctx, p.scale_log2);
    }
    if (tile < tile_end) compute_tile<D>(ra, qreg, st, tile, g, pos_eff, min_pos_eff, lo, max_lo, ctx, p.scale_log2);

    float l = st.l + __shfl_xor(st.l, 16);
    l += __shfl_xor(l, 32);

    // Publish this wavefront's piece: lane (n, g) holds channels 16c + 4g + i of column n.
    using MS = WaveMergeSmem<D>;
    {
        float *o_w = merge_lds + (wave * kWaveCols + n) * MS::kColStride + g * 4;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) *reinterpret_cast<f32x4 *>(o_w + c * 16) = st.o[c];
        if (g == 0) {
            float *ml = merge_lds + MS::kOutFloats + (wave * kWaveCols + n) * 2;
            ml[0] = st.m;
            ml[1] = l;
        }
    }
    __syncthreads();
    // Merge: thread t owns column t / 16 and D / 16 consecutive channels of it.
    constexpr int CH = D / 16;
    const int mc = threadIdx.x >> 4;
    const int ch0 = (threadIdx.x & 15) * CH;
    if (mc >= it.n_cols) return;
    float m_w[4], m_max = kNegSentinel;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        m_w[w] = merge_lds[MS::kOutFloats + (w * kWaveCols + mc) * 2];
        m_max = fmaxf(m_max, m_w[w]);
    }
    float acc[CH];
#pragma unroll
    for (int j = 0; j < CH; ++j) acc[j] = 0.f;
    float l_tot = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float wt = __builtin_amdgcn_exp2f(m_w[w] - m_max);
        l_tot += wt * merge_lds[MS::kOutFloats + (w * kWaveCols + mc) * 2 + 1];
        const float *o_w = merge_lds + (w * kWaveCols + mc) * MS::kColStride + ch0;
#pragma unroll
        for (int j = 0; j < CH; j += 4) {
            const f32x4 o4 = *reinterpret_cast<const f32x4 *>(o_w + j);
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[j + i] += wt * o4[i];
        }
    }
    const int mcol = it.col_begin + mc;
    const int mrow = mcol / G;
    const int mhead = kvh * G + (mcol - mrow * G);
    const UnitRange whole = unit_range(it, split);
    if (whole.part_row < 0) {
        const float inv = 1.0f / l_tot;
        uint16_t *op = p.out + ((int64_t)(q_start + mrow) * p.num_q_heads + mhead) * D + ch0;
#pragma unroll
        for (int j = 0; j < CH; j += 4) {
            const f32x4 o = {acc[j] * inv, acc[j + 1] * inv, acc[j + 2] * inv, acc[j + 3] * inv};
            *reinterpret_cast<u32x2 *>(op + j) = __builtin_bit_cast(u32x2, __builtin_convertvector(o, bf16x4));
        }
        return;
    }
    // Tile split across blocks: this block's (reference maximum, sum, unnormalised output).
    const int64_t prow = ((int64_t)(whole.part_row + mc) * p.num_kv_heads + kvh);
    float *po = p.part_o + prow * D + ch0;
#pragma unroll
    for (int j = 0; j < CH; j += 4) *reinterpret_cast<f32x4 *>(po + j) = f32x4{acc[j], acc[j + 1], acc[j + 2], acc[j + 3]};
    if ((threadIdx.x & 15) == 0) {
        p.part_ml[prow * 2 + 0] = m_max;
        p.part_ml[prow * 2 + 1] = l_tot;
    }
}

// ---------------------------------------------------------------------------------------
// Chunk-tile path: 4 waves x 32 columns, K/V tiles of 32 keys staged in LDS.
// ---------------------------------------------------------------------------------------
// LDS of the chunk-tile path: a ring of 4 K tiles and a ring of 4 V tiles (32 keys each).
// In the step that handles tile t the wave reads K(t+1) and V(t-1) while K(t+2), K(t+3), V(t+1)
// and V(t+2) are in flight from global memory straight into LDS (no staging registers).  Tile
// with index rel (relative to the unit's first tile) lives in slot rel % 4 of its ring.
constexpr int kRing = 4;

template <int D>
struct ChunkSmem {
    static constexpr int kTileElems = kTileKeys * D;  // one K tile or one V tile: 32 keys x D channels
    static constexpr int kVBase = kRing * kTileElems;
    static constexpr int kTotalElems = 2 * kRing * kTileElems;
};

// K rows sit unpadded in LDS (a direct global->LDS load writes 1 KiB of consecutive bytes per
// wavefront); the 16-byte chunks of row r are XOR-swizzled with this key so that the 16 lanes
// of a b128 read, which walk 16 different rows at the same logical chunk, hit distinct banks.
template <int D>
__device__ __forceinline__ int k_swizzle(int r) {
    return D == 128 ? (r & 15) : ((r >> 1) & 7);
}
// LDS element offset of the 8-slot half `hh` of V^T row `d` of page `u`: the two halves of a
// row are swapped on every other group of eight channels (conflict-free reads).
template <int D>
__device__ __forceinline__ int v_lds_off(int u, int d, int hh) {
    return ((u * D + d) * 2 + (hh ^ ((d >> 3) & 1))) * 8;
}

__device__ __forceinline__ bf16x8 lds_bf16x8(const uint16_t *p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p));
}

typedef void __attribute__((address_space(3))) *lds_ptr;

// A direct global -> LDS load moves 16 bytes per lane (1 KiB per wavefront): lane l fetches
// base + byte_off(l) and the wavefront's data lands at LDS byte address lds_addr + 16 l.
// Written as inline assembly on purpose: the compiler's wait-count bookkeeping treats the
// builtin form as a flat access that may return out of order with LDS reads, and from then on
// turns every wait for an LDS operand into a full drain of the LDS queue (one pipeline bubble
// per four MFMAs in the loop below).  The loads issued here are waited for by hand
// (SARATHI_WAIT_VMCNT), the only vector-memory accesses of the chunk loop.
// A whole page of one KV head (N loads of 1 KiB) behind ONE write of the LDS base register: the
// instruction's immediate offset is added to the global address and to the LDS address alike, so
// load j uses offset 1024 j and a lane offset that has 1024 j taken off (rel_off[j] = byte offset
// inside the page minus 1024 j, which is never negative: load j fetches the page's j-th KiB).
template <int N>
__device__ __forceinline__ void dma_load_page(const uint16_t *base, const int (&rel_off)[N], uint32_t lds_addr) {
    static_assert(N == 2 || N == 4, "pages of 2 KiB (d = 64) or 4 KiB (d = 128) per KV head");
    if constexpr (N == 4) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %1, %5\n\t"
                     "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
                     "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
                     "global_load_lds_dwordx4 %4, %5 offset:3072"
                     :
                     : "s"(lds_addr), "v"(rel_off[0]), "v"(rel_off[1]), "v"(rel_off[2]), "v"(rel_off[3]), "s"(base)
                     : "memory");
    } else {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %1, %3\n\t"
                     "global_load_lds_dwordx4 %2, %3 offset:1024"
                     :
                     : "s"(lds_addr), "v"(rel_off[0]), "v"(rel_off[1]), "s"(base)
                     : "memory");
    }
}
__device__ __forceinline__ uint32_t lds_address(const uint16_t *p) {
    return (uint32_t)(uintptr_t)(lds_ptr)(p);
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
#define SARATHI_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

constexpr int kCarry = 3;  // output-MFMA operands read one step ahead

// State a wave carries from one tile to the next in the software-pipelined chunk loop.
template <int D>
struct ChunkState {
    f32x16 oacc[D / 32];  // O^T accumulators: channel 32c + 8*(r/4) + 4h + r%4, column n
    // Two register sets used in turn by consecutive steps of the unrolled loop (a step reads one
    // and fills the other); steps outside that loop keep everything in set 0.
    f32x16 s[2];          // raw scores of the tile whose softmax is due (already masked)
    bf16x8 p[2][2];       // bf16 softmax weights of the previous tile (B operands of its output MFMAs)
    bf16x8 carry[kCarry]; // V operands of the next step's first output MFMAs, read at the end of this step
    float tmax;           // scaled maximum of the due scores over the column
    float m_ref;          // softmax reference, scaled base-2 units
    float l_run;          // this lane's share of the running sum
};

// One pipelined step.  Independent work of three tiles shares one basic block so that the
// matrix pipe and the vector ALU run side by side inside a single wavefront:
//   MFMA:  S^T(t+1) = K(t+1) Q^T    (HAS_NEXT)        O^T += V^T(t-1) P^T(t-1)      (HAS_PREV)
//   VALU:  P(t) = 2^(S(t)*scale - m_ref), row sums, bf16 packing; mask and maximum of S(t+1)
// k_chunk: this lane's (swizzled) K chunk offsets; K_OFF / V_OFF: element offsets of the ring
// slots read in this step (wave-uniform).
// Order of the MFMAs of a step: which kind slot i issues and its index within that kind.  A step
// with both kinds opens with three output MFMAs (their V operands were read at the end of the
// previous step, so the matrix pipe has work right after the barrier, before any read of this step
// returns), then all score MFMAs (one accumulator; the scores are complete a few slots before the
// end of the step, so that masking and the maximum of the next tile also run under MFMAs), then the
// remaining output MFMAs.
struct ChunkSlot {
    bool is_score;
    int sub;
};
constexpr ChunkSlot chunk_slot(int i, int n_s, int n_o) {
    const int lead = n_o < kCarry ? n_o : kCarry;
    if (i < lead) return ChunkSlot{false, i};
    if (i < lead + n_s) return ChunkSlot{true, i - lead};
    return ChunkSlot{false, i - n_s};
}
constexpr int chunk_last_score_slot(int n_s, int n_o) {
    return n_s == 0 ? -1 : (n_o < kCarry ? n_o : kCarry) + n_s - 1;
}

// PHASE >= 0: the tile's index inside the unit is PHASE modulo 4, which fixes the ring slots at
// compile time (K_OFF_RT / V_OFF_RT are ignored and the operand reads need no address
// arithmetic); PHASE < 0: slots given at run time.  The step reads register set PP and fills set
// PP ^ 1 (SWAP) or set PP again (the results are copied back).
// CARRY_IN: the operands of the first kCarry output MFMAs are in st.carry (read by the previous step);
// CARRY_OUT: this step reads them for the next step (whose previous tile, this step's current one,
// has been in LDS and visible since this step's barrier).
template <int D, bool HAS_PREV, bool HAS_NEXT, bool MASK_NEXT, bool CARRY_IN, bool CARRY_OUT, int PHASE = -1, int PP = 0,
          bool SWAP = false>
__device__ __forceinline__ void chunk_step(ChunkState<D> &st, const bf16x8 (&qreg)[D / 16], const uint16_t *smem,
                                           const int (&k_chunk)[D / 16], int v_rd, int K_OFF_RT, int V_OFF_RT, float scale,
                                           int next_key0, int pos_eff, int lo) {
    constexpr int TE_ = kTileKeys * D;
    static_assert(!CARRY_IN || HAS_PREV, "carried operands belong to output MFMAs");
    const int K_OFF = PHASE >= 0 ? ((PHASE + 1) & (kRing - 1)) * TE_ : K_OFF_RT;
    const int V_OFF = PHASE >= 0 ? ((PHASE + 3) & (kRing - 1)) * TE_ : V_OFF_RT;
    const int V_OFF_NEXT = (V_OFF + TE_) & (kRing * TE_ - 1);  // ring slot of the current tile
    constexpr int OUT = SWAP ? (PP ^ 1) : PP;
    constexpr int NS = D / 16;
    constexpr int NB = D / 32;
    constexpr int N_S = HAS_NEXT ? NS : 0;              // score MFMAs (one dependent chain through s_next)
    constexpr int N_O = HAS_PREV ? 2 * NB : 0;          // output MFMAs (NB accumulators, two pages each)
    constexpr int NM = N_S + N_O;
    constexpr int AHEAD = 3;                             // operand reads run this many MFMAs ahead
    auto is_score = [&](int i) { return chunk_slot(i, N_S, N_O).is_score; };
    auto sub_index = [&](int i) { return chunk_slot(i, N_S, N_O).sub; };

    // The step is laid out as NM slots fenced by scheduling barriers.  Slot i issues the LDS
    // read for MFMA i+AHEAD, then MFMA i, then its share of the vector-ALU work, which
    // executes while the matrix pipe is busy with MFMA i.
    auto operand = [&](int i) -> const uint16_t * {
        const int j = sub_index(i);
        if (is_score(i)) return smem + K_OFF + k_chunk[j < NS ? j : 0];
        // output MFMA j: page j / NB, channel block j % NB
        return smem + v_rd + (V_OFF + ((j / NB) * D + (j % NB) * 32) * 16);
    };
    static_assert(AHEAD == kCarry, "the operands carried between steps fill the read-ahead window");
    bf16x8 frag[AHEAD + 1];
    bf16x8 nxt[kCarry];
#pragma unroll
    for (int i = 0; i < AHEAD && i < NM; ++i) frag[i] = CARRY_IN ? st.carry[i] : lds_bf16x8(operand(i));

    f32x16 s_tmp;
    f32x16 &s_next = SWAP ? st.s[OUT] : s_tmp;
    const f32x16 &s_cur = st.s[PP];
    const bf16x8 p_old0 = st.p[PP][0], p_old1 = st.p[PP][1];

    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    uint32_t p_new[8];  // bf16 pairs of the current tile's weights: registers (2k, 2k+1)
    float e_even = 0.f;
    float psum = 0.f;
    float smax = -INFINITY;
    float neg_m = -st.m_ref;
    auto weight = [&](int r) {
        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[r], scale, neg_m));
        psum += e;
        if (r & 1) {
            const bf16x2 pk = __builtin_convertvector(f32x2{e_even, e}, bf16x2);
            p_new[r >> 1] = __builtin_bit_cast(uint32_t, pk);
        } else {
            e_even = e;
        }
    };
    // mask + running maximum of register r of the next tile (key next_key0 + 16*(r/8) + r%8)
    auto next_max = [&](int r) {
        if (MASK_NEXT) {  // causal bound and, under a sliding window, the column's first visible key
            const int key = next_key0 + (r >> 3) * 16 + (r & 7);
            s_next[r] = (key <= pos_eff && key >= lo) ? s_next[r] : -INFINITY;
        }
        smax = fmaxf(smax, s_next[r]);
    };
    constexpr int LAST_SCORE = chunk_last_score_slot(N_S, N_O);  // slot of the last score MFMA
    constexpr int MAX_FROM = LAST_SCORE + 2;  // first slot in which the finished scores may be touched
    int w_done = 0, m_done = 0;         // compile-time after unrolling
    // Slot boundaries.  The arithmetic below has no side effects, so nothing but data flow
    // would keep it inside its slot; an empty asm that "touches" the values a slot produced and
    // one input of the next slot's arithmetic (the negated reference) pins both, and the
    // scheduling barrier keeps the machine scheduler from undoing the layout.  Neither emits
    // an instruction.
    asm volatile("" : "+v"(neg_m), "+v"(psum));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NM; ++i) {
        bf16x8 &ahead = frag[(i + AHEAD) % (AHEAD + 1)];
        if (i + AHEAD < NM) ahead = lds_bf16x8(operand(i + AHEAD));
        else if (CARRY_OUT)  // operand j = i + AHEAD - NM of the next step: page j / NB, channel block j % NB of the current tile
            nxt[i + AHEAD - NM] = lds_bf16x8(smem + v_rd + (V_OFF_NEXT + (((i + AHEAD - NM) / NB) * D + ((i + AHEAD - NM) % NB) * 32) * 16));
        const bf16x8 a = frag[i % (AHEAD + 1)];
        const int j = sub_index(i);
        if (is_score(i)) {
            if (j == 0) {
                f32x16 zero;
#pragma unroll
                for (int r = 0; r < 16; ++r) zero[r] = 0.f;
                s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[0], zero, 0, 0, 0);
            } else {
                s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[j < NS ? j : 0], s_next, 0, 0, 0);
            }
        } else {
            st.oacc[j % NB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, (j / NB) ? p_old1 : p_old0, st.oacc[j % NB], 0, 0, 0);
        }
        // vector-ALU share of this slot
        const int w_from = w_done;
        const int w_target = 16 * (i + 1) / (NM > 0 ? NM : 1);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (r >= w_from && r < w_target) weight(r);
        w_done = w_target;
        if (HAS_NEXT && i >= MAX_FROM) {
            const int m_target = 16 * (i + 1 - MAX_FROM) / (NM > MAX_FROM ? NM - MAX_FROM : 1);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r >= m_done && r < m_target) next_max(r);
            m_done = m_target;
        }
        // pin: this slot's MFMA result and the weights made here.  The operand fetched ahead in
        // this slot is NOT pinned (that would make the slot wait for it); the scheduling barrier
        // alone keeps the read where it was issued.
        bf16x8 &older = frag[i % (AHEAD + 1)];
        if (is_score(i))
            asm volatile("" : "+v"(s_next), "+v"(older), "+v"(neg_m), "+v"(psum), "+v"(e_even));
        else if (i > LAST_SCORE)
            asm volatile("" : "+v"(st.oacc[j % NB]), "+v"(older), "+v"(neg_m), "+v"(psum), "+v"(e_even), "+v"(s_next), "+v"(smax));
        else
            asm volatile("" : "+v"(st.oacc[j % NB]), "+v"(older), "+v"(neg_m), "+v"(psum), "+v"(e_even));
#pragma unroll
        for (int r = 1; r < 16; r += 2)
            if (r >= w_from && r < w_target) asm volatile("" : "+v"(p_new[r >> 1]));
        __builtin_amdgcn_sched_barrier(0);
    }
    // whatever did not fit into the slots (steps without MFMAs, or too few of them)
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (r >= w_done) weight(r);
    if (HAS_NEXT) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (r >= m_done) next_max(r);
        // the other half-wave holds the other 16 keys of the column: one VALU half-swap, no LDS trip
        const auto halves = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(uint32_t, smax),
                                                             __builtin_bit_cast(uint32_t, smax), false, false);
        smax = fmaxf(__builtin_bit_cast(float, (uint32_t)halves[0]), __builtin_bit_cast(float, (uint32_t)halves[1]));
        st.tmax = smax * scale;  // scale > 0
        if (!SWAP) st.s[OUT] = s_tmp;
    }
    st.l_run += psum;
    if (CARRY_OUT) {
        static_assert(!CARRY_OUT || NM >= kCarry, "a step that reads ahead for the next one has at least kCarry slots");
#pragma unroll
        for (int j = 0; j < kCarry; ++j) st.carry[j] = nxt[j];
    }
    typedef __attribute__((ext_vector_type(4))) uint32_t pk4;
    st.p[OUT][0] = __builtin_bit_cast(bf16x8, pk4{p_new[0], p_new[1], p_new[2], p_new[3]});
    st.p[OUT][1] = __builtin_bit_cast(bf16x8, pk4{p_new[4], p_new[5], p_new[6], p_new[7]});
}

template <int D>
__device__ __forceinline__ void chunk_tile_path(const AttnParams &p, const TileDesc &it, int split, int kvh,
                                                uint16_t *smem) {
    constexpr int NS = D / 16;            // contraction steps of the score MFMAs
    constexpr int NB = D / 32;            // 32-channel blocks of the output
    constexpr int CPR = D / 8;            // 16-byte chunks per K row
    constexpr int PAGE_ELEMS = kPageSize * D;
    constexpr int LOADS_PER_PAGE = PAGE_ELEMS / 512;  // 1 KiB wavefront loads per page of one KV head
    using SM = ChunkSmem<D>;
    constexpr int TE = SM::kTileElems;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction; tell the compiler
    const int n = lane & 31;
    const int h = lane >> 5;
    const int seq = it.seq;
    const int ctx = it.ctx_len;
    const int q_start = it.q_start;
    const int prefix = ctx - it.q_len;
    const int G = p.group;
    const UnitRange ur = unit_range(it, split);

    // Columns of this wave; lanes (and whole waves) without a valid column shadow the tile's first column.
    const int wcol = wave * 32 + n;
    const bool col_valid = wcol < it.n_cols;
    const int col = it.col_begin + (col_valid ? wcol : 0);
    const int row = col / G;
    const int head = kvh * G + (col - row * G);
    const int pos_eff = min(prefix + row, ur.key_end - 1);
    const int wave_first_col = it.col_begin + ((wave * 32 < it.n_cols) ? wave * 32 : 0);
    const int min_pos_eff = min(prefix + wave_first_col / G, ur.key_end - 1);  // wave-uniform
    // Sliding window: first key this column sees, and the largest such key over the wave's valid
    // columns (wave-uniform; a wave without valid columns shadows the tile's first column).
    const int wave_last_col = it.col_begin + ((wave * 32 < it.n_cols) ? min(wave * 32 + 31, it.n_cols - 1) : 0);
    const int lo = p.window > 0 ? max(0, prefix + row - p.window + 1) : 0;
    const int max_lo = p.window > 0 ? max(0, prefix + wave_last_col / G - p.window + 1) : 0;

    bf16x8 qreg[NS];  // B operand of the score MFMAs: column n, channels 16s + 8h ..
    {
        const uint16_t *qp = p.q + ((int64_t)(q_start + row) * p.num_q_heads + head) * D + h * 8;
#pragma unroll
        for (int s = 0; s < NS; ++s) qreg[s] = load_bf16x8(qp + s * 16);
    }

    // Global -> LDS traffic of a tile: wave 0/1 move K page 0/1, wave 2/3 move V page 0/1, each
    // as LOADS_PER_PAGE direct loads of 1 KiB.  Lane l of load j fills physical 16-byte chunk
    // q = 64j + l of the page's LDS image and therefore fetches the logical chunk that lives there.
    // K pages run three tiles ahead of the step, V pages two (V is consumed two steps later than K).
    const bool moves_v = wave >= 2;
    const int my_page = wave & 1;
    int g_off[LOADS_PER_PAGE];  // this lane's byte offset inside the page of one KV head, per load, minus 1024 j
#pragma unroll
    for (int j = 0; j < LOADS_PER_PAGE; ++j) {
        const int q = j * 64 + lane;
        const int k_slot = q / CPR;
        const int k_elem = k_slot * D + ((q % CPR) ^ k_swizzle<D>(k_slot)) * 8;
        const int v_d = q >> 1;
        const int v_elem = (v_d * 2 + ((q & 1) ^ ((v_d >> 3) & 1))) * 8;
        g_off[j] = (moves_v ? v_elem : k_elem) * 2 - j * 1024;  // relative to the load's own KiB (see dma_load_page)
    }
    const const_i32_ptr bt = (const_i32_ptr)(p.block_table + (int64_t)seq * p.max_blocks);  // read-only: scalar loads
    const int n_pages_seq = (ctx + kPageSize - 1) / kPageSize;
    const int64_t page_stride = (int64_t)p.num_kv_heads * kPageSize * D;
    const uint16_t *cache_head = (moves_v ? p.v_cache : p.k_cache) + (int64_t)kvh * PAGE_ELEMS;
    const int64_t last_page_id = p.num_pages - 1;
    const int tile_begin = ur.key_begin / kTileKeys;
    const int tile_end = (ur.key_end + kTileKeys - 1) / kTileKeys;
    const int n_tiles = tile_end - tile_begin;
    const int my_lds_base = (moves_v ? SM::kVBase : 0) + my_page * PAGE_ELEMS;
    const uint32_t smem_addr = lds_address(smem);
    // page id of this wave's page of tile `tile` (a scalar load: issue it a step before it is needed)
    // The raw table entry and its clamp are separate so that the entry can be fetched a step
    // before it is needed and only then looked at (the clamp would otherwise wait for the load).
    auto page_raw = [&](int tile) -> int32_t { return bt[min(tile * 2 + my_page, n_pages_seq - 1)]; };
    auto page_clamp = [&](int32_t raw) -> int64_t {
        const int64_t pg = raw;
        return pg < 0 ? 0 : (pg > last_page_id ? last_page_id : pg);
    };
    auto page_of = [&](int tile) -> int64_t { return page_clamp(page_raw(tile)); };
    // this wave's page `pg` of tile `tile` -> ring slot (tile - tile_begin) % 4
    auto issue_page = [&](int tile, int64_t pg) {
        const uint16_t *src = cache_head + pg * page_stride;
        const uint32_t dst = smem_addr + (uint32_t)(my_lds_base + ((tile - tile_begin) & (kRing - 1)) * TE) * 2;
        dma_load_page<LOADS_PER_PAGE>(src, g_off, dst);
    };
    auto issue_tile = [&](int tile) { issue_page(tile, page_of(tile)); };
    const int my_ahead = moves_v ? 2 : 3;  // tiles this wave's loads run ahead of the step

    ChunkState<D> st;
#pragma unroll
    for (int c = 0; c < NB; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.oacc[c][r] = 0.f;
    st.m_ref = kNegSentinel;
    st.l_run = 0.f;
    st.tmax = kNegSentinel;

    // MFMA row n of the score tile is key  16u + 8h' + 4a + b  for n = 16u + 8a + 4h' + b.
    const int k_row = (n & 16) | ((n & 4) << 1) | ((n & 8) >> 1) | (n & 3);
    int k_chunk[NS];  // element offset of contraction step s inside this lane's K row (swizzled)
#pragma unroll
    for (int s = 0; s < NS; ++s) k_chunk[s] = k_row * D + ((s * 2 + h) ^ k_swizzle<D>(k_row)) * 8;
    const int v_rd = SM::kVBase + v_lds_off<D>(0, n, h);  // + slot*TE + (u*D + 32c)*16 elements
    const float scale = p.scale_log2;
    // first tile of the range in which some column of this wave needs masking (wave-uniform)
    const int mask_from = max(tile_begin, min(tile_end, (min_pos_eff + 1) / kTileKeys));
    // tiles below this index hold keys in front of some column's sliding window (wave-uniform; = tile_begin without one)
    const int mask_until = max(tile_begin, min(tile_end, (max_lo + kTileKeys - 1) / kTileKeys));

    // Prologue: the first tiles start loading; when they have landed the scores of tile 0 are
    // formed (as the "next" tile of an otherwise empty step).
#pragma unroll
    for (int i = 0; i < 3; ++i)
        if (i < my_ahead && i < n_tiles) issue_tile(tile_begin + i);
    SARATHI_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    {
#pragma unroll
        for (int r = 0; r < 16; ++r) st.s[0][r] = -INFINITY;  // "current" tile of the empty step: weights 0
        st.p[0][0] = st.p[0][1] = bf16x8{};
        const int key0 = tile_begin * kTileKeys + h * 8;
        if (tile_begin >= mask_from || tile_begin < mask_until)
            chunk_step<D, false, true, true, false, false>(st, qreg, smem, k_chunk, v_rd, 0, 0, scale, key0, pos_eff, lo);
        else
            chunk_step<D, false, true, false, false, false>(st, qreg, smem, k_chunk, v_rd, 0, 0, scale, key0, pos_eff, lo);
        st.l_run = 0.f;  // the empty step contributed exp2(-inf) = 0 terms only
    }

    int32_t pg_next = page_raw(tile_begin + my_ahead);  // table entry of the page the first step will fetch
    // Common head of a step for tile t, then the step proper.  Every loop below instantiates one
    // variant only, so its body stays a single basic block (plus the rare reference raise).
    // Every step but a unit's last fetches this wave's page of tile t + my_ahead; beyond the
    // unit's end that is a clamped, unused page landing in a free ring slot, which keeps the loop
    // body and the load counter the same for all steps.
    // pg_this: table entry of the page this step fetches; fetch_next: the step itself fetches the
    // entry of the step after it (single steps), or the caller brings entries in batches (the unrolled
    // group: while a scalar load is in flight every wait for an LDS read must wait for all of them,
    // so one batch per four steps costs a quarter of what one load per step did).
    auto step = [&](int tile, auto has_prev, auto has_next, auto mask_next, auto with_dma, auto phase, auto pp,
                    int32_t pg_this, auto fetch_next) {
        // Tile t+1 must have landed (only this wave's loads of one later tile may still be in
        // flight), and every wave must be done with the slots about to be overwritten (K of
        // tile t-1, V of tile t-2).
        if (decltype(with_dma)::value) SARATHI_WAIT_VMCNT(LOADS_PER_PAGE); else SARATHI_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const int rel = tile - tile_begin;
        if (decltype(with_dma)::value) {
            issue_page(tile + my_ahead, page_clamp(pg_this));
            if (decltype(fetch_next)::value) pg_next = page_raw(tile + my_ahead + 1);  // looked at in the next step only
        }
        // Raise the softmax reference of the columns whose due tile exceeds it by more than the slack
        // (rare).  Three things carry the old reference: the output accumulators (tiles up to t-2), the
        // running sum (up to t-1) and the bf16 weights of tile t-1, which still wait for their output
        // MFMAs in this step; all three are brought to the new one.  Columns that keep their
        // reference get alpha = 1 (both half-waves of a column see the same tmax and m_ref).
        if (__any(st.tmax > st.m_ref + kRescaleSlack)) {
            const float m_new = (st.tmax > st.m_ref + kRescaleSlack) ? st.tmax : st.m_ref;
            const float alpha = __builtin_amdgcn_exp2f(st.m_ref - m_new);
            st.l_run *= alpha;
            st.m_ref = m_new;
#pragma unroll
            for (int c = 0; c < NB; ++c) st.oacc[c] *= alpha;
            constexpr int kSet = decltype(pp)::value;
#pragma unroll
            for (int u = 0; u < 2; ++u)
                st.p[kSet][u] = __builtin_convertvector(__builtin_convertvector(st.p[kSet][u], f32x8) * alpha, bf16x8);
        }
        const int next_key0 = (tile + 1) * kTileKeys + h * 8;
        constexpr int kPhase = decltype(phase)::value;
        // every step with a predecessor finds its first V operands carried over; every step with a successor reads them
        chunk_step<D, decltype(has_prev)::value, decltype(has_next)::value, decltype(mask_next)::value,
                   decltype(has_prev)::value, decltype(has_next)::value, kPhase, decltype(pp)::value, (kPhase >= 0)>(
            st, qreg, smem, k_chunk, v_rd, ((rel + 1) & (kRing - 1)) * TE, ((rel + 3) & (kRing - 1)) * TE, scale, next_key0,
            pos_eff, lo);
    };
    using T = std::true_type;
    using F = std::false_type;
    using DYN = std::integral_constant<int, -1>;  // ring slots taken from the tile index at run time
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    using P3 = std::integral_constant<int, 3>;
    if (n_tiles == 1) {
        step(tile_begin, F{}, F{}, F{}, F{}, DYN{}, P0{}, pg_next, F{});
    } else {
        // first tile: nothing to accumulate yet
        if (tile_begin + 1 >= mask_from || tile_begin + 1 < mask_until) step(tile_begin, F{}, T{}, T{}, T{}, DYN{}, P0{}, pg_next, T{});
        else step(tile_begin, F{}, T{}, F{}, T{}, DYN{}, P0{}, pg_next, T{});
        // steady state, unmasked tiles: groups of four steps with the ring slots and the register
        // sets compiled in (the group starts at tile index 1 modulo 4 and leaves the state in set 0),
        // then single steps up to the causal diagonal
        int tile = tile_begin + 1;
        // tiles in front of a sliding window's start (none without a window), then single steps up to the
        // tile index the unrolled group expects
        for (; tile + 1 < tile_end && tile + 1 < mask_until; ++tile) step(tile, T{}, T{}, T{}, T{}, DYN{}, P0{}, pg_next, T{});
        for (; tile + 1 < tile_end && tile + 1 < mask_from && ((tile - tile_begin) & 3) != 1; ++tile)
            step(tile, T{}, T{}, F{}, T{}, DYN{}, P0{}, pg_next, T{});
        if (tile + 4 < tile_end && tile + 4 < mask_from) {
            // table entries of the pages the group's steps fetch; the next group's come in one batch
            int32_t e0 = pg_next, e1 = page_raw(tile + my_ahead + 1), e2 = page_raw(tile + my_ahead + 2),
                    e3 = page_raw(tile + my_ahead + 3);
            for (; tile + 4 < tile_end && tile + 4 < mask_from; tile += 4) {
                const int32_t n0 = page_raw(tile + my_ahead + 4), n1 = page_raw(tile + my_ahead + 5),
                              n2 = page_raw(tile + my_ahead + 6), n3 = page_raw(tile + my_ahead + 7);
                step(tile, T{}, T{}, F{}, T{}, P1{}, P0{}, e0, F{});
                step(tile + 1, T{}, T{}, F{}, T{}, P2{}, P1{}, e1, F{});
                step(tile + 2, T{}, T{}, F{}, T{}, P3{}, P0{}, e2, F{});
                step(tile + 3, T{}, T{}, F{}, T{}, P0{}, P1{}, e3, F{});
                e0 = n0, e1 = n1, e2 = n2, e3 = n3;
            }
            pg_next = e0;
        }
        for (; tile + 1 < tile_end && tile + 1 < mask_from; ++tile) step(tile, T{}, T{}, F{}, T{}, DYN{}, P0{}, pg_next, T{});
        // the tiles on the causal diagonal
        for (; tile + 1 < tile_end; ++tile) step(tile, T{}, T{}, T{}, T{}, DYN{}, P0{}, pg_next, T{});
        // last tile: no further scores to form, nothing more to fetch (and no load left in flight after it)
        step(tile_end - 1, T{}, F{}, F{}, F{}, DYN{}, P0{}, pg_next, F{});
    }
    // Epilogue: the output MFMAs of the last tile.  Only here can a tile hold slots at or beyond
    // ctx_len (a unit never extends past the sequence), whose V bits must be zeroed: stale cache
    // contents times a zero weight would still poison the accumulator if they were NaN or Inf.
    {
        const int last = tile_end - 1;
        const uint16_t *v_last = smem + v_rd + ((last - tile_begin) & (kRing - 1)) * TE;
        const bool tail = last * kTileKeys + kTileKeys > ctx;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                u32x4 v = *reinterpret_cast<const u32x4 *>(v_last + (u * D + c * 32) * 16);
                if (tail) {
                    const int key0 = last * kTileKeys + u * kPageSize + h * 8;
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        v[w] &= ((key0 + 2 * w < ctx) ? 0x0000FFFFu : 0u) | ((key0 + 2 * w + 1 < ctx) ? 0xFFFF0000u : 0u);
                }
                st.oacc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v), st.p[0][u],
                                                                      st.oacc[c], 0, 0, 0);
            }
        }
    }
    f32x16 (&oacc)[NB] = st.oacc;
    const float l_run = st.l_run;
    const float m_ref = st.m_ref;

    const float l = l_run + __shfl_xor(l_run, 32);
    // accumulator register r of block c: channel 32c + 8*(r/4) + 4h + r%4
    uint16_t *op = p.out + ((int64_t)(q_start + row) * p.num_q_heads + head) * D + h * 4;
    if (ur.part_row < 0) {
        if (!col_valid) return;
        const float inv = 1.0f / l;
#pragma unroll
        for (int c = 0; c < NB; ++c)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4 o = {oacc[c][q4 * 4 + 0], oacc[c][q4 * 4 + 1], oacc[c][q4 * 4 + 2], oacc[c][q4 * 4 + 3]};
                const bf16x4 o4 = __builtin_convertvector(o * inv, bf16x4);
                *reinterpret_cast<u32x2 *>(op + c * 32 + q4 * 8) = __builtin_bit_cast(u32x2, o4);
            }
        return;
    }
    // Split tile: publish this piece's (reference maximum, sum, unnormalised output).
    if (col_valid) {
        const int64_t prow = ((int64_t)(ur.part_row + wcol) * p.num_kv_heads + kvh);
        float *po = p.part_o + prow * D + h * 4;
#pragma unroll
        for (int c = 0; c < NB; ++c)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4 o = {oacc[c][q4 * 4 + 0], oacc[c][q4 * 4 + 1], oacc[c][q4 * 4 + 2], oacc[c][q4 * 4 + 3]};
                *reinterpret_cast<f32x4 *>(po + c * 32 + q4 * 8) = o;
            }
        if (h == 0) {
            p.part_ml[prow * 2 + 0] = m_ref;
            p.part_ml[prow * 2 + 1] = l;
        }
    }
}

// Chunk tiles: one block per (unit, KV head); one wavefront per SIMD so that the pipelined
// loop has the registers it needs, the matrix pipe / vector ALU overlap comes from inside the wave.
template <int D>
__global__ __launch_bounds__(256, 2) void attn_chunk_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ChunkSmem<D>::kTotalElems];
    const int kvh = blockIdx.x % p.num_kv_heads;  // consecutive blocks = the KV heads of one unit
    const int blk = blockIdx.x / p.num_kv_heads;
    constexpr uint32_t kTileMask = (1u << kUnitTileBits) - 1;
    const uint32_t u = p.units[blk];
    chunk_tile_path<D>(p, p.tiles[u & kTileMask], (int)(u >> kUnitTileBits), kvh, smem);
}

// Wave tiles (decodes, tiny chunks): one unit per block, its keys quartered among the four wavefronts.
template <int D, bool STREAM>
__global__ __launch_bounds__(256, 2) void attn_wave_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(16))) float merge_lds[WaveMergeSmem<D>::kTotalFloats];
    const int kvh = blockIdx.x % p.num_kv_heads;
    const int blk = blockIdx.x / p.num_kv_heads;
    constexpr uint32_t kTileMask = (1u << kUnitTileBits) - 1;
    const uint32_t u = p.units[p.num_tile_units + blk];
    wave16_path<D, STREAM>(p, p.tiles[u & kTileMask], (int)(u >> kUnitTileBits), kvh, merge_lds);
}

// Both kinds of unit in ONE launch (saves the second stream's fork and join).
//
// ROLES == false: the first num_tile_units * Hkv blocks run chunk tiles, the rest wave tiles.
//
// ROLES == true: a block decides what it runs when it starts.  Chunk blocks are compute-bound and
// wave blocks memory-bound, and they overlap only when they share a compute unit; two chunk blocks
// on one unit leave it without a memory stream.  So each block looks up its compute unit (hardware
// id registers), tries to become that unit's one chunk block (compare-and-swap on the unit's flag)
// and otherwise takes wave tiles; work is handed out by per-KV-head queue heads (atomic adds), each
// kind longest first, and a block whose preferred queue is empty takes from the other one.  The grid
// has exactly one block per work item and KV head, so the second queue cannot be empty too.  All
// atomics are relaxed: they only hand out indices into the read-only plan.  The host clears the
// scheduling words with a small fill kernel in front of every such launch, so nothing depends on what
// an earlier launch (or anybody else) left in them.
template <int D, bool ROLES, bool STREAM>
__global__ __launch_bounds__(256, 2) void attn_hybrid_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[ChunkSmem<D>::kTotalElems];
    const int kvh = blockIdx.x % p.num_kv_heads;
    int blk = blockIdx.x / p.num_kv_heads;
    constexpr uint32_t kTileMask = (1u << kUnitTileBits) - 1;
    const int n_wave_blocks = p.num_units - p.num_tile_units;
    bool chunk_role = blk < p.num_tile_units;
    __shared__ int32_t role[3];  // kind, index, "this block set its compute unit's flag"
    // compute unit, shader array and shader engine ids (bits 8..15 of HW_ID) and the XCC id
    auto my_cu_flag = [&]() -> int32_t * {
        const uint32_t hw = __builtin_amdgcn_s_getreg((7 << 11) | (8 << 6) | 4);
        const uint32_t xcc = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);
        return p.sched + (((xcc << 8) | hw) & (kSchedCuSlots - 1));
    };
    if (ROLES) {
        if (threadIdx.x == 0) {
            int32_t *flag = my_cu_flag();
            int32_t *heads = p.sched + kSchedCuSlots;
            int32_t expected = 0;
            const bool own = __hip_atomic_compare_exchange_strong(flag, &expected, 1, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                                  __HIP_MEMORY_SCOPE_AGENT);
            role[2] = own ? 1 : 0;
            int kind = own ? 1 : 0;  // 1 = chunk tiles, 0 = wave tiles
            int idx = __hip_atomic_fetch_add(heads + kind * kSchedMaxKvHeads + kvh, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (idx >= (kind ? p.num_tile_units : n_wave_blocks)) {
                kind ^= 1;
                idx = __hip_atomic_fetch_add(heads + kind * kSchedMaxKvHeads + kvh, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (idx >= (kind ? p.num_tile_units : n_wave_blocks)) idx = -1;  // cannot happen: one block per item
            }
            role[0] = kind;
            role[1] = idx;
        }
        __syncthreads();
        chunk_role = role[0] != 0;
        blk = role[1];
        if (blk >= 0 && !chunk_role) blk += p.num_tile_units;  // same numbering as the static split below
    }
    if (blk >= 0) {
        if (chunk_role) {
            const uint32_t u = p.units[blk];
            chunk_tile_path<D>(p, p.tiles[u & kTileMask], (int)(u >> kUnitTileBits), kvh, smem);
        } else {
            static_assert(sizeof(float) * WaveMergeSmem<D>::kTotalFloats <= sizeof(uint16_t) * ChunkSmem<D>::kTotalElems,
                          "the wave blocks' merge buffer lives in the chunk blocks' LDS");
            const uint32_t u = p.units[blk];
            wave16_path<D, STREAM>(p, p.tiles[u & kTileMask], (int)(u >> kUnitTileBits), kvh, reinterpret_cast<float *>(smem));
        }
    }
    // the compute unit is free for another chunk block
    if (ROLES && threadIdx.x == 0 && role[2]) __hip_atomic_store(my_cu_flag(), 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Per-call metadata, host -> device: a kernel that reads the pinned host buffer itself.  The runtime's copy
// goes through a copy kernel for a few kilobytes and through the DMA engine beyond that, and the DMA path
// leaves the stream idle for 10 us before and 13-23 us after the copy (kernel and copy trace of the
// decode-only batch, 13 KiB of metadata); a kernel of ours is followed by the next one at once.
__global__ __launch_bounds__(256) void upload_kernel(u32x4 *dst, const u32x4 *src, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

// The same for callers that own no pinned buffer: the bytes travel in the kernel's arguments (the runtime copies
// the argument block when the launch is enqueued, so the source is free at once).  3,840 bytes per launch.
constexpr uint32_t kArgPieceWords = 960;
struct ArgPiece {
    uint32_t w[kArgPieceWords];
};
__global__ __launch_bounds__(256) void upload_args_kernel(u32x4 *dst, ArgPiece piece, uint32_t n16) {
    const uint32_t i = threadIdx.x;
    if (i < n16) dst[i] = u32x4{piece.w[4 * i], piece.w[4 * i + 1], piece.w[4 * i + 2], piece.w[4 * i + 3]};
}

__global__ void zero_words_kernel(uint32_t *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// ---------------------------------------------------------------------------------------
// Split-KV merge: out = sum_i w_i O_i / sum_i w_i l_i with w_i = 2^(m_i - max_i m_i), pieces
// taken in index order.  A block merges 8 columns of one split tile for one KV head: D/4
// threads per column, each owning four channels, so a piece's row is read as one coalesced
// run and the loop over pieces is unrolled to keep several loads in flight.
// ---------------------------------------------------------------------------------------
constexpr int kMergeCols = 8;  // columns per block of the merge kernel (must match the planner)

struct ReduceParams {
    const TileDesc *tiles;
    const uint32_t *reduce_units;  // (8-column group << kUnitTileBits) | tile index
    const float *part_ml;
    const float *part_o;
    uint16_t *out;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t group;
};

template <int D>
__global__ __launch_bounds__(kMergeCols * D / 4) void splitkv_reduce_kernel(ReduceParams p) {
    constexpr int TPC = D / 4;  // threads per column
    const int kvh = blockIdx.x % p.num_kv_heads;
    const uint32_t u = p.reduce_units[blockIdx.x / p.num_kv_heads];
    const TileDesc it = p.tiles[u & ((1u << kUnitTileBits) - 1)];
    const int c = (int)(u >> kUnitTileBits) * kMergeCols + threadIdx.x / TPC;  // column inside the tile
    const int d4 = (threadIdx.x % TPC) * 4;
    if (c >= it.n_cols) return;
    const int col = it.col_begin + c;
    const int row = col / p.group;
    const int head = kvh * p.group + (col - row * p.group);
    const int64_t prow0 = ((int64_t)(it.part_row0 + c) * p.num_kv_heads + kvh);
    const int64_t split_stride = (int64_t)it.n_cols * p.num_kv_heads;
    const float *__restrict__ ml = p.part_ml;
    const float *__restrict__ po = p.part_o;
    // Loads first, arithmetic after: the pieces' rows were written by the attention launch and come from memory,
    // so a loop that loads, waits and accumulates piece by piece costs one memory latency per piece (and one more
    // per piece for the maxima).  Up to kBatch pieces are fetched at once (indices beyond the last piece are clamped
    // to it: a valid, unused read); the sums still run in index order.
    constexpr int kBatch = 4;
    const int n = it.n_splits;
    float m[kBatch], l[kBatch];
    f32x4 o[kBatch];
    auto fetch = [&](int base) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int64_t prow = prow0 + (int64_t)min(base + j, n - 1) * split_stride;
            const f32x2 v = *reinterpret_cast<const f32x2 *>(ml + prow * 2);
            m[j] = v[0];
            l[j] = v[1];
            o[j] = *reinterpret_cast<const f32x4 *>(po + prow * D + d4);
        }
    };
    fetch(0);
    float m_max = kNegSentinel;
#pragma unroll
    for (int j = 0; j < kBatch; ++j) m_max = fmaxf(m_max, m[j]);  // clamped entries repeat a valid piece
    for (int i = kBatch; i < n; ++i) m_max = fmaxf(m_max, ml[(prow0 + i * split_stride) * 2]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f;
    for (int base = 0;;) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (base + j < n) {
                const float w = __builtin_amdgcn_exp2f(m[j] - m_max);
                lsum += w * l[j];
                acc += o[j] * w;
            }
        }
        base += kBatch;
        if (base >= n) break;
        fetch(base);
    }
    const bf16x4 o4 = __builtin_convertvector(acc * (1.0f / lsum), bf16x4);
    uint16_t *op = p.out + ((int64_t)(it.q_start + row) * p.num_q_heads + head) * D + d4;
    *reinterpret_cast<u32x2 *>(op) = __builtin_bit_cast(u32x2, o4);
}

// ---------------------------------------------------------------------------------------
// KV append: byte copies into the paged pools.  A block fills the slots [lo, hi) of one cache
// page for one KV head (a page unit, built by the host: a decode has one, a chunk one per page
// it touches), one thread per channel.  K rows go over as 16-byte pieces (a page holds them
// slot-major, so the hi - lo rows are one contiguous run).  V pages are channel-major: thread c
// owns the 32-byte row of channel c, gathers the tokens' values of that channel (a wavefront
// reads 128 contiguous bytes per token) and, when the whole page is new, writes the row with
// two 16-byte stores (the block writes the 4 KiB page front to back); a partly filled page
// gets 2-byte stores into its new slots only, the others keep their bytes.
// ---------------------------------------------------------------------------------------
struct AppendParams {
    const uint16_t *k_new;
    const uint16_t *v_new;
    uint16_t *k_cache;
    uint16_t *v_cache;
    const int32_t *block_table;
    const AppendUnit *units;
    int64_t num_pages;
    int32_t max_blocks;
    int32_t num_kv_heads;
    // The first copy_blocks blocks move copy_n16 16-byte words from copy_src to copy_dst instead (the attention
    // metadata of the same iteration, pinned host memory -> workspace, riding in this launch).
    u32x4 *copy_dst;
    const u32x4 *copy_src;
    uint32_t copy_n16;
    uint32_t copy_blocks;
};

// Small batches carry their records in the kernel's arguments (the argument block is on the device when the
// blocks start; a record in pinned host memory is a read across the host link at the head of every block's
// chain of dependent loads: record -> block-table entry -> stores).
constexpr int kInlineAppendUnits = 224;
struct AppendParamsInline {
    AppendParams base;
    AppendUnit units[kInlineAppendUnits];
};
static_assert(sizeof(AppendParamsInline) <= 4096, "kernel arguments are limited to 4 KiB");

template <int D>
__device__ __forceinline__ void kv_append_block(const AppendParams &p, const AppendUnit *units) {
    constexpr int kPieces = D / 8;  // 16-byte pieces of one K row
    if (blockIdx.x < p.copy_blocks) {
        const uint32_t i = blockIdx.x * D + threadIdx.x;
        if (i < p.copy_n16) p.copy_dst[i] = p.copy_src[i];
        return;
    }
    const unsigned blk = blockIdx.x - p.copy_blocks;
    const int unit = (int)(blk / (unsigned)p.num_kv_heads);
    const int h = (int)(blk % (unsigned)p.num_kv_heads);
    const u32x4 rec = *reinterpret_cast<const u32x4 *>(units + unit);
    const int lo = (int)(rec[3] & 0xFFu), hi = (int)(rec[3] >> 8);
    const int n = hi - lo;
    const int64_t row_stride = (int64_t)p.num_kv_heads * D;
    const int64_t src = ((int64_t)(int)rec[2] * p.num_kv_heads + h) * D;
    const int tid = (int)threadIdx.x;
    // The block-table entry and the rows to move depend on the record only: all of these loads are issued
    // before the first is waited for (the table entry decides where the rows go, and whether they go at all).
    const int32_t *entry = p.block_table + (int64_t)(int)rec[0] * p.max_blocks + (int)rec[1];
    const int64_t page = *entry;

    // V: gather first (all loads in flight before any store)
    const uint16_t *vsrc = p.v_new + src + tid;
    uint16_t x[kPageSize];
#pragma unroll
    for (int i = 0; i < kPageSize; ++i) x[i] = (i < n) ? vsrc[i * row_stride] : (uint16_t)0;

    // K: n rows of D channels, destination contiguous
    constexpr int kRounds = (kPageSize * kPieces) / D;
    const uint16_t *ksrc = p.k_new + src;
    u32x4 krow[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int j = tid + r * D;
        const int i = j / kPieces, piece = j % kPieces;
        krow[r] = (i < n) ? *reinterpret_cast<const u32x4 *>(ksrc + i * row_stride + piece * 8) : u32x4{0, 0, 0, 0};
    }

    if (page < 0 || page >= p.num_pages) return;  // a corrupt table entry must not become a wild store
    const int64_t head_base = (page * p.num_kv_heads + h) * (int64_t)(kPageSize * D);
    uint16_t *kdst = p.k_cache + head_base + (int64_t)lo * D;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int j = tid + r * D;
        const int i = j / kPieces, piece = j % kPieces;
        if (i < n) *reinterpret_cast<u32x4 *>(kdst + i * D + piece * 8) = krow[r];
    }

    uint16_t *vdst = p.v_cache + head_base + (int64_t)tid * kPageSize;
    if (n == kPageSize) {
        u32x4 w0, w1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w0[e] = (uint32_t)x[2 * e] | ((uint32_t)x[2 * e + 1] << 16);
            w1[e] = (uint32_t)x[8 + 2 * e] | ((uint32_t)x[9 + 2 * e] << 16);
        }
        *reinterpret_cast<u32x4 *>(vdst) = w0;
        *reinterpret_cast<u32x4 *>(vdst + 8) = w1;
    } else {
#pragma unroll
        for (int i = 0; i < kPageSize; ++i)
            if (i < n) vdst[lo + i] = x[i];
    }
}

template <int D>
__global__ __launch_bounds__(D) void kv_append_kernel(AppendParams p) {
    kv_append_block<D>(p, p.units);
}
template <int D>
__global__ __launch_bounds__(D) void kv_append_inline_kernel(AppendParamsInline p) {
    kv_append_block<D>(p.base, p.units);
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
int launch_kv_append(const sarathi_config &cfg, const AppendMeta &m, const void *k_new, const void *v_new,
                     void *k_cache, void *v_cache, int64_t num_pages, void *stream) {
    if (m.num_units == 0) return (int)hipSuccess;
    AppendParams p;
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.k_cache = static_cast<uint16_t *>(k_cache);
    p.v_cache = static_cast<uint16_t *>(v_cache);
    p.block_table = m.block_table;
    p.units = m.units;
    p.num_pages = num_pages;
    p.max_blocks = m.max_blocks;
    p.num_kv_heads = cfg.num_kv_heads;
    p.copy_dst = static_cast<u32x4 *>(m.copy_dst);
    p.copy_src = static_cast<const u32x4 *>(m.copy_src);
    p.copy_n16 = (uint32_t)((m.copy_bytes + 15) / 16);
    p.copy_blocks = (p.copy_n16 + (uint32_t)cfg.head_dim - 1) / (uint32_t)cfg.head_dim;
    const unsigned blocks = p.copy_blocks + (unsigned)m.num_units * (unsigned)cfg.num_kv_heads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (m.units_host && m.num_units <= kInlineAppendUnits) {
        AppendParamsInline pi;
        pi.base = p;
        std::memcpy(pi.units, m.units_host, sizeof(AppendUnit) * (size_t)m.num_units);
        if (cfg.head_dim == 128)
            hipLaunchKernelGGL(kv_append_inline_kernel<128>, dim3(blocks), dim3(128), 0, st, pi);
        else
            hipLaunchKernelGGL(kv_append_inline_kernel<64>, dim3(blocks), dim3(64), 0, st, pi);
        return (int)hipGetLastError();
    }
    if (cfg.head_dim == 128)
        hipLaunchKernelGGL(kv_append_kernel<128>, dim3(blocks), dim3(128), 0, st, p);
    else
        hipLaunchKernelGGL(kv_append_kernel<64>, dim3(blocks), dim3(64), 0, st, p);
    return (int)hipGetLastError();
}

int launch_upload(void *dst, const void *pinned_src, size_t bytes, void *stream) {
    const size_t n = (bytes + 15) / 16;
    if (n == 0) return (int)hipSuccess;
    hipLaunchKernelGGL(upload_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(pinned_src), n);
    return (int)hipGetLastError();
}

int launch_upload_args(void *dst, const void *host_src, size_t bytes, void *stream) {
    static_assert(sizeof(ArgPiece) + 16 <= 4096, "kernel arguments are limited to 4 KiB");
    const char *src = static_cast<const char *>(host_src);
    char *d = static_cast<char *>(dst);
    for (size_t off = 0; off < bytes; off += sizeof(ArgPiece)) {
        const size_t n = bytes - off < sizeof(ArgPiece) ? bytes - off : sizeof(ArgPiece);
        ArgPiece piece;
        std::memcpy(piece.w, src + off, n);
        hipLaunchKernelGGL(upload_args_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream),
                           reinterpret_cast<u32x4 *>(d + off), piece, (uint32_t)((n + 15) / 16));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    return (int)hipSuccess;
}

// ---------------------------------------------------------------------------------------
// Scratch of the allocation-free entry point: one array in the device image of this library, so every GPU the
// library runs on holds its own copy until the process ends.  Host code never uses the array's name as an
// address: the device address is looked up once per device and used from then on.
// ---------------------------------------------------------------------------------------
constexpr size_t kStaticSchedBytes = (kSchedBytes + 255) / 256 * 256;
constexpr size_t kStaticScratchBytes = kStaticMetaBytes + kStaticSchedBytes + kStaticPartMlBytes + kStaticPartOBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch(StaticScratch *out) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static char *base_of_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    char *base;
    {
        std::lock_guard<std::mutex> guard(lock);
        if (!base_of_device[dev]) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return (int)e;
            if (!ptr) return (int)hipErrorInvalidSymbol;
            base_of_device[dev] = static_cast<char *>(ptr);
        }
        base = base_of_device[dev];
    }
    out->meta = base;
    out->sched = reinterpret_cast<int32_t *>(base + kStaticMetaBytes);
    out->part_ml = reinterpret_cast<float *>(base + kStaticMetaBytes + kStaticSchedBytes);
    out->part_o = reinterpret_cast<float *>(base + kStaticMetaBytes + kStaticSchedBytes + kStaticPartMlBytes);
    return (int)hipSuccess;
}

int launch_zero(void *ptr, size_t bytes, void *stream) {
    const size_t n = bytes / 4;
    if (n == 0) return (int)hipSuccess;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint32_t *>(ptr), n);
    return (int)hipGetLastError();
}

int launch_reduce(const sarathi_config &cfg, const AttnMeta &m, void *out, int32_t first, int32_t count, void *stream) {
    if (count <= 0) return (int)hipSuccess;
    static_assert(kMergeCols == kReduceCols, "planner and merge kernel must agree on columns per block");
    ReduceParams p;
    p.tiles = m.tiles;
    p.reduce_units = m.reduce_units + first;
    p.part_ml = m.part_ml;
    p.part_o = m.part_o;
    p.out = static_cast<uint16_t *>(out);
    p.num_q_heads = cfg.num_q_heads;
    p.num_kv_heads = cfg.num_kv_heads;
    p.group = cfg.num_q_heads / cfg.num_kv_heads;
    const unsigned blocks = (unsigned)count * (unsigned)cfg.num_kv_heads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cfg.head_dim == 128)
        hipLaunchKernelGGL(splitkv_reduce_kernel<128>, dim3(blocks), dim3(kMergeCols * 128 / 4), 0, st, p);
    else
        hipLaunchKernelGGL(splitkv_reduce_kernel<64>, dim3(blocks), dim3(kMergeCols * 64 / 4), 0, st, p);
    return (int)hipGetLastError();
}

int launch_attention(const sarathi_config &cfg, const AttnMeta &m, const void *q, const void *k_cache,
                     const void *v_cache, int64_t num_pages, float sm_scale, void *out, int which, void *stream) {
    if (m.num_units == 0) return (int)hipSuccess;
    AttnParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_cache = static_cast<const uint16_t *>(k_cache);
    p.v_cache = static_cast<const uint16_t *>(v_cache);
    p.out = static_cast<uint16_t *>(out);
    p.block_table = m.block_table;
    p.tiles = m.tiles;
    p.units = m.units;
    p.part_ml = m.part_ml;
    p.part_o = m.part_o;
    p.num_pages = num_pages;
    p.max_blocks = m.max_blocks;
    p.num_q_heads = cfg.num_q_heads;
    p.num_kv_heads = cfg.num_kv_heads;
    p.group = cfg.num_q_heads / cfg.num_kv_heads;
    p.num_tile_units = m.num_tile_units;
    p.num_units = m.num_units;
    p.scale_log2 = sm_scale * 1.4426950408889634f;
    p.sched = nullptr;
    p.window = m.window;
    const bool stream_kv = m.stream_kv != 0;
    const unsigned dyn_lds = (unsigned)m.lds_pad_bytes;  // diagnostic: unused LDS that lowers the blocks per compute unit
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned chunk_blocks = (unsigned)m.num_tile_units * (unsigned)cfg.num_kv_heads;
    const unsigned wave_blocks = (unsigned)(m.num_units - m.num_tile_units) * (unsigned)cfg.num_kv_heads;
    if (which == 4 || which == 5) {
        p.sched = m.sched;
        const dim3 grid(chunk_blocks + wave_blocks);
        auto launch = [&](auto d, auto roles, auto stream_hint) {
            hipLaunchKernelGGL((attn_hybrid_kernel<decltype(d)::value, decltype(roles)::value, decltype(stream_hint)::value>),
                               grid, dim3(256), dyn_lds, st, p);
        };
        auto pick_stream = [&](auto d, auto roles) {
            if (stream_kv) launch(d, roles, std::true_type{}); else launch(d, roles, std::false_type{});
        };
        auto pick_roles = [&](auto d) {
            if (which == 5) pick_stream(d, std::true_type{}); else pick_stream(d, std::false_type{});
        };
        if (cfg.head_dim == 128) pick_roles(std::integral_constant<int, 128>{});
        else pick_roles(std::integral_constant<int, 64>{});
        return (int)hipGetLastError();
    }
    if (chunk_blocks && (which & 1)) {
        if (cfg.head_dim == 128)
            hipLaunchKernelGGL(attn_chunk_kernel<128>, dim3(chunk_blocks), dim3(256), dyn_lds, st, p);
        else
            hipLaunchKernelGGL(attn_chunk_kernel<64>, dim3(chunk_blocks), dim3(256), dyn_lds, st, p);
    }
    if (wave_blocks && (which & 2)) {
        if (cfg.head_dim == 128) {
            if (stream_kv) hipLaunchKernelGGL((attn_wave_kernel<128, true>), dim3(wave_blocks), dim3(256), dyn_lds, st, p);
            else hipLaunchKernelGGL((attn_wave_kernel<128, false>), dim3(wave_blocks), dim3(256), dyn_lds, st, p);
        } else {
            if (stream_kv) hipLaunchKernelGGL((attn_wave_kernel<64, true>), dim3(wave_blocks), dim3(256), dyn_lds, st, p);
            else hipLaunchKernelGGL((attn_wave_kernel<64, false>), dim3(wave_blocks), dim3(256), dyn_lds, st, p);
        }
    }
    return (int)hipGetLastError();
}

}  // namespace sarathi
