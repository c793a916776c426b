// gfx950 kernels of libsarathi: KV append, hybrid-batch attention over the paged cache,
// and the split-KV merge.
//
// Attention kernel (16-column wave tile).  One wavefront owns one work item: 16 query
// COLUMNS (col = row*G + head_in_group, all sharing one KV head) against a key range, walked
// in tiles of 32 keys (two pages).  Both contractions run on v_mfma_f32_16x16x32_bf16 in the
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
// barriers; the softmax is per-lane work plus two cross-lane steps (lanes n, n+16, n+32, n+48).
//
// Masking is by select: keys beyond a column's position (causal mask inside a chunk, section
// 4.1 of the paper) or beyond the item's key range get score -inf; V of slots at or beyond
// ctx_len is zeroed so that stale cache contents (possibly NaN) cannot reach an accumulator.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "internal.h"

namespace sarathi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct AttnParams {
    const uint16_t *q;
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    uint16_t *out;
    const int32_t *block_table;
    const int32_t *q_start;
    const int32_t *q_len;
    const int32_t *ctx_len;
    const WorkItem *items;
    float *part_ml;
    float *part_o;
    int64_t num_pages;
    int32_t max_blocks;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t group;
    float scale_log2;  // sm_scale * log2(e): the softmax runs in base 2
};

constexpr float kNegSentinel = -1.0e30f;  // finite "no key seen yet" running maximum

__device__ __forceinline__ bf16x8 load_bf16x8(const uint16_t *p) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p));
}

template <int D>
struct TileRegs {
    bf16x8 k[2][D / 32];  // A operands of the two score MFMAs, per 32-channel step
    bf16x8 v[D / 16];     // A operands of the output MFMAs, per 16-channel tile
};

template <int D>
struct LaneGeom {
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    const int32_t *bt;     // this sequence's block-table row
    int64_t page_stride;   // elements per page (all KV heads)
    int64_t k_lane_off;    // element offset of this lane's K row start inside a page
    int64_t v_lane_off;    // element offset of this lane's V^T run inside a page
    int64_t last_page_id;  // num_pages - 1 (page ids are clamped: a corrupt table cannot fault)
    int32_t n_pages_seq;   // pages that hold positions < ctx_len
    int32_t k_pg_sel;      // which of the tile's two pages this lane's K rows come from
    int32_t v_pg_sel;
};

template <int D>
__device__ __forceinline__ void load_tile(const LaneGeom<D> &ge, int tile, TileRegs<D> &r) {
    // Pages at or beyond ceil(ctx_len/16) are never dereferenced: the index is clamped to the
    // sequence's last page and whatever is loaded for such keys is masked below.
    int pik = min(tile * 2 + ge.k_pg_sel, ge.n_pages_seq - 1);
    int piv = min(tile * 2 + ge.v_pg_sel, ge.n_pages_seq - 1);
    int64_t pk = ge.bt[pik];
    int64_t pv = ge.bt[piv];
    pk = pk < 0 ? 0 : (pk > ge.last_page_id ? ge.last_page_id : pk);
    pv = pv < 0 ? 0 : (pv > ge.last_page_id ? ge.last_page_id : pv);
    const uint16_t *kp = ge.k_cache + pk * ge.page_stride + ge.k_lane_off;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int s = 0; s < D / 32; ++s) r.k[b][s] = load_bf16x8(kp + b * 4 * D + s * 32);
    const uint16_t *vp = ge.v_cache + pv * ge.page_stride + ge.v_lane_off;
#pragma unroll
    for (int t = 0; t < D / 16; ++t) r.v[t] = load_bf16x8(vp + t * 16 * kPageSize);
}

template <int D>
struct SoftmaxState {
    f32x4 o[D / 16];  // O^T accumulators: channel 16t + 4g + i, column n
    float m;          // running maximum (base-2 scaled scores), identical in the 4 lanes of a column
    float l;          // this lane's share of the running sum (summed over g at the end)
};

template <int D>
__device__ __forceinline__ void compute_tile(TileRegs<D> &r, const bf16x8 (&qreg)[D / 32], SoftmaxState<D> &st,
                                             int tile, int g, int pos_eff, int min_pos_eff, int ctx,
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
    const float m_new = fmaxf(st.m, tmax);
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    f32x8 p;
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = __builtin_amdgcn_exp2f(t[j] - m_new);
        psum += p[j];
    }
    st.l = st.l * alpha + psum;
    st.m = m_new;
    const bf16x8 pT = __builtin_convertvector(p, bf16x8);
#pragma unroll
    for (int c = 0; c < D / 16; ++c) {
        st.o[c] *= alpha;
        st.o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.v[c], pT, st.o[c], 0, 0, 0);
    }
}

template <int D>
__global__ __launch_bounds__(64) void attn_wave16_kernel(AttnParams p) {
    const int lane = threadIdx.x;
    const int n = lane & 15;
    const int g = lane >> 4;
    const int kvh = blockIdx.x % p.num_kv_heads;  // consecutive blocks = the KV heads of one item
    const WorkItem it = p.items[blockIdx.x / p.num_kv_heads];
    const int seq = it.seq;
    const int q_len = p.q_len[seq];
    const int ctx = p.ctx_len[seq];
    const int q_start = p.q_start[seq];
    const int prefix = ctx - q_len;
    const int G = p.group;

    // Lanes beyond the tile's valid columns shadow column 0 of the tile and store nothing.
    const bool col_valid = n < it.n_cols;
    const int col = it.col_begin + (col_valid ? n : 0);
    const int row = col / G;
    const int head = kvh * G + (col - row * G);
    const int pos_eff = min(prefix + row, it.key_end - 1);                 // last key this column may see here
    const int min_pos_eff = min(prefix + it.col_begin / G, it.key_end - 1);  // the same for the tile's first column

    bf16x8 qreg[D / 32];
    {
        const uint16_t *qp = p.q + ((int64_t)(q_start + row) * p.num_q_heads + head) * D + g * 8;
#pragma unroll
        for (int s = 0; s < D / 32; ++s) qreg[s] = load_bf16x8(qp + s * 32);
    }

    LaneGeom<D> ge;
    ge.k_cache = p.k_cache;
    ge.v_cache = p.v_cache;
    ge.bt = p.block_table + (int64_t)seq * p.max_blocks;
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

    const int tile_begin = it.key_begin / kTileKeys;
    const int tile_end = (it.key_end + kTileKeys - 1) / kTileKeys;

    // Two register sets, ping-pong: the loads of tile i+1 are in flight while tile i computes.
    TileRegs<D> ra, rb;
    load_tile<D>(ge, tile_begin, ra);
    int tile = tile_begin;
    for (; tile + 1 < tile_end; tile += 2) {
        load_tile<D>(ge, tile + 1, rb);
        compute_tile<D>(ra, qreg, st, tile, g, pos_eff, min_pos_eff, ctx, p.scale_log2);
        if (tile + 2 < tile_end) load_tile<D>(ge, tile + 2, ra);
        compute_tile<D>(rb, qreg, st, tile + 1, g, pos_eff, min_pos_eff, ctx, p.scale_log2);
    }
    if (tile < tile_end) compute_tile<D>(ra, qreg, st, tile, g, pos_eff, min_pos_eff, ctx, p.scale_log2);

    float l = st.l + __shfl_xor(st.l, 16);
    l += __shfl_xor(l, 32);
    if (!col_valid) return;
    if (it.part_row < 0) {
        const float inv = 1.0f / l;
        uint16_t *op = p.out + ((int64_t)(q_start + row) * p.num_q_heads + head) * D + g * 4;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
            const bf16x4 o4 = __builtin_convertvector(st.o[c] * inv, bf16x4);
            *reinterpret_cast<u32x2 *>(op + c * 16) = __builtin_bit_cast(u32x2, o4);
        }
    } else {
        const int64_t prow = ((int64_t)(it.part_row + n) * p.num_kv_heads + kvh);
        float *po = p.part_o + prow * D + g * 4;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) *reinterpret_cast<f32x4 *>(po + c * 16) = st.o[c];
        if (g == 0) {
            p.part_ml[prow * 2 + 0] = st.m;
            p.part_ml[prow * 2 + 1] = l;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Split-KV merge: out = sum_i w_i O_i / sum_i w_i l_i with w_i = 2^(m_i - max_i m_i), splits
// taken in index order (fixed order => bitwise reproducible).
// ---------------------------------------------------------------------------------------
struct ReduceParams {
    const ReduceItem *items;
    const float *part_ml;
    const float *part_o;
    uint16_t *out;
    const int32_t *q_start;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t group;
};

template <int D>
__global__ __launch_bounds__(256) void splitkv_reduce_kernel(ReduceParams p) {
    const int kvh = blockIdx.x % p.num_kv_heads;
    const ReduceItem it = p.items[blockIdx.x / p.num_kv_heads];
    const int c = threadIdx.x >> 4;   // column of the tile handled by this group of 16 threads
    const int d0 = threadIdx.x & 15;  // channels d0, d0+16, ...
    if (c >= it.n_cols) return;
    const int col = it.col_begin + c;
    const int row = col / p.group;
    const int head = kvh * p.group + (col - row * p.group);
    float m_max = kNegSentinel;
    for (int i = 0; i < it.n_splits; ++i) {
        const int64_t prow = (int64_t)(it.part_row + i * it.n_cols + c) * p.num_kv_heads + kvh;
        m_max = fmaxf(m_max, p.part_ml[prow * 2]);
    }
    float acc[D / 16];
#pragma unroll
    for (int e = 0; e < D / 16; ++e) acc[e] = 0.f;
    float l = 0.f;
    for (int i = 0; i < it.n_splits; ++i) {
        const int64_t prow = (int64_t)(it.part_row + i * it.n_cols + c) * p.num_kv_heads + kvh;
        const float w = __builtin_amdgcn_exp2f(p.part_ml[prow * 2] - m_max);
        l += w * p.part_ml[prow * 2 + 1];
#pragma unroll
        for (int e = 0; e < D / 16; ++e) acc[e] += w * p.part_o[prow * D + d0 + 16 * e];
    }
    const float inv = 1.0f / l;
    uint16_t *op = p.out + ((int64_t)(p.q_start[it.seq] + row) * p.num_q_heads + head) * D + d0;
#pragma unroll
    for (int e = 0; e < D / 16; ++e) {
        const __bf16 b = (__bf16)(acc[e] * inv);
        op[16 * e] = __builtin_bit_cast(uint16_t, b);
    }
}

// ---------------------------------------------------------------------------------------
// KV append: byte copies into the paged pools.  One thread moves 8 channels of one
// (token, KV head): a 16-byte K store and eight 2-byte V stores (V pages are channel-major).
// ---------------------------------------------------------------------------------------
struct AppendParams {
    const uint16_t *k_new;
    const uint16_t *v_new;
    uint16_t *k_cache;
    uint16_t *v_cache;
    const int32_t *block_table;
    const int32_t *q_start;
    const int32_t *q_len;
    const int32_t *ctx_len;
    int64_t num_pages;
    int64_t total_threads;
    int32_t max_blocks;
    int32_t num_seqs;
    int32_t num_kv_heads;
};

template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(AppendParams p) {
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= p.total_threads) return;
    constexpr int kChunks = D / 8;
    const int chunk = (int)(tid % kChunks);
    const int h = (int)((tid / kChunks) % p.num_kv_heads);
    const int t = (int)(tid / ((int64_t)kChunks * p.num_kv_heads));
    // owning sequence: last s with q_start[s] <= t
    int lo = 0, hi = p.num_seqs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (p.q_start[mid] <= t) lo = mid; else hi = mid - 1;
    }
    const int s = lo;
    const int pos = p.ctx_len[s] - p.q_len[s] + (t - p.q_start[s]);
    int64_t page = p.block_table[(int64_t)s * p.max_blocks + pos / kPageSize];
    if (page < 0 || page >= p.num_pages) return;  // a corrupt table entry must not become a wild store
    const int slot = pos % kPageSize;
    const int64_t src = ((int64_t)t * p.num_kv_heads + h) * D + chunk * 8;
    const u32x4 kv = *reinterpret_cast<const u32x4 *>(p.k_new + src);
    const u32x4 vv = *reinterpret_cast<const u32x4 *>(p.v_new + src);
    const int64_t head_base = (page * p.num_kv_heads + h) * (int64_t)(kPageSize * D);
    *reinterpret_cast<u32x4 *>(p.k_cache + head_base + slot * D + chunk * 8) = kv;
    uint16_t *vdst = p.v_cache + head_base + (int64_t)(chunk * 8) * kPageSize + slot;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t word = vv[e >> 1];
        vdst[e * kPageSize] = (uint16_t)((e & 1) ? (word >> 16) : (word & 0xFFFFu));
    }
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
int launch_kv_append(const sarathi_config &cfg, const DeviceBatch &b, const void *k_new, const void *v_new,
                     void *k_cache, void *v_cache, int64_t num_pages, void *stream) {
    AppendParams p;
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.k_cache = static_cast<uint16_t *>(k_cache);
    p.v_cache = static_cast<uint16_t *>(v_cache);
    p.block_table = b.block_table;
    p.q_start = b.q_start;
    p.q_len = b.q_len;
    p.ctx_len = b.ctx_len;
    p.num_pages = num_pages;
    p.max_blocks = b.max_blocks;
    p.num_seqs = b.num_seqs;
    p.num_kv_heads = cfg.num_kv_heads;
    p.total_threads = (int64_t)b.num_tokens * cfg.num_kv_heads * (cfg.head_dim / 8);
    const int64_t blocks = (p.total_threads + 255) / 256;
    if (blocks == 0) return (int)hipSuccess;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cfg.head_dim == 128)
        hipLaunchKernelGGL(kv_append_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(kv_append_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, st, p);
    return (int)hipGetLastError();
}

int launch_attention(const sarathi_config &cfg, const DeviceBatch &b, const void *q, const void *k_cache,
                     const void *v_cache, int64_t num_pages, float sm_scale, void *out, const WorkItem *items,
                     int32_t num_items, float *part_ml, float *part_o, void *stream) {
    if (num_items == 0) return (int)hipSuccess;
    AttnParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_cache = static_cast<const uint16_t *>(k_cache);
    p.v_cache = static_cast<const uint16_t *>(v_cache);
    p.out = static_cast<uint16_t *>(out);
    p.block_table = b.block_table;
    p.q_start = b.q_start;
    p.q_len = b.q_len;
    p.ctx_len = b.ctx_len;
    p.items = items;
    p.part_ml = part_ml;
    p.part_o = part_o;
    p.num_pages = num_pages;
    p.max_blocks = b.max_blocks;
    p.num_q_heads = cfg.num_q_heads;
    p.num_kv_heads = cfg.num_kv_heads;
    p.group = cfg.num_q_heads / cfg.num_kv_heads;
    p.scale_log2 = sm_scale * 1.4426950408889634f;
    const unsigned blocks = (unsigned)num_items * (unsigned)cfg.num_kv_heads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cfg.head_dim == 128)
        hipLaunchKernelGGL(attn_wave16_kernel<128>, dim3(blocks), dim3(64), 0, st, p);
    else
        hipLaunchKernelGGL(attn_wave16_kernel<64>, dim3(blocks), dim3(64), 0, st, p);
    return (int)hipGetLastError();
}

int launch_reduce(const sarathi_config &cfg, const DeviceBatch &b, const ReduceItem *items, int32_t num_items,
                  const float *part_ml, const float *part_o, void *out, void *stream) {
    if (num_items == 0) return (int)hipSuccess;
    ReduceParams p;
    p.items = items;
    p.part_ml = part_ml;
    p.part_o = part_o;
    p.out = static_cast<uint16_t *>(out);
    p.q_start = b.q_start;
    p.num_q_heads = cfg.num_q_heads;
    p.num_kv_heads = cfg.num_kv_heads;
    p.group = cfg.num_q_heads / cfg.num_kv_heads;
    const unsigned blocks = (unsigned)num_items * (unsigned)cfg.num_kv_heads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cfg.head_dim == 128)
        hipLaunchKernelGGL(splitkv_reduce_kernel<128>, dim3(blocks), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(splitkv_reduce_kernel<64>, dim3(blocks), dim3(256), 0, st, p);
    return (int)hipGetLastError();
}

}  // namespace sarathi
