// gfx950 kernels of libsarathi: a linear layer over the token rows of a batch (paper sections
// 2.1 and 3.1),  y[t][n] = sum_k x[t][k] * w[n][k],  bf16 in, fp32 accumulation, bf16 out.
//
// Both operands are contiguous along the contraction index k, which is the per-lane operand
// shape of v_mfma_f32_32x32x16_bf16 (a lane holds one row and 8 consecutive k).  The weight tile
// is the A operand (rows = output features) and the token tile the B operand (columns = tokens),
// so an accumulator lane holds ONE token and runs of 4 consecutive features: the output row of
// a token is written in 8-byte pieces that a wavefront's accumulator tiles complete to 128
// contiguous bytes.
//
// Workgroup = 8 wavefronts = a 256-feature x BM-token tile (BM = 256; 128, 64 or 32 for small
// batches; 128 x 128 for matrices too small to fill the chip with wide tiles), wavefront = 64 features
// x BM/2 tokens of it (2 x 4 or 2 x 2 MFMA tiles; 32 x BM for the narrowest).  What bounds a tile
// shape on this chip is the path global memory -> LDS (64 bytes per clock and compute unit): a
// 128 x 128 tile needs 512 bytes of operands per MFMA, which is that path's whole bandwidth at
// full MFMA rate (measured: 0.30 of the MFMA peak, 0.40 with half of the loads made redundant);
// 256 x 256 needs half of it.  k advances in stages of 64, so that an LDS row is one full 128-byte
// line of its matrix row; a stage (256 x 64 weights, BM x 64 tokens) goes from global memory
// straight into LDS (global_load_lds_dwordx4: no staging registers) into a ring of two stages
// (BM = 256: 128 KiB), three (BM = 128: 144 KiB) or four, one workgroup per compute unit, one
// barrier per stage.  The eight 16-byte pieces of LDS row r are XOR-swizzled with (r >> 1) & 7 so that the
// 16 lanes of a b128 operand read, which walk 16 rows at one logical piece, hit distinct banks.
// Inside a stage the loop is skewed by one k16 step: the operands of step s+1 are read while the
// MFMAs of step s issue, and the last step's operands are carried over the barrier.
//
// Few tokens (a decode-heavy batch): one token tile covers the batch, the weights are read
// once, and the layer is bound by fetching them (section 3.1); when the grid would leave
// compute units idle the k range is cut into pieces (split-K) whose fp32 partial tiles a
// second small kernel adds up in piece order (bitwise reproducible).
//
// Workgroup -> tile mapping: blockIdx % 8 selects the XCD; an XCD owns the feature tiles
// n = xcd, xcd + 8, ... and runs all token tiles of a feature tile back to back, so that the
// weight tile they share is fetched into that XCD's L2 once.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "internal.h"

namespace sarathi {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 lbf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 lbf16x4;
typedef __attribute__((ext_vector_type(4))) float lf32x4;
typedef __attribute__((ext_vector_type(16))) float lf32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t lu32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t lu32x2;

constexpr int kLinBN = 256;      // features per workgroup tile
constexpr int kLinStageK = 64;   // k per stage: one 128-byte line of every row
constexpr int kLinXcds = 8;
constexpr int kLinThreads = 512;

typedef void __attribute__((address_space(3))) *lin_lds_ptr;

// One direct global -> LDS load of 16 bytes per lane: lane l fetches base + byte_off(l) and the
// wavefront's kilobyte lands at LDS byte address lds_addr + 16 l.  Inline assembly so that the
// compiler's wait-count pass does not treat later LDS operand reads as possibly overtaken by it;
// these loads are waited for by hand, they are the only vector-memory loads of the loop.
__device__ __forceinline__ void lin_dma_load_16(const uint16_t *base, int byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(byte_off), "s"(base)
                 : "memory");
}
// The same with the non-temporal hint, for the weights: every weight byte is fetched by one workgroup
// of a token tile, and a layer's weights are far more than the caches hold (+1 to +6 %).
__device__ __forceinline__ void lin_dma_load_16_stream(const uint16_t *base, int byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :
                 : "s"(lds_addr), "v"(byte_off), "s"(base)
                 : "memory");
}
// s_waitcnt with the vector-memory counter at n and the LDS counter at zero (gfx9 encoding: vmcnt in bits
// 3:0 and 15:14, expcnt 6:4 left at its maximum, lgkmcnt 11:8)
#define LIN_WAIT_VMCNT_AND_LDS(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0070)

struct LinearParams {
    const uint16_t *x;   // [T, K]
    const uint16_t *w;   // [N, K]
    uint16_t *y;         // [T, N]
    float *part;         // [splits, T, N] when splits > 1
    int32_t T, N, K;
    int32_t n_tiles, t_tiles, splits;
    int32_t k_per_split;  // multiple of 64
};

// BM tokens per tile; WT wavefronts side by side along the tokens (the other 8 / WT along the features);
// RING stages of LDS; BN features per tile (256, or 128 for matrices too small to fill the chip with wide tiles).
template <int BM, int WT, int RING, int KS = kLinStageK, int BN = kLinBN>
__global__ __launch_bounds__(kLinThreads, 1) void linear_kernel(LinearParams p) {
    constexpr int PIECES = KS / 8;              // 16-byte pieces of an LDS row
    constexpr int DMA_ROWS = 64 / PIECES;       // rows one 1 KiB load covers
    constexpr int W_ELEMS = BN * KS;
    constexpr int X_ELEMS = BM * KS;
    constexpr int STAGE = W_ELEMS + X_ELEMS;
    constexpr int W_ROWS = BN / 8;              // weight rows a wavefront moves per stage
    constexpr int W_LOADS = W_ROWS / DMA_ROWS;  // 1 KiB loads of weight rows per wavefront and stage
    constexpr int X_LOADS = BM >= 8 * DMA_ROWS ? BM / (8 * DMA_ROWS) : 1;  // the same for token rows
    constexpr int LOADS = W_LOADS + X_LOADS;    // all loads of a wavefront per stage
    constexpr int NI = BN * WT / 256;           // 32-feature MFMA tiles per wavefront: BN features / (8 / WT wavefronts) / 32
    constexpr int NJ = BM / WT / 32;            // 32-token MFMA tiles per wavefront
    constexpr int STEPS = KS / 16;
    static_assert(NI * (8 / WT) * 32 == BN && NJ * WT * 32 == BM, "the wavefronts' tiles cover the workgroup's");
    __shared__ __attribute__((aligned(16))) uint16_t smem[RING * STAGE];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // work item of this workgroup
    const int xcd = blockIdx.x % kLinXcds;
    int j = blockIdx.x / kLinXcds;
    const int t_tile = j % p.t_tiles;
    j /= p.t_tiles;
    const int split = j % p.splits;
    const int n_tile = xcd + kLinXcds * (j / p.splits);
    if (n_tile >= p.n_tiles) return;
    const int n0 = n_tile * BN;
    const int t0 = t_tile * BM;
    const int k_begin = split * p.k_per_split;
    const int k_end = min(p.K, k_begin + p.k_per_split);
    const int n_stages = (k_end - k_begin) / KS;
    auto row_key = [](int row) { return KS == 64 ? (row >> 1) & 7 : (row >> 2) & 3; };

    // ---- global -> LDS: wavefront w moves rows 32w .. 32w+31 of the weight tile (four loads of 8 rows) and
    // rows (BM/8)w .. of the token tile.  Lane l of a load fills physical piece l % 8 of row l / 8 and
    // therefore fetches the logical piece that lives there.  Rows past the matrix re-read its last row.
    int w_off[W_LOADS], x_off[X_LOADS];
#pragma unroll
    for (int i = 0; i < W_LOADS; ++i) {
        const int row = wave * W_ROWS + i * DMA_ROWS + lane / PIECES;
        const int piece = (lane % PIECES) ^ row_key(row);
        w_off[i] = ((min(n0 + row, p.N - 1) - n0) * p.K + piece * 8) * 2;
    }
#pragma unroll
    for (int i = 0; i < X_LOADS; ++i) {
        // fewer than 64 tokens: several wavefronts move the same rows (identical bytes to the same place), so
        // that every wavefront issues the same number of loads
        const int row = (wave * DMA_ROWS * X_LOADS) % BM + i * DMA_ROWS + lane / PIECES;
        const int piece = (lane % PIECES) ^ row_key(row);
        x_off[i] = ((min(t0 + row, p.T - 1) - t0) * p.K + piece * 8) * 2;
    }
    const uint16_t *w_base = p.w + (int64_t)n0 * p.K + k_begin;
    const uint16_t *x_base = p.x + (int64_t)t0 * p.K + k_begin;
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(lin_lds_ptr)(smem);
    auto issue_stage = [&](int stage, int slot) {
        // stages past the range re-read the last one into a free slot: every step issues the same
        // number of loads, so one wait count serves the whole loop
        const int s = min(stage, n_stages - 1);
        const uint32_t dst = smem_addr + (uint32_t)(slot * STAGE * 2);
        const uint16_t *wb = w_base + s * KS;
        const uint16_t *xb = x_base + s * KS;
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) lin_dma_load_16_stream(wb, w_off[i], dst + (uint32_t)((wave * W_ROWS + i * DMA_ROWS) * KS * 2));
#pragma unroll
        for (int i = 0; i < X_LOADS; ++i)
            lin_dma_load_16(xb, x_off[i], dst + (uint32_t)(W_ELEMS * 2 + ((wave * DMA_ROWS * X_LOADS) % BM + i * DMA_ROWS) * KS * 2));
    };

    // ---- operands: wavefront (wn, wt) owns features 32 NI wn.. and tokens 32 NJ wt.. of the tile
    const int wn = wave % (8 / WT), wt = wave / (8 / WT);
    const int r = lane & 31, g = lane >> 5;
    int a_row[NI], a_key[NI], b_row[NJ], b_key[NJ];  // element offset of the row inside a stage, and its swizzle key
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int ra = wn * (32 * NI) + i * 32 + r;
        a_row[i] = ra * KS;
        a_key[i] = row_key(ra);
    }
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        const int rb = wt * (32 * NJ) + jj * 32 + r;
        b_row[jj] = W_ELEMS + rb * KS;
        b_key[jj] = row_key(rb);
    }

    lf32x16 acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

    auto read_step = [&](const uint16_t *sp, int s, lbf16x8 (&a)[NI], lbf16x8 (&b)[NJ]) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
            a[i] = __builtin_bit_cast(lbf16x8, *reinterpret_cast<const lu32x4 *>(sp + a_row[i] + (((2 * s + g) ^ a_key[i]) * 8)));
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
            b[jj] = __builtin_bit_cast(lbf16x8, *reinterpret_cast<const lu32x4 *>(sp + b_row[jj] + (((2 * s + g) ^ b_key[jj]) * 8)));
    };
    auto mfma_step = [&](const lbf16x8 (&a)[NI], const lbf16x8 (&b)[NJ]) {
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
            for (int i = 0; i < NI; ++i)
                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[jj], acc[i][jj], 0, 0, 0);
    };
    lbf16x8 fa[2][NI], fb[2][NJ];  // two operand sets used in turn
#pragma unroll
    for (int i = 0; i < NI; ++i) fa[1][i] = lbf16x8{};  // the "last step of stage -1": zeros
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) fb[1][jj] = lbf16x8{};

#pragma unroll
    for (int st = 0; st < RING - 1; ++st) issue_stage(st, st);
    int slot = 0, fill_slot = RING - 1;
    for (int st = 0; st < n_stages; ++st) {
        // Stage st has landed when at most the loads of the RING-2 later stages are in flight.  The barrier
        // also says that every wavefront has its last operands of stage st-1 in registers (LDS counter at
        // zero), so the slot of stage st-1 may be overwritten by stage st+RING-1.
        LIN_WAIT_VMCNT_AND_LDS((RING - 2) * LOADS);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue_stage(st + RING - 1, fill_slot);
        const uint16_t *sp = smem + slot * STAGE;
        // STEPS is even: step s uses operand set s & 1; set 1 arrives holding the previous stage's last step
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            read_step(sp, s, fa[s & 1], fb[s & 1]);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(fa[(s & 1) ^ 1], fb[(s & 1) ^ 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
        slot = slot + 1 == RING ? 0 : slot + 1;
        fill_slot = fill_slot + 1 == RING ? 0 : fill_slot + 1;
    }
    mfma_step(fa[1], fb[1]);
    LIN_WAIT_VMCNT_AND_LDS(0);  // the padding loads past the range must land before the workgroup's LDS is given back

    // ---- output: accumulator element e of lane (r, g) of tile (i, jj) is feature 32i + 8(e/4) + 4g + e%4, token 32jj + r
#pragma unroll
    for (int jj = 0; jj < NJ; ++jj) {
        const int t = t0 + wt * (32 * NJ) + jj * 32 + r;
        if (t >= p.T) continue;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int f0 = n0 + wn * (32 * NI) + i * 32 + 4 * g;
            if (f0 >= p.N) continue;  // N is a multiple of 128, the tile 256 wide
            if (p.splits == 1) {
                uint16_t *yp = p.y + (int64_t)t * p.N + f0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const lf32x4 v = {acc[i][jj][4 * q], acc[i][jj][4 * q + 1], acc[i][jj][4 * q + 2], acc[i][jj][4 * q + 3]};
                    *reinterpret_cast<lu32x2 *>(yp + 8 * q) = __builtin_bit_cast(lu32x2, __builtin_convertvector(v, lbf16x4));
                }
            } else {
                float *pp = p.part + ((int64_t)split * p.T + t) * p.N + f0;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<lf32x4 *>(pp + 8 * q) =
                        lf32x4{acc[i][jj][4 * q], acc[i][jj][4 * q + 1], acc[i][jj][4 * q + 2], acc[i][jj][4 * q + 3]};
            }
        }
    }
}

// Adds the split-K pieces of every output element in piece order and rounds once to bf16.
__global__ __launch_bounds__(256) void linear_reduce_kernel(const float *part, uint16_t *y, int64_t elems, int splits) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= elems) return;
    lf32x4 sum = *reinterpret_cast<const lf32x4 *>(part + i);
    // four pieces are fetched before any is added (one memory latency per four pieces instead of one per piece;
    // indices past the last piece are clamped to it and not added); the additions keep the piece order
    for (int s = 1; s < splits; s += 4) {
        lf32x4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = *reinterpret_cast<const lf32x4 *>(part + (int64_t)min(s + j, splits - 1) * elems + i);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (s + j < splits) sum += v[j];
    }
    *reinterpret_cast<lu32x2 *>(y + i) = __builtin_bit_cast(lu32x2, __builtin_convertvector(sum, lbf16x4));
}

}  // namespace

LinearPlan plan_linear(int32_t T, int32_t N, int32_t K, size_t workspace_bytes) {
    // Rough cost of a tiling, in microseconds: rounds of workgroups (one per compute unit) x stages per piece x
    // the time of a stage (measured: ~1.95 us for a 256-token tile; ~1.3 us for the narrower ones, where
    // fetching the weights bounds it), plus, when the k range is cut into s pieces so that a small grid
    // fills the chip, the fp32 partial tiles (written, read back and added by a second kernel) at
    // ~3 TB/s and that kernel's launch.  Pieces keep at least 4 stages (256 k) and must fit the workspace.
    const int64_t k_stages = K / kLinStageK;
    const int64_t per_split_bytes = (int64_t)T * N * 4;
    const int64_t slots = 256;
    LinearPlan best_plan{};
    double best_cost = -1.0;
    auto consider = [&](int32_t feature_tile, int32_t token_tile) {
        const int64_t n_tiles = (N + feature_tile - 1) / feature_tile;
        const int64_t t_tiles = (T + token_tile - 1) / token_tile;
        const int64_t tiles = n_tiles * t_tiles;
        // a narrow tile next to others of its feature tile shares the weights and is bound by arithmetic (~15 % dearer
        // per token than the 256-token tile); alone it is bound by fetching them.  The 128 x 128 tile is bound by
        // the path global memory -> LDS: ~0.75 us for a quarter of the wide tile's arithmetic.
        // The 128 x 64 tile of small batches moves half the weight bytes of the 256-feature tiles per stage.
        const double stage_us = feature_tile == 128 ? (token_tile == 64 ? 0.7 : 0.75)
                                                    : token_tile == 256 ? 1.95 : (t_tiles >= 2 ? 1.12 : 1.3);
        for (int64_t s = 1; s <= 16 && (s == 1 || s * 4 <= k_stages); ++s) {
            if (s > 1 && (size_t)(s * per_split_bytes) > workspace_bytes) break;
            const int64_t rounds = (tiles * s + slots - 1) / slots;
            double c = (double)rounds * (double)((k_stages + s - 1) / s) * stage_us;
            if (s > 1) c += 8.0 * (double)s * T * N / 3.0e6 + 5.0;
            if (best_cost < 0.0 || c < 0.95 * best_cost) {
                best_cost = c;
                best_plan.feature_tile = feature_tile;
                best_plan.token_tile = token_tile;
                best_plan.n_tiles = (int32_t)n_tiles;
                best_plan.t_tiles = (int32_t)t_tiles;
                int32_t kps = (int32_t)((K + s - 1) / s);
                kps = (kps + kLinStageK - 1) / kLinStageK * kLinStageK;
                best_plan.k_per_split = s == 1 ? K : kps;
                best_plan.splits = s == 1 ? 1 : (K + kps - 1) / kps;
            }
        }
    };
    // Token tile: the smallest that holds a small batch; from 65 tokens on, 256 tokens per tile halve the
    // operand traffic per MFMA, 128 waste less of a ragged batch and give twice the workgroups, and 128 x 128
    // tiles give four times the workgroups to a matrix that is too small to fill the chip otherwise.
    // Small batches are bound by fetching the weights: 128-feature tiles give a large matrix enough workgroups
    // to fill the chip without cutting k (no partial tiles, no second kernel).
    if (T <= 32) { consider(256, 32); consider(128, 64); }
    else if (T <= 64) { consider(256, 64); consider(128, 64); }
    else {
        consider(256, 256);
        consider(256, 128);
        consider(128, 128);
    }
    return best_plan;
}

int launch_linear(const LinearPlan &pl, const void *x, const void *w, void *y, int32_t T, int32_t N, int32_t K,
                  void *workspace, void *stream) {
    LinearParams p;
    p.x = static_cast<const uint16_t *>(x);
    p.w = static_cast<const uint16_t *>(w);
    p.y = static_cast<uint16_t *>(y);
    p.part = static_cast<float *>(workspace);
    p.T = T; p.N = N; p.K = K;
    p.n_tiles = pl.n_tiles; p.t_tiles = pl.t_tiles; p.splits = pl.splits; p.k_per_split = pl.k_per_split;
    const int64_t n_rounds = (pl.n_tiles + kLinXcds - 1) / kLinXcds;
    const int64_t blocks = kLinXcds * n_rounds * pl.t_tiles * pl.splits;
    if (blocks > 0x7FFFFFFF) return (int)hipErrorInvalidValue;  // more workgroups than a grid holds
    hipStream_t st = static_cast<hipStream_t>(stream);
    // LDS: 6 x 24 KiB, 4 x 32 KiB, 2 x 64 KiB, 3 x 48 KiB, 3 x 40 KiB, 4 x 36 KiB
    if (pl.feature_tile == 128 && pl.token_tile == 64)
        hipLaunchKernelGGL((linear_kernel<64, 2, 6, kLinStageK, 128>), dim3((unsigned)blocks), dim3(kLinThreads), 0, st, p);
    else if (pl.feature_tile == 128)
        hipLaunchKernelGGL((linear_kernel<128, 2, 4, kLinStageK, 128>), dim3((unsigned)blocks), dim3(kLinThreads), 0, st, p);
    else if (pl.token_tile == 256)
        hipLaunchKernelGGL((linear_kernel<256, 2, 2>), dim3((unsigned)blocks), dim3(kLinThreads), 0, st, p);
    else if (pl.token_tile == 128)
        hipLaunchKernelGGL((linear_kernel<128, 2, 3>), dim3((unsigned)blocks), dim3(kLinThreads), 0, st, p);
    else if (pl.token_tile == 64)
        hipLaunchKernelGGL((linear_kernel<64, 1, 3>), dim3((unsigned)blocks), dim3(kLinThreads), 0, st, p);
    else
        hipLaunchKernelGGL((linear_kernel<32, 1, 4>), dim3((unsigned)blocks), dim3(kLinThreads), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return (int)e;
    const int64_t elems = (int64_t)T * N;
    hipLaunchKernelGGL(linear_reduce_kernel, dim3((unsigned)((elems / 4 + 255) / 256)), dim3(256), 0, st, p.part, p.y, elems, pl.splits);
    return (int)hipGetLastError();
}

}  // namespace sarathi
