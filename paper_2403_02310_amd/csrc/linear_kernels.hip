// gfx950 kernels of libsarathi: a linear layer over the token rows of a batch (paper sections
// 2.1 and 3.1),  y[t][n] = sum_k x[t][k] * w[n][k],  bf16 in, fp32 accumulation, bf16 out.
//
// Both operands are contiguous along the contraction index k, which is the per-lane operand
// shape of v_mfma_f32_32x32x16_bf16 (a lane holds one row and 8 consecutive k).  The weight tile
// is the A operand (rows = output features) and the token tile the B operand (columns = tokens),
// so an accumulator lane holds ONE token and runs of 4 consecutive features: the output row of
// a token is written in 8-byte pieces that a wavefront's 2 x 2 accumulator tiles complete to
// 128 contiguous bytes.
//
// Workgroup = 4 wavefronts = a 128-feature x 128-token tile, wavefront = 64 x 64 of it (2 x 2
// MFMA tiles, 64 accumulator registers).  k advances in stages of 32: a stage is a 128 x 32
// weight tile and a 128 x 32 token tile (8 KiB each) brought from global memory straight into
// LDS (global_load_lds_dwordx4: no staging registers) into a ring of four stages (64 KiB, two
// workgroups per compute unit); loads run three stages ahead, one barrier per stage.  LDS rows
// are 64 bytes; the four 16-byte pieces of row r are XOR-swizzled with (r >> 2) & 3 so that the 16
// lanes of a b128 operand read, which walk 16 rows at one logical piece, hit distinct banks.
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

constexpr int kLinTile = 128;    // features and tokens per workgroup tile
constexpr int kLinStageK = 32;   // k per stage
constexpr int kLinRing = 4;      // stages in the LDS ring
constexpr int kLinStageElems = 2 * kLinTile * kLinStageK;  // weight tile then token tile
constexpr int kLinXcds = 8;

typedef void __attribute__((address_space(3))) *lin_lds_ptr;

// One direct global -> LDS load of 16 bytes per lane: lane l fetches base + byte_off(l) and the
// wavefront's kilobyte lands at LDS byte address lds_addr + 16 l.  Inline assembly so that the
// compiler's wait-count pass does not treat later LDS operand reads as possibly overtaken by it;
// these loads are waited for by hand (LIN_WAIT_VMCNT), the only vector-memory loads of the loop.
__device__ __forceinline__ void lin_dma_load_16(const uint16_t *base, int byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(byte_off), "s"(base)
                 : "memory");
}
#define LIN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

struct LinearParams {
    const uint16_t *x;   // [T, K]
    const uint16_t *w;   // [N, K]
    uint16_t *y;         // [T, N]
    float *part;         // [splits, T, N] when splits > 1
    int32_t T, N, K;
    int32_t n_tiles, t_tiles, splits;
    int32_t k_per_split;  // multiple of 32
};

__global__ __launch_bounds__(256, 2) void linear_kernel(LinearParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t smem[kLinRing * kLinStageElems];
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
    const int n0 = n_tile * kLinTile;
    const int t0 = t_tile * kLinTile;
    const int k_begin = split * p.k_per_split;
    const int k_end = min(p.K, k_begin + p.k_per_split);
    const int n_stages = (k_end - k_begin) / kLinStageK;

    // ---- global -> LDS: wavefront w moves rows 32w .. 32w+31 of the weight tile and of the token tile,
    // two loads of 16 rows each.  Lane l of a load fills physical piece l % 4 of row l / 4 and
    // therefore fetches the logical piece that lives there.
    int w_off[2], x_off[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = wave * 32 + i * 16 + (lane >> 2);
        const int piece = (lane & 3) ^ ((row >> 2) & 3);
        w_off[i] = (row * p.K + piece * 8) * 2;                  // feature rows always exist (N % 128 == 0)
        const int tok = min(t0 + row, p.T - 1) - t0;             // token rows past the batch re-read its last row
        x_off[i] = (tok * p.K + piece * 8) * 2;
    }
    const uint16_t *w_base = p.w + (int64_t)n0 * p.K + k_begin;
    const uint16_t *x_base = p.x + (int64_t)t0 * p.K + k_begin;
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(lin_lds_ptr)(smem);
    auto issue_stage = [&](int stage) {
        // stages past the range re-read the last one into a free slot: every step issues the same
        // number of loads, so one wait count serves the whole loop
        const int s = min(stage, n_stages - 1);
        const uint32_t dst = smem_addr + (uint32_t)((stage & (kLinRing - 1)) * kLinStageElems * 2) + (uint32_t)(wave * 32 * kLinStageK * 2);
        const uint16_t *wb = w_base + s * kLinStageK;
        const uint16_t *xb = x_base + s * kLinStageK;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            lin_dma_load_16(wb, w_off[i], dst + i * 1024);
            lin_dma_load_16(xb, x_off[i], dst + kLinTile * kLinStageK * 2 + i * 1024);
        }
    };

    // ---- operands: wavefront (wn, wt) owns features 64wn.. and tokens 64wt.. of the tile
    const int wn = wave & 1, wt = wave >> 1;
    const int r = lane & 31, g = lane >> 5;
    int a_off[2][2], b_off[2][2];  // [sub-tile][k16 step] element offsets inside a stage
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int ra = wn * 64 + i * 32 + r;
            const int rb = wt * 64 + i * 32 + r;
            a_off[i][s] = ra * kLinStageK + (((2 * s + g) ^ ((ra >> 2) & 3)) * 8);
            b_off[i][s] = kLinTile * kLinStageK + rb * kLinStageK + (((2 * s + g) ^ ((rb >> 2) & 3)) * 8);
        }

    lf32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

    issue_stage(0);
    issue_stage(1);
    issue_stage(2);
    for (int st = 0; st < n_stages; ++st) {
        // stage st has landed when at most the loads of the two later stages are in flight; the barrier
        // also says that every wavefront is done with the slot stage st+3 is about to overwrite
        LIN_WAIT_VMCNT(8);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue_stage(st + 3);
        const uint16_t *sp = smem + (st & (kLinRing - 1)) * kLinStageElems;
        lbf16x8 a[2][2], b[2][2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i][s] = __builtin_bit_cast(lbf16x8, *reinterpret_cast<const lu32x4 *>(sp + a_off[i][s]));
                b[i][s] = __builtin_bit_cast(lbf16x8, *reinterpret_cast<const lu32x4 *>(sp + b_off[i][s]));
            }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
                    acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i][s], b[jj][s], acc[i][jj], 0, 0, 0);
    }
    LIN_WAIT_VMCNT(0);  // the padding loads past the range must land before the workgroup's LDS is given back

    // ---- output: accumulator element e of lane (r, g) of tile (i, jj) is feature 32i + 8(e/4) + 4g + e%4, token 32jj + r
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
        const int t = t0 + wt * 64 + jj * 32 + r;
        if (t >= p.T) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int f0 = n0 + wn * 64 + i * 32 + 4 * g;
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
    for (int s = 1; s < splits; ++s) sum += *reinterpret_cast<const lf32x4 *>(part + (int64_t)s * elems + i);
    *reinterpret_cast<lu32x2 *>(y + i) = __builtin_bit_cast(lu32x2, __builtin_convertvector(sum, lbf16x4));
}

}  // namespace

LinearPlan plan_linear(int32_t T, int32_t N, int32_t K, size_t workspace_bytes) {
    LinearPlan pl;
    pl.n_tiles = N / kLinTile;
    pl.t_tiles = (T + kLinTile - 1) / kLinTile;
    pl.splits = 1;
    pl.k_per_split = K;
    // Fewer workgroups than the chip holds at once (two per compute unit): cut k so that the
    // weights stream through all compute units.  A piece keeps at least 8 stages (256 k).
    const int64_t tiles = (int64_t)pl.n_tiles * pl.t_tiles;
    const int64_t slots = 512;
    if (tiles < slots) {
        int64_t want = (slots + tiles - 1) / tiles;
        const int64_t max_by_k = K / 256 > 0 ? K / 256 : 1;
        if (want > max_by_k) want = max_by_k;
        if (want > 16) want = 16;
        const int64_t per_split_bytes = (int64_t)T * N * 4;
        while (want > 1 && (size_t)(want * per_split_bytes) > workspace_bytes) --want;
        if (want > 1) {
            int32_t kps = (int32_t)((K + want - 1) / want);
            kps = (kps + kLinStageK - 1) / kLinStageK * kLinStageK;
            pl.k_per_split = kps;
            pl.splits = (K + kps - 1) / kps;
        }
    }
    return pl;
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
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(linear_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.splits == 1) return (int)e;
    const int64_t elems = (int64_t)T * N;
    hipLaunchKernelGGL(linear_reduce_kernel, dim3((unsigned)((elems / 4 + 255) / 256)), dim3(256), 0, st, p.part, p.y, elems, pl.splits);
    return (int)hipGetLastError();
}

}  // namespace sarathi
