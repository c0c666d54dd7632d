// The paper's FC(h) predictor (Section 3, table of predictor architectures): the whole hidden
// layer output, flattened in storage order (D = C*S values per request), through FC(D->H) and
// ReLU.  This is the one place in the lookup where a large dense contraction appears:
// [n x D] x [D x H] with D up to ~800 K, i.e. ~0.8 TFLOP and ~2.4 GB of operands per layer at
// the ResNet-50 stage-1 shape -- balanced between the MFMA and the HBM roofline.
//
// Design: a workgroup of 4 waves (2 x 2) owns a (64*MT) x (64*NT) output tile and one slice of
// the reduction axis (split-K across workgroups: the output is only n x H, far too few tiles
// to fill 256 CUs otherwise).  Each wave keeps an MT x NT grid of 32x32 accumulators (256
// AGPRs at MT = NT = 4), so one A fragment feeds NT MFMAs and one B fragment MT MFMAs.  Both
// operands are contiguous along the reduction axis -- the activation row as stored, the
// weights repacked at creation into MFMA fragment order -- so fragments are 16-byte loads
// straight from global memory, double buffered; the 4 waves of a workgroup share them through
// L1/L2.  Split partial tiles go to a workspace and are added in split order by a second
// kernel (bias, ReLU, fp32 + bf16 features), which keeps the result bit-reproducible.
// The grid is linear and XCD-aware: the workgroups that share an operand slice (same split,
// different tiles) get consecutive slots on one XCD, so the slice is fetched into one L2.
#pragma once

#include "head_kernels.h"

namespace gati {

struct FlatArgs {
    const void* act;           // [rows, D] activation rows as stored (bf16 or f32)
    const int32_t* row_index;  // [n] or null
    const int32_t* n_dev;
    int n_max;
    long D;                    // elements per row, multiple of kStep
    const void* Wp;            // packed W1: [Hb/32][KS][64][kLane]
    int KS;                    // D / kStep
    int Hb;                    // padded hidden width (multiple of 64*NT)
    int rows_b;                // padded rows (multiple of 64*MT)
    int splits, ks_per_split;
    int tiles_m, tiles_n;
    float* partial;            // [splits][rows_b][Hb]
};

template <bool BF16, int MT, int NT>
__global__ __launch_bounds__(256) void fc_flat_kernel(FlatArgs a) {
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep, kLane = M::kLane;
    constexpr int kElem = BF16 ? 2 : 4;

    const int n = active_rows(a.n_dev, a.n_max);
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, kb = lane >> 5;

    // linear grid -> (tile, split); 8 XCDs take consecutive block ids round robin
    const int tiles = a.tiles_m * a.tiles_n;
    int tile, split;
    if ((a.splits & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        tile = j % tiles;
        split = xcd * (a.splits >> 3) + j / tiles;
    } else {
        tile = blockIdx.x % tiles;
        split = blockIdx.x / tiles;
    }
    const int tile_m = tile / a.tiles_n, tile_n = tile - tile_m * a.tiles_n;
    const int row_base = (tile_m * 2 + (wave >> 1)) * (MT * 32);
    if (row_base >= n) return;                               // no barriers below: a wave may leave alone
    const int col_tile0 = (tile_n * 2 + (wave & 1)) * NT;    // in 32-column tiles

    const int ks0 = split * a.ks_per_split;
    const int ks1 = min(a.KS, ks0 + a.ks_per_split);
    const int steps = ks1 - ks0;

    // A: lane (r, kb) streams row (row_base + 32*mt + r); rows past n re-read row n-1
    const frag_t* ap[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = min(row_base + mt * 32 + r, n - 1);
        const long src = a.row_index ? (long)a.row_index[row] : (long)row;
        ap[mt] = reinterpret_cast<const frag_t*>(static_cast<const char*>(a.act) +
                                                 (src * a.D + (long)ks0 * kStep + kb * kLane) * kElem);
    }
    const frag_t* bp = reinterpret_cast<const frag_t*>(a.Wp) + ((long)col_tile0 * a.KS + ks0) * 64 + lane;
    const long b_tile = (long)a.KS * 64;

    f32x16_t acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[mt][nt][j] = 0.f;

    // two k-steps per stage, two stages in flight
    constexpr int U = 2;
    frag_t af[2][U][MT], bf[2][U][NT];
    const int last = steps - 1;
    auto load_stage = [&](int buf, int first) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = min(first + u, last);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) af[buf][u][mt] = ap[mt][k * 2];     // kStep elements = 2 fragments
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bf[buf][u][nt] = bp[nt * b_tile + (long)k * 64];
        }
    };
    if (steps > 0) load_stage(0, 0);
    for (int ks = 0; ks < steps; ks += 2 * U) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int cur = ks + half * U;
            if (cur + U < steps) load_stage(half ^ 1, cur + U);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (cur + u < steps) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            acc[mt][nt] = M::mma(af[half][u][mt], bf[half][u][nt], acc[mt][nt]);
                }
            }
        }
    }

    float* out = a.partial + (long)split * a.rows_b * a.Hb;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int row = row_base + mt * 32 + mfma_row(j, kb);
                const int col = (col_tile0 + nt) * 32 + r;
                out[(long)row * a.Hb + col] = acc[mt][nt][j];
            }
}

struct FlatReduceArgs {
    const float* partial;      // [splits][rows_b][Hb]
    const float* bias;         // [>= ldp], zero padded
    const int32_t* n_dev;
    int n_max;
    int splits, rows_b, Hb;
    float* p;                  // [rows, ldp] fp32 features = relu(sum of splits + bias)
    __bf16* p16;               // same rounded to bf16, or null
    int ldp;                   // feature stride (<= Hb), columns [0, ldp) are written
};

// One lane per 4 consecutive features of one row; splits added in order.
__global__ __launch_bounds__(256) void fc_flat_reduce_kernel(FlatReduceArgs a) {
    const int n = active_rows(a.n_dev, a.n_max);
    const int vec_per_row = a.ldp >> 2;
    const long total = (long)n * vec_per_row;
    const long split_stride = (long)a.rows_b * a.Hb;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const int row = (int)(idx / vec_per_row);
        const int col = (int)(idx - (long)row * vec_per_row) * 4;
        const float* src = a.partial + (long)row * a.Hb + col;
        f32x4_t s = {0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < a.splits; ++sp) s += *reinterpret_cast<const f32x4_t*>(src + sp * split_stride);
        const f32x4_t b = *reinterpret_cast<const f32x4_t*>(a.bias + col);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float v = fmaxf(s[k] + b[k], 0.f);
            a.p[(long)row * a.ldp + col + k] = v;
            if (a.p16) a.p16[(long)row * a.ldp + col + k] = (__bf16)v;
        }
    }
}

}  // namespace gati
