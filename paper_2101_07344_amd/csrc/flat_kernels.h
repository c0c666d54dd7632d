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
// straight from global memory into a register ring several k-steps deep; the 4 waves of a workgroup share them through
// L1/L2.  Within every block of 4 k-steps the reduction index is permuted so that a lane's four
// A fragments are 64 contiguous bytes of its row (lanes kb = 0 / 1 take the two halves of a
// 128-byte line): the line is requested whole while the four loads are in flight, instead of
// in 32-byte pieces.  The weights are packed with the same permutation (pack_weights_flat).
// Split partial tiles go to a workspace and are added in split order by a second
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
    long D;                    // elements per row, multiple of 64
    const void* Wp;            // packed W1: [Hb/32][KS][64][kLane]
    int KS;                    // D / kStep
    int Hb;                    // padded hidden width (multiple of 64*NT)
    int rows_b;                // padded rows (multiple of 64*MT)
    int splits, ks_per_split;  // ks_per_split is a multiple of 4 (whole permutation blocks)
    int tiles_m, tiles_n;
    float* partial;            // [splits][rows_b][Hb]
};

template <bool BF16, int MT, int NT, int RING>
__global__ __launch_bounds__(256) void fc_flat_kernel(FlatArgs a) {
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep;
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
                                                 (src * a.D + (long)ks0 * kStep) * kElem) + kb * 4;
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

    // Register ring of RING k-steps: the fragments of k-step ks + RING - 1 are requested before
    // the MFMAs of k-step ks are issued, so RING - 1 k-steps (each 16 MFMAs at MT = NT = 4) of
    // work cover the memory latency.  With one wave per SIMD this lead, not bandwidth, is what
    // sets the MFMA duty cycle.  Slots past the end re-read the last k-step and are not used.
    frag_t af[RING][MT], bf[RING][NT];
    const int last = steps - 1;
    auto load_step = [&](int slot, int k_raw) {
        const int k = min(k_raw, last);
        // k-step k = 4*block + v reads fragment 8*block + 4*kb + v of the row (kb is in ap)
        const int fa = (k >> 2) * 8 + (k & 3);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[slot][mt] = ap[mt][fa];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bf[slot][nt] = bp[nt * b_tile + (long)k * 64];
    };
    if (steps > 0) {
#pragma unroll
        for (int s = 0; s < RING - 1; ++s) load_step(s, s);
    }
    for (int ks = 0; ks < steps; ks += RING) {
#pragma unroll
        for (int s = 0; s < RING; ++s) {
            // slot (s + RING - 1) % RING was consumed by the previous k-step
            load_step((s + RING - 1) % RING, ks + s + RING - 1);
            if (ks + s < steps) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[mt][nt] = M::mma(af[s][mt], bf[s][nt], acc[mt][nt]);
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

// The same contraction with the operands shared through LDS, for the full-size 256 x 256
// workgroup tile (MT = NT = 4).  Loading every fragment straight into the registers of each
// wave that needs it makes the two waves of a tile row (column) fetch the same A (B) fragments
// twice, and the vector memory pipeline -- 32 scattered 128-byte lines per A fragment -- then
// caps the MFMA duty cycle near a quarter.  Here the 4 waves split the 16 fragments of a k-step
// (8 row blocks of A, 8 column blocks of B) four each, park them in LDS in fragment order
// (lane i's 16 bytes at slot 16*i, so both the store and the later ds_read_b128 are
// conflict-free), and after one barrier per stage every wave reads the 4 + 4 fragments of its
// own 128 x 128 quadrant.  Two LDS slots of U = 2 k-steps (64 KB) and P stages of global loads
// in flight in registers, so a load has P stages of MFMA work to cover its latency.
template <bool BF16, int P>
__global__ __launch_bounds__(256) void fc_flat_lds_kernel(FlatArgs a) {
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep;
    constexpr int kElem = BF16 ? 2 : 4;
    constexpr int U = 2;
    __shared__ frag_t lds[2][U][16][64];          // [slot][k-step][A row blocks 0-7, B column blocks 8-15][lane]

    const int n = active_rows(a.n_dev, a.n_max);
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, kb = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

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
    const int tile_row0 = tile_m * 256;
    if (tile_row0 >= n) return;                              // whole workgroup leaves together

    const int ks0 = split * a.ks_per_split;
    const int ks1 = min(a.KS, ks0 + a.ks_per_split);
    const int steps = ks1 - ks0;                             // a multiple of 4
    const int stages = (steps + U - 1) / U;
    const int last = steps - 1;

    // loader role: this wave fetches row blocks 2*wave, 2*wave+1 of A and the same column blocks of B
    const frag_t* apg[2];
    const frag_t* bpg[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int row = min(tile_row0 + (2 * wave + q) * 32 + r, n - 1);   // rows past n re-read row n-1
        const long src = a.row_index ? (long)a.row_index[row] : (long)row;
        apg[q] = reinterpret_cast<const frag_t*>(static_cast<const char*>(a.act) +
                                                 (src * a.D + (long)ks0 * kStep) * kElem) + kb * 4;
        bpg[q] = reinterpret_cast<const frag_t*>(a.Wp) + ((long)(tile_n * 8 + 2 * wave + q) * a.KS + ks0) * 64 + lane;
    }
    frag_t g[P][U][4];                                      // stage q waits in g[q % P]
    auto gload = [&](frag_t (&gs)[U][4], int first_k) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = min(first_k + u, last);
            const int fa = (k >> 2) * 8 + (k & 3);           // see fc_flat_kernel: permuted k within blocks of 4
            gs[u][0] = apg[0][fa];
            gs[u][1] = apg[1][fa];
            gs[u][2] = bpg[0][(long)k * 64];
            gs[u][3] = bpg[1][(long)k * 64];
        }
    };
    auto lwrite = [&](int slot, const frag_t (&gs)[U][4]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            lds[slot][u][2 * wave][lane] = gs[u][0];
            lds[slot][u][2 * wave + 1][lane] = gs[u][1];
            lds[slot][u][8 + 2 * wave][lane] = gs[u][2];
            lds[slot][u][8 + 2 * wave + 1][lane] = gs[u][3];
        }
    };

    f32x16_t acc[4][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[mt][nt][j] = 0.f;

    if (stages > 0) {
        gload(g[0], 0);
        lwrite(0, g[0]);
#pragma unroll
        for (int q = 1; q <= P; ++q)
            if (q < stages) gload(g[q % P], q * U);
    }
    __syncthreads();
    for (int s0 = 0; s0 < stages; s0 += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int s = s0 + p;
            if (s < stages) {                                // uniform over the workgroup
                const int slot = s & 1;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (s * U + u < steps) {
                        frag_t af[4], bf[4];
#pragma unroll
                        for (int m = 0; m < 4; ++m) af[m] = lds[slot][u][4 * wm + m][lane];
#pragma unroll
                        for (int nn = 0; nn < 4; ++nn) bf[nn] = lds[slot][u][8 + 4 * wn + nn][lane];
#pragma unroll
                        for (int m = 0; m < 4; ++m)
#pragma unroll
                            for (int nn = 0; nn < 4; ++nn) acc[m][nn] = M::mma(af[m], bf[nn], acc[m][nn]);
                    }
                }
                if (s + 1 < stages) {
                    // every wave finished reading that slot before the previous barrier
                    lwrite(slot ^ 1, g[(p + 1) % P]);
                    if (s + 1 + P < stages) gload(g[(p + 1) % P], (s + 1 + P) * U);
                }
                __syncthreads();
            }
        }
    }

    const int row_base = tile_row0 + wm * 128;
    const int col_tile0 = tile_n * 8 + wn * 4;
    float* out = a.partial + (long)split * a.rows_b * a.Hb;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
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
