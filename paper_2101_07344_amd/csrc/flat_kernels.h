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
// weights repacked at creation into MFMA fragment order.  Within every block of 4 k-steps the
// reduction index is permuted so that the eight 16-byte chunks of a row's 128-byte line are
// (k-step j&3, lane half j>>2): a lane's four A fragments of the block are 64 contiguous bytes
// of its row.  The weights are packed with the same permutation (pack_weights_flat).
// Two kernels: fc_flat_kernel (small tiles, MT = NT = 1 or 2: 16-byte fragment loads straight
// from global memory into a register ring several k-steps deep, the waves sharing them through
// L1/L2) and fc_flat_lds_kernel (the full 256 x 256 tile, operands staged through LDS).
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
// workgroup tile (four waves, each a 128 x 128 quadrant held in 16 accumulator tiles).
//
// Why not load fragments straight into the registers of each wave that needs them: the two waves
// of a tile row (column) then fetch the same A (B) fragments twice, and -- worse -- an A fragment
// load touches 32 rows x 32 bytes, a quarter of each 128-byte line.  The other three quarters are
// wanted by the next three k-steps, but by then 64 KB has passed through the 32 KB vector L1 and
// the line is gone: counters showed every activation line crossing L2 -> L1 four times and the
// MFMA pipe busy a third of the time.
//
// Here a stage is U = 4 k-steps = one whole 128-byte line per activation row.  The four waves
// split the stage's loads (64 rows x 128 B of A and 2 column blocks x 4 k-steps of packed B
// each, all full lines), park them in one of two 64 KB LDS slots, and after ONE barrier per
// stage every wave reads the 4 + 4 fragments per k-step of its quadrant with ds_read_b128.
//
// LDS slot layout: fragment (u, f) -- k-step u of the stage, f = 0..7 the A row blocks, 8..15 the
// B column blocks -- is 1 KB at u*16 KB + f*1 KB.  A B fragment is stored lane-major (lane l at
// 16*l).  An A fragment is two 512-byte halves (kb = 0, 1), and inside a half row r sits at
// (r>>3)*128 + (((r&7) + u + 4*kb) & 7)*16: the rotation by the chunk number u + 4*kb makes the
// eight lanes that hold the eight 16-byte chunks of ONE row (a loader's natural, coalesced
// assignment) hit eight different bank groups, while a reader's eight consecutive rows still
// cover one whole 128-byte group.  Neither side has bank conflicts.
//
// P stages of global loads (16 x 16 bytes per lane each) are in flight in registers; each group of
// four registers is reloaded P+1 stages ahead right after its LDS stores, so a load has P whole
// stages of MFMA work (P x 2048 MFMA cycles per wave) to cover its latency.
template <bool BF16, int P>
__global__ __launch_bounds__(256) void fc_flat_lds_kernel(FlatArgs a) {
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep;
    constexpr int kElem = BF16 ? 2 : 4;
    constexpr int U = 4;
    constexpr int kSlot = U * 16 * 1024;                     // bytes per LDS slot
    extern __shared__ __align__(16) unsigned char flat_lds[];   // 2 slots

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
    const int steps = ks1 - ks0;                             // a multiple of 4: whole stages
    const int stages = steps / U;

    // ---- loader role: rows [64*wave, 64*wave+64) of A, column blocks 2*wave, 2*wave+1 of B ----
    // load i of a stage covers 8 rows x 128 B: lane -> (row lane>>3, 16-byte chunk j = lane&7).
    // Chunk j of a line belongs to k-step j&3, half j>>2 (the k order inside a block of 4 k-steps
    // is the permuted one fc_flat_kernel documents; the packed weights follow it).
    const int row_in = lane >> 3, j = lane & 7;
    const frag_t* apg[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = min(tile_row0 + wave * 64 + i * 8 + row_in, n - 1);   // rows past n re-read row n-1
        const long src = a.row_index ? (long)a.row_index[row] : (long)row;
        apg[i] = reinterpret_cast<const frag_t*>(static_cast<const char*>(a.act) +
                                                 (src * a.D + (long)ks0 * kStep) * kElem) + j;
    }
    const frag_t* bpg[2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
        bpg[q] = reinterpret_cast<const frag_t*>(a.Wp) + ((long)(tile_n * 8 + 2 * wave + q) * a.KS + ks0) * 64 + lane;
    // LDS store offsets: A load i goes to row block 2*wave + (i>>2), rows (i&3)*8 + row_in
    const int wa_off = (j & 3) * 16384 + wave * 2048 + (j >> 2) * 512 + ((row_in + j) & 7) * 16;
    const int wb_off = (8 + 2 * wave) * 1024 + lane * 16;
    // LDS read offsets of this wave's quadrant
    int ra_off[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        ra_off[u] = u * 16384 + wm * 4096 + kb * 512 + (r >> 3) * 128 + (((r & 7) + u + 4 * kb) & 7) * 16;
    const int rb_off = (8 + 4 * wn) * 1024 + lane * 16;

    frag_t g[P][16];                                         // stage q waits in g[q % P]: 8 A loads, 2 x 4 B loads
    auto gload = [&](frag_t (&g)[16], int t_raw, int first, int count) {
        const int t = min(t_raw, stages - 1);                // the tail re-reads the last stage
#pragma unroll
        for (int e = first; e < first + count; ++e) {
            if (e < 8) g[e] = apg[e][(long)t * 8];
            else g[e] = bpg[(e - 8) >> 2][(long)(t * U + ((e - 8) & 3)) * 64];
        }
    };
    auto lstore = [&](int slot, const frag_t (&g)[16], int first, int count) {
        unsigned char* base = flat_lds + slot * kSlot;
#pragma unroll
        for (int e = first; e < first + count; ++e) {
            if (e < 8)
                *reinterpret_cast<frag_t*>(base + wa_off + (e >> 2) * 1024 + (e & 3) * 128) = g[e];
            else
                *reinterpret_cast<frag_t*>(base + wb_off + ((e - 8) & 3) * 16384 + ((e - 8) >> 2) * 1024) = g[e];
        }
    };
    auto lread = [&](frag_t (&af)[4], frag_t (&bf)[4], int slot, int u) {
        const unsigned char* base = flat_lds + slot * kSlot;
#pragma unroll
        for (int m = 0; m < 4; ++m) af[m] = *reinterpret_cast<const frag_t*>(base + ra_off[u] + m * 1024);
#pragma unroll
        for (int nn = 0; nn < 4; ++nn) bf[nn] = *reinterpret_cast<const frag_t*>(base + u * 16384 + rb_off + nn * 1024);
    };

    f32x16_t acc[4][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) acc[mt][nt][jj] = 0.f;

    frag_t ax[4], bx[4], ay[4], by[4];                       // fragments of even / odd k-steps
    auto mma_rows = [&](const frag_t (&af)[4], const frag_t (&bf)[4], int m0) {
#pragma unroll
        for (int m = m0; m < m0 + 2; ++m)
#pragma unroll
            for (int nn = 0; nn < 4; ++nn) acc[m][nn] = M::mma(af[m], bf[nn], acc[m][nn]);
    };
    // One stage, order fixed by hand with scheduling fences: every LDS read is issued half a k-step
    // or more before its MFMAs, the LDS stores of stage s+1 and the reloads for stage s+2 are spread
    // between MFMA groups, and the single barrier sits inside the last k-step.  A slot is overwritten
    // only after the barrier that follows the last MFMA-consumed read of it, and read only after the
    // barrier that follows its stores.  Every global load is issued unconditionally: a load under a
    // branch would make the compiler wait for ALL outstanding loads before each LDS store, because
    // the wait counter only orders loads that are certain to have been issued.
    auto stage = [&](int s, frag_t (&gs)[16]) {
        const int slot = s & 1;
        lread(ay, by, slot, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ax, bx, 0);
        __builtin_amdgcn_sched_barrier(0);
        lstore(slot ^ 1, gs, 0, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ax, bx, 2);
        __builtin_amdgcn_sched_barrier(0);
        lread(ax, bx, slot, 2);
        gload(gs, s + 1 + P, 0, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ay, by, 0);
        __builtin_amdgcn_sched_barrier(0);
        lstore(slot ^ 1, gs, 4, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ay, by, 2);
        __builtin_amdgcn_sched_barrier(0);
        lread(ay, by, slot, 3);
        gload(gs, s + 1 + P, 4, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ax, bx, 0);
        __builtin_amdgcn_sched_barrier(0);
        lstore(slot ^ 1, gs, 8, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ax, bx, 2);
        __builtin_amdgcn_sched_barrier(0);
        lstore(slot ^ 1, gs, 12, 4);
        gload(gs, s + 1 + P, 8, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ay, by, 0);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        lread(ax, bx, slot ^ 1, 0);
        gload(gs, s + 1 + P, 12, 4);
        __builtin_amdgcn_sched_barrier(0);
        mma_rows(ay, by, 2);
        __builtin_amdgcn_sched_barrier(0);
    };
    if (stages > 0) {                                        // uniform over the workgroup
        gload(g[0], 0, 0, 16);
        lstore(0, g[0], 0, 16);
#pragma unroll
        for (int q = 1; q <= P; ++q) gload(g[q % P], q, 0, 16);
        __syncthreads();
        lread(ax, bx, 0, 0);
        int s0 = 0;
        for (; s0 + P <= stages; s0 += P) {
#pragma unroll
            for (int p = 0; p < P; ++p) stage(s0 + p, g[(p + 1) % P]);
        }
#pragma unroll
        for (int p = 0; p < P - 1; ++p)                      // the last stages % P stages
            if (s0 + p < stages) stage(s0 + p, g[(p + 1) % P]);
    }

    const int row_base = tile_row0 + wm * 128;
    const int col_tile0 = tile_n * 8 + wn * 4;
    float* out = a.partial + (long)split * a.rows_b * a.Hb;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                const int row = row_base + mt * 32 + mfma_row(jj, kb);
                const int col = (col_tile0 + nt) * 32 + r;
                out[(long)row * a.Hb + col] = acc[mt][nt][jj];
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

// FC(h) for rows whose length is not a multiple of 64 elements (the MFMA kernels consume whole
// 128-byte lines): one wave per (row, hidden unit), lanes stride over the row, fp32 products added
// lane-wise and then by the wave butterfly -- a fixed order.  W1 is kept as stored, [H, D], in the
// cache's element type.  Slow (no operand reuse); a correctness path for odd shapes.
struct FlatGenericArgs {
    const void* act;           // [rows, D]
    const int32_t* row_index;
    const int32_t* n_dev;
    int n_max;
    long D;
    int H;
    const void* W;             // [H, D] bf16 or f32
    const float* bias;         // [H]
    float* p;                  // [rows, ldp]
    __bf16* p16;               // or null
    int ldp;
};

template <bool BF16>
__global__ __launch_bounds__(256) void fc_flat_generic_kernel(FlatGenericArgs a) {
    const int n = active_rows(a.n_dev, a.n_max);
    const int lane = threadIdx.x & 63;
    const long wave = (long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const long nwaves = (long)gridDim.x * (blockDim.x >> 6);
    const long total = (long)n * a.H;
    for (long w = wave; w < total; w += nwaves) {
        const long i = w / a.H;
        const int j = (int)(w - i * a.H);
        const long r = a.row_index ? (long)a.row_index[i] : i;
        float s = 0.f;
        if constexpr (BF16) {
            const uint16_t* x = static_cast<const uint16_t*>(a.act) + r * a.D;
            const uint16_t* wt = static_cast<const uint16_t*>(a.W) + (long)j * a.D;
            for (long e = lane; e < a.D; e += 64)
                s = fmaf(__uint_as_float((uint32_t)x[e] << 16), __uint_as_float((uint32_t)wt[e] << 16), s);
        } else {
            const float* x = static_cast<const float*>(a.act) + r * a.D;
            const float* wt = static_cast<const float*>(a.W) + (long)j * a.D;
            for (long e = lane; e < a.D; e += 64) s = fmaf(x[e], wt[e], s);
        }
        s = wave_sum(s);
        if (lane == 0) {
            const float v = fmaxf(s + a.bias[j], 0.f);
            a.p[i * a.ldp + j] = v;
            if (a.p16) a.p16[i * a.ldp + j] = (__bf16)v;
        }
    }
}

}  // namespace gati
