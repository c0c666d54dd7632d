// The predictor's two FC layers, the class distribution and the selector (paper, Section 3:
// predictor Input -> Hidden(h), ReLU -> Output; selector: a projection of the predictor's
// output onto a binary decision).
//
// Both FC layers are real dense contractions (rows x C x H and rows x H x K), so they run
// on the matrix cores: v_mfma_f32_32x32x16_bf16 for bf16 caches, v_mfma_f32_32x32x2_f32 for
// fp32 caches, fp32 accumulation in both.  The GEMMs are small (at most a few GFLOP) and
// latency-bound, so the design goal is many short workgroups rather than big tiles:
//   * one workgroup = one 32-row x (32*NT)-column output tile; its 4 waves split the
//     reduction axis (split-K) and meet in LDS, added in a fixed order;
//   * the weights are repacked once, at cache creation, into MFMA fragment order, so a
//     wave's B operand for consecutive k-steps is one contiguous, fully coalesced stream;
//   * the A operand (pooled features / hidden activations) is row-major with the reduction
//     axis contiguous, which is the per-lane fragment the 32x32 MFMA wants.
//
// Fragment layout (wave of 64 lanes, r = lane % 32, kb = lane / 32), per k-step of
// kStep = 16 (bf16) or 8 (fp32) reduction elements, kLane = kStep/2 per lane:
//   A: lane holds A[m = r][k = kLane*kb .. kLane*kb + kLane-1]
//   B: lane holds B[k = kLane*kb .. ][n = r]
//   D: acc[j] is D[m = 8*(j/4) + 4*kb + j%4][n = r]
// Packed weights: Wp[((nt*KS + ks)*64 + lane)*kLane + e] = W[nt*32 + r][ks*kStep + kb*kLane + e].
#pragma once

#include "common.h"
#include "compact_kernels.h"

namespace gati {

__device__ __forceinline__ int mfma_row(int j, int kb) { return 8 * (j >> 2) + 4 * kb + (j & 3); }

template <bool BF16> struct Mma;

template <> struct Mma<true> {
    typedef bf16x8_t frag_t;            // 16 bytes: 8 bf16
    static constexpr int kStep = 16, kLane = 8;
    static __device__ __forceinline__ f32x16_t mma(frag_t a, frag_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

template <> struct Mma<false> {
    typedef f32x4_t frag_t;             // 16 bytes: 4 fp32
    static constexpr int kStep = 8, kLane = 4;
    // MFMA number e multiplies element e of every lane, i.e. k = e (lanes 0-31) and k = 4 + e
    // (lanes 32-63).  A and B use the same order, so 4 MFMAs cover the 8 k values.
    static __device__ __forceinline__ f32x16_t mma(frag_t a, frag_t b, f32x16_t c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], c, 0, 0, 0);
        return c;
    }
};

// Per-(row, column tile) summary of the logits, combined across tiles by finalize_kernel.
struct __attribute__((aligned(16))) TileStat {
    float max;    // largest logit of the tile (-inf if the tile holds only padding classes)
    float sum;    // sum over the tile of exp(z - max)
    float wsum;   // sum over the tile of ws_prob[k] * exp(z - max)
    int arg;      // lowest class index attaining max
};

struct FcArgs {
    const void* A;         // [rows_pad, K] row-major operand (bf16 or f32), zero in padding columns
    const void* Wp;        // packed weights, see above
    const float* bias;     // [N]
    int Kdim;              // padded reduction length (multiple of 4*kStep)
    int N;                 // padded output width (multiple of 32*NT)
    int n_max;
    const int32_t* n_dev;
    // epilogue of the hidden layer
    void* h;               // [rows_pad, N] bf16 or f32: relu(A W^T + bias)
    const float* p32;      // [rows_pad, ldp] fp32 pooled features (selector half); null = not this kernel's job
    const float* ws_pool;  // [ldp]
    float* u_pool;         // [rows_pad] out: ws_pool . p32[row]
    int ldp;
    // epilogue of the output layer
    int K;                 // real number of classes (<= N)
    const float* ws_prob;  // [N] selector weights of the class probabilities, zero padded
    float* logits;         // [n, K] or null
    TileStat* stats;       // [rows_pad, N/(32*NT)]
    // heads whose classes fit one column tile: the tile's summary is the row's, and this kernel writes class,
    // confidence and hit flag itself (u_pool must come from an earlier launch); stats is then unused
    int fin;
    float fin_bs, fin_tau;
    int fin_softmax_only;
    int32_t* fin_class;    // [n]
    float* fin_conf;       // [n]
    uint8_t* fin_hit;      // [n]
};

// One row's per-tile softmax summaries merged in tile order: the running (max, sum, wsum) is
// rescaled when a later tile raises the maximum; an earlier tile keeps the class on equality.
__device__ __forceinline__ void merge_tile_stats(const TileStat* st, int n_tiles, float* m_out, float* sum_out,
                                                 float* wsum_out, int* arg_out) {
    float m = -INFINITY, sum = 0.f, wsum = 0.f;
    int arg = 0;
    constexpr int B = 16;                      // summaries requested together (K = 1000: all of a row's)
    for (int t0 = 0; t0 < n_tiles; t0 += B) {
        TileStat s[B];
#pragma unroll
        for (int u = 0; u < B; ++u) s[u] = st[min(t0 + u, n_tiles - 1)];
#pragma unroll
        for (int u = 0; u < B; ++u) {
            if (t0 + u < n_tiles && s[u].max > -INFINITY) {
                if (s[u].max > m) {
                    const float w = expf(m - s[u].max);   // m = -inf -> 0
                    sum *= w; wsum *= w;
                    m = s[u].max; arg = s[u].arg;
                }
                const float w = expf(s[u].max - m);
                sum = fmaf(s[u].sum, w, sum);
                wsum = fmaf(s[u].wsum, w, wsum);
            }
        }
    }
    *m_out = m; *sum_out = sum; *wsum_out = wsum; *arg_out = arg;
}

// One row's class, confidence and hit flag from its per-tile summaries;
// confidence = logistic(bs + u_pool + sum_k ws[k] softmax(z)[k]).
// softmax_only: no selector network, confidence = largest class probability = 1 / sum_k exp(z_k - max).
__device__ __forceinline__ bool finish_row(const TileStat* st, int n_tiles, float u_pool, float bs, float tau,
                                           bool softmax_only, int32_t* cls_out, float* conf_out,
                                           uint8_t* hit_out) {
    float m, sum, wsum;
    int arg;
    merge_tile_stats(st, n_tiles, &m, &sum, &wsum, &arg);
    const float u = bs + u_pool + wsum / sum;
    const float conf = softmax_only ? 1.f / sum : 1.f / (1.f + expf(-u));
    const bool is_hit = conf > tau;
    *cls_out = arg;
    *conf_out = conf;
    *hit_out = is_hit ? 1 : 0;
    return is_hit;
}

// Pooled-feature half of the selector, fp32: u_pool[row] = ws_pool . p32[row].  The 32 rows of a
// row tile are shared out over the column blocks of the grid row, and a block's rows over its 4
// waves: a wave's 64 lanes stride over one row and add up in a fixed order (lane partials ->
// wave butterfly).  Nothing is shared between waves, so there is no barrier; rows up to the
// padded row count exist in p32, so the loads do not wait for the device-side row count.
__device__ __forceinline__ void selector_pool_part(const FcArgs& a, int row0, int tile_x, const int32_t* n_dev, int n_max, int n_tiles_x) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rpb = (32 + n_tiles_x - 1) / n_tiles_x;   // rows per block
    const f32x4_t* wv = reinterpret_cast<const f32x4_t*>(a.ws_pool);
    const int nvec = a.ldp / 4;
    for (int q = wave; q < rpb; q += 4) {
        const int rr = tile_x * rpb + q;                // wave-uniform
        if (rr >= 32) break;
        const f32x4_t* pr = reinterpret_cast<const f32x4_t*>(a.p32 + (long)(row0 + rr) * a.ldp);
        float s = 0.f;
        for (int k0 = 0; k0 < nvec; k0 += 64 * 4) {
            f32x4_t x[4], w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = min(k0 + u * 64 + lane, nvec - 1);
                x[u] = pr[k]; w[u] = wv[k];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (k0 + u * 64 + lane < nvec) {
                    s = fmaf(x[u][0], w[u][0], s); s = fmaf(x[u][1], w[u][1], s);
                    s = fmaf(x[u][2], w[u][2], s); s = fmaf(x[u][3], w[u][3], s);
                }
            }
        }
        s = wave_sum(s);
        if (lane == 0 && row0 + rr < active_rows(n_dev, n_max)) a.u_pool[row0 + rr] = s;
    }
}

// grid = (N/(32*NT), ceil(n_max/32)), block = 256.
// HIDDEN: epilogue bias + ReLU -> h, plus a share of the pooled-feature half of the selector's
// dot product (fp32).
// !HIDDEN: epilogue bias -> logits (optional store) and the tile's softmax/argmax summary.
// U: k-steps per pipeline stage (two stages in registers): 4 when a wave's share of the reduction is
// at most 8 k-steps (everything is in flight at once with half the registers), else 8.
// ASTAGE (bf16, Kdim a multiple of 256): long reductions -- the output layer over a thousand features
// or more, the hidden layer over a thousand channels or more.  A lane's A fragment is 16 bytes of ITS row, so a wave-wide fragment load touches 32
// different 128-byte lines and uses 32 bytes of each: the texture path, which takes a line per clock,
// is then busy 4x longer on A than the bytes need and the kernel is bound by it (counters at
// F = 4096: waves stalled on issue 70 % of the time, 7.5 M line accesses per launch).  Here every wave
// loads its A block of 32 rows x 128 bytes (4 k-steps) with whole lines -- 8 lanes per row, 4 loads --
// parks it in its own 4 KB of LDS (16-byte chunks of a row rotated by the row number, so neither the
// stores nor the fragment reads conflict) and reads the fragments back.  The region is the wave's
// slice of `red`, which it writes only after its last fragment read: no barrier is involved.
template <bool BF16, int NT, bool HIDDEN, int U, bool ASTAGE = false>
__global__ __launch_bounds__(256) void fc_kernel(FcArgs a) {
    static_assert(!ASTAGE || BF16, "staged A: bf16 operands");
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep, kLane = M::kLane;
    // split-K partial tiles, [wave][tile*16 + j][lane]; the staged-A instance parks two 4 KB blocks per wave there
    __shared__ float red[4][ASTAGE ? 32 : NT * 16][64];

    // tile of this workgroup.  The long-reduction output layer deals the tiles out so that one XCD (consecutive
    // workgroup ids go round the 8 XCDs) owns 8 of every 16 row tiles x (column tiles / 4): its L2 then holds
    // 8 activation tiles and a quarter of the weights instead of all activation tiles and an eighth of the weights
    int bx = blockIdx.x, by = blockIdx.y;
    if constexpr (ASTAGE && !HIDDEN) {
        if ((gridDim.x & 3) == 0 && (gridDim.y & 15) == 0) {
            const int lin = blockIdx.y * gridDim.x + blockIdx.x;
            const int xcd = lin & 7, j = lin >> 3;                       // j: 0 .. gx*gy/8 - 1 within the XCD
            const int cpx = gridDim.x >> 2;                              // column tiles per XCD
            const int per = 8 * cpx;                                     // tiles of one XCD per block of 16 row tiles
            const int blk = j / per, jj = j - blk * per;
            by = blk * 16 + (jj & 7) * 2 + (xcd & 1);                    // even / odd row tiles: a batch that fills only
                                                                         // its first row tiles still keeps every XCD busy
            bx = (xcd >> 1) * cpx + (jj >> 3);
        }
    }
    const int row0 = by * 32;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, kb = lane >> 5;
    const int n_tiles_x = a.N / (32 * NT);

    // ---- split-K MFMA over this wave's quarter of the reduction axis ----
    const int KS = a.Kdim / kStep;
    const int ksw = KS >> 2;                    // k-steps per wave
    const int ks0 = wave * ksw;
    const int nt0 = bx * NT;
    // A advances kStep elements = 2 fragments of 16 bytes per k-step
    const frag_t* ap = reinterpret_cast<const frag_t*>(
        static_cast<const char*>(a.A) + ((long)(row0 + r) * a.Kdim + (long)ks0 * kStep + kb * kLane) * (BF16 ? 2 : 4));
    const frag_t* bp = reinterpret_cast<const frag_t*>(a.Wp) + ((long)nt0 * KS + ks0) * 64 + lane;
    const long b_tile = (long)KS * 64;          // fragments between consecutive column tiles

    f32x16_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][j] = 0.f;

    const int n = active_rows(a.n_dev, a.n_max);
    if (row0 >= n) return;      // before any load: a stack's late layers launch many more row tiles than they fill

    // Software pipeline, two stages of U k-steps in registers.  What this kernel costs is a chain of
    // dependent memory round trips, so as much as fits is requested up front: both stages, the
    // epilogue's bias / selector weights and the selector's pooled half before the first MFMA, and a
    // stage is refilled as soon as its MFMAs are issued.  Reductions of up to 16 k-steps per wave
    // (C <= 1024 in bf16) are one round trip.  Slots past the end re-read the last k-step (in
    // bounds) and are skipped by the MFMA loop.
    frag_t af[2][U], bf[2][NT][U];
    const int last = ksw - 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if (!ASTAGE && (half == 0 || U < ksw)) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = min(half * U + u, last);
                af[half][u] = ap[k * 2];
#pragma unroll
                for (int t = 0; t < NT; ++t) bf[half][t][u] = bp[t * b_tile + (long)k * 64];
            }
        }
    }
    // epilogue operands of this thread's output slots (tj = q*4 + wave), requested now
    float ep_bias[4 * NT], ep_ws[4 * NT];
#pragma unroll
    for (int q = 0; q < 4 * NT; ++q) {
        const int col = (nt0 + ((q * 4 + wave) >> 4)) * 32 + r;     // < N: bias and ws_prob are padded to N
        ep_bias[q] = a.bias[col];
        ep_ws[q] = HIDDEN ? 0.f : a.ws_prob[col];
    }
    if constexpr (HIDDEN) {
        if (a.p32) selector_pool_part(a, row0, bx, a.n_dev, a.n_max, n_tiles_x);   // null: this launch has no selector half
    }
    if constexpr (ASTAGE) {
        constexpr int PD = 3;                               // blocks in flight in registers (A and W)
        const int NB = ksw >> 2;                            // blocks of 4 k-steps = one 128-byte line per row
        unsigned char* const my = reinterpret_cast<unsigned char*>(&red[wave][0][0]);   // 8 KB: two blocks
        const char* const abase = static_cast<const char*>(a.A) + ((long)row0 * a.Kdim + (long)ks0 * kStep) * 2;
        int aoff[4], rd[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 8 * i + (lane >> 3);
            aoff[i] = row * a.Kdim * 2 + (((lane & 7) - row) & 7) * 16;     // load i, lane -> (row, chunk): slot 64 i + lane
            rd[i] = (r * 8 + ((2 * i + kb + r) & 7)) * 16;                  // k-step i of the block, this lane's fragment
        }
        auto gload_a = [&](u32x4_t (&g)[4], int b) {
            const long o = (long)min(b, NB - 1) * 128;      // past the end: the last block again, never multiplied
#pragma unroll
            for (int i = 0; i < 4; ++i) g[i] = *reinterpret_cast<const u32x4_t*>(abase + aoff[i] + o);
        };
        auto gload_w = [&](frag_t (&w)[NT][4], int b) {
            const long k0 = (long)min(b, NB - 1) * 4;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) w[t][j] = bp[t * b_tile + (k0 + j) * 64];
        };
        auto lstore = [&](int buf, const u32x4_t (&g)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4_t*>(my + buf * 4096 + (64 * i + lane) * 16) = g[i];
        };
        u32x4_t ga[PD][4];
        frag_t bw[PD][NT][4];
#pragma unroll
        for (int p = 0; p < PD; ++p) { gload_a(ga[p], p); gload_w(bw[p], p); }
        lstore(0, ga[0]);
        gload_a(ga[0], PD);
        for (int b0 = 0; b0 < NB; b0 += PD) {
#pragma unroll
            for (int p = 0; p < PD; ++p) {
                const int b = b0 + p;
                if (b < NB) {                               // uniform
                    frag_t fa[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) fa[j] = *reinterpret_cast<const frag_t*>(my + (b & 1) * 4096 + rd[j]);
                    lstore((b + 1) & 1, ga[(p + 1) % PD]);  // block b+1, multiplied in the next iteration
                    gload_a(ga[(p + 1) % PD], b + 1 + PD);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int t = 0; t < NT; ++t) acc[t] = M::mma(fa[j], bw[p][t][j], acc[t]);
                    gload_w(bw[p], b + PD);
                }
            }
        }
    } else
    for (int ks = 0; ks < ksw; ks += 2 * U) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int cur = ks + half * U;          // first k-step of the stage in buffer `half`
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (cur + u < ksw) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[t] = M::mma(af[half][u], bf[half][t][u], acc[t]);
                }
            }
            const int nxt = cur + 2 * U;
            if (nxt < ksw) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = min(nxt + u, last);
                    af[half][u] = ap[k * 2];
#pragma unroll
                    for (int t = 0; t < NT; ++t) bf[half][t][u] = bp[t * b_tile + (long)k * 64];
                }
            }
        }
    }

#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) red[wave][t * 16 + j][lane] = acc[t][j];
    __syncthreads();

    // ---- fixed-order sum of the four partial tiles; thread (wave, lane) takes slots q*4 + wave ----
    float z[4 * NT];
#pragma unroll
    for (int q = 0; q < 4 * NT; ++q) {
        const int tj = q * 4 + wave;
        z[q] = (red[0][tj][lane] + red[1][tj][lane]) + (red[2][tj][lane] + red[3][tj][lane]);
    }

    if constexpr (HIDDEN) {
#pragma unroll
        for (int q = 0; q < 4 * NT; ++q) {
            const int tj = q * 4 + wave;
            const int col = (nt0 + (tj >> 4)) * 32 + r;
            const int row = row0 + mfma_row(tj & 15, kb);
            const float v = fmaxf(z[q] + ep_bias[q], 0.f);
            if constexpr (BF16)
                static_cast<__bf16*>(a.h)[(long)row * a.N + col] = (__bf16)v;
            else
                static_cast<float*>(a.h)[(long)row * a.N + col] = v;
        }
    } else {
        constexpr int TW = 32 * NT;                 // tile width in classes
        __shared__ float zt[32][TW + 1];
        __shared__ float wst[TW];
        const int col_base = nt0 * 32;
#pragma unroll
        for (int q = 0; q < 4 * NT; ++q) {
            const int tj = q * 4 + wave;
            const int lc = (tj >> 4) * 32 + r;
            const int col = col_base + lc;
            const int lr = mfma_row(tj & 15, kb);
            const bool valid = col < a.K;
            const float v = z[q] + (valid ? ep_bias[q] : 0.f);
            if (a.logits && valid && row0 + lr < n) a.logits[(long)(row0 + lr) * a.K + col] = v;
            zt[lr][lc] = valid ? v : -INFINITY;
            if ((tj & 15) == 0 && kb == 0) wst[lc] = ep_ws[q];      // one holder per column: output row 0 of its tile
        }
        __syncthreads();
        // 8 lanes per row; lane `sub` takes classes sub, sub+8, ...
        const int lr = tid >> 3, sub = tid & 7;
        float bm = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int c = sub; c < TW; c += 8) {
            const float v = zt[lr][c];
            if (v > bm) { bm = v; bi = col_base + c; }     // ascending c: lowest index on equality
        }
#pragma unroll
        for (int m = 4; m >= 1; m >>= 1) {
            const float ov = __shfl_xor(bm, m, 64);
            const int oi = __shfl_xor(bi, m, 64);
            if (ov > bm || (ov == bm && oi < bi)) { bm = ov; bi = oi; }
        }
        float ps = 0.f, pt = 0.f;
#pragma unroll
        for (int c = sub; c < TW; c += 8) {
            const float v = zt[lr][c];
            if (v > -INFINITY) {
                const float e = expf(v - bm);
                ps += e;
                pt = fmaf(e, wst[c], pt);
            }
        }
#pragma unroll
        for (int m = 4; m >= 1; m >>= 1) {
            ps += __shfl_xor(ps, m, 64);
            pt += __shfl_xor(pt, m, 64);
        }
        if (sub == 0) {
            TileStat s;
            s.max = bm; s.sum = ps; s.wsum = pt; s.arg = bi;
            if (a.fin) {
                const int row = row0 + lr;
                if (row < n)
                    finish_row(&s, 1, a.u_pool[row], a.fin_bs, a.fin_tau, a.fin_softmax_only != 0, &a.fin_class[row],
                               &a.fin_conf[row], &a.fin_hit[row]);
            } else {
                a.stats[(long)(row0 + lr) * n_tiles_x + bx] = s;
            }
        }
        if (a.p32) selector_pool_part(a, row0, bx, a.n_dev, a.n_max, n_tiles_x);   // predictors without a hidden-layer kernel
    }
}

// Input of the hidden-layer selector (Section 3, "Selector Network Design"): one operand row
// [features ; class probabilities] per active row, in the element type of the cache's matrix
// products, so that the selector's first layer is one more fc_kernel launch.
struct SelInArgs {
    const TileStat* stats;   // [rows_pad, n_tiles]
    int n_tiles;
    const float* logits;     // [n, K]
    const void* feat;        // [rows_pad, Cp] features as the predictor's FC reads them (bf16 or f32)
    void* sel_in;            // [rows_pad, ld] out: features in columns [0, Cp), q in [Cp, Cp+K), zeros after
    int Cp, K, ld;
    int n_max;
    const int32_t* n_dev;
};

template <bool BF16>
__global__ __launch_bounds__(256) void selector_input_kernel(SelInArgs a) {
    const int n = active_rows(a.n_dev, a.n_max);
    constexpr int kElem = BF16 ? 2 : 4;
    for (int row = blockIdx.x; row < n; row += gridDim.x) {
        float m, sum, wsum;
        int arg;
        merge_tile_stats(a.stats + (long)row * a.n_tiles, a.n_tiles, &m, &sum, &wsum, &arg);   // every lane: same values
        const float inv = 1.f / sum;
        char* dst = static_cast<char*>(a.sel_in) + (long)row * a.ld * kElem;
        const u32x4_t* src = reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.feat) + (long)row * a.Cp * kElem);
        const int nvec = a.Cp * kElem / 16;                   // Cp is a multiple of 64 elements
        for (int v = threadIdx.x; v < nvec; v += 256) reinterpret_cast<u32x4_t*>(dst)[v] = src[v];
        const float* z = a.logits + (long)row * a.K;
        const int nq = a.ld - a.Cp;
        for (int k = threadIdx.x; k < nq; k += 256) {
            const float q = k < a.K ? expf(z[k] - m) * inv : 0.f;
            if constexpr (BF16) reinterpret_cast<__bf16*>(dst)[a.Cp + k] = (__bf16)q;
            else reinterpret_cast<float*>(dst)[a.Cp + k] = q;
        }
    }
}

struct FinalizeArgs {
    const TileStat* stats;   // [rows_pad, n_tiles]
    int n_tiles;
    const float* u_pool;     // [rows_pad]
    float bs, tau;
    int softmax_only;        // 1: no selector network, threshold on the top class probability
    // selector with a hidden layer: u = bs + vs . g[row] replaces u_pool (null = not that selector)
    const void* sel_g;       // [rows_pad, ldg] hidden vector, bf16 or f32
    const float* sel_vs;     // [Hs]
    int sel_hs, ldg, g_bf16;
    int n_max;
    const int32_t* n_dev;
    int32_t* pred_class;     // [n]
    float* confidence;       // [n]
    uint8_t* hit;            // [n]
    // optional fused miss compaction (ids_out null = lookup only)
    const int32_t* ids_in;   // [n] or null (identity)
    int32_t* ids_out;        // [n]
    int32_t* n_miss;         // device scalar, may alias n_dev
};

// The finish: one workgroup of 1024 lanes, 1024 rows per step, turns each row's tile summaries
// into class / confidence / hit; with ids_out it also compacts the misses in the same pass.
// Batches beyond 1024 rows: launched without ids_out over several workgroups of 256 lanes (the rows
// are independent), and compact_misses_kernel follows -- one launch more, but the summaries of
// thousands of rows no longer pass through a single CU.
// (Folding this into the output-layer kernel through last-arriver tickets was tried and lost:
// device-scope fences between workgroups on different XCDs cost more than the extra launch.)
__global__ __launch_bounds__(1024) void finalize_kernel(FinalizeArgs a) {
    __shared__ CompactState<16> st;
    const int n = active_rows(a.n_dev, a.n_max);   // read before n_miss is written (they may alias)
    const int tid = threadIdx.x;
    const bool compact = a.ids_out != nullptr;     // only ever launched as one workgroup of 1024 lanes
    if (tid == 0) st.carry = 0;
    // without compaction the rows may be dealt out over several (smaller) workgroups
    for (int base = blockIdx.x * blockDim.x; base < n; base += gridDim.x * blockDim.x) {
        const int i = base + tid;
        const bool live = i < n;
        bool is_hit = false;
        if (live) {
            float u_in;
            if (a.sel_g) {                                  // second layer of the selector, in unit order
                u_in = 0.f;                                 // rows are padded to 32 units: whole 16-byte loads
                if (a.g_bf16) {
                    const u32x4_t* g = reinterpret_cast<const u32x4_t*>(static_cast<const __bf16*>(a.sel_g) + (long)i * a.ldg);
                    for (int j0 = 0; j0 < a.sel_hs; j0 += 16) {
                        const u32x4_t v0 = g[j0 / 8], v1 = g[j0 / 8 + 1];
                        const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const float gv = __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
                            if (j0 + e < a.sel_hs) u_in = fmaf(a.sel_vs[j0 + e], gv, u_in);
                        }
                    }
                } else {
                    const f32x4_t* g = reinterpret_cast<const f32x4_t*>(static_cast<const float*>(a.sel_g) + (long)i * a.ldg);
                    for (int j0 = 0; j0 < a.sel_hs; j0 += 8) {
                        const f32x4_t v0 = g[j0 / 4], v1 = g[j0 / 4 + 1];
                        const float w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (j0 + e < a.sel_hs) u_in = fmaf(a.sel_vs[j0 + e], w[e], u_in);
                    }
                }
            } else {
                u_in = a.u_pool[i];
            }
            is_hit = finish_row(a.stats + (long)i * a.n_tiles, a.n_tiles, u_in, a.bs, a.tau, a.softmax_only != 0,
                                &a.pred_class[i], &a.confidence[i], &a.hit[i]);
        }
        if (compact) {
            const int slot = compact_step<16>(st, live && !is_hit, tid);
            if (slot >= 0) a.ids_out[slot] = a.ids_in ? a.ids_in[i] : i;
        }
    }
    if (compact && tid == 0) *a.n_miss = st.carry;
}

}  // namespace gati
