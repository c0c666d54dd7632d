// Kernels of one retraining step of a learned cache (Section 3, "Training Learned Caches";
// Section 5, "Retraining Learned Caches"): forward and backward pass of the predictors of the
// paper's table of architectures (pooling, FC(h), Conv(k,s) as a product over gathered windows;
// all end in FC -> softmax) and of the selector, with the SGD update fused into the
// weight-gradient products.  All arithmetic is fp32; the products run on the fp32 MFMA
// (32x32x2), whose accumulation is an fp32 FMA chain.  gfx950, 64-wide waves.
#pragma once

#include "common.h"

namespace gati {

// ---------------------------------------------------------------------------------------------
// D[M][N] = sum_k A(m,k) * B(k,n), then an epilogue.
//   A(m,k) = TA ? A[k*lda + m] : A[m*lda + k]
//   B(k,n) = TB ? B[n*ldb + k] : B[k*ldb + n]
// Workgroup: 256 threads = 4 waves, 64 x 64 output tile, one 32 x 32 MFMA tile per wave.  A stage
// is 32 values of k; the two operand tiles are staged through LDS as [k][m] and [k][n] (row
// length 65 floats), from which lane l reads the MFMA operands (k = l/32, m or n = l%32) without
// bank conflicts.  Out-of-range elements are read as zero, so M, N and Kd are arbitrary.
// With gridDim.z > 1 the reduction is split: slice z handles stages z, z + gridDim.z, ... and
// writes its raw sums to part[z][M][N]; gemm_epilogue_kernel adds the slices in a fixed order.
enum GemmEpilogue {
    EPI_BIAS = 0,       // out = acc + bias[n]
    EPI_BIAS_RELU = 1,  // out = max(acc + bias[n], 0)
    EPI_MASK = 2,       // out = mask[m][n] > 0 ? acc : 0      (mask has the leading dimension of out)
    EPI_SGD = 3         // out = out - lr * acc
};

struct GemmArgs {
    const float* A; int lda;
    const float* B; int ldb;
    int M, N, Kd;
    float* out; int ldo;
    const float* bias;   // EPI_BIAS, EPI_BIAS_RELU
    const float* mask;   // EPI_MASK
    float lr;            // EPI_SGD
    float* part;         // [gridDim.z][M][N] when the reduction is split
    int veca, vecb;      // 16-byte loads allowed for A / B (base and leading dimension aligned)
};

constexpr int kGemmTile = 64, kGemmK = 32, kGemmLd = 65;

template <int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, int r, int c, float acc) {
    float* o = g.out + (size_t)r * g.ldo + c;
    if constexpr (EPI == EPI_BIAS) *o = acc + g.bias[c];
    else if constexpr (EPI == EPI_BIAS_RELU) *o = fmaxf(acc + g.bias[c], 0.0f);
    else if constexpr (EPI == EPI_MASK) *o = g.mask[(size_t)r * g.ldo + c] > 0.0f ? acc : 0.0f;
    else *o = *o - g.lr * acc;
}

// Four consecutive elements along the contiguous axis of an operand, zero where out of range.
// `major` is the index along the strided axis (limit nmajor), `minor` along the contiguous one.
__device__ __forceinline__ f32x4_t gemm_load4(const float* __restrict__ p, int ld, int major, int minor,
                                              int nmajor, int nminor, int vec) {
    f32x4_t v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (major >= nmajor) return v;
    const float* q = p + (size_t)major * ld + minor;
    if (vec && minor + 3 < nminor) return *reinterpret_cast<const f32x4_t*>(q);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (minor + i < nminor) v[i] = q[i];
    return v;
}

// One operand's 64 x 32 stage, two 16-byte pieces per thread.
//   KC (k contiguous in memory: A plain, B transposed): thread -> k quad t%8, row t/8 and t/8 + 32
//   else (m contiguous: A transposed, B plain):          thread -> m quad t%16, k t/16 and t/16 + 16
template <bool KC>
__device__ __forceinline__ void gemm_fetch(const float* __restrict__ p, int ld, int m0, int k0, int nm, int nk,
                                           int vec, int t, f32x4_t (&v)[2]) {
    if constexpr (KC) {
        const int kq = (t & 7) * 4, m = t >> 3;
        v[0] = gemm_load4(p, ld, m0 + m, k0 + kq, nm, nk, vec);
        v[1] = gemm_load4(p, ld, m0 + m + 32, k0 + kq, nm, nk, vec);
    } else {
        const int mq = (t & 15) * 4, k = t >> 4;
        v[0] = gemm_load4(p, ld, k0 + k, m0 + mq, nk, nm, vec);
        v[1] = gemm_load4(p, ld, k0 + k + 16, m0 + mq, nk, nm, vec);
    }
}

template <bool KC>
__device__ __forceinline__ void gemm_stash(float* __restrict__ s, int t, const f32x4_t (&v)[2]) {
    if constexpr (KC) {
        const int kq = (t & 7) * 4, m = t >> 3;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[(kq + i) * kGemmLd + m] = v[0][i];
            s[(kq + i) * kGemmLd + m + 32] = v[1][i];
        }
    } else {
        const int mq = (t & 15) * 4, k = t >> 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[k * kGemmLd + mq + i] = v[0][i];
            s[(k + 16) * kGemmLd + mq + i] = v[1][i];
        }
    }
}

template <bool TA, bool TB, int EPI>
__global__ __launch_bounds__(256) void train_gemm_kernel(GemmArgs g) {
    __shared__ float As[kGemmK * kGemmLd];
    __shared__ float Bs[kGemmK * kGemmLd];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int m0 = blockIdx.y * kGemmTile, n0 = blockIdx.x * kGemmTile;
    const int wm = (wave & 1) * 32, wn = (wave >> 1) * 32;
    const int stages = (g.Kd + kGemmK - 1) / kGemmK;
    const int nz = gridDim.z, z = blockIdx.z;

    f32x16_t acc;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;

    f32x4_t va[2], vb[2];
    int s = z;
    if (s < stages) {
        gemm_fetch<!TA>(g.A, g.lda, m0, s * kGemmK, g.M, g.Kd, g.veca, t, va);
        gemm_fetch<TB>(g.B, g.ldb, n0, s * kGemmK, g.N, g.Kd, g.vecb, t, vb);
    }
    for (; s < stages; s += nz) {
        __syncthreads();                       // the previous stage's LDS reads are done
        gemm_stash<!TA>(As, t, va);
        gemm_stash<TB>(Bs, t, vb);
        __syncthreads();
        if (s + nz < stages) {                 // next stage's loads fly during the MFMAs
            gemm_fetch<!TA>(g.A, g.lda, m0, (s + nz) * kGemmK, g.M, g.Kd, g.veca, t, va);
            gemm_fetch<TB>(g.B, g.ldb, n0, (s + nz) * kGemmK, g.N, g.Kd, g.vecb, t, vb);
        }
        const float* ap = As + (lane >> 5) * kGemmLd + wm + (lane & 31);
        const float* bp = Bs + (lane >> 5) * kGemmLd + wn + (lane & 31);
#pragma unroll
        for (int kk = 0; kk < kGemmK; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[kk * kGemmLd], bp[kk * kGemmLd], acc, 0, 0, 0);
    }

    const int c = n0 + wn + (lane & 31);
    if (c >= g.N) return;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int r = m0 + wm + 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3);
        if (r >= g.M) continue;
        if (nz > 1) g.part[((size_t)z * g.M + r) * g.N + c] = acc[j];
        else gemm_epilogue<EPI>(g, r, c, acc[j]);
    }
}

// Sum of the reduction slices, slice 0 first, then the epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_epilogue_kernel(GemmArgs g, int nz) {
    const long total = (long)g.M * g.N;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        float acc = g.part[i];
        for (int z = 1; z < nz; ++z) acc += g.part[(size_t)z * total + i];
        gemm_epilogue<EPI>(g, (int)(i / g.N), (int)(i % g.N), acc);
    }
}

// ---------------------------------------------------------------------------------------------
// Per training sample (one wave per row): softmax of the logits, the distillation-style target
// t = (1 - alpha) onehot(label) + alpha Y, the predictor's loss term and logit gradient
// (q - t)/n; the selector's ground truth G = [argmax z == argmax Y] (lowest index on ties), its
// confidence c = logistic(ws . [p ; q] + bs), the false-positive-weighted cross-entropy term and
// its gradient with respect to the score.
struct TrainRowArgs {
    float* z;              // [n][K] in: logits; out: dz = (q - t)/n
    float* q;              // [n][K] out: class probabilities
    const float* p; int ldp;   // [n][ldp] pooled features
    const int32_t* labels; // [n]
    const float* Y; int ldy;   // [n][ldy] base model's class distribution
    const float* ws;       // [C + K]
    const float* bs;       // device scalar
    int n, C, K;
    float alpha, fp_weight;
    // selector with a hidden layer: this kernel only prepares its input rows X = [p ; q] and the ground
    // truth, and train_selector_hidden_kernel does the rest (X null: the linear selector, finished here)
    float* X; int ldx;     // [n][ldx]
    float* G;              // [n] 1.0 where argmax z == argmax Y
    float* du;             // [n] d(selector loss)/d(score)
    float* lp;             // [n] predictor loss term (not yet divided by n)
    float* ls;             // [n] selector loss term
};

__device__ __forceinline__ void wave_argmax(float& v, int& i) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const float ov = __shfl_xor(v, m, 64);
        const int oi = __shfl_xor(i, m, 64);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
}

// log(1 + exp(x)) without overflow.
__device__ __forceinline__ float softplus(float x) { return fmaxf(x, 0.0f) + log1pf(expf(-fabsf(x))); }

// NK > 0: the row's logits and teacher probabilities stay in registers (K <= 64*NK), so global
// memory is read once; NK == 0: any K, the row is re-read from memory in each pass.
template <int NK>
__global__ __launch_bounds__(256) void train_row_kernel(TrainRowArgs a) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.n) return;
    float* z = a.z + (size_t)row * a.K;
    float* q = a.q + (size_t)row * a.K;
    const float* Y = a.Y + (size_t)row * a.ldy;
    const float* p = a.p + (size_t)row * a.ldp;
    constexpr int R = NK > 0 ? NK : 1;
    float zr[R], yr[R];
    const int chunks = NK > 0 ? NK : (a.K + 63) / 64;

    if constexpr (NK > 0) {
#pragma unroll
        for (int j = 0; j < NK; ++j) {
            const int k = lane + 64 * j;
            zr[j] = k < a.K ? z[k] : -INFINITY;
            yr[j] = k < a.K ? Y[k] : -INFINITY;
        }
    }
    // the selector's feature half does not depend on the softmax: issue its loads early
    float u = 0.0f;
    const bool hidden = a.X != nullptr;                      // uniform
    const bool nosel = !hidden && a.ws == nullptr;           // uniform: no selector network to train
    float* x = hidden ? a.X + (size_t)row * a.ldx : nullptr;
    if (hidden) for (int c = lane; c < a.C; c += 64) x[c] = p[c];
    else if (!nosel) for (int c = lane; c < a.C; c += 64) u += a.ws[c] * p[c];

    float zm = -INFINITY, ym = -INFINITY;
    int zi = 0x7fffffff, yi = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < chunks; ++j) {
        const int k = lane + 64 * j;
        if (k < a.K) {
            const float zv = NK > 0 ? zr[NK > 0 ? j : 0] : z[k], yv = NK > 0 ? yr[NK > 0 ? j : 0] : Y[k];
            if (zv > zm) { zm = zv; zi = k; }
            if (yv > ym) { ym = yv; yi = k; }
        }
    }
    wave_argmax(zm, zi);
    wave_argmax(ym, yi);

    float se = 0.0f;
#pragma unroll
    for (int j = 0; j < chunks; ++j) {
        const int k = lane + 64 * j;
        if (k < a.K) se += expf((NK > 0 ? zr[NK > 0 ? j : 0] : z[k]) - zm);
    }
    se = wave_sum(se);
    const float log_se = logf(se), inv_se = 1.0f / se, inv_n = 1.0f / (float)a.n;

    const int label = a.labels[row];
    float lp = 0.0f;
#pragma unroll
    for (int j = 0; j < chunks; ++j) {
        const int k = lane + 64 * j;
        if (k < a.K) {
            const float zc = (NK > 0 ? zr[NK > 0 ? j : 0] : z[k]) - zm;
            const float yv = NK > 0 ? yr[NK > 0 ? j : 0] : Y[k];
            const float qk = expf(zc) * inv_se;
            const float tk = a.alpha * yv + (k == label ? 1.0f - a.alpha : 0.0f);
            lp -= tk * (zc - log_se);
            if (hidden) x[a.C + k] = qk;
            else if (!nosel) u += a.ws[a.C + k] * qk;
            q[k] = qk;
            z[k] = (qk - tk) * inv_n;
        }
    }
    lp = wave_sum(lp);
    if (hidden) {
        if (lane == 0) { a.lp[row] = lp; a.G[row] = zi == yi ? 1.0f : 0.0f; }
        return;
    }
    if (nosel) {
        if (lane == 0) { a.du[row] = 0.0f; a.lp[row] = lp; a.ls[row] = 0.0f; }
        return;
    }
    u = wave_sum(u) + *a.bs;
    if (lane == 0) {
        const float conf = 1.0f / (1.0f + expf(-u));
        const float G = zi == yi ? 1.0f : 0.0f;
        a.du[row] = (G * (conf - 1.0f) + a.fp_weight * (1.0f - G) * conf) * inv_n;
        a.lp[row] = lp;
        a.ls[row] = G * softplus(-u) + a.fp_weight * (1.0f - G) * softplus(u);
    }
}

// Selector with a hidden layer (Section 3, "Selector Network Design"), one wave per sample: from the
// hidden vector g = relu(Ws [p ; q] + cs) (a product kernel wrote it) the score u = vs . g + bs, the
// confidence, the weighted cross-entropy term, its gradient du with respect to u, and the gradient
// with respect to the hidden pre-activations, dg_j = du vs_j [g_j > 0].
struct TrainSelHiddenArgs {
    const float* g;        // [n][Hs]
    float* dg;             // [n][Hs] out
    const float* vs;       // [Hs]
    const float* bs;       // device scalar
    const float* G;        // [n]
    int n, Hs;
    float fp_weight;
    float* du;             // [n]
    float* ls;             // [n]
};

__global__ __launch_bounds__(256) void train_selector_hidden_kernel(TrainSelHiddenArgs a) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.n) return;
    const float* g = a.g + (size_t)row * a.Hs;
    float u = 0.0f;
    for (int j = lane; j < a.Hs; j += 64) u += a.vs[j] * g[j];
    u = wave_sum(u) + *a.bs;
    const float conf = 1.0f / (1.0f + expf(-u));
    const float G = a.G[row];
    const float du = (G * (conf - 1.0f) + a.fp_weight * (1.0f - G) * conf) / (float)a.n;
    float* dg = a.dg + (size_t)row * a.Hs;
    for (int j = lane; j < a.Hs; j += 64) dg[j] = g[j] > 0.0f ? du * a.vs[j] : 0.0f;
    if (lane == 0) {
        a.du[row] = du;
        a.ls[row] = G * softplus(-u) + a.fp_weight * (1.0f - G) * softplus(u);
    }
}

// out[c] -= lr * sum_i scale_i X[i][c] (scale null: 1): the two bias gradients and the two halves
// of the selector's weight gradient, all in one launch.  A workgroup of 16 waves owns 64 columns of
// one job; rows are dealt round-robin to the waves, four independent partial sums per thread, and
// the partials are added in a fixed order.
struct ColsumJob {
    const float* X; int ld; int cols;
    const float* scale;
    float* out;
    int first_block;     // this job's first workgroup in the launch
    int rows;            // rows of X to add up
};
struct ColsumArgs { ColsumJob job[4]; float lr; };

__global__ __launch_bounds__(1024) void train_colsums_kernel(ColsumArgs a) {
    __shared__ float part[16][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int j = 0;
#pragma unroll
    for (int t = 1; t < 4; ++t)
        if ((int)blockIdx.x >= a.job[t].first_block) j = t;
    const ColsumJob job = a.job[j];
    const int c = (blockIdx.x - job.first_block) * 64 + lane;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (c < job.cols) {
        for (int i0 = w; i0 < job.rows; i0 += 64) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = i0 + 16 * r;
                if (i < job.rows) acc[r] += (job.scale ? job.scale[i] : 1.0f) * job.X[(size_t)i * job.ld + c];
            }
        }
    }
    part[w][lane] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    __syncthreads();
    if (w == 0 && c < job.cols) {
        float s = 0.0f;
#pragma unroll
        for (int t = 0; t < 16; ++t) s += part[t][lane];
        job.out[c] -= a.lr * s;
    }
}

// Conv(k,s) predictor as a matrix product: row (i, oy, ox) of Xc holds the C*k*k input values under
// that output position, in (channel, dy, dx) order -- the order of a filter's weights -- so the
// convolution is Xc W1^T and its weight gradient dh^T Xc.  One lane per element, consecutive lanes
// along a row of Xc.
struct Im2colArgs {
    const float* x; int ldx;     // [n][ldx] maps, channel-major: x[i][c*ih*iw + y*iw + xx]
    float* Xc;                   // [n*oh*ow][C*k*k]
    int n, C, ih, iw, k, s, oh, ow;
};

__global__ __launch_bounds__(256) void train_im2col_kernel(Im2colArgs a) {
    const int kk = a.k * a.k, Cin = a.C * kk, P = a.oh * a.ow;
    const long total = (long)a.n * P * Cin;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const long rowp = idx / Cin;
        const int col = (int)(idx - rowp * Cin);
        const int i = (int)(rowp / P), pix = (int)(rowp - (long)i * P);
        const int c = col / kk, tap = col - c * kk;
        const int dy = tap / a.k, dx = tap - dy * a.k;
        const int oy = pix / a.ow, ox = pix - oy * a.ow;
        a.Xc[idx] = a.x[(size_t)i * a.ldx + (size_t)c * a.ih * a.iw + (size_t)(oy * a.s + dy) * a.iw + ox * a.s + dx];
    }
}

// bs -= lr * sum du; losses = (sum lp / n, sum ls / n).  One workgroup.
__global__ __launch_bounds__(256) void train_scalar_kernel(const float* __restrict__ du, const float* __restrict__ lp,
                                                           const float* __restrict__ ls, int n, float lr, float* bs,
                                                           float* losses) {
    __shared__ float part[3][4];
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f;
    for (int i = threadIdx.x; i < n; i += 256) { s0 += du[i]; s1 += lp[i]; s2 += ls[i]; }
    s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2);
    if ((threadIdx.x & 63) == 0) { part[0][threadIdx.x >> 6] = s0; part[1][threadIdx.x >> 6] = s1; part[2][threadIdx.x >> 6] = s2; }
    __syncthreads();
    if (threadIdx.x == 0) {
        *bs -= lr * ((part[0][0] + part[0][1]) + (part[0][2] + part[0][3]));
        if (losses) {
            losses[0] = ((part[1][0] + part[1][1]) + (part[1][2] + part[1][3])) / (float)n;
            losses[1] = ((part[2][0] + part[2][1]) + (part[2][2] + part[2][3])) / (float)n;
        }
    }
}

}  // namespace gati
