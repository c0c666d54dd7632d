// The predictor's two FC layers, the class distribution and the selector (paper, Section 3:
// predictor Input -> Hidden(h), ReLU -> Output; selector: a projection of the predictor's
// output onto a binary decision).
//
// Both FC layers are real dense contractions (rows x C x H and rows x H x K), so they run
// on the matrix cores: v_mfma_f32_32x32x16_bf16 for bf16 caches, v_mfma_f32_32x32x2_f32 for
// fp32 caches, fp32 accumulation in both.  A and B operands are both contiguous along the
// reduction axis ([rows, C] x [H, C]^T), which is exactly the per-lane fragment the 32x32
// MFMA wants (8 consecutive k for one row / column), so fragments are loaded straight from
// global memory / L2 with 16-byte loads; the matrices are a few MB and stay cache resident.
//
// Fragment layout used here (wave of 64 lanes, r = lane % 32, kb = lane / 32):
//   A: lane holds A[m = r][k = 8*kb .. 8*kb+7]      (bf16; f32: one k per MFMA)
//   B: lane holds B[k = 8*kb .. 8*kb+7][n = r]
//   D: acc[j] is D[m = 8*(j/4) + 4*kb + j%4][n = r]
#pragma once

#include "common.h"

namespace gati {

__device__ __forceinline__ int mfma_row(int j, int kb) { return 8 * (j >> 2) + 4 * kb + (j & 3); }

// One 32x32 tile step over 16 (bf16) or 8 (f32) values of the reduction axis.
template <bool BF16> struct MmaStep;

template <> struct MmaStep<true> {
    static constexpr int kStep = 16;     // reduction elements consumed per call
    static constexpr int kLane = 8;      // consecutive k held by one lane
    // A from fp32 memory (rounded to bf16, nearest even), B from bf16 memory.
    static __device__ __forceinline__ bf16x8_t load_a_f32(const float* p) {
        const float4 x = *reinterpret_cast<const float4*>(p);
        const float4 y = *reinterpret_cast<const float4*>(p + 4);
        bf16x8_t a;
        a[0] = (__bf16)x.x; a[1] = (__bf16)x.y; a[2] = (__bf16)x.z; a[3] = (__bf16)x.w;
        a[4] = (__bf16)y.x; a[5] = (__bf16)y.y; a[6] = (__bf16)y.z; a[7] = (__bf16)y.w;
        return a;
    }
    static __device__ __forceinline__ bf16x8_t load_bf16(const void* p) {
        return *reinterpret_cast<const bf16x8_t*>(p);
    }
    static __device__ __forceinline__ f32x16_t mma(bf16x8_t a, bf16x8_t b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

template <> struct MmaStep<false> {
    static constexpr int kStep = 8;
    static constexpr int kLane = 4;
    // Lane (r, kb) holds k = 4*kb .. 4*kb+3; MFMA number j multiplies element j of every
    // lane, i.e. k = j and k = 4 + j.  A and B use the same order, so the sum over the 8 k
    // values is complete after 4 MFMAs.
    static __device__ __forceinline__ f32x16_t mma(const float4& a, const float4& b, f32x16_t c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, c, 0, 0, 0);
        return c;
    }
};

struct Fc1Args {
    const float* p;        // [rows_pad, Cp] pooled features, fp32, zero in the padding columns
    const void* W1;        // [Hp, Cp] bf16 or f32, zero padded
    const float* b1;       // [Hp]
    void* h;               // [rows_pad, Hp] bf16 or f32
    const float* ws_pool;  // [Cp] selector weights of the pooled features, zero padded
    float* u_pool;         // [rows_pad] out: ws_pool . p[row]
    int Cp, Hp;
    int n_max;
    const int32_t* n_dev;
};

// grid = (Hp/32 + 1, rows_pad/32), block = one wave.  Column tile Hp/32 is not a tile of the
// hidden layer: that wave computes the pooled-feature half of the selector's dot product in
// fp32 for the 32 rows, so it overlaps with the MFMA tiles instead of serialising later.
template <bool BF16>
__global__ __launch_bounds__(64) void fc1_kernel(Fc1Args a) {
    using Step = MmaStep<BF16>;
    const int n = active_rows(a.n_dev, a.n_max);
    const int row0 = blockIdx.y * 32;
    if (row0 >= n) return;
    const int lane = threadIdx.x;
    const int ct = blockIdx.x;

    if (ct == a.Hp / 32) {
        const float4* wv = reinterpret_cast<const float4*>(a.ws_pool);
        const int nvec = a.Cp / 4;
        for (int rr = 0; rr < 32 && row0 + rr < n; ++rr) {
            const float4* pr = reinterpret_cast<const float4*>(a.p + (long)(row0 + rr) * a.Cp);
            float acc = 0.f;
            for (int k = lane; k < nvec; k += 64) {
                const float4 x = pr[k], w = wv[k];
                acc = fmaf(x.x, w.x, acc); acc = fmaf(x.y, w.y, acc);
                acc = fmaf(x.z, w.z, acc); acc = fmaf(x.w, w.w, acc);
            }
            acc = wave_sum(acc);
            if (lane == 0) a.u_pool[row0 + rr] = acc;
        }
        return;
    }

    const int r = lane & 31, kb = lane >> 5;
    f32x16_t acc;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.f;
    const float* arow = a.p + (long)(row0 + r) * a.Cp + kb * Step::kLane;

    if constexpr (BF16) {
        const __bf16* brow = static_cast<const __bf16*>(a.W1) + (long)(ct * 32 + r) * a.Cp + kb * 8;
        for (int k0 = 0; k0 < a.Cp; k0 += 64) {   // Cp is a multiple of 64
            bf16x8_t af[4], bf[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                af[u] = Step::load_a_f32(arow + k0 + 16 * u);
                bf[u] = Step::load_bf16(brow + k0 + 16 * u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = Step::mma(af[u], bf[u], acc);
        }
    } else {
        const float* brow = static_cast<const float*>(a.W1) + (long)(ct * 32 + r) * a.Cp + kb * 4;
        for (int k0 = 0; k0 < a.Cp; k0 += 32) {
            float4 af[4], bf[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                af[u] = *reinterpret_cast<const float4*>(arow + k0 + 8 * u);
                bf[u] = *reinterpret_cast<const float4*>(brow + k0 + 8 * u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = Step::mma(af[u], bf[u], acc);
        }
    }

    const int col = ct * 32 + r;
    const float bias = a.b1[col];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int row = row0 + mfma_row(j, kb);
        const float v = fmaxf(acc[j] + bias, 0.f);
        if constexpr (BF16)
            static_cast<__bf16*>(a.h)[(long)row * a.Hp + col] = (__bf16)v;
        else
            static_cast<float*>(a.h)[(long)row * a.Hp + col] = v;
    }
}

struct Fc2Args {
    const void* h;        // [rows_pad, Hp] bf16 or f32
    const void* W2;       // [Kp, Hp] bf16 or f32, zero padded
    const float* b2;      // [Kp]
    const float* ws_prob; // [Kp] selector weights of the class probabilities, zero padded
    const float* u_pool;  // [rows_pad]
    float bs, tau;
    int Hp, K, Kp;
    int n_max;
    const int32_t* n_dev;
    int32_t* pred_class;
    float* confidence;
    uint8_t* hit;
    float* logits;        // [n, K] or null
};

// One workgroup of NW waves owns 32 rows.  Per pass it forms NW*TPW*32 logits per row in
// registers (TPW 32x32 tiles per wave), then reduces them to the row's running maximum,
// argmax, sum of exponentials and probability-weighted selector sum; wider class counts
// take several passes with the usual rescaling by exp(old max - new max).  Finally
// confidence = logistic(bs + u_pool + sum_k ws[k] prob[k]) and hit = confidence > tau.
template <bool BF16, int TPW>
__global__ __launch_bounds__(256) void fc2_head_kernel(Fc2Args a) {
    using Step = MmaStep<BF16>;
    constexpr int kPartials = 4 * 32;               // partial columns per row at most (4 waves)
    __shared__ float s_f[32][kPartials + 1];
    __shared__ float s_g[32][kPartials + 1];        // second float plane (reinterpreted as int for argmax)
    __shared__ float row_max[32], row_sum[32], row_wsum[32];
    __shared__ int row_arg[32];

    const int n = active_rows(a.n_dev, a.n_max);
    const int row0 = blockIdx.x * 32;
    if (row0 >= n) return;
    const int tid = threadIdx.x;
    const int nw = blockDim.x >> 6;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, kb = lane >> 5;
    const int tpr = blockDim.x >> 5;                // lanes that share one row in the reductions
    const int red_row = tid / tpr, red_sub = tid - red_row * tpr;
    const int npart = nw * 32;

    if (tid < 32) { row_max[tid] = -INFINITY; row_sum[tid] = 0.f; row_wsum[tid] = 0.f; row_arg[tid] = 0; }
    __syncthreads();

    const int chunk_cols = nw * TPW * 32;
    for (int chunk0 = 0; chunk0 < a.Kp; chunk0 += chunk_cols) {
        const int colbase = chunk0 + wave * TPW * 32;
        f32x16_t acc[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[t][j] = 0.f;

        if constexpr (BF16) {
            const __bf16* arow = static_cast<const __bf16*>(a.h) + (long)(row0 + r) * a.Hp + kb * 8;
            const __bf16* bbase = static_cast<const __bf16*>(a.W2) + (long)(colbase + r) * a.Hp + kb * 8;
            for (int k0 = 0; k0 < a.Hp; k0 += 32) {   // Hp is a multiple of 32
                const bf16x8_t a0 = Step::load_bf16(arow + k0);
                const bf16x8_t a1 = Step::load_bf16(arow + k0 + 16);
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    if (colbase + t * 32 < a.Kp) {     // wave-uniform
                        const __bf16* bp = bbase + (long)t * 32 * a.Hp + k0;
                        const bf16x8_t b0 = Step::load_bf16(bp);
                        const bf16x8_t b1 = Step::load_bf16(bp + 16);
                        acc[t] = Step::mma(a0, b0, acc[t]);
                        acc[t] = Step::mma(a1, b1, acc[t]);
                    }
                }
            }
        } else {
            const float* arow = static_cast<const float*>(a.h) + (long)(row0 + r) * a.Hp + kb * 4;
            const float* bbase = static_cast<const float*>(a.W2) + (long)(colbase + r) * a.Hp + kb * 4;
            for (int k0 = 0; k0 < a.Hp; k0 += 16) {
                const float4 a0 = *reinterpret_cast<const float4*>(arow + k0);
                const float4 a1 = *reinterpret_cast<const float4*>(arow + k0 + 8);
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    if (colbase + t * 32 < a.Kp) {
                        const float* bp = bbase + (long)t * 32 * a.Hp + k0;
                        const float4 b0 = *reinterpret_cast<const float4*>(bp);
                        const float4 b1 = *reinterpret_cast<const float4*>(bp + 8);
                        acc[t] = Step::mma(a0, b0, acc[t]);
                        acc[t] = Step::mma(a1, b1, acc[t]);
                    }
                }
            }
        }

        // logits of this pass: bias, optional store, mask of the padding classes
        float wsq[TPW];
        bool valid[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int col = colbase + t * 32 + r;
            valid[t] = col < a.K;
            const float bias = valid[t] ? a.b2[col] : 0.f;
            wsq[t] = valid[t] ? a.ws_prob[col] : 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float z = acc[t][j] + bias;
                acc[t][j] = valid[t] ? z : -INFINITY;
                const int row = row0 + mfma_row(j, kb);
                if (a.logits && valid[t] && row < n) a.logits[(long)row * a.K + col] = z;
            }
        }

        // (1) row maximum and argmax (lowest index among equals)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float pm = -INFINITY;
            int pi = 0x7fffffff;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const float v = acc[t][j];
                if (v > pm) { pm = v; pi = colbase + t * 32 + r; }
            }
            const int lr = mfma_row(j, kb);
            s_f[lr][wave * 32 + r] = pm;
            s_g[lr][wave * 32 + r] = __int_as_float(pi);
        }
        __syncthreads();
        {
            float bm = -INFINITY;
            int bi = 0x7fffffff;
            for (int c = red_sub; c < npart; c += tpr) {
                const float v = s_f[red_row][c];
                const int i = __float_as_int(s_g[red_row][c]);
                if (v > bm || (v == bm && i < bi)) { bm = v; bi = i; }
            }
            for (int m = tpr >> 1; m >= 1; m >>= 1) {
                const float ov = __shfl_xor(bm, m, 64);
                const int oi = __shfl_xor(bi, m, 64);
                if (ov > bm || (ov == bm && oi < bi)) { bm = ov; bi = oi; }
            }
            if (red_sub == 0) {
                const float old = row_max[red_row];
                if (bm > old) {                      // an earlier pass keeps the class on equality
                    const float scale = expf(old - bm);   // old = -inf -> 0
                    row_sum[red_row] *= scale;
                    row_wsum[red_row] *= scale;
                    row_max[red_row] = bm;
                    row_arg[red_row] = bi;
                }
            }
        }
        __syncthreads();

        // (2) sum of exponentials and selector-weighted sum, relative to the running maximum
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int lr = mfma_row(j, kb);
            const float m = row_max[lr];
            float ps = 0.f, pt = 0.f;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if (valid[t]) {
                    const float e = expf(acc[t][j] - m);
                    ps += e;
                    pt = fmaf(e, wsq[t], pt);
                }
            }
            s_f[lr][wave * 32 + r] = ps;
            s_g[lr][wave * 32 + r] = pt;
        }
        __syncthreads();
        {
            float ss = 0.f, st = 0.f;
            for (int c = red_sub; c < npart; c += tpr) { ss += s_f[red_row][c]; st += s_g[red_row][c]; }
            for (int m = tpr >> 1; m >= 1; m >>= 1) {
                ss += __shfl_xor(ss, m, 64);
                st += __shfl_xor(st, m, 64);
            }
            if (red_sub == 0) { row_sum[red_row] += ss; row_wsum[red_row] += st; }
        }
        __syncthreads();
    }

    if (red_sub == 0) {
        const int row = row0 + red_row;
        if (row < n) {
            const float u = a.bs + a.u_pool[row] + row_wsum[red_row] / row_sum[red_row];
            const float conf = 1.f / (1.f + expf(-u));
            a.pred_class[row] = row_arg[red_row];
            a.confidence[row] = conf;
            a.hit[row] = conf > a.tau ? 1 : 0;
        }
    }
}

}  // namespace gati
