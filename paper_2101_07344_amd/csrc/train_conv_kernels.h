// First layer of the Conv(k,s) predictor (Section 3, table of predictor architectures) inside the
// retraining step (Section 5, "Retraining Learned Caches"), computed on the activation maps
// themselves: forward h = relu(conv(x, W1) + b1), the filter gradient
// dW1[o][c][dy][dx] = sum over samples and positions of dh[i][p][o] * x[i][c][s*y+dy][s*x+dx]
// and the bias gradient db1[o] = sum of dh[i][p][o], for up to 8 filters of 3 x 3 or 5 x 5 taps.
// The product over gathered windows (train_kernels.h) needs a window matrix k*k/s*s times the size
// of the activation and a 64-wide product tile for 8 filters; here every map is read once per
// kernel and all arithmetic is fp32 FMA on the vector units (k*k*8 FMAs per value read from LDS).
//
// Work layout shared by both kernels: a workgroup is 4 waves; `wpc` (1, 2 or 4) waves share a
// channel, so a workgroup step covers cw = 4 / wpc channels; the lanes of a channel's waves are
// dealt the output positions.  Maps (and, in the gradient kernel, the hidden gradients) are staged
// through LDS in passes, with 16-byte loads that are issued one pass ahead where the caller's rows
// allow it (`vec`), element by element otherwise; the filter values of a wave's channel are the
// same for all its lanes and come through the scalar cache.  Every sum has a fixed order.
// gfx950, 64-wide waves.
#pragma once

#include "common.h"

namespace gati {

constexpr int kConvTrainXFloats = 4096;    // forward: activation values staged per pass
constexpr int kConvTrainRedFloats = 2048;  // forward: with the staged values, room for the sums of 3 positions per lane (256*3*8)
constexpr int kConvTrainGXFloats = 6272;   // filter gradient: activation values staged per pass (two 56 x 56 maps)
constexpr int kConvTrainDFloats = 5632;    // filter gradient: hidden gradients staged per pass, [sample][position][8]
constexpr int kConvTrainMaxP = 704;        // output positions per map the kernels take
constexpr int kConvTrainFilters = 8;
constexpr int kConvTrainGradLds = (kConvTrainGXFloats + kConvTrainDFloats + kConvTrainMaxP) * 4;

struct ConvTrainArgs {
    const float* x; int ldx;          // [n][ldx] maps, channel-major: x[i][c*ih*iw + y*iw + xx]
    int n, C, ih, iw, s, oh, ow, H;   // H filters (<= 8)
    float* W1;                        // [H][C*k*k]
    float* W1t;                       // [C][k*k][8]: the filters as the forward pass reads them, zero past H
    float* b1;                        // [H]
    float* h;                         // forward out: [n][oh*ow][H]
    const float* dh;                  // gradient in: [n][oh*ow][H], zero where h is zero
    float* part;                      // filter gradient partial sums [splits][C][8][k*k]; forward: [csplit][n][oh*ow][8]
    float* bpart;                     // bias gradient partial sums [splits][8]
    int wpc;                          // waves per channel
    int sg;                           // forward: samples per workgroup (> 1 only when several fit one wave)
    int cpw;                          // forward: channels per wave and pass
    int csplit;                       // forward: workgroups that share a sample group's channels
    int ns;                           // gradient: samples per pass
    int rows_per_split;               // gradient: samples per workgroup (a multiple of ns)
    int splits;
    int vec;                          // 16-byte staging loads: rows, runs and (gradient) H == 8 allow them
    float lr;
};

// W1t[c][tap][o] = W1[o][c][tap], zero for o >= H.  One thread per value of W1t.
__global__ __launch_bounds__(256) void train_conv_pack_kernel(ConvTrainArgs a, int kk2) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.C * kk2 * 8) return;
    const int o = idx & 7, ct = idx >> 3;
    a.W1t[idx] = o < a.H ? a.W1[(size_t)o * a.C * kk2 + ct] : 0.0f;
}

// Four consecutive values at offset r (a multiple of 4) of a run of which the first `rem` (a multiple of 4)
// exist; zeros past them.  Branch-free: the load is redirected to the run's start.
__device__ __forceinline__ f32x4_t conv_train_load4(const float* __restrict__ p, int r, int rem) {
    const bool in = r < rem;
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(p + (in ? r : 0));
    const f32x4_t z = {0.0f, 0.0f, 0.0f, 0.0f};
    return in ? v : z;
}

// grid = (ceil(n / sg), csplit), block = 256.  PP: output positions (of the workgroup's sg samples) per lane.
// With csplit > 1 the channels are shared out over gridDim.y workgroups, which leave their raw sums in
// part[split][n][oh*ow][8] for train_conv_finish_kernel.
// The next pass's loads are issued before the present pass is multiplied and parked in LDS after it.
template <int KK, int PP>
__global__ __launch_bounds__(256) void train_conv_fwd_kernel(ConvTrainArgs a) {
    constexpr int KK2 = KK * KK;
    constexpr int XV = kConvTrainXFloats / 1024;     // 16-byte loads per lane and pass
    __shared__ __attribute__((aligned(16))) float lds[kConvTrainXFloats + kConvTrainRedFloats];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wpc = a.wpc, cw = 4 / wpc;
    const int ch = wave / wpc, wpos = wave - ch * wpc;
    const int S = a.ih * a.iw, P = a.oh * a.ow;
    const int cc = cw * a.cpw;                       // channels per pass
    const int i0 = blockIdx.x * a.sg;
    const int sgl = min(a.sg, a.n - i0);             // samples this workgroup has
    const int nl = 64 * wpc;                         // lanes per channel

    int xb[PP], out_i[PP], out_p[PP];
#pragma unroll
    for (int pp = 0; pp < PP; ++pp) {
        const int item = wpos * 64 + lane + pp * nl;
        int si = item / P, pix = item - si * P;
        out_i[pp] = si < sgl ? si : -1;
        out_p[pp] = pix;
        if (si >= sgl) { si = 0; pix = 0; }          // reads stay inside the staged maps, nothing is stored
        const int oy = pix / a.ow, ox = pix - oy * a.ow;
        xb[pp] = si * cc * S + oy * a.s * a.iw + ox * a.s;
    }
    float acc[PP][8];
#pragma unroll
    for (int pp = 0; pp < PP; ++pp)
#pragma unroll
        for (int o = 0; o < 8; ++o) acc[pp][o] = 0.0f;

    // a pass stages [sample][channel of the pass][S] activations, channels past the last one as zeros; the filter
    // values of a wave's channel are the same for all its lanes and come through the scalar cache
    const int run = cc * S;
    // vec: the 16-byte piece e4 = j*256 + tid of the staged activations is piece r4 of sample si's run
    int xcode[XV];
#pragma unroll
    for (int j = 0; j < XV; ++j) {
        const int e4 = j * 256 + tid, run4 = max(run >> 2, 1);
        const int si = e4 / run4;
        xcode[j] = (a.vec && si < sgl) ? ((si << 16) | (e4 - si * run4)) : -1;
    }
    f32x4_t xs[XV];
    auto prefetch = [&](int c0) {
        const float* xrow = a.x + (size_t)i0 * a.ldx + (size_t)c0 * S;
        const int xrem = (a.C - c0) * S;             // values left in a sample's run from channel c0 on
#pragma unroll
        for (int j = 0; j < XV; ++j)
            if (xcode[j] >= 0) xs[j] = conv_train_load4(xrow + (size_t)(xcode[j] >> 16) * a.ldx, (xcode[j] & 0xffff) * 4, xrem);
    };
    auto park = [&](int c0) {
        f32x4_t* l4 = reinterpret_cast<f32x4_t*>(lds);
#pragma unroll
        for (int j = 0; j < XV; ++j)
            if (xcode[j] >= 0) l4[j * 256 + tid] = xs[j];
        if (!a.vec) {
            const int xrem = (a.C - c0) * S;
            for (int si = 0; si < sgl; ++si) {
                const float* xrow = a.x + (size_t)(i0 + si) * a.ldx + (size_t)c0 * S;
#pragma unroll 8
                for (int r = tid; r < run; r += 256) lds[si * run + r] = r < xrem ? xrow[r] : 0.0f;
            }
        }
    };
    auto compute = [&](int c0) {
        for (int j = 0; j < a.cpw; ++j) {
            const int cl = ch * a.cpw + j;
            const float* xc = lds + cl * S;
            const f32x4_t* wc = reinterpret_cast<const f32x4_t*>(a.W1t + (size_t)min(c0 + cl, a.C - 1) * KK2 * 8);
#pragma unroll
            for (int dy = 0; dy < KK; ++dy) {
                const float* xr = xc + dy * a.iw;
#pragma unroll
                for (int dx = 0; dx < KK; ++dx) {
                    const f32x4_t w0 = wc[(dy * KK + dx) * 2], w1 = wc[(dy * KK + dx) * 2 + 1];
#pragma unroll
                    for (int pp = 0; pp < PP; ++pp) {
                        const float xv = xr[xb[pp] + dx];
#pragma unroll
                        for (int o = 0; o < 4; ++o) {
                            acc[pp][o] = fmaf(xv, w0[o], acc[pp][o]);
                            acc[pp][4 + o] = fmaf(xv, w1[o], acc[pp][4 + o]);
                        }
                    }
                }
            }
        }
    };

    // this workgroup's share of the channels: whole passes
    const int passes = (a.C + cc - 1) / cc, ppw = (passes + a.csplit - 1) / a.csplit;
    const int c_begin = blockIdx.y * ppw * cc, c_end = min(a.C, c_begin + ppw * cc);
    if (c_begin < c_end) prefetch(c_begin);
    for (int c0 = c_begin; c0 < c_end; c0 += cc) {
        park(c0);
        __syncthreads();
        if (c0 + cc < c_end) prefetch(c0 + cc);
        compute(c0);
        __syncthreads();
    }

    // sum over the channel lanes (fixed order), bias, ReLU
    float* red = lds;                                // [cw][nl*PP][8]; every read of the staged data is behind the barrier
#pragma unroll
    for (int pp = 0; pp < PP; ++pp) {
        const int item = wpos * 64 + lane + pp * nl;
        f32x4_t* dst = reinterpret_cast<f32x4_t*>(red + ((size_t)ch * nl * PP + item) * 8);
        dst[0] = f32x4_t{acc[pp][0], acc[pp][1], acc[pp][2], acc[pp][3]};
        dst[1] = f32x4_t{acc[pp][4], acc[pp][5], acc[pp][6], acc[pp][7]};
    }
    __syncthreads();
    if (ch == 0) {
#pragma unroll
        for (int pp = 0; pp < PP; ++pp) {
            if (out_i[pp] < 0) continue;
            const int item = wpos * 64 + lane + pp * nl;
            const size_t at = (size_t)(i0 + out_i[pp]) * P + out_p[pp];
            for (int o = 0; o < a.H; ++o) {
                float v = 0.0f;
                for (int c = 0; c < cw; ++c) v += red[((size_t)c * nl * PP + item) * 8 + o];
                if (a.csplit == 1) a.h[at * a.H + o] = fmaxf(v + a.b1[o], 0.0f);
                else a.part[((size_t)blockIdx.y * a.n * P + at) * 8 + o] = v;
            }
        }
    }
}

// h = relu(sum of the channel splits' sums, in split order, + b1).  One thread per hidden value.
__global__ __launch_bounds__(256) void train_conv_finish_kernel(ConvTrainArgs a) {
    const size_t np = (size_t)a.n * a.oh * a.ow;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= np * a.H) return;
    const size_t at = idx / a.H;
    const int o = (int)(idx - at * a.H);
    float v = 0.0f;
    for (int sp = 0; sp < a.csplit; ++sp) v += a.part[((size_t)sp * np + at) * 8 + o];
    a.h[idx] = fmaxf(v + a.b1[o], 0.0f);
}

// grid = (ceil(C / cw), splits), block = 256, dynamic LDS kConvTrainGradLds.  FS: a position's 8 filters are
// split over FS neighbouring lanes (the 5 x 5 filter would otherwise need 200 accumulators per lane).
template <int KK, int FS>
__global__ __launch_bounds__(256) void train_conv_wgrad_kernel(ConvTrainArgs a) {
    constexpr int KK2 = KK * KK, OF = 8 / FS;
    constexpr int XV = (kConvTrainGXFloats + 1023) / 1024, DV = (kConvTrainDFloats + 1023) / 1024;
    extern __shared__ __attribute__((aligned(16))) float dyn[];
    float* const dl = dyn + kConvTrainGXFloats;                                   // staged hidden gradients
    int* offs = reinterpret_cast<int*>(dyn + kConvTrainGXFloats + kConvTrainDFloats);   // position -> offset of its window's corner
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wpc = a.wpc, cw = 4 / wpc;
    const int ch = wave / wpc, wpos = wave - ch * wpc;
    const int S = a.ih * a.iw, P = a.oh * a.ow;
    const int c0 = blockIdx.x * cw;
    const int split = blockIdx.y;
    const int s_begin = split * a.rows_per_split, s_end = min(a.n, s_begin + a.rows_per_split);
    const int fs = lane & (FS - 1), pl = (wpos * 64 + lane) / FS, npl = 64 * wpc / FS;

    for (int pix = tid; pix < P; pix += 256) {
        const int oy = pix / a.ow, ox = pix - oy * a.ow;
        offs[pix] = oy * a.s * a.iw + ox * a.s;
    }
    const int si_first = pl / P, pix_first = pl - si_first * P;

    float acc[KK2][OF], bsum[OF];
#pragma unroll
    for (int o = 0; o < OF; ++o) bsum[o] = 0.0f;
#pragma unroll
    for (int t = 0; t < KK2; ++t)
#pragma unroll
        for (int o = 0; o < OF; ++o) acc[t][o] = 0.0f;

    // a pass stages [sample][channel of the workgroup][S] activations and [sample][position][8] hidden gradients
    const int run = cw * S;
    const int xrem = (a.C - c0) * S;
    int xcode[XV];
#pragma unroll
    for (int j = 0; j < XV; ++j) {
        const int e4 = j * 256 + tid, run4 = max(run >> 2, 1);
        const int si = e4 / run4;
        xcode[j] = (a.vec && si < a.ns) ? ((si << 16) | (e4 - si * run4)) : -1;
    }
    // vec: the next pass's loads are issued before the present pass is multiplied and parked in LDS after it
    f32x4_t xs[XV], dv[DV];
    auto prefetch = [&](int sp, int nsl) {
        if (!a.vec) return;
        const float* xrow = a.x + (size_t)sp * a.ldx + (size_t)c0 * S;
#pragma unroll
        for (int j = 0; j < XV; ++j)
            if (xcode[j] >= 0 && (xcode[j] >> 16) < nsl)
                xs[j] = conv_train_load4(xrow + (size_t)(xcode[j] >> 16) * a.ldx, (xcode[j] & 0xffff) * 4, xrem);
        const f32x4_t* drow = reinterpret_cast<const f32x4_t*>(a.dh + (size_t)sp * P * 8);
        const int d4 = nsl * P * 2;
#pragma unroll
        for (int j = 0; j < DV; ++j)
            if (j * 256 + tid < d4) dv[j] = drow[j * 256 + tid];
    };
    auto park = [&](int sp, int nsl) {
        if (a.vec) {
            f32x4_t* x4 = reinterpret_cast<f32x4_t*>(dyn);
            f32x4_t* d4l = reinterpret_cast<f32x4_t*>(dl);
            const int d4 = nsl * P * 2;
#pragma unroll
            for (int j = 0; j < XV; ++j)
                if (xcode[j] >= 0 && (xcode[j] >> 16) < nsl) x4[j * 256 + tid] = xs[j];
#pragma unroll
            for (int j = 0; j < DV; ++j)
                if (j * 256 + tid < d4) d4l[j * 256 + tid] = dv[j];
        } else {
            for (int si = 0; si < nsl; ++si) {
                const float* xrow = a.x + (size_t)(sp + si) * a.ldx + (size_t)c0 * S;
#pragma unroll 8
                for (int r = tid; r < run; r += 256) dyn[si * run + r] = r < xrem ? xrow[r] : 0.0f;
            }
            const float* drow = a.dh + (size_t)sp * P * a.H;
            const int dfl = nsl * P * 8;
#pragma unroll 8
            for (int e = tid; e < dfl; e += 256) {
                const int o = e & 7;
                dl[e] = o < a.H ? drow[(size_t)(e >> 3) * a.H + o] : 0.0f;
            }
        }
    };
    auto compute = [&](int items) {
        int si = si_first, pix = pix_first;
        for (int it = pl; it < items; it += npl) {
            const float* xr = dyn + (si * cw + ch) * S + offs[pix];
            float d[OF];
            const f32x4_t* dp = reinterpret_cast<const f32x4_t*>(dl + (size_t)it * 8 + fs * OF);
#pragma unroll
            for (int q = 0; q < OF / 4; ++q) {
                const f32x4_t v = dp[q];
                d[4 * q] = v[0]; d[4 * q + 1] = v[1]; d[4 * q + 2] = v[2]; d[4 * q + 3] = v[3];
            }
#pragma unroll
            for (int o = 0; o < OF; ++o) bsum[o] += d[o];
#pragma unroll
            for (int dy = 0; dy < KK; ++dy)
#pragma unroll
                for (int dx = 0; dx < KK; ++dx) {
                    const float xv = xr[dy * a.iw + dx];
#pragma unroll
                    for (int o = 0; o < OF; ++o) acc[dy * KK + dx][o] = fmaf(xv, d[o], acc[dy * KK + dx][o]);
                }
            pix += npl;
            while (pix >= P) { pix -= P; ++si; }
        }
    };

    if (s_begin < s_end) prefetch(s_begin, min(a.ns, s_end - s_begin));
    for (int sp = s_begin; sp < s_end; sp += a.ns) {
        const int nsl = min(a.ns, s_end - sp);
        park(sp, nsl);
        __syncthreads();                              // the first one also publishes the position table
        if (sp + a.ns < s_end) prefetch(sp + a.ns, min(a.ns, s_end - sp - a.ns));
        compute(nsl * P);
        __syncthreads();
    }
    __syncthreads();                                  // a workgroup without samples: the table's writes before `red`

    // lanes of a wave that hold the same filters (butterfly, fixed order), then the waves of a channel
    float* red = dyn;                                 // [wave][tap][8], then [wave][8] for the bias
    float* bred = dyn + 4 * KK2 * 8;
#pragma unroll
    for (int t = 0; t < KK2; ++t)
#pragma unroll
        for (int o = 0; o < OF; ++o) {
            float v = acc[t][o];
#pragma unroll
            for (int m = FS; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
            if (lane < FS) red[(wave * KK2 + t) * 8 + fs * OF + o] = v;
        }
#pragma unroll
    for (int o = 0; o < OF; ++o) {
        float v = bsum[o];
#pragma unroll
        for (int m = FS; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
        if (lane < FS) bred[wave * 8 + fs * OF + o] = v;
    }
    __syncthreads();
    for (int e = tid; e < cw * KK2 * 8; e += 256) {
        const int chh = e / (KK2 * 8), r = e - chh * KK2 * 8, t = r >> 3, o = r & 7;
        const int c = c0 + chh;
        if (c >= a.C) continue;
        float v = 0.0f;
        for (int wp = 0; wp < wpc; ++wp) v += red[((chh * wpc + wp) * KK2 + t) * 8 + o];
        a.part[(((size_t)split * a.C + c) * 8 + o) * KK2 + t] = v;
    }
    // every channel's lanes see every position once: the workgroup of channel 0 adds up the bias gradient
    if (blockIdx.x == 0 && tid < 8) {
        float v = 0.0f;
        for (int wp = 0; wp < wpc; ++wp) v += bred[wp * 8 + tid];
        a.bpart[split * 8 + tid] = v;
    }
}

// W1 -= lr * (sum of the split partial gradients, in split order), b1 likewise.  One thread per filter value.
__global__ __launch_bounds__(256) void train_conv_update_kernel(ConvTrainArgs a, int kk2) {
    const int total = a.H * a.C * kk2;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx < a.H) {
        float g = 0.0f;
        for (int sp = 0; sp < a.splits; ++sp) g += a.bpart[sp * 8 + idx];
        a.b1[idx] = a.b1[idx] - a.lr * g;
    }
    if (idx >= total) return;
    const int o = idx / (a.C * kk2), r = idx - o * a.C * kk2, c = r / kk2, t = r - c * kk2;
    float g = 0.0f;
    for (int sp = 0; sp < a.splits; ++sp) g += a.part[(((size_t)sp * a.C + c) * 8 + o) * kk2 + t];
    a.W1[idx] = a.W1[idx] - a.lr * g;
}

}  // namespace gati
