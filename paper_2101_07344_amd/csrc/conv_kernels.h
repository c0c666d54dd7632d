// The paper's Conv(k,s) predictor (Section 3, table of predictor architectures): the hidden
// layer is a convolution of the layer's C x in_h x in_w activation with Co filters of k x k,
// stride s, no padding, then ReLU; the output FC reads the Co*oh*ow hidden values
// (feature order [co][oy][ox]).
//
// The convolution is a dense contraction over (channel, dy, dx): per request
// 2*Co*oh*ow*C*k*k flop against C*in_h*in_w elements read once, i.e. tens of flop per byte
// -- far above what the vector ALUs sustain at HBM speed -- so it runs on the matrix cores as
// an implicit GEMM:  D[pixel][co] = sum over k-steps (channel block cb, tap dy, dx) of
// X[pixel + tap][channels of cb] * W[channels of cb, tap][co].
//
//   * one workgroup = one request x one band of output rows (all Co filters); its 4 waves
//     deal out the band's 32-pixel tiles, TPW per wave, accumulators in registers for the
//     whole reduction;
//   * the input band of one channel block (kStep = 16 bf16 / 8 fp32 channels) is staged in
//     LDS exactly as it lies in memory (16-byte coalesced loads; the next block's loads are in
//     flight in registers while the current block is multiplied), and read k*k times from
//     there, once per tap: the A fragment of a tap is the lane's pixel shifted by
//     dy*in_w + dx, its kLane channels one LDS plane apart;
//   * the filters are repacked at cache creation into MFMA B-fragment order with the
//     reduction index ordered (cb, dy, dx, channel in block), so a tap's fragment is one
//     16-byte load per lane.
// Two staging modes, chosen on the host: `whole` (small maps: the kStep channel planes of a
// block are one contiguous piece of memory, copied as is) and banded (large maps: a band of
// rows_in input rows per channel; needs in_w*elem and S*elem to be multiples of 16).
// conv_generic_kernel takes everything else (any shape or alignment; one lane per output).
#pragma once

#include "head_kernels.h"

namespace gati {

struct ConvArgs {
    const void* act;           // [rows, C, in_h*in_w]
    const int32_t* row_index;  // [n] or null
    const int32_t* n_dev;
    int n_max;
    int C, S, in_h, in_w, k, s, oh, ow, Co;
    const void* Wp;            // packed filters [Cop/32][KS][64][kLane], KS = (C/kStep)*k*k
    const float* Wplain;       // [Co, C, k, k] fp32 (bf16 caches: already rounded), generic kernel
    const float* bias;         // [Cop]
    int CB;                    // channel blocks C / kStep
    int R, nbands;             // output rows per band, bands per request
    int rows_in;               // input rows staged per band ((R-1)*s + k; whole: in_h)
    int whole;                 // staging mode
    float* out;                // [n, out_stride] fp32 features
    __bf16* out16;             // bf16 copy (the output FC's operand) or null
    int out_stride;
};

template <bool BF16>
__device__ __forceinline__ typename Mma<BF16>::frag_t conv_a_fragment(const unsigned char* xb, int pos, int pitch, int kb);

// bf16: 8 channels, one 2-byte LDS read each, packed pairwise
template <>
__device__ __forceinline__ Mma<true>::frag_t conv_a_fragment<true>(const unsigned char* xb, int pos, int pitch, int kb) {
    const uint16_t* x = reinterpret_cast<const uint16_t*>(xb) + (kb * 8) * pitch + pos;
    u32x4_t w;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t lo = x[(2 * e) * pitch], hi = x[(2 * e + 1) * pitch];
        w[e] = lo | (hi << 16);
    }
    return __builtin_bit_cast(Mma<true>::frag_t, w);
}

template <>
__device__ __forceinline__ Mma<false>::frag_t conv_a_fragment<false>(const unsigned char* xb, int pos, int pitch, int kb) {
    const float* x = reinterpret_cast<const float*>(xb) + (kb * 4) * pitch + pos;
    f32x4_t w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = x[e * pitch];
    return w;
}

// TPW: 32-pixel tiles per wave (a band holds at most 128*TPW output pixels); NTC: 32-filter tiles.
template <bool BF16, int TPW, int NTC>
__global__ __launch_bounds__(256) void conv_relu_kernel(ConvArgs a) {
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep;
    constexpr int kElem = BF16 ? 2 : 4;
    constexpr int kMaxVec = 2048;                            // 32 KB per buffer: kStep * pitch * kElem <= 32 KB
    __shared__ u32x4_t xs[2][kMaxVec];

    const int n = active_rows(a.n_dev, a.n_max);
    const int i = blockIdx.x / a.nbands;
    const int b = blockIdx.x - i * a.nbands;
    if (i >= n) return;                                      // whole workgroup
    const long r = a.row_index ? (long)a.row_index[i] : (long)i;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int m = lane & 31, kb = lane >> 5;

    const int oy0 = b * a.R;
    const int Rb = min(a.R, a.oh - oy0);
    const int Pb = Rb * a.ow;                                // output pixels of this band (raster order)
    const int y0 = a.whole ? 0 : oy0 * a.s;                  // first input row held in LDS
    const int rows_here = a.whole ? a.in_h : min(a.rows_in, a.in_h - y0);
    const int pitch = a.whole ? a.S : a.rows_in * a.in_w;    // elements per channel plane in LDS
    // staging: `whole` copies kStep*S contiguous elements; banded copies kStep chunks of rows_here rows
    const int vpc_full = pitch * kElem / 16;                 // banded: LDS vectors per channel
    const int vpc_here = rows_here * a.in_w * kElem / 16;    // banded: vectors actually loaded per channel
    const int total_vec = a.whole ? kStep * a.S * kElem / 16 : kStep * vpc_here;
    const unsigned char* row_base = static_cast<const unsigned char*>(a.act) + r * (long)a.C * a.S * kElem;

    // per-thread source / destination of its up to 8 vectors of a block (the same for every block)
    constexpr int LPT = kMaxVec / 256;
    long src_off[LPT];
    int dst_idx[LPT];
#pragma unroll
    for (int q = 0; q < LPT; ++q) {
        const int v = min(tid + 256 * q, total_vec - 1);     // surplus threads repeat the last vector
        if (a.whole) {
            src_off[q] = (long)v * 16;
            dst_idx[q] = v;
        } else {
            const int cl = v / vpc_here, vv = v - cl * vpc_here;
            src_off[q] = ((long)cl * a.S + (long)y0 * a.in_w) * kElem + (long)vv * 16;
            dst_idx[q] = cl * vpc_full + vv;
        }
    }
    const long block_stride = (long)kStep * a.S * kElem;     // bytes from one channel block to the next
    u32x4_t stage[LPT];
    auto issue = [&](int cb) {
        const unsigned char* base = row_base + (long)cb * block_stride;
#pragma unroll
        for (int q = 0; q < LPT; ++q) stage[q] = load_stream(reinterpret_cast<const u32x4_t*>(base + src_off[q]));
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int q = 0; q < LPT; ++q)
            if (tid + 256 * q < total_vec) xs[buf][dst_idx[q]] = stage[q];
    };

    // the lane's pixel (A-fragment row m) in each of the wave's tiles, as an LDS element position
    const int tiles = (Pb + 31) >> 5;
    int pos[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int q = min((wave + 4 * t) * 32 + m, Pb - 1);  // pixels past the band repeat its last pixel
        const int oyl = q / a.ow, ox = q - oyl * a.ow;
        pos[t] = ((a.whole ? oy0 + oyl : oyl) * a.s) * a.in_w + ox * a.s;
    }

    f32x16_t acc[TPW][NTC];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[t][nt][j] = 0.f;

    const int k2 = a.k * a.k;
    const long KS = (long)a.CB * k2;
    const frag_t* wp = reinterpret_cast<const frag_t*>(a.Wp) + lane;

    issue(0);
    park(0);
    __syncthreads();
    for (int cb = 0; cb < a.CB; ++cb) {
        issue(min(cb + 1, a.CB - 1));                        // unconditional: the last block is loaded twice
        const unsigned char* xb = reinterpret_cast<const unsigned char*>(xs[cb & 1]);
        int dy = 0, dx = 0;
        for (int tap = 0; tap < k2; ++tap) {
            frag_t wf[NTC];
#pragma unroll
            for (int nt = 0; nt < NTC; ++nt) wf[nt] = wp[((long)nt * KS + (long)cb * k2 + tap) * 64];
            const int off = dy * a.in_w + dx;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if (wave + 4 * t < tiles) {                  // wave-uniform
                    const frag_t xf = conv_a_fragment<BF16>(xb, pos[t] + off, pitch, kb);
#pragma unroll
                    for (int nt = 0; nt < NTC; ++nt) acc[t][nt] = M::mma(xf, wf[nt], acc[t][nt]);
                }
            }
            if (++dx == a.k) { dx = 0; ++dy; }
        }
        if (cb + 1 < a.CB) park((cb + 1) & 1);               // that buffer was last read before the previous barrier
        __syncthreads();
    }

    // bias, ReLU, features [co][oy][ox]: a band's pixels are contiguous within a filter's plane
    const int OHW = a.oh * a.ow;
    float* orow = a.out + (long)i * a.out_stride + oy0 * a.ow;
    __bf16* orow16 = a.out16 ? a.out16 + (long)i * a.out_stride + oy0 * a.ow : nullptr;
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        if (wave + 4 * t >= tiles) continue;
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt) {
            const int co = nt * 32 + m;                      // D column
            if (co >= a.Co) continue;
            const float bv = a.bias[co];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int q = (wave + 4 * t) * 32 + mfma_row(j, kb);
                if (q < Pb) {
                    const float v = fmaxf(acc[t][nt][j] + bv, 0.f);
                    orow[(long)co * OHW + q] = v;
                    if (orow16) orow16[(long)co * OHW + q] = (__bf16)v;
                }
            }
        }
    }
}

// Any shape, layout NCS: one lane per hidden value, scalar loads, fp32 accumulation in
// (channel, dy, dx) order.
template <bool BF16>
__global__ __launch_bounds__(256) void conv_generic_kernel(ConvArgs a) {
    const int n = active_rows(a.n_dev, a.n_max);
    const int OHW = a.oh * a.ow;
    const long F = (long)a.Co * OHW;
    const long total = (long)n * F;
    const long stride = (long)gridDim.x * blockDim.x;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const long i = idx / F;
        const int f = (int)(idx - i * F);
        const int co = f / OHW, q = f - co * OHW;
        const int oy = q / a.ow, ox = q - oy * a.ow;
        const long r = a.row_index ? (long)a.row_index[i] : i;
        float acc = 0.f;
        for (int c = 0; c < a.C; ++c) {
            const long plane = (r * a.C + c) * (long)a.S;
            const float* w = a.Wplain + ((long)co * a.C + c) * a.k * a.k;
            for (int dy = 0; dy < a.k; ++dy)
                for (int dx = 0; dx < a.k; ++dx) {
                    const long e = plane + (long)(oy * a.s + dy) * a.in_w + ox * a.s + dx;
                    float x;
                    if constexpr (BF16) x = __uint_as_float((uint32_t)static_cast<const uint16_t*>(a.act)[e] << 16);
                    else x = static_cast<const float*>(a.act)[e];
                    acc = fmaf(w[dy * a.k + dx], x, acc);
                }
        }
        const float v = fmaxf(acc + a.bias[co], 0.f);
        a.out[i * a.out_stride + f] = v;
        if (a.out16) a.out16[i * a.out_stride + f] = (__bf16)v;
    }
}

}  // namespace gati
