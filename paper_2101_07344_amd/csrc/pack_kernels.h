// Device-side repacking of fp32 master weights (as a trainer holds them: plain row-major) into the
// layouts the lookup kernels read, so that retrained weights reach a serving cache without a trip
// through the host (paper, Section 5, "Retraining Learned Caches": retrained predictor and selector
// replace the old ones while serving goes on).  One lane per destination element; every destination
// element is written (padding as zero), so nothing of the old weights survives.  Rounding to bf16 is
// nearest-even, the same as the host packing of gati_cache_create.
#pragma once

#include "common.h"
#include "conv_kernels.h"

namespace gati {

// Where column i of a destination matrix comes from in the source row:
//   i < F                      feature column; with perm_P > 0 the source keeps hidden values in
//                              [position][filter] order while the destination wants [filter][position]:
//                              i = o*perm_P + p  ->  p*perm_H + o
//   F <= i < F + gap           zero (the destination pads its feature part)
//   F + gap <= i               source column F + (i - F - gap), zero past the source's cols_src columns
struct ColMap {
    int F, gap, cols_src, perm_P, perm_H;
};

__device__ __forceinline__ int map_col(const ColMap& m, int i) {
    if (i < m.F) {
        if (m.perm_P > 0) { const int o = i / m.perm_P, p = i - o * m.perm_P; return p * m.perm_H + o; }
        return i;
    }
    if (i < m.F + m.gap) return -1;
    const int s = m.F + (i - m.F - m.gap);
    return s < m.cols_src ? s : -1;
}

template <bool BF16> struct PackElem;
template <> struct PackElem<true> { typedef __bf16 type; static __device__ __forceinline__ __bf16 cvt(float v) { return (__bf16)v; } };
template <> struct PackElem<false> { typedef float type; static __device__ __forceinline__ float cvt(float v) { return v; } };

// MFMA fragment order of head_kernels.h: out[((nt*KS + ks)*64 + l)*kLane + e] =
// W[nt*32 + l%32][map(ks*kStep + (l/32)*kLane + e)], zero outside [rows, mapped columns].
template <bool BF16>
__global__ __launch_bounds__(256) void pack_fc_kernel(const float* __restrict__ W, int ld, int rows, int rows_p, int cols_p,
                                                      ColMap m, typename PackElem<BF16>::type* __restrict__ out) {
    constexpr int kStep = BF16 ? 16 : 8, kLane = kStep / 2;
    const int KS = cols_p / kStep;
    const long total = (long)rows_p * cols_p;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int e = (int)(idx % kLane);
        const int l = (int)((idx / kLane) % 64);
        const long t = idx / (kLane * 64);
        const int ks = (int)(t % KS), nt = (int)(t / KS);
        const int row = nt * 32 + (l & 31), col = ks * kStep + (l >> 5) * kLane + e;
        const int sc = map_col(m, col);
        out[idx] = PackElem<BF16>::cvt(row < rows && sc >= 0 ? W[(long)row * ld + sc] : 0.f);
    }
}

// W1 of the FC(h) predictor (flat_kernels.h): as above, but within every block of 4 k-steps lane
// half kb owns 2*kStep consecutive inputs: fragment (nt, ks, lane, e) holds
// W[nt*32 + lane%32][(ks/4)*4*kStep + (lane/32)*2*kStep + (ks%4)*kLane + e].  cols % (4*kStep) == 0.
template <bool BF16>
__global__ __launch_bounds__(256) void pack_flat_kernel(const float* __restrict__ W, long cols, int rows, int rows_p,
                                                        typename PackElem<BF16>::type* __restrict__ out) {
    constexpr int kStep = BF16 ? 16 : 8, kLane = kStep / 2;
    const long KS = cols / kStep;
    const long total = (long)rows_p * cols;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int e = (int)(idx % kLane);
        const int l = (int)((idx / kLane) % 64);
        const long t = idx / (kLane * 64);
        const long ks = t % KS;
        const int nt = (int)(t / KS);
        const int row = nt * 32 + (l & 31);
        const long col = (ks >> 2) * 4 * kStep + (long)(l >> 5) * 2 * kStep + (ks & 3) * kLane + e;
        out[idx] = PackElem<BF16>::cvt(row < rows ? W[(long)row * cols + col] : 0.f);
    }
}

// Filters of the Conv(k,s) predictor (conv_kernels.h): fragment order over the reduction index
// (channel block, tap padded to conv_taps_padded(k), channel in block); source W1 [Co][C][k*k].
template <bool BF16>
__global__ __launch_bounds__(256) void pack_conv_kernel(const float* __restrict__ W, int Co, int C, int k, int rows_p,
                                                        typename PackElem<BF16>::type* __restrict__ out) {
    constexpr int kStep = BF16 ? 16 : 8, kLane = kStep / 2;
    const int k2 = k * k, IT = conv_taps_padded(k);
    const int CB = (C + kStep - 1) / kStep, Kd = CB * IT * kStep, KS = Kd / kStep;
    const long total = (long)rows_p * Kd;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int e = (int)(idx % kLane);
        const int l = (int)((idx / kLane) % 64);
        const long t = idx / (kLane * 64);
        const int ks = (int)(t % KS), nt = (int)(t / KS);
        const int o = nt * 32 + (l & 31);
        const int col = ks * kStep + (l >> 5) * kLane + e;       // ((cb*IT + tap)*kStep + channel in block)
        const int cin = col % kStep, tap = (col / kStep) % IT, cb = col / (kStep * IT);
        const int c = cb * kStep + cin;
        out[idx] = PackElem<BF16>::cvt(o < Co && c < C && tap < k2 ? W[((long)o * C + c) * k2 + tap] : 0.f);
    }
}

// Filters of conv_rows_kernel (conv_rows_kernels.h): A fragments [channel group][row parity][lane][8 bf16];
// lane (m, kb) holds tap row t = m / 8 of filter o = m % 8, element e = horizontal tap e of channel
// 2*group + kb (slot 8) or tap e % 4 of channel 4*group + 2*kb + e / 4 (slot 4), row offset dy = parity + s*t.
__global__ __launch_bounds__(256) void pack_conv_rows_kernel(const float* __restrict__ W, int Co, int C, int k, int s, int slot,
                                                             long total, __bf16* __restrict__ out) {
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int e = (int)(idx & 7), l = (int)((idx >> 3) & 63);
        const long g = idx >> 9;
        const int pi = (int)(g % s), cg = (int)(g / s);
        const int m = l & 31, kb = l >> 5, t = m >> 3, o = m & 7;
        const int ch = slot == 8 ? 2 * cg + kb : 4 * cg + 2 * kb + (e >> 2);
        const int dx = slot == 8 ? e : (e & 3), dy = pi + s * t;
        out[idx] = (__bf16)(o < Co && dy < k && dx < k ? W[(((long)o * C + ch) * k + dy) * k + dx] : 0.f);
    }
}

// dst[i] = src[map(i)] (fp32), zero where the map says so; BF16VAL rounds the value to bf16 and keeps it
// as fp32 (the plain copies that the generic kernels read).
template <bool BF16VAL>
__global__ __launch_bounds__(256) void pack_vector_kernel(const float* __restrict__ src, long n_dst, ColMap m, float* __restrict__ dst) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n_dst; i += (long)gridDim.x * 256) {
        const int sc = map_col(m, (int)i);
        float v = sc >= 0 ? src[sc] : 0.f;
        if constexpr (BF16VAL) v = (float)(__bf16)v;
        dst[i] = v;
    }
}

// Plain element-type conversion of a whole matrix (FC(h) rows of odd length keep W1 as stored).
template <bool BF16>
__global__ __launch_bounds__(256) void pack_plain_kernel(const float* __restrict__ src, long n, typename PackElem<BF16>::type* __restrict__ dst) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) dst[i] = PackElem<BF16>::cvt(src[i]);
}

}  // namespace gati
