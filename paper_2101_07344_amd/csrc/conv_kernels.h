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
//     LDS exactly as it lies in memory (16-byte coalesced loads) and read k*k times from
//     there, once per tap: the A fragment of a tap is the lane's pixel shifted by
//     dy*in_w + dx, its kLane channels one LDS plane apart;
//   * the filters are repacked at cache creation into MFMA B-fragment order with the
//     reduction index ordered (cb, dy, dx, channel in block), so a tap's fragment is one
//     16-byte load per lane.
// Two staging modes, chosen on the host: `whole` (small maps: the kStep channel planes of a
// block are one contiguous piece of memory, copied as is) and banded (large maps: a band of
// rows_in input rows per channel; needs in_w*elem and S*elem to be multiples of 16).
// For bf16 maps whose rows of 8 positions are 16-byte aligned (S a multiple of 8; banded: in_w
// too) the block is transposed on its way into LDS (TR): a thread loads the same 8 positions
// of 8 channels, swaps them in registers and stores 8 records of [position][8 channels], so an
// A fragment is ONE 16-byte LDS read instead of eight 2-byte reads and four packs -- the
// untransposed form is bound by LDS and VALU instruction issue, several times over the MFMA
// time.  Records of a group of 8 positions are stored XOR-swizzled by the group index so the
// transposing stores of neighbouring lanes (256 bytes apart) do not fall on one bank.
// conv_generic_kernel takes everything else (any shape, alignment or layout; one lane per output).
#pragma once

#include "head_kernels.h"

namespace gati {

// Filter fragments are prefetched through a register ring of kConvRing slots; a channel block's
// k*k taps are padded to a multiple of it with all-zero fragments (conv_taps_padded).
constexpr int kConvRing = 4;
inline __host__ __device__ int conv_taps_padded(int k) { return (k * k + kConvRing - 1) / kConvRing * kConvRing; }

struct ConvArgs {
    const void* act;           // [rows, C, in_h*in_w]
    const int32_t* row_index;  // [n] or null
    const int32_t* n_dev;
    int n_max;
    int C, S, in_h, in_w, k, s, oh, ow, Co;
    const void* Wp;            // packed filters [Cop/32][KS][64][kLane], KS = (C/kStep)*conv_taps_padded(k)
    const float* Wplain;       // [Co, C, k, k] fp32 (bf16 caches: already rounded), generic kernel
    const float* bias;         // [Cop]
    int CB;                    // channel blocks C / kStep
    int R, nbands;             // output rows per band, bands per request
    int rows_in;               // input rows staged per band ((R-1)*s + k; whole: in_h)
    int whole;                 // staging mode
    float* out;                // [n, out_stride] fp32 features
    __bf16* out16;             // bf16 copy (the output FC's operand) or null
    int out_stride;
    // split of the channel blocks over ksplit workgroups (small maps: too few workgroups otherwise);
    // ksplit > 1: raw sums go to partial[split][n_max][out_stride], conv_reduce_kernel finishes
    int ksplit, cb_per_split;
    float* partial;
    int bps;                   // channel blocks staged per LDS fill (whole mode without transposition:
                               // consecutive blocks are contiguous in memory; else 1)
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

// Transposed staging: position p's record of 16 channels (32 bytes) sits at slot
// (p & ~7) | ((p ^ (p >> 3)) & 7); lane half kb reads its 8 channels with one 16-byte load.
__device__ __forceinline__ Mma<true>::frag_t conv_a_fragment_tr(const unsigned char* xb, int p, int kb) {
    const int slot = (p & ~7) | ((p ^ (p >> 3)) & 7);
    return *reinterpret_cast<const Mma<true>::frag_t*>(xb + slot * 32 + kb * 16);
}

// TPW: 32-pixel tiles per wave (a band holds at most 128*TPW output pixels; every wave computes TPW
// tiles, the ones past the band on repeated pixels, unstored); NTC: 32-filter tiles.
template <bool BF16, int TPW, int NTC, bool TR>
__global__ __launch_bounds__(256, (TPW * NTC <= 2 ? 4 : (TPW * NTC <= 4 ? 3 : 1))) void conv_relu_kernel(ConvArgs a) {
    static_assert(BF16 || !TR, "transposed staging is for bf16 maps");
    using M = Mma<BF16>;
    using frag_t = typename M::frag_t;
    constexpr int kStep = M::kStep;
    constexpr int kElem = BF16 ? 2 : 4;
    constexpr int kMaxVec = 2048;                            // 32 KB: kStep * pitch * kElem <= 32 KB
    __shared__ u32x4_t xs[1][kMaxVec];

    const int n = active_rows(a.n_dev, a.n_max);
    const int split = blockIdx.x % a.ksplit;
    const int ib = blockIdx.x / a.ksplit;
    const int i = ib / a.nbands;
    const int b = ib - i * a.nbands;
    if (i >= n) return;                                      // whole workgroup
    const int cb0 = split * a.cb_per_split, cb1 = min(a.CB, cb0 + a.cb_per_split);
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
    int src_off[LPT];                                        // within one request's C*S*elem < 2^31 bytes
    int dst_idx[LPT];
    // TR: thread (chunk = tid & 127, half h = tid >> 7) owns positions 8*chunk .. 8*chunk+7 of channels 8h .. 8h+7
    const int tr_chunk = tid & 127, tr_h = tid >> 7;
    const int tr_chunks = (a.whole ? a.S : rows_here * a.in_w) >> 3;      // chunks that exist in this band
    if constexpr (TR) {
        const int ch = min(tr_chunk, tr_chunks - 1);
#pragma unroll
        for (int q = 0; q < LPT; ++q) src_off[q] = ((tr_h * 8 + q) * a.S + y0 * a.in_w + ch * 8) * kElem;
    } else {
#pragma unroll
        for (int q = 0; q < LPT; ++q) {
            const int v = min(tid + 256 * q, total_vec - 1);     // surplus threads repeat the last vector
            if (a.whole) {
                src_off[q] = v * 16;
                dst_idx[q] = v;
            } else {
                const int cl = v / vpc_here, vv = v - cl * vpc_here;
                src_off[q] = (cl * a.S + y0 * a.in_w) * kElem + vv * 16;
                dst_idx[q] = cl * vpc_full + vv;
            }
        }
    }
    const long block_stride = (long)kStep * a.S * kElem;     // bytes from one channel block to the next
    u32x4_t stage[LPT];
    int stage_vec = total_vec;                               // vectors of the fill being staged
    auto issue = [&](int cb, int nblk) {
        const unsigned char* base = row_base + (long)cb * block_stride;
        if (a.bps > 1) {                                     // several contiguous blocks: plain copy
            stage_vec = nblk * total_vec;
#pragma unroll
            for (int q = 0; q < LPT; ++q)
                stage[q] = load_stream(reinterpret_cast<const u32x4_t*>(base) + min(tid + 256 * q, stage_vec - 1));
        } else {
#pragma unroll
            for (int q = 0; q < LPT; ++q) stage[q] = load_stream(reinterpret_cast<const u32x4_t*>(base + src_off[q]));
        }
    };
    auto park = [&](int buf) {
        if constexpr (TR) {
            // stage[e] = channel 8h+e, positions 0..7 of the chunk (two per dword); record j wants
            // the 8 channels of position j: dword q = (channel 2q, channel 2q+1)
            if (tr_chunk < tr_chunks) {
                unsigned char* dst = reinterpret_cast<unsigned char*>(xs[buf]) + tr_chunk * 256 + tr_h * 16;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    u32x4_t rec;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t lo = stage[2 * q][j >> 1], hi = stage[2 * q + 1][j >> 1];
                        rec[q] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
                    }
                    *reinterpret_cast<u32x4_t*>(dst + ((j ^ (tr_chunk & 7)) * 32)) = rec;
                }
            }
        } else {
#pragma unroll
            for (int q = 0; q < LPT; ++q)
                if (tid + 256 * q < stage_vec) xs[buf][a.bps > 1 ? tid + 256 * q : dst_idx[q]] = stage[q];
        }
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
    // Filter fragments run WD-1 iterations ahead of their use in a register ring (they come from
    // L2: every workgroup reads the same few hundred KB).  A block's taps are walked in
    // IT = conv_taps_padded(k) iterations so that ring slots are compile-time; a padded iteration
    // multiplies the block's first tap by an all-zero fragment.  Nothing in the loop is conditional:
    // a load under a branch would make the compiler drain the whole load queue at every use, and
    // an MFMA under a branch makes it shuttle the accumulators between register files.
    constexpr int WD = kConvRing;
    const int IT = conv_taps_padded(a.k);
    const int KS = a.CB * IT;
    const frag_t* wp = reinterpret_cast<const frag_t*>(a.Wp) + lane;
    frag_t wring[WD][NTC];
    int pcb = cb0, ptap = 0;                                 // (block, tap) the next ring load is for
    auto wload = [&](int slot) {
        const int kc = min(pcb, a.CB - 1) * IT + ptap;
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt) wring[slot][nt] = wp[((long)nt * KS + kc) * 64];
        if (++ptap == IT) { ptap = 0; ++pcb; }
    };
#pragma unroll
    for (int d = 0; d < WD - 1; ++d) wload(d);

    // One LDS buffer per workgroup, no load/compute overlap inside it: up to four workgroups share
    // a CU and cover each other's loads.  (Double buffering inside the workgroup loses to this:
    // the filter loads issued during a block's arithmetic sit behind the next block's activation
    // loads in the in-order load queue, so the first filter use of every block waits for HBM.)
    for (int cbs = cb0; cbs < cb1; cbs += a.bps) {
        const int nblk = min(a.bps, cb1 - cbs);
        issue(cbs, nblk);
        park(0);
        __syncthreads();
      for (int bj = 0; bj < nblk; ++bj) {
        const unsigned char* xb = reinterpret_cast<const unsigned char*>(xs[0]) + (long)bj * total_vec * 16;
        // the A fragments of tap t+1 are read from LDS before the MFMAs of tap t, so the read latency
        // is covered by arithmetic; (dy, dx) below are those of the NEXT tap
        auto fragments = [&](frag_t (&f)[TPW], int off) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if constexpr (TR) f[t] = conv_a_fragment_tr(xb, pos[t] + off, kb);
                else f[t] = conv_a_fragment<BF16>(xb, pos[t] + off, pitch, kb);
            }
        };
        frag_t xf[TPW], xn[TPW];
        fragments(xf, 0);                                    // tap 0
        int dy = 0, dx = 1;
        if (dx == a.k) { dx = 0; dy = 1; }
        for (int tap0 = 0; tap0 < IT; tap0 += WD) {
#pragma unroll
            for (int u = 0; u < WD; ++u) {                   // ring slot = u
                wload((u + WD - 1) % WD);
                fragments(xn, tap0 + u + 1 < k2 ? dy * a.in_w + dx : 0);   // past the last tap: any valid position
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int nt = 0; nt < NTC; ++nt) acc[t][nt] = M::mma(xf[t], wring[u][nt], acc[t][nt]);
#pragma unroll
                for (int t = 0; t < TPW; ++t) xf[t] = xn[t];
                if (++dx == a.k) { dx = 0; ++dy; }
            }
        }
      }
        __syncthreads();                                     // every wave is done with the buffer
    }

    // features [co][oy][ox]: a band's pixels are contiguous within a filter's plane.  One split: bias
    // and ReLU here; several: raw sums to this split's slab
    const int OHW = a.oh * a.ow;
    const bool last = a.ksplit == 1;
    float* orow = (last ? a.out : a.partial + (long)split * a.n_max * a.out_stride) + (long)i * a.out_stride + oy0 * a.ow;
    __bf16* orow16 = (last && a.out16) ? a.out16 + (long)i * a.out_stride + oy0 * a.ow : nullptr;
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
                    const float v = last ? fmaxf(acc[t][nt][j] + bv, 0.f) : acc[t][nt][j];
                    orow[(long)co * OHW + q] = v;
                    if (orow16) orow16[(long)co * OHW + q] = (__bf16)v;
                }
            }
        }
    }
}

// Sum of the channel-block splits in split order, bias, ReLU, fp32 + bf16 features.
__global__ __launch_bounds__(256) void conv_reduce_kernel(ConvArgs a) {
    const int n = active_rows(a.n_dev, a.n_max);
    const int OHW = a.oh * a.ow;
    const int F = a.Co * OHW;
    const long total = (long)n * F;
    const long stride = (long)gridDim.x * blockDim.x;
    const long slab = (long)a.n_max * a.out_stride;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const long i = idx / F;
        const int f = (int)(idx - i * F);
        const long o = i * a.out_stride + f;
        float sum = 0.f;
        for (int sp = 0; sp < a.ksplit; ++sp) sum += a.partial[sp * slab + o];
        const float v = fmaxf(sum + a.bias[f / OHW], 0.f);
        a.out[o] = v;
        if (a.out16) a.out16[o] = (__bf16)v;
    }
}

// Any shape, either layout: one lane per hidden value, scalar loads, fp32 accumulation in
// (channel, dy, dx) order.  nsc_layout = 1: the map is stored [position][channel].
template <bool BF16>
__global__ __launch_bounds__(256) void conv_generic_kernel(ConvArgs a, int nsc_layout) {
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
        const long pos_step = nsc_layout ? a.C : 1;
        float acc = 0.f;
        for (int c = 0; c < a.C; ++c) {
            const long plane = nsc_layout ? r * a.S * (long)a.C + c : (r * a.C + c) * (long)a.S;
            const float* w = a.Wplain + ((long)co * a.C + c) * a.k * a.k;
            for (int dy = 0; dy < a.k; ++dy)
                for (int dx = 0; dx < a.k; ++dx) {
                    const long e = plane + ((long)(oy * a.s + dy) * a.in_w + ox * a.s + dx) * pos_step;
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
