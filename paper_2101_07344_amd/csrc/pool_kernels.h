// Global average pooling of the activation tensor: pooled[i,c] = mean_s x[row(i),c,s].
// (Pooling predictor of the paper's Section 3 table of predictor architectures, with the
// pool extent taken over the whole spatial / token axis.)
//
// This is the stage that moves nearly all the bytes of a lookup, so every variant is a
// pure streaming read: 16-byte loads, many independent loads in flight per lane, fp32
// accumulation in a fixed order (no float atomics: results are bit-reproducible).
// All kernels are persistent: a fixed grid strides over the work, and the true row count
// is read on the device.
#pragma once

#include "common.h"

namespace gati {

struct PoolArgs {
    const void* act;           // activation tensor, device
    const int32_t* row_index;  // [n] source rows, or null for the identity
    const int32_t* n_dev;      // device row count, or null
    int n_max;
    int C, S;
    float inv_S;
    float* out;                // [n, out_stride] fp32
    __bf16* out16;             // same values rounded to bf16 (nearest even), same stride; or null
    int out_stride;
};

// Store one pooled mean (and its bf16 copy, the FC1 operand of bf16 caches).
__device__ __forceinline__ void store_pooled(const PoolArgs& a, long idx, float v) {
    a.out[idx] = v;
    if (a.out16) a.out16[idx] = (__bf16)v;
}

// ---------------------------------------------------------------------------------------
// [n,C,S], S*elem a multiple of 16 bytes: one wave sums one channel at a time, CPI channels
// per iteration so that LPC*CPI 16-byte loads per lane are in flight before the first add.
// vpc = 16-byte vectors per channel; a channel needs ceil(vpc/64) loads per lane, taken in
// chunks of LPC.
// ---------------------------------------------------------------------------------------
template <typename Tag, int LPC, int CPI>
__global__ __launch_bounds__(256) void pool_ncs_wave_kernel(PoolArgs a, int vpc) {
    const int n = active_rows(a.n_dev, a.n_max);
    const int lane = threadIdx.x & 63;
    const int waves_per_block = blockDim.x >> 6;
    const unsigned wave = blockIdx.x * waves_per_block + (threadIdx.x >> 6);
    const unsigned nwaves = gridDim.x * waves_per_block;
    const unsigned gpr = (unsigned)(a.C + CPI - 1) / CPI;  // channel groups per row
    const unsigned total = (unsigned)n * gpr;

    for (unsigned g = wave; g < total; g += nwaves) {
        const unsigned i = g / gpr;
        const int c0 = (int)(g - i * gpr) * CPI;
        const long r = a.row_index ? (long)a.row_index[i] : (long)i;
        const u32x4_t* base =
            reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.act) +
                                             ((r * a.C + c0) * (long)a.S) * Tag::kBytes);
        float s[CPI];
#pragma unroll
        for (int q = 0; q < CPI; ++q) s[q] = 0.f;

        for (int b = 0; b < vpc; b += 64 * LPC) {
            // Every load is unconditional and in bounds: slots past the end of the channel
            // (or past the last channel) re-read the last valid vector and are zeroed after.
            u32x4_t v[CPI][LPC];
#pragma unroll
            for (int q = 0; q < CPI; ++q) {
                const int qc = min(q, a.C - 1 - c0);
#pragma unroll
                for (int u = 0; u < LPC; ++u) {
                    const int idx = b + u * 64 + lane;
                    v[q][u] = load_stream(base + (long)qc * vpc + min(idx, vpc - 1));
                }
            }
#pragma unroll
            for (int q = 0; q < CPI; ++q) {
#pragma unroll
                for (int u = 0; u < LPC; ++u)
                    v[q][u] = keep_or_zero(v[q][u], (b + u * 64 + lane < vpc) && (c0 + q < a.C));
            }
#pragma unroll
            for (int q = 0; q < CPI; ++q) {
#pragma unroll
                for (int u = 0; u < LPC; ++u) s[q] += vec_sum<Tag>(v[q][u]);
            }
        }
        float mine = 0.f;
#pragma unroll
        for (int q = 0; q < CPI; ++q) {
            const float t = wave_sum(s[q]);
            mine = (lane == q) ? t : mine;
        }
        if (lane < CPI && c0 + lane < a.C)
            store_pooled(a, (long)i * a.out_stride + c0 + lane, mine * a.inv_S);
    }
}

// Split of one 16-byte vector at the channel boundary it may straddle: pa = sum of its first cnt
// elements, pb = sum of the rest.  bf16: the boundary becomes a bit mask over the four element
// pairs, built once per lane, and the pairs are added with the dot-product instruction.
template <typename Tag> struct SplitMask;
template <> struct SplitMask<F32Tag> {
    __device__ __forceinline__ void set(int) {}
    __device__ __forceinline__ void split(const u32x4_t& v, int cnt, float& pa, float& pb) const {
        float e[4];
        vec_unpack<F32Tag>(v, e);
        pa = 0.f; pb = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            pa += (k < cnt) ? e[k] : 0.f;
            pb += (k < cnt) ? 0.f : e[k];
        }
    }
};
template <> struct SplitMask<BF16Tag> {
    uint32_t m[4];     // bits of the elements that belong to the first channel
    __device__ __forceinline__ void set(int cnt) {
#pragma unroll
        for (int d = 0; d < 4; ++d)
            m[d] = (2 * d < cnt ? 0x0000ffffu : 0u) | (2 * d + 1 < cnt ? 0xffff0000u : 0u);
    }
    __device__ __forceinline__ void split(const u32x4_t& v, int, float& pa, float& pb) const {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        pa = 0.f; pb = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            pa = add_bf16_pair(w[d] & m[d], pa);
            pb = add_bf16_pair(w[d] & ~m[d], pb);
        }
    }
};

// ---------------------------------------------------------------------------------------
// [n,C,S] with short or 16-byte-unaligned channels (S = 49, 196, 64, ...), wave-granular.
// A sample's channels are one flat, contiguous stream, so a wave takes a tile of `gt` whole
// channels whose byte size is a multiple of 16 (at most 256 vectors) and reads it with fully
// coalesced 16-byte loads.  A vector may straddle one channel boundary (S >= elements per
// vector): each lane splits its vector into the part that belongs to the channel of its
// first element (a) and the part that belongs to the next channel (b) and parks both in the
// wave's own LDS strip; then `tpc` lanes per channel add up that channel's partial sums in a
// fixed order.  Nothing is shared between waves, so there is no workgroup barrier: the LDS
// unit serves one wave's instructions in order.  The next tile's loads are issued before the
// current tile's second phase, so every wave keeps a tile in flight.
// Requirements (checked on the host): gt*S % kVec == 0, C*S % kVec == 0, gt*S/kVec <= 256,
// S >= kVec, gt << tpc_log2 <= 64.
// ---------------------------------------------------------------------------------------
template <typename Tag>
__global__ __launch_bounds__(256) void pool_ncs_segw_kernel(PoolArgs a, int gt, int tiles_per_row,
                                                            int tpc_log2, unsigned magic_S) {
    constexpr int V = Tag::kVec;
    constexpr int J = 4;                 // loads per lane per tile
    constexpr int kMaxVec = 64 * J;
    __shared__ float sA[4][kMaxVec];
    __shared__ float sB[4][kMaxVec];

    const int n = active_rows(a.n_dev, a.n_max);
    const unsigned total = (unsigned)n * (unsigned)tiles_per_row;
    const int lane = threadIdx.x & 63;
    const int wib = threadIdx.x >> 6;
    const unsigned wave = blockIdx.x * (blockDim.x >> 6) + wib;
    const unsigned nwaves = gridDim.x * (blockDim.x >> 6);
    float* A = sA[wib];
    float* B = sB[wib];
    const int tpc = 1 << tpc_log2;
    const int lc = lane >> tpc_log2;     // tile-local channel this lane helps to finish
    const int sub = lane & (tpc - 1);

    // tile w -> (active row i, first channel, channel count, base pointer)
    auto tile_of = [&](unsigned w, unsigned& i, int& c_first, int& nch) -> const u32x4_t* {
        i = w / (unsigned)tiles_per_row;
        const int t = (int)(w - i * (unsigned)tiles_per_row);
        const long r = a.row_index ? (long)a.row_index[i] : (long)i;
        c_first = t * gt;
        nch = min(gt, a.C - c_first);
        return reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.act) +
                                                ((r * a.C + c_first) * (long)a.S) * Tag::kBytes);
    };

    // Where a lane's j-th vector lies relative to the channel boundaries is the same in every tile
    // (tiles start on a channel): cnt[j] = elements of the vector that belong to the channel of its
    // first element, found once.  (Recomputing it per tile, with the selects below on all 8 bf16
    // elements, kept the vector ALUs 87 % busy and the kernel below HBM speed.)
    int cnt[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const unsigned o = (unsigned)(lane + 64 * j) * V;    // first element, tile-local
        const unsigned ch = __umulhi(o, magic_S);            // o / S
        cnt[j] = a.S - (int)(o - ch * (unsigned)a.S);
    }
    SplitMask<Tag> mask[J];
#pragma unroll
    for (int j = 0; j < J; ++j) mask[j].set(cnt[j]);

    u32x4_t v[J];
    unsigned i = 0;
    int c_first = 0, nch = 0;
    if (wave < total) {
        const u32x4_t* base = tile_of(wave, i, c_first, nch);
        const int tv = (nch * a.S) / V;
#pragma unroll
        for (int j = 0; j < J; ++j) v[j] = load_stream(base + min(lane + 64 * j, tv - 1));
    }
    for (unsigned w = wave; w < total; w += nwaves) {
        const int tile_vecs = (nch * a.S) / V;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int idx = lane + 64 * j;
            if (idx < tile_vecs) {
                float pa, pb;
                mask[j].split(v[j], cnt[j], pa, pb);
                A[idx] = pa;
                B[idx] = pb;
            }
        }
        // this tile's identity, then start the next tile's loads
        const unsigned ci = i;
        const int cc = c_first, cn = nch;
        const unsigned wn = w + nwaves;
        if (wn < total) {
            const u32x4_t* base = tile_of(wn, i, c_first, nch);
            const int tv = (nch * a.S) / V;
#pragma unroll
            for (int j = 0; j < J; ++j) v[j] = load_stream(base + min(lane + 64 * j, tv - 1));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float acc = 0.f;
        const bool live = lc < cn;
        if (live) {
            const int start = lc * a.S;
            const int lo = (start + V - 1) / V;
            const int hi = (start + a.S + V - 1) / V;
            for (int k = lo + sub; k < hi; k += tpc) acc += A[k];
            if (sub == 0 && (start % V) != 0) acc += B[lo - 1];
        }
        for (int m = tpc >> 1; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
        if (live && sub == 0) store_pooled(a, (long)ci * a.out_stride + cc + lc, acc * a.inv_S);
        // keep the next tile's LDS writes behind this tile's reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---------------------------------------------------------------------------------------
// [n,C,S] with short or 16-byte-unaligned channels (S = 49, 196, 64, ...).  A sample's
// channels are one flat, contiguous stream, so a workgroup takes a tile of `gt` whole
// channels whose byte size is a multiple of 16 and reads it with fully coalesced 16-byte
// loads.  A vector may straddle one channel boundary (S >= elements per vector): each lane
// splits its vector into the part that belongs to the channel of its first element (a) and
// the part that belongs to the next channel (b), parks both in LDS, and after a barrier
// `tpc` lanes per channel add up that channel's partial sums in a fixed order.
// Requirements (checked on the host): gt*S % kVec == 0, C*S % kVec == 0, gt*S/kVec <= 1024,
// S >= kVec, gt << tpc_log2 <= 256.
// ---------------------------------------------------------------------------------------
template <typename Tag>
__global__ __launch_bounds__(256) void pool_ncs_seg_kernel(PoolArgs a, int gt, int tiles_per_row,
                                                           int tpc_log2, unsigned magic_S) {
    constexpr int V = Tag::kVec;
    constexpr int kMaxVec = 1024;
    __shared__ float sA[2][kMaxVec];
    __shared__ float sB[2][kMaxVec];

    const int n = active_rows(a.n_dev, a.n_max);
    const unsigned total = (unsigned)n * (unsigned)tiles_per_row;
    const int tid = threadIdx.x;
    const int tpc = 1 << tpc_log2;
    const int lc = tid >> tpc_log2;   // tile-local channel this lane helps to finish
    const int sub = tid & (tpc - 1);
    int buf = 0;

    for (unsigned w = blockIdx.x; w < total; w += gridDim.x, buf ^= 1) {
        const unsigned i = w / (unsigned)tiles_per_row;
        const int t = (int)(w - i * (unsigned)tiles_per_row);
        const long r = a.row_index ? (long)a.row_index[i] : (long)i;
        const int c_first = t * gt;
        const int nch = min(gt, a.C - c_first);
        const int tile_vecs = (nch * a.S) / V;
        const u32x4_t* base =
            reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.act) +
                                             ((r * a.C + c_first) * (long)a.S) * Tag::kBytes);
        u32x4_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)   // unconditional, clamped into the tile; extras are ignored below
            v[j] = load_stream(base + min(tid + 256 * j, tile_vecs - 1));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + 256 * j;
            if (idx < tile_vecs) {
                const unsigned o = (unsigned)idx * V;            // first element, tile-local
                const unsigned ch = __umulhi(o, magic_S);        // o / S
                const int cnt = a.S - (int)(o - ch * (unsigned)a.S);  // elements left in that channel
                float e[V];
                vec_unpack<Tag>(v[j], e);
                float pa = 0.f, pb = 0.f;
#pragma unroll
                for (int k = 0; k < V; ++k) {
                    pa += (k < cnt) ? e[k] : 0.f;
                    pb += (k < cnt) ? 0.f : e[k];
                }
                sA[buf][idx] = pa;
                sB[buf][idx] = pb;
            }
        }
        __syncthreads();
        float acc = 0.f;
        const bool live = lc < nch;
        if (live) {
            const int start = lc * a.S;
            const int lo = (start + V - 1) / V;
            const int hi = (start + a.S + V - 1) / V;
            for (int k = lo + sub; k < hi; k += tpc) acc += sA[buf][k];
            if (sub == 0 && (start % V) != 0) acc += sB[buf][lo - 1];
        }
        for (int m = tpc >> 1; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
        if (live && sub == 0) store_pooled(a, (long)i * a.out_stride + c_first + lc, acc * a.inv_S);
        // The other LDS buffer is written next; the barrier of the next iteration orders
        // this iteration's reads against the writes two iterations ahead.
    }
}

// ---------------------------------------------------------------------------------------
// [n,S,C] (tokens / channels-last), wave-granular: a lane owns one 16-byte vector of channels
// and walks down the token axis.  A wave covers GW channel-vectors of one row and splits the
// tokens over its 64/GW lane groups, whose partial sums are added with lane shuffles in a
// fixed order; no LDS, no barrier.  Requires C % kVec == 0.
// ---------------------------------------------------------------------------------------
template <typename Tag, int GW>
__global__ __launch_bounds__(256) void pool_nsc_kernel(PoolArgs a, int cvb_per_row) {
    constexpr int V = Tag::kVec;
    constexpr int NG = 64 / GW;    // token slices per wave
    constexpr int UN = 8;          // loads in flight per lane

    const int n = active_rows(a.n_dev, a.n_max);
    const unsigned total = (unsigned)n * (unsigned)cvb_per_row;
    const int lane = threadIdx.x & 63;
    const unsigned wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const unsigned nwaves = gridDim.x * (blockDim.x >> 6);
    const int gl = lane % GW;
    const int grp = lane / GW;
    const int CV = a.C / V;

    for (unsigned w = wave; w < total; w += nwaves) {
        const unsigned i = w / (unsigned)cvb_per_row;
        const int cb = (int)(w - i * (unsigned)cvb_per_row);
        const long r = a.row_index ? (long)a.row_index[i] : (long)i;
        const int cv = cb * GW + gl;
        const bool ok = cv < CV;
        const u32x4_t* base =
            reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.act) +
                                             (r * a.S * (long)a.C) * Tag::kBytes) + min(cv, CV - 1);
        float acc[V];
#pragma unroll
        for (int k = 0; k < V; ++k) acc[k] = 0.f;
        for (int s0 = grp; s0 < a.S; s0 += NG * UN) {
            u32x4_t v[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u)   // unconditional, clamped to the last token
                v[u] = load_stream(base + (long)min(s0 + u * NG, a.S - 1) * CV);
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                v[u] = keep_or_zero(v[u], ok && (s0 + u * NG < a.S));
                float e[V];
                vec_unpack<Tag>(v[u], e);
#pragma unroll
                for (int k = 0; k < V; ++k) acc[k] += e[k];
            }
        }
        // add the token slices: lanes gl, gl+GW, gl+2GW, ... hold the same channels
#pragma unroll
        for (int m = 32; m >= GW; m >>= 1) {
#pragma unroll
            for (int k = 0; k < V; ++k) acc[k] += __shfl_xor(acc[k], m, 64);
        }
        if (grp == 0 && ok) {
            const long o = (long)i * a.out_stride + (long)cv * V;
#pragma unroll
            for (int k = 0; k < V; ++k) store_pooled(a, o + k, acc[k] * a.inv_S);
        }
    }
}

// ---------------------------------------------------------------------------------------
// [n,S,C] with many tokens, wave-granular units: one wave owns (row, block of CVB channel
// vectors) and nothing else -- no LDS, no barrier, no other wave to wait for.  Its 64 lanes are
// 64/CVB token phases x CVB channel vectors, R loads per lane in flight; the token phases meet by
// lane shuffles in a fixed order.  Units leave the chip as they finish and the dispatcher brings
// in the next ones, so a launch with few rows still spreads over every CU and has no slow
// workgroup-sized tail (timestamps of the row-per-workgroup kernel showed workgroup end times
// spread over 40 % of the launch).  The row index is requested before the device-side row count
// is known (both scalar loads fly together).  Requires C % kVec == 0.
// ---------------------------------------------------------------------------------------
template <typename Tag, int R, int CVB>
__global__ __launch_bounds__(64) void pool_nsc_unit_kernel(PoolArgs a, int cvb_per_row) {
    constexpr int V = Tag::kVec;
    constexpr int TP = 64 / CVB;                       // token phases per load instruction
    const int lane = threadIdx.x;
    const int cvl = lane % CVB, tp = lane / CVB;
    const int CV = a.C / V;
    const unsigned w = blockIdx.x;
    const unsigned i = w / (unsigned)cvb_per_row;      // < n_max by the grid size
    const long r = a.row_index ? (long)a.row_index[i] : (long)i;
    const int n = active_rows(a.n_dev, a.n_max);
    if (i >= (unsigned)n) return;
    const int cb = (int)(w - i * (unsigned)cvb_per_row);
    const int cv = cb * CVB + cvl;
    const u32x4_t* base =
        reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.act) + (r * a.S * (long)a.C) * Tag::kBytes) +
        min(cv, CV - 1);
    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.f;
    for (int t0 = tp; t0 < a.S; t0 += TP * R) {
        u32x4_t v[R];
#pragma unroll
        for (int u = 0; u < R; ++u)        // unconditional, clamped to the last token
            v[u] = load_stream(base + (long)min(t0 + u * TP, a.S - 1) * CV);
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const u32x4_t x = keep_or_zero(v[u], t0 + u * TP < a.S);
            float e[V];
            vec_unpack<Tag>(x, e);
#pragma unroll
            for (int k = 0; k < V; ++k) acc[k] += e[k];
        }
    }
#pragma unroll
    for (int m = 32; m >= CVB; m >>= 1) {
#pragma unroll
        for (int k = 0; k < V; ++k) acc[k] += __shfl_xor(acc[k], m, 64);
    }
    if (tp == 0 && cv < CV) {
        const long o = (long)i * a.out_stride + (long)cv * V;
#pragma unroll
        for (int k = 0; k < V; ++k) store_pooled(a, o + k, acc[k] * a.inv_S);
    }
}

// ---------------------------------------------------------------------------------------
// Adaptive average pool of [n,C,in_h*in_w] to [n,C,out_h,out_w] with ReLU (the hidden layer of
// the paper's Pool(h) predictor).  Same flat-stream tiling as pool_ncs_segw: a wave loads a
// tile of whole channels (16-byte coalesced, at most 64*J vectors) and parks the raw elements
// in its own LDS strip; then `tpo` lanes per output window add up the window's rows in a fixed
// order.  Window i of an axis covers [floor(i*in/out), ceil((i+1)*in/out)).
// ---------------------------------------------------------------------------------------
// One output window of a tile, by its index o = local_channel * out_h*out_w + window: where its
// first element lies in the tile's flat element stream, its extent, and its element count.  Built
// on the host so that the kernel does no integer division (those made it ALU-bound).
struct __attribute__((aligned(16))) AdaptiveWindow {
    int start;   // local_channel * S + y0 * in_w + x0
    int rows;    // y1 - y0
    int cols;    // x1 - x0
    float area;  // rows * cols
};

struct AdaptiveArgs {
    int in_h, in_w, out_h, out_w;
    int gt, tiles_per_row, tpo_log2;
    const AdaptiveWindow* win;   // [gt * out_h * out_w], tiled kernel only
};

template <typename Tag> __device__ __forceinline__ float lds_elem(const u32x4_t* raw, int idx);
template <> __device__ __forceinline__ float lds_elem<F32Tag>(const u32x4_t* raw, int idx) {
    return reinterpret_cast<const float*>(raw)[idx];
}
template <> __device__ __forceinline__ float lds_elem<BF16Tag>(const u32x4_t* raw, int idx) {
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(raw)[idx] << 16);
}

// WW > 0: every window is WW columns wide (known on the host), so a window row's LDS reads are
// unrolled and all in flight together; with a run-time width each element's read waits for the
// one before it and the kernel is bound by LDS latency instead of HBM.  (Also unrolling the
// window rows, with clamped reads for the rows a lane does not own, was slower.)
// PAIR (bf16 only): 1 = every window row starts on an even element and WW is even, two elements
// per 32-bit LDS read; 2 = 32-bit reads from the even element at or before the row start, the
// candidates outside the window masked to zero; 0 = 16-bit reads.  Pairs are added by the bf16
// dot-product instruction, so a row's elements are not added strictly left to right.
template <typename Tag, int J, int WPB, int WW, int PAIR>
__global__ __launch_bounds__(WPB * 64) void pool_ncs_adaptive_kernel(PoolArgs a, AdaptiveArgs g) {
    constexpr int V = Tag::kVec;
    __shared__ u32x4_t raw_all[WPB][64 * J];

    const int n = active_rows(a.n_dev, a.n_max);
    const unsigned total = (unsigned)n * (unsigned)g.tiles_per_row;
    const int lane = threadIdx.x & 63;
    const int wib = threadIdx.x >> 6;
    const unsigned wave = blockIdx.x * WPB + wib;
    const unsigned nwaves = gridDim.x * WPB;
    u32x4_t* raw = raw_all[wib];
    const int OO = g.out_h * g.out_w;
    const int tpo = 1 << g.tpo_log2;
    const int sub = lane & (tpo - 1);

    auto tile_of = [&](unsigned w, unsigned& i, int& c_first, int& nch) -> const u32x4_t* {
        i = w / (unsigned)g.tiles_per_row;
        const int t = (int)(w - i * (unsigned)g.tiles_per_row);
        const long r = a.row_index ? (long)a.row_index[i] : (long)i;
        c_first = t * g.gt;
        nch = min(g.gt, a.C - c_first);
        return reinterpret_cast<const u32x4_t*>(static_cast<const char*>(a.act) +
                                                ((r * a.C + c_first) * (long)a.S) * Tag::kBytes);
    };

    constexpr int kWinRegs = 4;
    const int per_it = 64 >> g.tpo_log2;            // windows per step of the wave
    const int my_win = lane >> g.tpo_log2;
    AdaptiveWindow wreg[kWinRegs];
#pragma unroll
    for (int it = 0; it < kWinRegs; ++it) wreg[it] = g.win[min(it * per_it + my_win, g.gt * OO - 1)];

    u32x4_t v[J];
    unsigned i = 0;
    int c_first = 0, nch = 0;
    if (wave < total) {
        const u32x4_t* base = tile_of(wave, i, c_first, nch);
        const int tv = (nch * a.S) / V;
#pragma unroll
        for (int j = 0; j < J; ++j) v[j] = load_stream(base + min(lane + 64 * j, tv - 1));
    }
    for (unsigned w = wave; w < total; w += nwaves) {
        const int tile_vecs = (nch * a.S) / V;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int idx = lane + 64 * j;
            if (idx < tile_vecs) raw[idx] = v[j];
        }
        const unsigned ci = i;
        const int cc = c_first, cn = nch;
        const unsigned wn = w + nwaves;
        if (wn < total) {          // next tile's loads fly while this tile's windows are summed
            const u32x4_t* base = tile_of(wn, i, c_first, nch);
            const int tv = (nch * a.S) / V;
#pragma unroll
            for (int j = 0; j < J; ++j) v[j] = load_stream(base + min(lane + 64 * j, tv - 1));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int n_out = cn * OO;
        auto window = [&](int o, const AdaptiveWindow& wd) {
            const bool live = o < n_out;
            float acc = 0.f;
            if (live) {
                for (int y = sub; y < wd.rows; y += tpo) {
                    const int rb = wd.start + y * g.in_w;          // first element of the window row
                    if constexpr (WW > 0 && PAIR == 1) {
                        uint32_t e2[WW / 2];
                        const uint32_t* r2 = reinterpret_cast<const uint32_t*>(raw) + (rb >> 1);
#pragma unroll
                        for (int x = 0; x < WW / 2; ++x) e2[x] = r2[x];
#pragma unroll
                        for (int x = 0; x < WW / 2; ++x) acc = add_bf16_pair(e2[x], acc);
                    } else if constexpr (WW > 0 && PAIR == 2) {
                        // The row starts at any element: NP aligned pairs hold candidates k = 0 .. 2*NP-1, the
                        // window is k = odd .. odd + WW - 1.  Only the first and the last pair can hold a
                        // candidate outside the window; it is masked to +0.0 before the pair is added.
                        constexpr int NP = WW / 2 + 1;
                        const bool odd = rb & 1;
                        const uint32_t* r2 = reinterpret_cast<const uint32_t*>(raw);
                        const int last_pair = tile_vecs * 4 - 1;              // 8 elements per vector
                        uint32_t e2[NP];
#pragma unroll
                        for (int x = 0; x < NP; ++x) e2[x] = r2[min((rb >> 1) + x, last_pair)];
                        e2[0] &= odd ? 0xffff0000u : 0xffffffffu;
                        if constexpr (WW % 2 == 0) e2[NP - 1] &= odd ? 0x0000ffffu : 0u;
                        else e2[NP - 1] &= odd ? 0xffffffffu : 0x0000ffffu;
#pragma unroll
                        for (int x = 0; x < NP; ++x) acc = add_bf16_pair(e2[x], acc);
                    } else if constexpr (WW > 0) {
                        float e[WW];
#pragma unroll
                        for (int x = 0; x < WW; ++x) e[x] = lds_elem<Tag>(raw, rb + x);
#pragma unroll
                        for (int x = 0; x < WW; ++x) acc += e[x];          // same order as the loop below
                    } else {
                        for (int x = 0; x < wd.cols; ++x) acc += lds_elem<Tag>(raw, rb + x);
                    }
                }
            }
            for (int m = tpo >> 1; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
            if (live && sub == 0)      // (cc + local channel) * OO + window = cc * OO + o
                store_pooled(a, (long)ci * a.out_stride + (long)cc * OO + o, fmaxf(acc / wd.area, 0.f));
        };
        // a lane meets the same windows in every tile: the first kWinRegs steps' table entries wait in registers
#pragma unroll
        for (int it = 0; it < kWinRegs; ++it)
            if (it * per_it < n_out) window(it * per_it + my_win, wreg[it]);
        for (int ob = kWinRegs * per_it; ob < n_out; ob += per_it) {
            const int o = ob + my_win;
            window(o, g.win[min(o, n_out - 1)]);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// Adaptive pool for shapes the tiled kernel cannot take: one lane per output window, scalar loads.
// nsc_layout = 0: [n,C,S] rows, consecutive lanes take consecutive features (c*OO + window).
// nsc_layout = 1: [n,S,C] rows (channels-last maps): consecutive lanes take consecutive channels of one
// window, so a wave's loads fall on consecutive addresses; feature order stays [c][oy][ox].
template <typename Tag>
__global__ __launch_bounds__(256) void pool_adaptive_generic_kernel(PoolArgs a, AdaptiveArgs g, int nsc_layout) {
    const int n = active_rows(a.n_dev, a.n_max);
    const int OO = g.out_h * g.out_w;
    const long F = (long)a.C * OO;
    const long total = (long)n * F;
    const long stride = (long)gridDim.x * blockDim.x;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const long i = idx / F;
        const int q = (int)(idx - i * F);
        const int c = nsc_layout ? q % a.C : q / OO;
        const int wi = nsc_layout ? q / a.C : q - c * OO;
        const int f = c * OO + wi;
        const int oy = wi / g.out_w, ox = wi - oy * g.out_w;
        const int y0 = (oy * g.in_h) / g.out_h, y1 = ((oy + 1) * g.in_h + g.out_h - 1) / g.out_h;
        const int x0 = (ox * g.in_w) / g.out_w, x1 = ((ox + 1) * g.in_w + g.out_w - 1) / g.out_w;
        const long r = a.row_index ? (long)a.row_index[i] : i;
        const long first = nsc_layout ? r * a.S * (long)a.C + c : (r * a.C + c) * (long)a.S;
        const long step = nsc_layout ? a.C : 1;
        float s = 0.f;
        for (int y = y0; y < y1; ++y)
            for (int x = x0; x < x1; ++x) {
                const long e = first + (long)(y * g.in_w + x) * step;
                if (Tag::kBytes == 4) s += static_cast<const float*>(a.act)[e];
                else s += __uint_as_float((uint32_t)static_cast<const uint16_t*>(a.act)[e] << 16);
            }
        store_pooled(a, i * a.out_stride + f, fmaxf(s / (float)((y1 - y0) * (x1 - x0)), 0.f));
    }
}

// ---------------------------------------------------------------------------------------
// Any shape, layout and alignment: one lane per (row, channel), scalar loads.  Slow; only
// for shapes the vector kernels cannot take.
// ---------------------------------------------------------------------------------------
template <typename Tag>
__global__ __launch_bounds__(256) void pool_generic_kernel(PoolArgs a, int nsc_layout) {
    const int n = active_rows(a.n_dev, a.n_max);
    const long total = (long)n * a.C;
    const long stride = (long)gridDim.x * blockDim.x;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const long i = idx / a.C;
        const int c = (int)(idx - i * a.C);
        const long r = a.row_index ? (long)a.row_index[i] : i;
        const long first = nsc_layout ? (r * a.S * (long)a.C + c) : ((r * a.C + c) * (long)a.S);
        const long step = nsc_layout ? a.C : 1;
        float s = 0.f;
        if (Tag::kBytes == 4) {
            const float* x = static_cast<const float*>(a.act);
            for (int k = 0; k < a.S; ++k) s += x[first + k * step];
        } else {
            const uint16_t* x = static_cast<const uint16_t*>(a.act);
            for (int k = 0; k < a.S; ++k) s += __uint_as_float((uint32_t)x[first + k * step] << 16);
        }
        store_pooled(a, i * a.out_stride + c, s * a.inv_S);
    }
}

}  // namespace gati
