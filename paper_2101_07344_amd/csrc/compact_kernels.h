// Stable stream compaction of the miss set (paper, Section 1: requests that miss keep
// running on the base model and meet the next layer's cache; Appendix A.1: earlier hits
// remove samples from later caches).  Pure integer work: wave ballots, popcount prefix
// within the wave, a scan of the per-wave totals in LDS.
#pragma once

#include "common.h"

namespace gati {

struct CompactArgs {
    const uint8_t* hit;      // [n] any non-zero byte = hit
    const int32_t* ids_in;   // [n] or null (identity)
    const int32_t* n_dev;    // device count or null
    int n_max;
    int32_t* ids_out;        // [n]
    int32_t* n_miss;         // device scalar (may alias n_dev)
};

// Shared state of a workgroup-wide stable compaction over NW waves.
template <int NW> struct CompactState {
    int wave_total[NW];
    int wave_offset[NW];
    int carry, carry_next;
};

// One step: every lane of the workgroup brings one flag; returns the output slot of a
// surviving lane (running offset + survivors before it, in lane order) or -1.  Wave ballots,
// popcount prefix within the wave, a scan of the NW wave totals by the first NW lanes.
// Must be called by all lanes of the workgroup; st.carry must be set before the first step
// (with a barrier in between, which the first call provides).
template <int NW>
__device__ __forceinline__ int compact_step(CompactState<NW>& st, bool keep, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    const unsigned long long mask = __ballot(keep);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) st.wave_total[wave] = __popcll(mask);
    __syncthreads();
    if (tid < NW) {
        const int v = st.wave_total[tid];
        int incl = v;
#pragma unroll
        for (int d = 1; d < NW; d <<= 1) {
            const int o = __shfl_up(incl, d, 64);
            if (tid >= d) incl += o;
        }
        st.wave_offset[tid] = st.carry + incl - v;
        if (tid == NW - 1) st.carry_next = st.carry + incl;
    }
    __syncthreads();
    const int slot = keep ? st.wave_offset[wave] + before : -1;
    // carry is next read after the first barrier of the following step
    if (tid == 0) st.carry = st.carry_next;
    return slot;
}

// One workgroup of 1024 lanes walks the list 1024 entries at a time, carrying the running
// output offset; the batch sizes of a serving system (up to a few thousand in-flight
// requests per layer) take one to four steps.  The order of survivors is their incoming order.
__global__ __launch_bounds__(1024) void compact_misses_kernel(CompactArgs a) {
    __shared__ CompactState<16> st;
    const int n = active_rows(a.n_dev, a.n_max);   // read before n_miss is written (they may alias)
    const int tid = threadIdx.x;
    if (tid == 0) st.carry = 0;
    for (int base = 0; base < n; base += 1024) {
        const int i = base + tid;
        const bool miss = (i < n) && (a.hit[i] == 0);
        const int slot = compact_step<16>(st, miss, tid);
        if (slot >= 0) a.ids_out[slot] = a.ids_in ? a.ids_in[i] : i;
    }
    if (tid == 0) *a.n_miss = st.carry;
}

// ---------------------------------------------------------------------------------------
// Long lists: two launches over many workgroups instead of one workgroup walking the list.
// The list is cut into `chunks` equal spans of `steps` x 1024 entries; workgroup b owns span b.
//   compact_count_kernel    counts[b] = misses in span b; also records the clamped row count, so
//                           that the second launch never reads n_dev (which n_miss may alias)
//   compact_scatter_kernel  offset of span b = counts[0] + ... + counts[b-1] (every workgroup adds
//                           them up itself: at most 1024 integers), then the same stable
//                           workgroup-wide compaction as above, starting at that offset; the last
//                           workgroup also writes the total.
// No workgroup waits for another one: the launch boundary is the only dependence.
// scratch: kCompactScratchWords int32 of device memory, word 0 = row count, words 1.. = counts.
// ---------------------------------------------------------------------------------------
constexpr int kCompactMaxChunks = 1024;
constexpr int kCompactScratchWords = 1 + kCompactMaxChunks;

struct CompactWideArgs {
    CompactArgs c;
    int32_t* scratch;   // [kCompactScratchWords]
    int steps;          // 1024-entry steps per workgroup
};

__global__ __launch_bounds__(1024) void compact_count_kernel(CompactWideArgs a) {
    __shared__ int wave_total[16];
    const int n = active_rows(a.c.n_dev, a.c.n_max);
    const int tid = threadIdx.x;
    const long first = (long)blockIdx.x * a.steps * 1024;
    int mine = 0;
    for (int s = 0; s < a.steps; ++s) {
        const long i = first + (long)s * 1024 + tid;
        mine += (i < n && a.c.hit[i] == 0) ? 1 : 0;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) mine += __shfl_xor(mine, m, 64);
    if ((tid & 63) == 0) wave_total[tid >> 6] = mine;
    __syncthreads();
    if (tid == 0) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += wave_total[w];
        a.scratch[1 + blockIdx.x] = t;
        if (blockIdx.x == 0) a.scratch[0] = n;
    }
}

__global__ __launch_bounds__(1024) void compact_scatter_kernel(CompactWideArgs a) {
    __shared__ CompactState<16> st;
    __shared__ int wave_total[16];
    const int n = a.scratch[0];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    // misses in the spans before this one (gridDim.x <= 1024: one count per lane)
    int before = (tid < b) ? a.scratch[1 + tid] : 0;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) before += __shfl_xor(before, m, 64);
    if ((tid & 63) == 0) wave_total[tid >> 6] = before;
    __syncthreads();
    if (tid == 0) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += wave_total[w];
        st.carry = t;
    }
    const long first = (long)b * a.steps * 1024;
    for (int s = 0; s < a.steps; ++s) {
        const long i = first + (long)s * 1024 + tid;
        const bool miss = (i < n) && (a.c.hit[i] == 0);
        const int slot = compact_step<16>(st, miss, tid);      // its first barrier publishes st.carry
        if (slot >= 0) a.c.ids_out[slot] = a.c.ids_in ? a.c.ids_in[i] : (int32_t)i;
    }
    if (b == (int)gridDim.x - 1 && tid == 0) *a.c.n_miss = st.carry;
}

}  // namespace gati
