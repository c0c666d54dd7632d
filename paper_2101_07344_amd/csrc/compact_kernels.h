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

}  // namespace gati
