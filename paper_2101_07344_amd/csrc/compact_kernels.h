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

// One workgroup of 1024 lanes walks the list 1024 entries at a time, carrying the running
// output offset; the batch sizes of a serving system (up to a few thousand in-flight
// requests per layer) take one to four steps.  The order of survivors is their incoming order.
__global__ __launch_bounds__(1024) void compact_misses_kernel(CompactArgs a) {
    __shared__ int wave_total[16];
    __shared__ int wave_offset[16];
    __shared__ int carry, carry_next;
    const int n = active_rows(a.n_dev, a.n_max);   // read before n_miss is written (they may alias)
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;

    for (int base = 0; base < n; base += 1024) {
        const int i = base + tid;
        const bool miss = (i < n) && (a.hit[i] == 0);
        const unsigned long long mask = __ballot(miss);
        const int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_total[wave] = __popcll(mask);
        __syncthreads();
        if (tid < 16) {
            // exclusive scan of the 16 wave totals by the first 16 lanes of wave 0
            const int v = wave_total[tid];
            int incl = v;
#pragma unroll
            for (int d = 1; d < 16; d <<= 1) {
                const int o = __shfl_up(incl, d, 64);
                if (tid >= d) incl += o;
            }
            wave_offset[tid] = carry + incl - v;
            if (tid == 15) carry_next = carry + incl;
        }
        __syncthreads();
        if (miss) a.ids_out[wave_offset[wave] + before] = a.ids_in ? a.ids_in[i] : i;
        // carry is next read after the first barrier of the following step
        if (tid == 0) carry = carry_next;
    }
    if (tid == 0) *a.n_miss = carry;
}

}  // namespace gati
