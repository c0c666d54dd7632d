// Conv(k,s) with few filters (Section 3, table of predictor architectures; the paper's convolution
// predictors have a handful of filters) on channel-major bf16 maps, formulated over INPUT rows so that
// the map is used exactly as it lies in memory -- no transposition on the way into LDS:
//
//   for an input row iy of channel c, P[t][o][x] = sum_dx W[o][c][dy_t][dx] * X[c][iy][s*x + dx]
//   is what that row adds to output row y = (iy - dy_t) / s, where dy_t = (iy mod s) + s*t are the
//   k/s taps (rounded up) whose row offset has the parity of iy.
//
// As one MFMA (32 x 32 x 16, bf16): the 32 rows of D are (t, o) -- up to 4 tap rows x 8 filters --
// its 32 columns are output pixels x of one or several input rows (a "tile"), and the reduction
// index is (channel, dx): SLOT = 8 horizontal taps of 2 channels, or SLOT = 4 taps of 4 channels.
// A lane's B fragment is then SLOT consecutive elements of an input row starting at s*x: one
// LDS read of bytes that were copied from global memory unchanged.  Taps past k meet zero weights.
// The filters are repacked at cache creation into A fragments per (channel group, row parity).
// A tile's accumulators stay in registers over all channels; since D's row index lives in the
// register number (t = j / 4), a tap row's share is a group of four registers, and the shares
// are added into the output rows through LDS at the end, in the fixed order of dy.
//
// One workgroup = one request -- or 2 on small maps, whose tiles then share every filter
// fragment that is fetched -- (x one share of the channels when few requests would leave CUs
// idle: the shares are summed in order by conv_reduce_kernel).  Its 8 waves split into row
// parities (s = 2), then into tile sets, then -- small maps, fewer tiles than waves -- into channel
// parts.  A fill is CC channels of the map followed by their filter fragments; fills go from global
// memory straight into a ring of LDS slots (global_load_lds: lane l of a wave-wide load lands at
// base + 16*l, counted by vmcnt), three fills ahead of the one being multiplied, so no register
// holds data in transit and ~90 KB per CU are in flight.
#pragma once

#include "conv_kernels.h"

namespace gati {

constexpr int kRowsSlotVec = 2048;       // 32 KB per fill (16-byte vectors)
constexpr int kRowsDepth = 4;            // LDS slots: one being multiplied, three in flight
constexpr int kRowsWaves = 8;            // waves per workgroup: two per SIMD, so one multiplies while the other waits
constexpr int kRowsThreads = kRowsWaves * 64;
constexpr int kRowsLoads = kRowsSlotVec / kRowsThreads;   // wave-wide loads per wave and fill: always this many (surplus
                                                          // ones land in a spare KB), so the wait below can name a count
constexpr int kRowsLdsBytes = kRowsDepth * kRowsSlotVec * 16 + 1024;
constexpr int kRowsFilters = 8;          // filters per MFMA row block
constexpr int kRowsMaxTiles = 7;         // tiles per wave: 7 x 16 accumulators

struct ConvRowsArgs {
    const void* act;           // [rows, C, in_h*in_w] bf16
    const int32_t* row_index;  // [n] or null
    const int32_t* n_dev;
    int n_max;
    int C, S, in_h, in_w, k, s, oh, ow, Co;
    const void* Wr;            // [C / KC][s][64 lanes] x 16 bytes: A fragments, see pack_conv_rows
    const float* bias;
    int rb, ntq;               // requests per workgroup (1 or 2); tiles per row parity of one request
    int CC;                    // channels per fill: CC*S*2 bytes are a multiple of 16
    int xw_log2;               // a tile gives every input row it holds 2^xw_log2 >= ow pixel lanes
    int rs_log2;               // the rows of one tile are 2^rs_log2 apart (among the rows of their parity)
    int nwt_log2, ws;          // waves of one parity: 2^nwt_log2 tile sets x ws channel parts (waves past that only load)
    float* out;                // [n, out_stride] fp32 features, order [filter][oy][ox]
    __bf16* out16;             // bf16 copy or null
    int out_stride;
    int ksplit, fills_per_split;
    float* partial;            // [ksplit][n_max][out_stride] raw sums when ksplit > 1
};

// 16 bytes of LDS at a 4-byte aligned address.
struct __attribute__((packed, aligned(4))) lds_u32x4 { uint32_t w[4]; };

// One wave-wide load of 64 x 16 bytes from global memory (base + the lane's byte offset) straight into LDS:
// lane l lands at dst + 16*l; dst is wave-uniform and travels in M0.  Written as assembly so that the compiler
// does not order every later LDS read behind it (it would wait for ALL outstanding loads before the first
// fragment read of a fill); the kernel waits by count instead (wait_loads), and barriers separate a slot's
// writers and readers.
__device__ __forceinline__ void lds_direct_load(const void* base, uint32_t lane_off, void* dst) {
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)dst);
    const uint64_t b = (uint64_t)(uintptr_t)base;
    // (the builtin returns a signed int: without the casts the low half would sign-extend into the high one)
    const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32) |
                        (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(m0), "v"(lane_off), "s"(sb) : "memory");
}
// Wait until at most N of this wave's vector-memory loads are outstanding (they complete in order).
template <int N>
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

// SLOT: horizontal taps per channel in the reduction index (8: stride 2, even row length; 4: k <= 3).
// TPW: tiles per wave.
template <int SLOT, int TPW>
__global__ __launch_bounds__(kRowsThreads) void conv_rows_kernel(ConvRowsArgs a) {
    using frag_t = Mma<true>::frag_t;
    constexpr int KC = 16 / SLOT;                            // channels per MFMA
    constexpr int UG = TPW >= 4 ? 1 : (TPW == 2 ? 2 : 4);    // channel groups whose fragments are in flight per wave
    constexpr int D = kRowsDepth, QF = kRowsLoads, NW = kRowsWaves, NT = kRowsThreads;
    extern __shared__ __align__(16) unsigned char rows_lds[];    // D slots, then the spare KB

    const int n = active_rows(a.n_dev, a.n_max);
    const int split = blockIdx.x % a.ksplit;
    const int i0 = (blockIdx.x / a.ksplit) * a.rb;           // first of this workgroup's requests
    if (i0 >= n) return;                                     // whole workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: what follows from it stays in scalar registers
    const int nn = lane & 31, kb = lane >> 5;

    // wave -> (row parity, tile set, channel part)
    const int pi = wave % a.s;
    const int wc = wave / a.s;
    const int wt = wc & ((1 << a.nwt_log2) - 1);
    const int wp = wc >> a.nwt_log2;
    // lane -> (input row within the tile, output column)
    const int xs = nn & ((1 << a.xw_log2) - 1), jrow = nn >> a.xw_log2;
    const int x = min(xs, a.ow - 1);
    const int rpt_log2 = 5 - a.xw_log2;

    const int nva = a.CC * a.S * 2 / 16;                     // vectors of one request's part of a fill
    const int ca = (nva + 63) >> 6;                          // ... in whole KB
    int iy[TPW];                                             // the lane's input row per tile; past the map: unused
    int tq[TPW];                                             // the tile's request among the workgroup's
    int boff[TPW][SLOT == 8 ? 1 : 2];                        // LDS byte offset of the lane's fragment in channel group 0
    int bsh[TPW][SLOT == 8 ? 1 : 2];                         // SLOT 4: 16 when the fragment starts on an odd element
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        // tile tau holds the rows rho = block*RS*rpt + i + RS*j (block = tau / RS, i = tau % RS, j < rpt): the
        // rows of a tile are RS apart, which the plan picks so that they fall on different LDS banks
        const int tall = wt + (t << a.nwt_log2);             // tile among those of all the workgroup's requests
        const int q = min(tall / a.ntq, a.rb - 1);
        const int tau = tall - q * a.ntq;                    // a surplus tile (past the last request's) lands past the map
        const int rho = ((tau >> a.rs_log2) << (a.rs_log2 + rpt_log2)) + (tau & ((1 << a.rs_log2) - 1)) + (jrow << a.rs_log2);
        tq[t] = q;
        iy[t] = i0 + q < n ? pi + a.s * rho : a.in_h;        // a request past n: every row "past the map"
        const int e0 = min(pi + a.s * rho, a.in_h - 1) * a.in_w + a.s * x;
        const int part = q * ca * 1024;                      // the request's part of the fill
        if constexpr (SLOT == 8) {
            boff[t][0] = part + (kb * a.S + e0) * 2;         // even element by plan: 4-byte aligned
            bsh[t][0] = 0;
        } else {
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int e = (2 * kb + g) * a.S + e0;
                boff[t][g] = part + (e >> 1) * 4;
                bsh[t][g] = (e & 1) * 16;
            }
        }
    }
    const int gbytes = KC * a.S * 2;                         // one channel group further on
    auto bfrag = [&](const unsigned char* slot, int t, int cg) -> frag_t {
        const unsigned char* p = slot + cg * gbytes;
        u32x4_t w;
        if constexpr (SLOT == 8) {
            const lds_u32x4 v = *reinterpret_cast<const lds_u32x4*>(p + boff[t][0]);
            w[0] = v.w[0]; w[1] = v.w[1]; w[2] = v.w[2]; w[3] = v.w[3];
        } else {
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const uint32_t* q = reinterpret_cast<const uint32_t*>(p + boff[t][g]);
                const uint32_t d0 = q[0], d1 = q[1];
                w[2 * g] = __builtin_amdgcn_alignbit(d1, d0, bsh[t][g]);
                w[2 * g + 1] = d1 >> bsh[t][g];
            }
        }
        return __builtin_bit_cast(frag_t, w);
    };

    // One fill: per request CC channels of its map (nva vectors, contiguous in memory, padded to whole KB), then
    // the channels' A fragments (whole KB).  A wave-wide load moves one KB, so every load has one source: one
    // request's map or the fragments; only a map part's last KB may be partial -- its surplus lanes repeat the
    // last vector (the pad they fill is read by the last rows' fragments past the window, against zero weights).
    const int G = a.CC / KC;
    const int cw = G * a.s;                                  // KB of fragments
    const int cm = a.rb * ca;                                // KB of map
    const int chunks = cm + cw;                              // <= kRowsSlotVec / 64 by plan
    const int fill0 = split * a.fills_per_split;
    const int fill1 = min(a.C / a.CC, fill0 + a.fills_per_split);
    unsigned char* const spare = rows_lds + D * kRowsSlotVec * 16;
    const uint32_t off_full = lane * 16;
    const uint32_t off_tail = min(lane, nva - 1 - (ca - 1) * 64) * 16;
    // This wave's QF loads of a fill, the same for every fill: which KB, of which request's map or of the
    // fragments, as a base address and a step from one fill to the next
    const unsigned char* l_base[QF];
    int l_step[QF], l_dst[QF];
    uint32_t l_off[QF];
    bool l_live[QF];
#pragma unroll
    for (int q = 0; q < QF; ++q) {
        const int c = min(wave + NW * q, chunks - 1);        // wave-uniform
        const bool is_w = c >= cm;
        const int part = min(c / ca, a.rb - 1), cq = c - part * ca;
        const int iq = min(i0 + part, n - 1);                // a request past n: the last one again, computed and dropped
        const long row = a.row_index ? (long)a.row_index[iq] : (long)iq;
        l_base[q] = is_w ? static_cast<const unsigned char*>(a.Wr) + (long)(c - cm) * 1024
                         : static_cast<const unsigned char*>(a.act) + row * a.C * a.S * 2 + (long)cq * 1024;
        l_step[q] = is_w ? cw * 1024 : nva * 16;
        l_dst[q] = c * 1024;
        l_live[q] = wave + NW * q < chunks;
        l_off[q] = (!is_w && cq == ca - 1) ? off_tail : off_full;
    }
    // Fill `f` into slot `slot`.  Always QF loads per wave: KBs past the fill, and whole fills past the last
    // one, re-read valid vectors into the spare KB.
    auto issue = [&](int f, int slot) {
        const bool live = f < fill1;
        const int fc = min(f, fill1 - 1);
        unsigned char* sb = rows_lds + slot * (kRowsSlotVec * 16);
#pragma unroll
        for (int q = 0; q < QF; ++q)
            lds_direct_load(l_base[q] + (long)fc * l_step[q], l_off[q], (live && l_live[q]) ? sb + l_dst[q] : spare);
    };

    f32x16_t acc[TPW];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][j] = 0.f;

    // The multiplication is one stream of rounds (UG channel groups x TPW tiles) over all fills: every fragment is
    // read one round ahead of its MFMA, the last round of a fill reads the first groups of the NEXT fill.  Before
    // that round the wave makes sure the next fill has landed (its own loads by count, everyone's by the
    // barrier); past the barrier nobody reads the current slot any more, so the fill D ahead goes there.
    const int rounds = G / a.ws / UG;                        // rounds per wave and fill: whole by plan
    const bool active = wp < a.ws;                           // a wave without a channel part (few channels) only loads
    frag_t bf[UG][TPW], af[UG];
    auto preload = [&](const unsigned char* slot) {
        const unsigned char* const alds = slot + cm * 1024 + (pi * 64 + lane) * 16;
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            const int cg = wp + u * a.ws;
            af[u] = *reinterpret_cast<const frag_t*>(alds + cg * a.s * 1024);
#pragma unroll
            for (int t = 0; t < TPW; ++t) bf[u][t] = bfrag(slot, t, cg);
        }
    };
    // multiply what the ring holds, refill it with round `rd` of the fill in `slot`
    auto round = [&](const unsigned char* slot, int rd) {
        const unsigned char* const alds = slot + cm * 1024 + (pi * 64 + lane) * 16;
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            const int cgn = wp + (rd * UG + u) * a.ws;
            const frag_t an = *reinterpret_cast<const frag_t*>(alds + cgn * a.s * 1024);
            __builtin_amdgcn_sched_barrier(0);               // keep this read ahead of the MFMAs that hide it
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                acc[t] = Mma<true>::mma(af[u], bf[u][t], acc[t]);
                bf[u][t] = bfrag(slot, t, cgn);
            }
            af[u] = an;
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) issue(fill0 + d, d);
    wait_loads<(D - 1) * QF>();                              // the first fill
    __syncthreads();
    if (active) preload(rows_lds);
    int cur = 0;
    for (int f = fill0; f < fill1; ++f) {
        const unsigned char* slot = rows_lds + cur * (kRowsSlotVec * 16);
        if (active)
            for (int rd = 1; rd < rounds; ++rd) round(slot, rd);
        wait_loads<(D - 2) * QF>();                          // fill f+1: D-2 younger fills are in flight behind it
        __syncthreads();
        issue(f + D, cur);
        cur = cur + 1 == D ? 0 : cur + 1;
        // past the last fill this reads a slot that holds an older fill: finite data, multiplied by nobody
        if (active) round(rows_lds + cur * (kRowsSlotVec * 16), 0);
    }
    wait_loads<0>();                                         // the surplus loads of the last rounds
    __syncthreads();

    // shares of the tap rows -> output rows, through LDS (the slots are free now), in the order
    // (channel part, dy): within one round no two lanes meet in an output element
    const int OHW = a.oh * a.ow;
    const int F = a.Co * OHW;
    float* const obuf = reinterpret_cast<float*>(rows_lds);  // [request][filter][oy][ox]
    for (int idx = tid; idx < a.rb * F; idx += NT) obuf[idx] = 0.f;
    for (int wpp = 0; wpp < a.ws; ++wpp) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            for (int pp = 0; pp < a.s; ++pp) {
                __syncthreads();
                const int dy = pp + a.s * t;
                if (wp != wpp || pi != pp || dy >= a.k) continue;        // wave-uniform
#pragma unroll
                for (int tl = 0; tl < TPW; ++tl) {
                    const int y = (iy[tl] - dy) / a.s;                   // exact: iy and dy have the same parity
                    if (xs < a.ow && iy[tl] < a.in_h && iy[tl] >= dy && y < a.oh) {
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            const int o = 4 * kb + jj;
                            if (o < a.Co) obuf[tq[tl] * F + o * OHW + y * a.ow + x] += acc[tl][4 * t + jj];
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    // one split: bias and ReLU here; several: raw sums to this split's slab
    const bool last = a.ksplit == 1;
    for (int q = 0; q < a.rb && i0 + q < n; ++q) {
        float* orow = (last ? a.out : a.partial + (long)split * a.n_max * a.out_stride) + (long)(i0 + q) * a.out_stride;
        __bf16* orow16 = (last && a.out16) ? a.out16 + (long)(i0 + q) * a.out_stride : nullptr;
        for (int idx = tid; idx < F; idx += NT) {
            float v = obuf[q * F + idx];
            if (last) v = fmaxf(v + a.bias[idx / OHW], 0.f);
            orow[idx] = v;
            if (orow16) orow16[idx] = (__bf16)v;
        }
    }
}

}  // namespace gati
