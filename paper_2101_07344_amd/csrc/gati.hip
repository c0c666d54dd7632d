// C ABI of the learned-cache lookup library (see include/gati.h): argument checking, the
// cache object (device weights in the kernels' private layout + a per-cache workspace), and
// the choice of kernel variant per shape.  gfx950 only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/gati.h"
#include "common.h"
#include "compact_kernels.h"
#include "conv_kernels.h"
#include "conv_rows_kernels.h"
#include "flat_kernels.h"
#include "head_kernels.h"
#include "pack_kernels.h"
#include "pool_kernels.h"
#include "trainer_view.h"

using namespace gati;

namespace {

enum PoolVariant { POOL_NCS_WAVE = 0, POOL_NCS_SEG = 1, POOL_NSC_VEC = 2, POOL_GENERIC = 3, POOL_NCS_SEGW = 4, POOL_NSC_UNIT = 5,
                   POOL_NCS_ADAPTIVE = 6, POOL_ADAPTIVE_GENERIC = 7, POOL_FC_FLAT = 8, POOL_CONV = 9, POOL_CONV_GENERIC = 10,
                   POOL_FC_FLAT_GENERIC = 11, POOL_CONV_ROWS = 12 };

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace

struct gati_cache {
    gati_cache_desc_t desc;
    int device = 0;
    int num_cu = 256;
    bool bf16 = false;
    int elem = 4;
    bool pool_fc = false;     // no separate hidden-FC kernel: the features feed the output FC (Pool(h), FC(h))
    bool flat_fc = false;     // the paper's FC(h): the features are relu(W1 x + b1) over the flattened row
    // FC(h) plan: wave register tile MT=NT=flat_t, padded sizes, split-K
    int flat_t = 1, Hb = 0, rows_b = 0, flat_KS = 0, flat_splits = 1, flat_ks_per = 0, flat_tiles_m = 0, flat_tiles_n = 0;
    float* flat_partial = nullptr;   // [splits][rows_b][Hb]
    bool flat_generic = false;       // FC(h) rows of a length the MFMA kernels cannot take: W1 kept as stored
    int F = 0;                // features the pooling step produces per row (C, or C*out_h*out_w)
    // padded sizes: Cp % 64 == 0 (Cp pads F) and Hp % 64 == 0 (reduction axes: 4 waves x whole
    // k-steps), Kp % (32*fc2_nt) == 0, rows_pad % 32 == 0
    int Cp = 0, Hp = 0, Kp = 0, rows_pad = 0;
    // device weights, packed in MFMA fragment order (head_kernels.h)
    void* W1 = nullptr;       // [Hp/32][Cp/kStep][64][kLane] bf16 | f32
    void* W2 = nullptr;       // [Kp/32][Hp/kStep][64][kLane] bf16 | f32
    float* b1 = nullptr;      // [Hp]
    float* b2 = nullptr;      // [Kp]
    float* ws_pool = nullptr; // [Cp]
    float* ws_prob = nullptr; // [Kp]
    float bs = 0.f, tau = 0.5f;
    // workspace
    float* p = nullptr;       // [rows_pad, Cp] pooled features, fp32
    void* p16 = nullptr;      // [rows_pad, Cp] the same rounded to bf16 (bf16 caches only)
    void* h = nullptr;        // [rows_pad, Hp]
    float* u_pool = nullptr;  // [rows_pad]
    TileStat* stats = nullptr; // [rows_pad, Kp/(32*fc2_nt)]
    // pooling plan
    PoolVariant variant = POOL_GENERIC;
    int vpc = 0;              // ncs_wave: 16-byte vectors per channel
    int wave_cfg = 0;         // ncs_wave: index into the (LPC, CPI) table
    int gt = 0, tiles_per_row = 0, tpc_log2 = 0;  // ncs_seg
    unsigned magic_S = 0;
    int gw = 64, cvb_per_row = 0;                 // nsc_vec
    AdaptiveWindow* ad_win = nullptr;   // ncs_adaptive: [gt * out_h * out_w] window table
    int ad_j = 4, ad_tpo_log2 = 0, ad_ww = 0, ad_pair = 0;   // ncs_adaptive (tile in gt / tiles_per_row; common window width or 0; LDS read mode)
    int pool_blocks_per_cu = 16;  // persistent grid = CUs x this (more blocks than fit: finer tail balance)
    // head plan: column tiles per workgroup of the output layer
    int fc2_nt = 1;
    // selector with a hidden layer: Hs units (padded Hsp), operand rows [features(Cp) ; prob] of width Sin
    int Hs = 0, Hsp = 0, Sin = 0;
    void* Ws = nullptr;       // [Hsp/32][Sin/kStep][64][kLane] bf16 | f32
    float* cs = nullptr;      // [Hsp]
    float* vs = nullptr;      // [Hsp]
    void* sel_in = nullptr;   // [rows_pad, Sin]
    void* sel_g = nullptr;    // [rows_pad, Hsp]
    float* zbuf = nullptr;    // [max_rows, K] logits when the caller keeps none
    // Conv(k,s) predictor: Co = desc.H filters; plan of conv_relu_kernel
    bool conv_fc = false;
    int conv_oh = 0, conv_ow = 0, conv_R = 0, conv_nbands = 1, conv_rows_in = 0, conv_whole = 0, conv_tpw = 8, conv_ntc = 1, conv_tr = 0, conv_ksplit = 1, conv_cb_per = 0, conv_bps = 1;
    float* conv_partial = nullptr;   // [ksplit][max_rows][Cp] when ksplit > 1
    // plan of conv_rows_kernel (few filters, bf16, channel-major): taps per channel in the reduction index,
    // tiles per wave, channels per LDS fill, pixel lanes per input row, waves per tile set / channel part
    int rows_slot = 0, rows_tpw = 0, rows_cc = 0, rows_xw_log2 = 0, rows_rs_log2 = 0, rows_nwt_log2 = 0, rows_ws = 1, rows_fills_per = 0, rows_rb = 1, rows_ntq = 1;
    float* W1plain = nullptr; // [Co, C, k, k] fp32 (rounded to bf16 values in bf16 caches)
    // gati_cache_fork: a fork shares its owner's weights, tables and selector scalars and has a workspace of its own
    gati_cache* owner = nullptr;
    int forks = 0;            // live forks of an owner
};

namespace {

void free_all(gati_cache* c) {
    void* workspace[] = {c->p, c->p16, c->h, c->u_pool, c->stats, c->flat_partial, c->sel_in, c->sel_g, c->zbuf,
                         c->conv_partial};
    for (void* q : workspace)
        if (q) (void)hipFree(q);
    if (c->owner) return;      // weights and tables belong to the owner
    void* weights[] = {c->W1, c->W2, c->b1, c->b2, c->ws_pool, c->ws_prob, c->Ws, c->cs, c->vs, c->W1plain, c->ad_win};
    for (void* q : weights)
        if (q) (void)hipFree(q);
}

// where the selector scalars of a cache live: in the cache that owns the weights
inline const gati_cache* weights_of(const gati_cache* c) { return c->owner ? c->owner : c; }

// Device copy of a host array (src == NULL: zeros).  *dst == NULL allocates; otherwise the existing
// allocation of the same size is overwritten (weight replacement).
gati_status_t upload(void** dst, const void* src, size_t bytes) {
    hipError_t e = hipSuccess;
    if (!*dst) {
        e = hipMalloc(dst, bytes);
        if (e != hipSuccess) { *dst = nullptr; (void)hipGetLastError(); return GATI_ERR_OOM; }
    }
    e = src ? hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice) : hipMemset(*dst, 0, bytes);
    if (e != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    return GATI_OK;
}

// Conv(k,s) with at most 8 filters on channel-major bf16 maps: the plan of conv_rows_kernel, or false.
bool plan_conv_rows(gati_cache* c) {
    const gati_cache_desc_t& d = c->desc;
    const int k = d.conv_k, s = d.conv_s, oh = c->conv_oh, ow = c->conv_ow;
    if (!c->bf16 || d.layout != GATI_LAYOUT_NCS || d.H > kRowsFilters) return false;
    if (s != 1 && s != 2) return false;
    int slot;
    if (k <= 3) slot = 4;                                    // a fragment may start on an odd element
    else if (s == 2 && k <= 8 && d.in_w % 2 == 0) slot = 8;  // fragments start on even elements only
    else return false;
    if ((k + s - 1) / s > 4) return false;                   // tap rows of one parity: D has room for 4
    const int KC = 16 / slot;
    if (ow > 32 || (long)d.H * oh * ow * 4 > (long)kRowsSlotVec * 16) return false;
    if (d.C % KC != 0 || ((long)d.C * d.S * 2) % 16 != 0 || (long)d.C * d.S >= (1L << 30)) return false;
    int xw = 0;
    while ((1 << xw) < ow) ++xw;
    const int rpt = 32 >> xw;                                // input rows per tile
    const int nwc = kRowsWaves / s;                          // waves per row parity
    const int rows_c = (d.in_h + s - 1) / s;                 // rows of parity 0, the larger class
    // several rows per tile: how far apart (1, 2 or 4 rows of the parity) they should be so that the first
    // dwords of the 32 pixel lanes' fragments fall on as many different LDS banks as possible
    int rs_log2 = 0;
    if (rpt > 1) {
        int best = 1 << 30;
        for (int cand = 0; cand <= 2; ++cand) {
            int per_bank[32] = {0}, worst = 0;
            for (int j = 0; j < rpt; ++j)
                for (int xx = 0; xx < std::min(ow, 32 / rpt); ++xx) {
                    const int dword = ((j << cand) * s * d.in_w + s * xx) / 2;
                    worst = std::max(worst, ++per_bank[dword & 31]);
                }
            if (worst < best) { best = worst; rs_log2 = cand; }
        }
    }
    const int rs = 1 << rs_log2;
    const int ntc = (rows_c + rs * rpt - 1) / (rs * rpt) * rs;   // tiles per parity
    // Requests per workgroup: the filter fragments of a fill are fetched once per workgroup (from L2, but through
    // the same path as the map, which takes ~24 GB/s per CU whatever it carries), so on small maps, where they
    // are a sizeable share of a fill, 2 requests share them (4 were measured too: slower on the 7 x 7 maps, where
    // the gain should have been largest, 1475 -> 866 GB/s: the fills get too small).
    const long map_bytes = (long)d.S * 2 * KC, frag_bytes = (long)s * 1024;      // per channel group and request
    for (int rb : {2, 1}) {
        if (rb == 2 && 4 * frag_bytes < map_bytes) continue;
        if (rb > 1 && d.max_rows < 2 * rb) continue;
        const int tiles = rb * ntc;                              // tiles per parity of one workgroup
        int nwt_log2 = 0;
        while ((2 << nwt_log2) <= std::min(nwc, tiles)) ++nwt_log2;
        const int nwt = 1 << nwt_log2;
        const int need = (tiles + nwt - 1) / nwt;
        int tpw = 0;
        for (int cand : {1, 2, 4, kRowsMaxTiles})
            if (cand >= need) { tpw = cand; break; }
        if (!tpw || (slot == 4 && tpw > 4)) continue;           // 7 tiles of two-part fragments do not fit the registers
        const int ug = tpw >= 4 ? 1 : (tpw == 2 ? 2 : 4);
        // channels per fill: whole 16-byte vectors, whole rounds of every wave, a divisor of C; the requests' map
        // parts (each rounded up to whole KB) and the fill's filter fragments share one LDS slot.  Waves left over
        // once the tiles are dealt out split the channels of a fill, as far as C has channels for them.
        int ws = nwc / nwt, cc = 0;
        for (; ws >= 1 && !cc; ws /= 2) {
            int unit = KC * ws * ug;
            while (((long)unit * d.S * 2) % 16 != 0) unit *= 2;
            for (int cand = unit; cand <= d.C; cand += unit) {
                if (d.C % cand != 0) continue;
                if ((long)rb * round_up((int)((long)cand * d.S * 2), 1024) + (long)(cand / KC) * s * 1024 > (long)kRowsSlotVec * 16) break;
                cc = cand;
            }
            if (cc) break;
        }
        if (!cc || (long)rb * d.H * oh * ow * 4 > (long)kRowsDepth * kRowsSlotVec * 16) continue;
        const int fills = d.C / cc;
        // few workgroups: share the channels of a request among several (fixed at creation, so results do not
        // depend on how many rows a call has)
        const long groups = (d.max_rows + rb - 1) / rb;
        int ks = (int)((2L * c->num_cu + groups - 1) / groups);
        if (rb > 1) ks = 1;
        ks = std::max(1, std::min(std::min(ks, fills), 16));
        c->rows_fills_per = (fills + ks - 1) / ks;
        c->conv_ksplit = (fills + c->rows_fills_per - 1) / c->rows_fills_per;
        c->rows_slot = slot; c->rows_tpw = tpw; c->rows_cc = cc; c->rows_xw_log2 = xw; c->rows_rs_log2 = rs_log2;
        c->rows_nwt_log2 = nwt_log2; c->rows_ws = ws; c->rows_rb = rb; c->rows_ntq = ntc;
        return true;
    }
    return false;
}

typedef void (*conv_rows_fn)(ConvRowsArgs);
conv_rows_fn conv_rows_instance(int slot, int tpw) {
    switch (slot * 16 + tpw) {
    case 8 * 16 + 1: return conv_rows_kernel<8, 1>;
    case 8 * 16 + 2: return conv_rows_kernel<8, 2>;
    case 8 * 16 + 4: return conv_rows_kernel<8, 4>;
    case 8 * 16 + 7: return conv_rows_kernel<8, 7>;
    case 4 * 16 + 1: return conv_rows_kernel<4, 1>;
    case 4 * 16 + 2: return conv_rows_kernel<4, 2>;
    default: return conv_rows_kernel<4, 4>;
    }
}

// Conv(k,s): staging mode and band height of conv_relu_kernel, or the generic kernel.
void plan_conv(gati_cache* c) {
    const gati_cache_desc_t& d = c->desc;
    const int k_step = c->bf16 ? 16 : 8;
    const int oh = c->conv_oh, ow = c->conv_ow;
    c->variant = POOL_CONV_GENERIC;
    if (d.layout == GATI_LAYOUT_NSC) return;      // channels-last maps: the generic kernel
    if (plan_conv_rows(c)) { c->variant = POOL_CONV_ROWS; return; }
    c->conv_ntc = d.H > 32 ? 2 : 1;
    const int max_pixels = c->conv_ntc == 2 ? 512 : 1024;   // 4 waves x TPW tiles x 32 pixels
    c->conv_tpw = c->conv_ntc == 2 ? 4 : 8;
    if (d.C % k_step != 0 || ((long)d.C * d.S * c->elem) % 16 != 0) return;
    if (d.S <= 1024) {
        // small map: the whole planes of a channel block are staged; bands only split the output rows
        c->conv_whole = 1;
        c->conv_rows_in = d.in_h;
        c->conv_R = std::min(oh, std::max(1, max_pixels / ow));
        if (ow > max_pixels) return;
    } else {
        if ((d.in_w * c->elem) % 16 != 0 || ((long)d.S * c->elem) % 16 != 0) return;
        int R = std::min(oh, max_pixels / ow);
        while (R >= 1 && (long)((R - 1) * d.conv_s + d.conv_k) * d.in_w > 1024) --R;
        if (R < 1) return;
        c->conv_whole = 0;
        c->conv_R = R;
        c->conv_rows_in = (R - 1) * d.conv_s + d.conv_k;
    }
    c->conv_nbands = (oh + c->conv_R - 1) / c->conv_R;
    // 32-pixel tiles per wave: the smallest of 1, 2, 4, 8 that covers the tallest band
    const int tiles = (c->conv_R * ow + 31) / 32;
    int tpw = 1;
    while (tpw * 4 < tiles) tpw *= 2;
    c->conv_tpw = tpw;
    // bf16 maps whose 8-position chunks are 16-byte aligned in every channel: transposed staging
    c->conv_tr = (c->bf16 && d.S % 8 == 0 && (c->conv_whole || d.in_w % 8 == 0)) ? 1 : 0;
    // a workgroup walks its channel blocks one after another: when max_rows x bands gives fewer than
    // ~4 workgroups per CU, split the blocks over several (fixed at creation, so results do not
    // depend on how many rows a call has)
    const int CB = d.C / k_step;
    const long wgs = (long)d.max_rows * c->conv_nbands;
    int ks = (int)((4L * c->num_cu + wgs - 1) / wgs);
    if (wgs < 8L * c->num_cu) ks = std::max(ks, CB / 8);     // and keep a workgroup's chain to ~8 blocks
    ks = std::max(1, std::min(std::min(ks, CB / 2), 16));
    c->conv_cb_per = (CB + ks - 1) / ks;
    c->conv_ksplit = (CB + c->conv_cb_per - 1) / c->conv_cb_per;
    // small maps copied as they lie: as many channel blocks per LDS fill as the 32 KB buffer holds
    c->conv_bps = (c->conv_whole && !c->conv_tr) ? std::max(1, std::min(c->conv_cb_per, 1024 / d.S)) : 1;
    c->variant = POOL_CONV;
}

template <bool BF16>
hipError_t launch_conv_t(const gati_cache* c, const void* act, const int32_t* row_index, int n_max,
                         const int32_t* n_dev, float* out, void* out16, int out_stride, hipStream_t st) {
    const gati_cache_desc_t& d = c->desc;
    ConvArgs a;
    a.act = act; a.row_index = row_index; a.n_dev = n_dev; a.n_max = n_max;
    a.C = d.C; a.S = d.S; a.in_h = d.in_h; a.in_w = d.in_w; a.k = d.conv_k; a.s = d.conv_s;
    a.oh = c->conv_oh; a.ow = c->conv_ow; a.Co = d.H;
    a.Wp = c->W1; a.Wplain = c->W1plain; a.bias = c->b1;
    a.CB = d.C / (BF16 ? 16 : 8);
    a.R = c->conv_R; a.nbands = c->conv_nbands; a.rows_in = c->conv_rows_in; a.whole = c->conv_whole;
    a.out = out; a.out16 = static_cast<__bf16*>(out16); a.out_stride = out_stride;
    a.ksplit = 1; a.cb_per_split = a.CB; a.partial = nullptr; a.bps = c->conv_bps;
    if (n_max == 0) return hipSuccess;
    if (c->variant == POOL_CONV_ROWS && (reinterpret_cast<uintptr_t>(act) & 15u) == 0) {
        if constexpr (BF16) {
            ConvRowsArgs ra;
            ra.act = act; ra.row_index = row_index; ra.n_dev = n_dev; ra.n_max = n_max;
            ra.C = d.C; ra.S = d.S; ra.in_h = d.in_h; ra.in_w = d.in_w; ra.k = d.conv_k; ra.s = d.conv_s;
            ra.oh = c->conv_oh; ra.ow = c->conv_ow; ra.Co = d.H;
            ra.Wr = c->W1; ra.bias = c->b1; ra.CC = c->rows_cc; ra.xw_log2 = c->rows_xw_log2; ra.rs_log2 = c->rows_rs_log2;
            ra.rb = c->rows_rb; ra.ntq = c->rows_ntq;
            ra.nwt_log2 = c->rows_nwt_log2; ra.ws = c->rows_ws;
            ra.out = out; ra.out16 = static_cast<__bf16*>(out16); ra.out_stride = out_stride;
            ra.ksplit = 1; ra.fills_per_split = d.C / c->rows_cc; ra.partial = nullptr;
            if (c->conv_ksplit > 1 && out_stride <= c->Cp) {
                ra.ksplit = c->conv_ksplit; ra.fills_per_split = c->rows_fills_per; ra.partial = c->conv_partial;
            }
            const int grid = (n_max + ra.rb - 1) / ra.rb * ra.ksplit;
            conv_rows_instance(c->rows_slot, c->rows_tpw)<<<grid, kRowsThreads, kRowsLdsBytes, st>>>(ra);
            if (ra.ksplit > 1) {
                hipError_t e = hipGetLastError();
                if (e != hipSuccess) return e;
                a.ksplit = ra.ksplit; a.partial = ra.partial;
                const long items = (long)n_max * c->F;
                conv_reduce_kernel<<<(int)std::min<long>((items + 255) / 256, (long)c->num_cu * 8), 256, 0, st>>>(a);
            }
        }
    } else if (c->variant != POOL_CONV || (reinterpret_cast<uintptr_t>(act) & 15u) != 0) {
        const long items = (long)n_max * c->F;
        const int blocks = (int)std::min<long>((items + 255) / 256, (long)c->num_cu * 16);
        conv_generic_kernel<BF16><<<blocks, 256, 0, st>>>(a, d.layout == GATI_LAYOUT_NSC ? 1 : 0);
    } else {
        // the split slabs are laid out for out_stride == Cp (the cache's own feature buffer and
        // gati_cache_pool's F-wide output both fit: out_stride <= Cp)
        if (c->conv_ksplit > 1 && out_stride <= c->Cp) {
            a.ksplit = c->conv_ksplit; a.cb_per_split = c->conv_cb_per; a.partial = c->conv_partial;
        }
        const int grid = n_max * c->conv_nbands * a.ksplit;
        const int key = c->conv_ntc * 16 + c->conv_tpw;
#define GATI_CONV(TRV)                                                                        \
    switch (key) {                                                                            \
    case 16 + 1: conv_relu_kernel<BF16, 1, 1, TRV><<<grid, 256, 0, st>>>(a); break;           \
    case 16 + 2: conv_relu_kernel<BF16, 2, 1, TRV><<<grid, 256, 0, st>>>(a); break;           \
    case 16 + 4: conv_relu_kernel<BF16, 4, 1, TRV><<<grid, 256, 0, st>>>(a); break;           \
    case 16 + 8: conv_relu_kernel<BF16, 8, 1, TRV><<<grid, 256, 0, st>>>(a); break;           \
    case 32 + 1: conv_relu_kernel<BF16, 1, 2, TRV><<<grid, 256, 0, st>>>(a); break;           \
    case 32 + 2: conv_relu_kernel<BF16, 2, 2, TRV><<<grid, 256, 0, st>>>(a); break;           \
    default: conv_relu_kernel<BF16, 4, 2, TRV><<<grid, 256, 0, st>>>(a); break;               \
    }
        if constexpr (BF16) {
            if (c->conv_tr) { GATI_CONV(true) } else { GATI_CONV(false) }
        } else {
            GATI_CONV(false)
        }
#undef GATI_CONV
        if (a.ksplit > 1) {
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            const long items = (long)n_max * c->F;
            conv_reduce_kernel<<<(int)std::min<long>((items + 255) / 256, (long)c->num_cu * 8), 256, 0, st>>>(a);
        }
    }
    return hipGetLastError();
}

// Pick the pooling kernel for a shape.  Everything the vector kernels assume is checked here.
void plan_pool(gati_cache* c) {
    const int C = c->desc.C, S = c->desc.S;
    const int V = 16 / c->elem;
    c->variant = POOL_GENERIC;
    if (c->pool_fc) {
        c->variant = POOL_ADAPTIVE_GENERIC;
        if (c->desc.layout == GATI_LAYOUT_NCS && S >= V && ((long)C * S) % V == 0) {
            int g0 = 1;
            while (((long)g0 * S) % V != 0) ++g0;
            const long vec0 = (long)g0 * S / V;            // vectors of the smallest aligned tile
            const int J = vec0 <= 256 ? 4 : vec0 <= 512 ? 8 : vec0 <= 1024 ? 16 : 0;
            if (J) {
                const int max_mult = (int)((64L * J) / vec0);
                int mult = max_mult;
                for (int m = max_mult; m >= (max_mult + 1) / 2; --m)
                    if (C % (m * g0) == 0) { mult = m; break; }
                int gt = mult * g0;
                if (gt > C) gt = round_up(C, g0);
                c->gt = gt;
                c->tiles_per_row = (C + gt - 1) / gt;
                c->ad_j = J;
                // lanes per output window: split the window's rows when windows are big
                const int win_rows = (c->desc.in_h + c->desc.out_h - 1) / c->desc.out_h;
                const int win_cols = (c->desc.in_w + c->desc.out_w - 1) / c->desc.out_w;
                int t = 0;
                while (win_rows * win_cols > 16 && (2 << t) <= win_rows && t < 3) ++t;
                c->ad_tpo_log2 = t;
                // a window width shared by every window lets the kernel unroll a window row
                int ww = -1;
                for (int ox = 0; ox < c->desc.out_w; ++ox) {
                    const int x0 = (ox * c->desc.in_w) / c->desc.out_w;
                    const int x1 = ((ox + 1) * c->desc.in_w + c->desc.out_w - 1) / c->desc.out_w;
                    ww = (ww == -1 || ww == x1 - x0) ? x1 - x0 : 0;
                }
                c->ad_ww = (ww == 4 || ww == 7 || ww == 14) ? ww : 0;
                // bf16 LDS read mode of the kernel: aligned pairs for the 14-wide windows of an even map
                // that out_w divides (row starts 14*ox + even), offset pairs for the narrow ones
                c->ad_pair = 0;
                if (c->bf16 && c->ad_ww == 14 && c->desc.in_w % 2 == 0 && S % 2 == 0 && c->desc.in_w % c->desc.out_w == 0)
                    c->ad_pair = 1;
                else if (c->bf16 && c->ad_ww > 0)
                    c->ad_pair = 2;
                c->variant = POOL_NCS_ADAPTIVE;
            }
        }
        return;
    }
    if (c->desc.layout == GATI_LAYOUT_NSC) {
        if (C % V == 0) {
            const int CV = C / V;
            // widest lane group that wastes the fewest lanes on the last channel block
            int best = 64, best_waste = round_up(CV, 64) - CV;
            for (int gw : {32, 16}) {
                const int waste = round_up(CV, gw) - CV;
                if (waste < best_waste) { best = gw; best_waste = waste; }
            }
            c->gw = best;
            c->cvb_per_row = (CV + best - 1) / best;
            c->variant = POOL_NSC_VEC;
            // many tokens: one wave per (row, block of channel vectors) walks all of them
            if (S >= 32) {
                c->gw = (CV % 32 == 0 || CV > 48) ? 32 : 16;
                c->cvb_per_row = (CV + c->gw - 1) / c->gw;
                c->variant = POOL_NSC_UNIT;
            }
        }
        return;
    }
    // [n,C,S]
    if ((long)S * c->elem % 16 == 0 && S / V >= 32) {
        c->vpc = S / V;
        const int lpc = (c->vpc + 63) / 64;
        // (LPC, CPI) table index: 0:(1,8) 1:(2,4) 2:(4,2) 3:(8,2) 4:(16,1)
        c->wave_cfg = lpc <= 1 ? 0 : lpc <= 2 ? 1 : lpc <= 4 ? 2 : lpc <= 8 ? 3 : 4;
        c->variant = POOL_NCS_WAVE;
        return;
    }
    if (S >= V && ((long)C * S) % V == 0 && (long)S < 65536) {
        // smallest channel count whose byte size is a multiple of 16
        int g0 = 1;
        while (((long)g0 * S) % V != 0) ++g0;
        c->magic_S = (unsigned)(((1ull << 32) / (unsigned long long)S) + 1ull);
        // wave-granular tiles: at most 256 vectors and 64 channels per wave
        {
            int max_mult = (int)((256L * V) / ((long)g0 * S));
            if (max_mult * g0 > 64) max_mult = 64 / g0;
            if (max_mult >= 1) {
                int mult = max_mult;
                for (int m = max_mult; m >= (max_mult + 1) / 2; --m)
                    if (C % (m * g0) == 0) { mult = m; break; }
                int gt = mult * g0;
                if (gt > C) gt = round_up(C, g0);
                c->gt = gt;
                c->tiles_per_row = (C + gt - 1) / gt;
                int tpc_log2 = 0;
                const int partials = (S + V - 1) / V + 1;
                while ((gt << (tpc_log2 + 1)) <= 64 && (2 << tpc_log2) <= partials / 2) ++tpc_log2;
                c->tpc_log2 = tpc_log2;
                c->variant = POOL_NCS_SEGW;
                return;
            }
        }
        const int max_mult = (int)((1024L * V) / ((long)g0 * S));   // tile <= 1024 vectors
        if (max_mult >= 1) {
            int mult = max_mult;
            for (int m = max_mult; m >= (max_mult + 1) / 2; --m)
                if (C % (m * g0) == 0) { mult = m; break; }
            int gt = mult * g0;
            if (gt > 256) gt = 256 / g0 * g0;
            if (gt >= g0 && gt > 0) {
                if (gt > C) gt = round_up(C, g0);   // C*S % V == 0 makes C a multiple of g0
                c->gt = gt;
                c->tiles_per_row = (C + gt - 1) / gt;
                int tpc_log2 = 0;
                const int partials = (S + V - 1) / V + 1;
                while ((gt << (tpc_log2 + 1)) <= 256 && (2 << tpc_log2) <= partials / 2 && tpc_log2 < 6)
                    ++tpc_log2;
                c->tpc_log2 = tpc_log2;
                c->magic_S = (unsigned)(((1ull << 32) / (unsigned long long)S) + 1ull);
                c->variant = POOL_NCS_SEG;
            }
        }
    }
}

// Weights [rows, cols] (row-major, fp32, host) -> MFMA fragment order, zero padded to
// [rows_p, cols_p]; element type bf16 (nearest even) or fp32.
template <typename T, typename Conv>
void pack_weights(const float* W, int rows, int cols, int rows_p, int cols_p, int k_step, std::vector<T>& out,
                  Conv conv) {
    const int k_lane = k_step / 2, KS = cols_p / k_step;
    out.assign((size_t)rows_p * cols_p, conv(0.f));
    for (int nt = 0; nt < rows_p / 32; ++nt)
        for (int ks = 0; ks < KS; ++ks)
            for (int l = 0; l < 64; ++l)
                for (int e = 0; e < k_lane; ++e) {
                    const int row = nt * 32 + (l & 31), col = ks * k_step + (l >> 5) * k_lane + e;
                    if (row < rows && col < cols)
                        out[(((size_t)nt * KS + ks) * 64 + l) * k_lane + e] = conv(W[(size_t)row * cols + col]);
                }
}

// W1 of the FC(h) predictor: as pack_weights, but within every block of 4 k-steps lane half kb
// owns 2*k_step consecutive inputs (see flat_kernels.h): fragment (nt, ks, lane, e) holds
// W[nt*32 + lane%32][(ks/4)*4*k_step + (lane/32)*2*k_step + (ks%4)*k_lane + e].
template <typename T, typename Conv>
void pack_weights_flat(const float* W, int rows, long cols, int rows_p, int k_step, std::vector<T>& out, Conv conv) {
    const int k_lane = k_step / 2;
    const long KS = cols / k_step;
    out.assign((size_t)rows_p * cols, conv(0.f));
    for (int nt = 0; nt < rows_p / 32; ++nt)
        for (long ks = 0; ks < KS; ++ks)
            for (int l = 0; l < 64; ++l) {
                const int row = nt * 32 + (l & 31);
                if (row >= rows) continue;
                const long col0 = (ks >> 2) * 4 * k_step + (long)(l >> 5) * 2 * k_step + (ks & 3) * k_lane;
                T* dst = &out[(((size_t)nt * KS + ks) * 64 + l) * k_lane];
                const float* src = &W[(size_t)row * cols + col0];
                for (int e = 0; e < k_lane; ++e) dst[e] = conv(src[e]);
            }
}

// Filters of the Conv(k,s) predictor as a [Co, Kd] matrix whose reduction index is ordered
// (channel block, tap dy*k+dx padded with zeros to conv_taps_padded(k), channel in block): the
// order conv_relu_kernel walks.  Returns Kd.
int conv_reorder(const gati_cache_desc_t* d, const float* W1, int k_step, std::vector<float>& out) {
    const int k = d->conv_k, k2 = k * k, IT = conv_taps_padded(k);
    const int CB = (d->C + k_step - 1) / k_step, Kd = CB * IT * k_step;
    out.assign((size_t)d->H * Kd, 0.f);
    for (int o = 0; o < d->H; ++o)
        for (int c = 0; c < d->C; ++c)
            for (int t = 0; t < k2; ++t)
                out[(size_t)o * Kd + ((size_t)(c / k_step) * IT + t) * k_step + c % k_step] =
                    W1[((size_t)o * d->C + c) * k2 + t];
    return Kd;
}

// Filters of conv_rows_kernel as MFMA A fragments: [channel group][row parity][lane][8 bf16].  Lane
// (m, kb): row m = tap row t (m / 8) x filter o (m % 8); its element e is horizontal tap e of channel
// 2*group + kb (slot 8), or tap e % 4 of channel 4*group + 2*kb + e / 4 (slot 4); the tap row's offset
// is dy = parity + s*t.  Everything outside the filter is zero.
void pack_conv_rows(const gati_cache* c, const float* W1, std::vector<uint16_t>& out) {
    const gati_cache_desc_t& d = c->desc;
    const int k = d.conv_k, s = d.conv_s, slot = c->rows_slot, KC = 16 / slot;
    out.assign((size_t)(d.C / KC) * s * 64 * 8, 0);
    for (int cg = 0; cg < d.C / KC; ++cg)
        for (int pi = 0; pi < s; ++pi)
            for (int l = 0; l < 64; ++l)
                for (int e = 0; e < 8; ++e) {
                    const int m = l & 31, kb = l >> 5, t = m >> 3, o = m & 7;
                    const int ch = slot == 8 ? 2 * cg + kb : 4 * cg + 2 * kb + (e >> 2);
                    const int dx = slot == 8 ? e : (e & 3), dy = pi + s * t;
                    if (o < d.H && dy < k && dx < k)
                        out[(((size_t)cg * s + pi) * 64 + l) * 8 + e] =
                            f32_to_bf16_rne(W1[(((size_t)o * d.C + ch) * k + dy) * k + dx]);
                }
}

template <typename Tag>
hipError_t launch_pool_t(const gati_cache* c, PoolArgs a, PoolVariant variant, hipStream_t st) {
    // grid cap per CU: the wave kernel streams fastest with a wave per channel group and no grid-stride
    // loop (7.03 against 6.86 TB/s at 16 blocks per CU), so it has no cap; the tiled kernels do best with 12-24;
    // the adaptive-pool kernel with 48 for its large (J >= 8) tiles (6.8 against 6.4 TB/s inside a stack pass;
    // 128 drops to 5.9) and 24 otherwise
    int per_cu = c->pool_blocks_per_cu;
    if (variant == POOL_NCS_SEGW) per_cu = 12;      // 5.70 / 4.22 TB/s at S = 196 / 49 against 5.61 / 4.11 at 16
    else if (variant == POOL_NCS_ADAPTIVE) per_cu = c->ad_j >= 8 ? 48 : 24;
    const int max_blocks = c->num_cu * per_cu;
    switch (variant) {
    case POOL_NCS_WAVE: {
        static const int cpi_of[] = {8, 4, 2, 2, 1};
        const long groups = (long)a.n_max * ((a.C + cpi_of[c->wave_cfg] - 1) / cpi_of[c->wave_cfg]);
        // a wave per channel group and no loop, however many groups (the kernel's wave-stride loop only
        // serves launches beyond 2^24 workgroups): at 4096 rows of [256, 3136] the 64-blocks-per-CU grid
        // that earlier builds looped over read 6.72 TB/s, one workgroup per four groups 6.92
        const int blocks = (int)std::min<long>((groups + 3) / 4, 1L << 24);
        switch (c->wave_cfg) {
        case 0: pool_ncs_wave_kernel<Tag, 1, 8><<<blocks, 256, 0, st>>>(a, c->vpc); break;
        case 1: pool_ncs_wave_kernel<Tag, 2, 4><<<blocks, 256, 0, st>>>(a, c->vpc); break;
        case 2: pool_ncs_wave_kernel<Tag, 4, 2><<<blocks, 256, 0, st>>>(a, c->vpc); break;
        case 3: pool_ncs_wave_kernel<Tag, 8, 2><<<blocks, 256, 0, st>>>(a, c->vpc); break;
        default: pool_ncs_wave_kernel<Tag, 16, 1><<<blocks, 256, 0, st>>>(a, c->vpc); break;
        }
        break;
    }
    case POOL_NCS_SEGW: {
        const long tiles = (long)a.n_max * c->tiles_per_row;
        const int blocks = (int)std::min<long>((tiles + 3) / 4, max_blocks);
        pool_ncs_segw_kernel<Tag><<<blocks, 256, 0, st>>>(a, c->gt, c->tiles_per_row, c->tpc_log2, c->magic_S);
        break;
    }
    case POOL_NCS_SEG: {
        const long tiles = (long)a.n_max * c->tiles_per_row;
        const int blocks = (int)std::min<long>(tiles, max_blocks);
        pool_ncs_seg_kernel<Tag><<<blocks, 256, 0, st>>>(a, c->gt, c->tiles_per_row, c->tpc_log2, c->magic_S);
        break;
    }
    case POOL_NSC_VEC: {
        const long items = (long)a.n_max * c->cvb_per_row;
        const int blocks = (int)std::min<long>((items + 3) / 4, max_blocks);
        if (c->gw == 64) pool_nsc_kernel<Tag, 64><<<blocks, 256, 0, st>>>(a, c->cvb_per_row);
        else if (c->gw == 32) pool_nsc_kernel<Tag, 32><<<blocks, 256, 0, st>>>(a, c->cvb_per_row);
        else pool_nsc_kernel<Tag, 16><<<blocks, 256, 0, st>>>(a, c->cvb_per_row);
        break;
    }
    case POOL_NSC_UNIT: {
        const long units = (long)a.n_max * c->cvb_per_row;       // < 2^31: checked at creation (max_rows x features)
        if (c->gw == 32) pool_nsc_unit_kernel<Tag, 8, 32><<<(int)units, 64, 0, st>>>(a, c->cvb_per_row);
        else pool_nsc_unit_kernel<Tag, 8, 16><<<(int)units, 64, 0, st>>>(a, c->cvb_per_row);
        break;
    }
    case POOL_NCS_ADAPTIVE:
    case POOL_ADAPTIVE_GENERIC: {
        AdaptiveArgs g;
        g.in_h = c->desc.in_h; g.in_w = c->desc.in_w; g.out_h = c->desc.out_h; g.out_w = c->desc.out_w;
        g.gt = c->gt; g.tiles_per_row = c->tiles_per_row; g.tpo_log2 = c->ad_tpo_log2; g.win = c->ad_win;
        if (variant == POOL_ADAPTIVE_GENERIC) {
            const long items = (long)a.n_max * c->F;
            const int blocks = (int)std::min<long>((items + 255) / 256, max_blocks);
            pool_adaptive_generic_kernel<Tag><<<blocks, 256, 0, st>>>(a, g, c->desc.layout == GATI_LAYOUT_NSC ? 1 : 0);
            break;
        }
        const long tiles = (long)a.n_max * c->tiles_per_row;
        const int wpb = c->ad_j == 16 ? 2 : 4;
        const int blocks = (int)std::min<long>((tiles + wpb - 1) / wpb, max_blocks);
#define GATI_ADAPTIVE(JJ, WPB)                                                                                  \
    switch (c->ad_ww * 4 + c->ad_pair) {                                                                        \
    case 4 * 4 + 2: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 4, 2><<<blocks, WPB * 64, 0, st>>>(a, g); break;    \
    case 4 * 4: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 4, 0><<<blocks, WPB * 64, 0, st>>>(a, g); break;        \
    case 7 * 4: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 7, 0><<<blocks, WPB * 64, 0, st>>>(a, g); break;        \
    case 7 * 4 + 2: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 7, 2><<<blocks, WPB * 64, 0, st>>>(a, g); break;    \
    case 14 * 4 + 2: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 14, 2><<<blocks, WPB * 64, 0, st>>>(a, g); break;  \
    case 14 * 4 + 1: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 14, 1><<<blocks, WPB * 64, 0, st>>>(a, g); break;  \
    case 14 * 4: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 14, 0><<<blocks, WPB * 64, 0, st>>>(a, g); break;      \
    default: pool_ncs_adaptive_kernel<Tag, JJ, WPB, 0, 0><<<blocks, WPB * 64, 0, st>>>(a, g); break;           \
    }
        if (c->ad_j == 4) { GATI_ADAPTIVE(4, 4) }
        else if (c->ad_j == 8) { GATI_ADAPTIVE(8, 4) }
        else { GATI_ADAPTIVE(16, 2) }
#undef GATI_ADAPTIVE
        break;
    }
    default: {
        const long items = (long)a.n_max * a.C;
        const int blocks = (int)std::min<long>((items + 255) / 256, max_blocks);
        pool_generic_kernel<Tag><<<blocks, 256, 0, st>>>(a, c->desc.layout == GATI_LAYOUT_NSC ? 1 : 0);
        break;
    }
    }
    return hipGetLastError();
}

// Two 64 KB LDS slots of the 256 x 256 FC(h) kernel: above the 64 KB a kernel gets by default, so
// the limit is raised for the device when a cache that uses the kernel is created.
constexpr int kFlatLdsBytes = 2 * 4 * 16 * 1024;

hipError_t raise_flat_lds_limit(bool bf16) {
    const void* kern = bf16 ? reinterpret_cast<const void*>(fc_flat_lds_kernel<true, 2>)
                            : reinterpret_cast<const void*>(fc_flat_lds_kernel<false, 2>);
    return hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kFlatLdsBytes);
}

// FC(h): features = relu(W1 x + b1) over the flattened rows: split-K MFMA tiles, then the
// fixed-order reduction of the splits.
template <bool BF16>
hipError_t launch_flat_t(const gati_cache* c, const void* act, const int32_t* row_index, int n_max,
                         const int32_t* n_dev, float* out, void* out16, int out_stride, hipStream_t st) {
    if (c->flat_generic) {
        FlatGenericArgs ga;
        ga.act = act; ga.row_index = row_index; ga.n_dev = n_dev; ga.n_max = n_max;
        ga.D = (long)c->desc.C * c->desc.S; ga.H = c->desc.H; ga.W = c->W1; ga.bias = c->b1;
        ga.p = out; ga.p16 = static_cast<__bf16*>(out16); ga.ldp = out_stride;
        const long waves = (long)n_max * ga.H;
        fc_flat_generic_kernel<BF16><<<(int)std::min<long>((waves + 3) / 4, (long)c->num_cu * 16), 256, 0, st>>>(ga);
        return hipGetLastError();
    }
    FlatArgs f;
    f.act = act; f.row_index = row_index; f.n_dev = n_dev; f.n_max = n_max;
    f.D = (long)c->desc.C * c->desc.S; f.Wp = c->W1; f.KS = c->flat_KS; f.Hb = c->Hb; f.rows_b = c->rows_b;
    f.splits = c->flat_splits; f.ks_per_split = c->flat_ks_per;
    f.tiles_n = c->flat_tiles_n;
    f.tiles_m = std::min(c->flat_tiles_m, (n_max + 64 * c->flat_t - 1) / (64 * c->flat_t));
    f.partial = c->flat_partial;
    const int grid = f.tiles_m * f.tiles_n * f.splits;
    if (c->flat_t == 4) fc_flat_lds_kernel<BF16, 2><<<grid, 256, kFlatLdsBytes, st>>>(f);
    else if (c->flat_t == 2) fc_flat_kernel<BF16, 2, 2, 6><<<grid, 256, 0, st>>>(f);
    else fc_flat_kernel<BF16, 1, 1, 8><<<grid, 256, 0, st>>>(f);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    FlatReduceArgs r;
    r.partial = c->flat_partial; r.bias = c->b1; r.n_dev = n_dev; r.n_max = n_max;
    r.splits = c->flat_splits; r.rows_b = c->rows_b; r.Hb = c->Hb;
    r.p = out; r.p16 = static_cast<__bf16*>(out16); r.ldp = out_stride;
    const long vecs = (long)n_max * (out_stride / 4);
    const int blocks = (int)std::min<long>((vecs + 255) / 256, c->num_cu * 8);
    fc_flat_reduce_kernel<<<blocks, 256, 0, st>>>(r);
    return hipGetLastError();
}

hipError_t launch_pool(const gati_cache* c, const void* act, const int32_t* row_index, int n_max,
                       const int32_t* n_dev, float* out, void* out16, int out_stride, hipStream_t st) {
    if (c->flat_fc)
        return c->bf16 ? launch_flat_t<true>(c, act, row_index, n_max, n_dev, out, out16, out_stride, st)
                       : launch_flat_t<false>(c, act, row_index, n_max, n_dev, out, out16, out_stride, st);
    if (c->conv_fc)
        return c->bf16 ? launch_conv_t<true>(c, act, row_index, n_max, n_dev, out, out16, out_stride, st)
                       : launch_conv_t<false>(c, act, row_index, n_max, n_dev, out, out16, out_stride, st);
    PoolArgs a;
    a.out16 = static_cast<__bf16*>(out16);
    a.act = act; a.row_index = row_index; a.n_dev = n_dev; a.n_max = n_max;
    a.C = c->desc.C; a.S = c->desc.S; a.inv_S = 1.0f / (float)c->desc.S;
    a.out = out; a.out_stride = out_stride;
    // the vector kernels need 16-byte aligned rows; rows are multiples of 16 bytes by plan
    PoolVariant v = c->variant;
    if ((reinterpret_cast<uintptr_t>(act) & 15u) != 0) {
        if (v == POOL_NCS_ADAPTIVE) v = POOL_ADAPTIVE_GENERIC;
        else if (v != POOL_ADAPTIVE_GENERIC) v = POOL_GENERIC;
    }
    return c->bf16 ? launch_pool_t<BF16Tag>(c, a, v, st) : launch_pool_t<F32Tag>(c, a, v, st);
}

constexpr int kCompactSingleMax = 4096;   // up to here one workgroup walks the list (one launch, no table)

// FC1 (+ pooled half of the selector), FC2 (+ per-tile softmax summaries), then the per-row
// finish; with ids_out the finish also compacts the misses.
template <bool BF16>
hipError_t launch_head_t(const gati_cache* c, int n_max, const int32_t* n_dev, int32_t* pred_class,
                         float* confidence, uint8_t* hit, float* logits, const int32_t* ids_in,
                         int32_t* ids_out, int32_t* n_miss, hipStream_t st) {
    const int row_tiles = (n_max + 31) / 32;
    hipError_t e = hipSuccess;
    const bool sel_hidden = c->desc.selector == GATI_SEL_HIDDEN;
    // a wave's share of the reduction beyond 8 k-steps: the kernel instance with the deeper load pipeline
    auto deep = [](const FcArgs& f) { return f.Kdim / (BF16 ? 16 : 8) / 4 > 8; };
    // a layer with ReLU (predictor FC1, selector first layer): over 1024 inputs and more, the instance that fetches its
    // operand rows by whole lines
    auto launch_hidden = [&](const FcArgs& f, int col_tiles) {
        if constexpr (BF16) {
            if (f.Kdim >= 1024 && f.Kdim % 256 == 0) {
                fc_kernel<true, 1, true, 8, true><<<dim3(col_tiles, row_tiles), 256, 0, st>>>(f);
                return;
            }
        }
        if (deep(f)) fc_kernel<BF16, 1, true, 8><<<dim3(col_tiles, row_tiles), 256, 0, st>>>(f);
        else fc_kernel<BF16, 1, true, 4><<<dim3(col_tiles, row_tiles), 256, 0, st>>>(f);
    };
    if (sel_hidden && !logits) logits = c->zbuf;     // the selector's first layer reads the class probabilities
    FcArgs f2 = {};
    if (!c->pool_fc) {
        FcArgs f1 = {};
        f1.A = BF16 ? c->p16 : (const void*)c->p; f1.Wp = c->W1; f1.bias = c->b1; f1.Kdim = c->Cp; f1.N = c->Hp;
        f1.n_max = n_max; f1.n_dev = n_dev; f1.h = c->h;
        if (!sel_hidden) { f1.p32 = c->p; f1.ws_pool = c->ws_pool; f1.u_pool = c->u_pool; f1.ldp = c->Cp; }
        launch_hidden(f1, c->Hp / 32);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        f2.A = c->h; f2.Kdim = c->Hp;
    } else {
        // Pool(h): the ReLU'd pooled features are the hidden layer; the output-layer kernel also
        // computes the selector's pooled half
        f2.A = BF16 ? c->p16 : (const void*)c->p; f2.Kdim = c->Cp;
        if (!sel_hidden) { f2.p32 = c->p; f2.ws_pool = c->ws_pool; f2.ldp = c->Cp; }
    }
    f2.u_pool = c->u_pool;
    f2.Wp = c->W2; f2.bias = c->b2; f2.N = c->Kp;
    f2.n_max = n_max; f2.n_dev = n_dev;
    f2.K = c->desc.K; f2.ws_prob = c->ws_prob; f2.logits = logits; f2.stats = c->stats;
    const int n_tiles = c->Kp / (32 * c->fc2_nt);
    // few classes (one column tile): the output layer finishes its rows itself, and what is left of the finish
    // is the compaction of the flags
    const bool fused_finish = n_tiles == 1 && !sel_hidden && !c->pool_fc && (!ids_out || n_max <= kCompactSingleMax);
    if (fused_finish) {
        f2.fin = 1; f2.fin_bs = weights_of(c)->bs; f2.fin_tau = weights_of(c)->tau;
        f2.fin_softmax_only = c->desc.selector == GATI_SEL_SOFTMAX ? 1 : 0;
        f2.fin_class = pred_class; f2.fin_conf = confidence; f2.fin_hit = hit;
    }
    if (c->fc2_nt == 2) {
        // a thousand features or more (Pool(h), Conv(k,s), the hidden layer of FC(h)): the instance that fetches its
        // activation rows by whole lines
        if constexpr (BF16) {
            if (f2.Kdim >= 1024 && f2.Kdim % 256 == 0) {
                fc_kernel<true, 2, false, 8, true><<<dim3(n_tiles, row_tiles), 256, 0, st>>>(f2);
                goto output_layer_launched;
            }
        }
        if (deep(f2)) fc_kernel<BF16, 2, false, 8><<<dim3(n_tiles, row_tiles), 256, 0, st>>>(f2);
        else fc_kernel<BF16, 2, false, 4><<<dim3(n_tiles, row_tiles), 256, 0, st>>>(f2);
    } else {
        if (deep(f2)) fc_kernel<BF16, 1, false, 8><<<dim3(n_tiles, row_tiles), 256, 0, st>>>(f2);
        else fc_kernel<BF16, 1, false, 4><<<dim3(n_tiles, row_tiles), 256, 0, st>>>(f2);
    }
output_layer_launched:
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (fused_finish) {
        if (!ids_out) return hipSuccess;
        CompactArgs ca;
        ca.hit = hit; ca.ids_in = ids_in; ca.n_dev = n_dev; ca.n_max = n_max; ca.ids_out = ids_out; ca.n_miss = n_miss;
        compact_misses_kernel<<<1, 1024, 0, st>>>(ca);
        return hipGetLastError();
    }

    FinalizeArgs fa = {};
    if (sel_hidden) {
        // [features ; prob] operand rows, then the selector's first layer as one more FC launch
        SelInArgs si = {};
        si.stats = c->stats; si.n_tiles = n_tiles; si.logits = logits;
        si.feat = BF16 ? c->p16 : (const void*)c->p; si.sel_in = c->sel_in;
        si.Cp = c->Cp; si.K = c->desc.K; si.ld = c->Sin; si.n_max = n_max; si.n_dev = n_dev;
        selector_input_kernel<BF16><<<std::max(1, std::min(n_max, c->num_cu * 4)), 256, 0, st>>>(si);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        FcArgs fs = {};
        fs.A = c->sel_in; fs.Wp = c->Ws; fs.bias = c->cs; fs.Kdim = c->Sin; fs.N = c->Hsp;
        fs.n_max = n_max; fs.n_dev = n_dev; fs.h = c->sel_g;
        launch_hidden(fs, c->Hsp / 32);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        fa.sel_g = c->sel_g; fa.sel_vs = c->vs; fa.sel_hs = c->Hs; fa.ldg = c->Hsp; fa.g_bf16 = BF16 ? 1 : 0;
    }
    fa.stats = c->stats; fa.n_tiles = n_tiles; fa.u_pool = c->u_pool; fa.bs = weights_of(c)->bs; fa.tau = weights_of(c)->tau;
    fa.softmax_only = c->desc.selector == GATI_SEL_SOFTMAX ? 1 : 0;
    fa.n_max = n_max; fa.n_dev = n_dev; fa.pred_class = pred_class; fa.confidence = confidence; fa.hit = hit;
    fa.ids_in = ids_in; fa.ids_out = ids_out; fa.n_miss = n_miss;
    if (n_max > 1024 && (!ids_out || n_max <= kCompactSingleMax)) {
        // many rows: the per-row finish over several workgroups, then (with ids_out) the compaction by itself
        fa.ids_out = nullptr;
        finalize_kernel<<<(n_max + 255) / 256, 256, 0, st>>>(fa);
        if (!ids_out) return hipGetLastError();
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        CompactArgs ca;
        ca.hit = hit; ca.ids_in = ids_in; ca.n_dev = n_dev; ca.n_max = n_max; ca.ids_out = ids_out; ca.n_miss = n_miss;
        compact_misses_kernel<<<1, 1024, 0, st>>>(ca);
        return hipGetLastError();
    }
    finalize_kernel<<<1, 1024, 0, st>>>(fa);
    return hipGetLastError();
}

// Repack the host weights into the kernels' layouts and copy them to the device (allocating on
// first use).  Everything the packing needs is already planned in *c.
gati_status_t upload_weights(gati_cache* c, const gati_cache_weights_t* w) {
    const gati_cache_desc_t* desc = &c->desc;
    const bool flat_fc = c->flat_fc, conv_fc = c->conv_fc;
    const bool pool_fc = desc->predictor == GATI_PRED_POOL_FC;
    const bool no_hidden_kernel = c->pool_fc;
    const bool sel_hidden = desc->selector == GATI_SEL_HIDDEN;
    const int C = c->F, H = no_hidden_kernel ? c->F : desc->H, K = desc->K;   // C: features; H: inputs of the output FC
    gati_status_t st = GATI_OK;
    try {
        // weights in MFMA fragment order, zero padded
        if (c->bf16) {
            std::vector<uint16_t> t1, t2;
            if (flat_fc && c->flat_generic) {
                const size_t cnt = (size_t)desc->H * desc->C * desc->S;
                t1.resize(cnt);
                for (size_t q = 0; q < cnt; ++q) t1[q] = f32_to_bf16_rne(w->W1[q]);
                st = upload(&c->W1, t1.data(), cnt * 2);
            } else if (flat_fc) {
                const int D = desc->C * desc->S;
                pack_weights_flat(w->W1, desc->H, (long)D, c->Hb, 16, t1, f32_to_bf16_rne);
                st = upload(&c->W1, t1.data(), t1.size() * 2);
            } else if (conv_fc) {
                std::vector<float> wr, plain;
                if (c->variant == POOL_CONV_ROWS) {
                    pack_conv_rows(c, w->W1, t1);
                } else {
                    const int kd = conv_reorder(desc, w->W1, 16, wr);
                    pack_weights(wr.data(), desc->H, kd, round_up(desc->H, 32), kd, 16, t1, f32_to_bf16_rne);
                }
                st = upload(&c->W1, t1.data(), t1.size() * 2);
                plain.resize((size_t)desc->H * desc->C * desc->conv_k * desc->conv_k);
                for (size_t q = 0; q < plain.size(); ++q) {
                    const uint32_t bits = (uint32_t)f32_to_bf16_rne(w->W1[q]) << 16;
                    std::memcpy(&plain[q], &bits, 4);
                }
                if (st == GATI_OK) st = upload((void**)&c->W1plain, plain.data(), plain.size() * 4);
            } else if (!pool_fc) {
                pack_weights(w->W1, H, C, c->Hp, c->Cp, 16, t1, f32_to_bf16_rne);
                st = upload(&c->W1, t1.data(), t1.size() * 2);
            }
            pack_weights(w->W2, K, H, c->Kp, c->Hp, 16, t2, f32_to_bf16_rne);
            if (st == GATI_OK) st = upload(&c->W2, t2.data(), t2.size() * 2);
        } else {
            std::vector<float> t1, t2;
            auto same = [](float x) { return x; };
            if (flat_fc && c->flat_generic) {
                st = upload(&c->W1, w->W1, (size_t)desc->H * desc->C * desc->S * 4);
            } else if (flat_fc) {
                const int D = desc->C * desc->S;
                pack_weights_flat(w->W1, desc->H, (long)D, c->Hb, 8, t1, same);
                st = upload(&c->W1, t1.data(), t1.size() * 4);
            } else if (conv_fc) {
                std::vector<float> wr;
                const int kd = conv_reorder(desc, w->W1, 8, wr);
                pack_weights(wr.data(), desc->H, kd, round_up(desc->H, 32), kd, 8, t1, same);
                st = upload(&c->W1, t1.data(), t1.size() * 4);
                if (st == GATI_OK)
                    st = upload((void**)&c->W1plain, w->W1, (size_t)desc->H * desc->C * desc->conv_k * desc->conv_k * 4);
            } else if (!pool_fc) {
                pack_weights(w->W1, H, C, c->Hp, c->Cp, 8, t1, same);
                st = upload(&c->W1, t1.data(), t1.size() * 4);
            }
            pack_weights(w->W2, K, H, c->Kp, c->Hp, 8, t2, same);
            if (st == GATI_OK) st = upload(&c->W2, t2.data(), t2.size() * 4);
        }
        std::vector<float> b1(c->Hp, 0.f), b2(c->Kp, 0.f), wp(c->Cp, 0.f), wq(c->Kp, 0.f);
        if (!pool_fc) std::memcpy(b1.data(), w->b1, (size_t)desc->H * 4);   // conv_fc: one bias per filter
        std::memcpy(b2.data(), w->b2, (size_t)K * 4);
        if (desc->selector == GATI_SEL_LINEAR) {      // otherwise both halves stay zero: the per-tile selector sums are unused
            std::memcpy(wp.data(), w->ws, (size_t)C * 4);
            std::memcpy(wq.data(), w->ws + C, (size_t)K * 4);
        }
        if (st == GATI_OK) st = upload((void**)&c->b1, b1.data(), b1.size() * 4);
        if (st == GATI_OK) st = upload((void**)&c->b2, b2.data(), b2.size() * 4);
        if (st == GATI_OK) st = upload((void**)&c->ws_pool, wp.data(), wp.size() * 4);
        if (st == GATI_OK) st = upload((void**)&c->ws_prob, wq.data(), wq.size() * 4);
        if (sel_hidden) {
            // first layer over operand rows [features padded to Cp ; probabilities padded to Sin - Cp]
            c->Hs = desc->selector_hidden;
            c->Hsp = round_up(c->Hs, 32);
            c->Sin = c->Cp + round_up(K, 64);
            std::vector<float> wide((size_t)c->Hs * c->Sin, 0.f), cs(c->Hsp, 0.f), vs(c->Hsp, 0.f);
            for (int j = 0; j < c->Hs; ++j) {
                std::memcpy(&wide[(size_t)j * c->Sin], w->Ws + (size_t)j * (C + K), (size_t)C * 4);
                std::memcpy(&wide[(size_t)j * c->Sin + c->Cp], w->Ws + (size_t)j * (C + K) + C, (size_t)K * 4);
            }
            std::memcpy(cs.data(), w->cs, (size_t)c->Hs * 4);
            std::memcpy(vs.data(), w->vs, (size_t)c->Hs * 4);
            if (c->bf16) {
                std::vector<uint16_t> t;
                pack_weights(wide.data(), c->Hs, c->Sin, c->Hsp, c->Sin, 16, t, f32_to_bf16_rne);
                if (st == GATI_OK) st = upload(&c->Ws, t.data(), t.size() * 2);
            } else {
                std::vector<float> t;
                pack_weights(wide.data(), c->Hs, c->Sin, c->Hsp, c->Sin, 8, t, [](float x) { return x; });
                if (st == GATI_OK) st = upload(&c->Ws, t.data(), t.size() * 4);
            }
            if (st == GATI_OK) st = upload((void**)&c->cs, cs.data(), cs.size() * 4);
            if (st == GATI_OK) st = upload((void**)&c->vs, vs.data(), vs.size() * 4);
        }
    } catch (const std::bad_alloc&) {
        st = GATI_ERR_OOM;
    }
    return st;
}

// Workspace of a cache (or of a fork), zeroed once: the padding columns of p are never written and must read as 0.
gati_status_t alloc_workspace(gati_cache* c) {
    const gati_cache_desc_t* desc = &c->desc;
    const bool sel_hidden = desc->selector == GATI_SEL_HIDDEN;
    gati_status_t st = upload((void**)&c->p, nullptr, (size_t)c->rows_pad * c->Cp * 4);
    if (st == GATI_OK && c->bf16) st = upload(&c->p16, nullptr, (size_t)c->rows_pad * c->Cp * 2);
    if (st == GATI_OK && !c->pool_fc) st = upload(&c->h, nullptr, (size_t)c->rows_pad * c->Hp * (c->bf16 ? 2 : 4));
    if (st == GATI_OK && c->flat_fc && !c->flat_generic)
        st = upload((void**)&c->flat_partial, nullptr, (size_t)c->flat_splits * c->rows_b * c->Hb * 4);
    if (st == GATI_OK && c->conv_fc && c->conv_ksplit > 1)
        st = upload((void**)&c->conv_partial, nullptr, (size_t)c->conv_ksplit * desc->max_rows * c->Cp * 4);
    if (st == GATI_OK) st = upload((void**)&c->u_pool, nullptr, (size_t)c->rows_pad * 4);
    if (st == GATI_OK && sel_hidden) st = upload(&c->sel_in, nullptr, (size_t)c->rows_pad * c->Sin * c->elem);
    if (st == GATI_OK && sel_hidden) st = upload(&c->sel_g, nullptr, (size_t)c->rows_pad * c->Hsp * c->elem);
    if (st == GATI_OK && sel_hidden) st = upload((void**)&c->zbuf, nullptr, (size_t)desc->max_rows * desc->K * 4);
    if (st == GATI_OK)
        st = upload((void**)&c->stats, nullptr, (size_t)c->rows_pad * (c->Kp / (32 * c->fc2_nt)) * sizeof(TileStat));
    return st;
}

bool on_cache_device(const gati_cache* c) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == c->device;
}

// ---- compaction of long lists: two launches that share a small table of per-span counts ----
constexpr int kMaxDevices = 64;
std::mutex g_compact_mu;
int32_t* g_compact_ws[kMaxDevices];       // gati_compact_misses: allocated on a device's first long list
int32_t* g_compact_static[kMaxDevices];   // gati_compact_misses_static: this device's copy of `scratch`

hipError_t launch_compact(const CompactArgs& c, int32_t* table, hipStream_t st) {
    if (c.n_max <= kCompactSingleMax) {
        compact_misses_kernel<<<1, 1024, 0, st>>>(c);
        return hipGetLastError();
    }
    CompactWideArgs a;
    a.c = c; a.scratch = table;
    const long steps_total = ((long)c.n_max + 1023) / 1024;
    a.steps = (int)((steps_total + kCompactMaxChunks - 1) / kCompactMaxChunks);
    const int chunks = (int)((steps_total + a.steps - 1) / a.steps);   // <= kCompactMaxChunks
    compact_count_kernel<<<chunks, 1024, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    compact_scatter_kernel<<<chunks, 1024, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace

// The count table of gati_compact_misses_static: device memory that exists from the moment the
// library is loaded, one copy per GPU.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) int32_t scratch[kCompactScratchWords];

extern "C" {

const char* gati_status_string(gati_status_t s) {
    switch (s) {
    case GATI_OK: return "ok";
    case GATI_ERR_INVALID_ARG: return "invalid argument";
    case GATI_ERR_UNSUPPORTED: return "unsupported configuration";
    case GATI_ERR_OOM: return "out of memory";
    case GATI_ERR_DEVICE: return "HIP device error";
    }
    return "unknown status";
}

gati_status_t gati_cache_create(const gati_cache_desc_t* desc, const gati_cache_weights_t* w,
                                gati_cache_t** out) {
    if (!desc || !w || !out) return GATI_ERR_INVALID_ARG;
    if (desc->predictor != GATI_PRED_GAP_MLP && desc->predictor != GATI_PRED_POOL_FC &&
        desc->predictor != GATI_PRED_FC_MLP && desc->predictor != GATI_PRED_CONV_FC)
        return GATI_ERR_INVALID_ARG;
    const bool flat_fc = desc->predictor == GATI_PRED_FC_MLP;
    const bool pool_fc = desc->predictor == GATI_PRED_POOL_FC;
    const bool conv_fc = desc->predictor == GATI_PRED_CONV_FC;
    const bool no_hidden_kernel = pool_fc || flat_fc || conv_fc;
    int conv_oh = 0, conv_ow = 0;
    if (conv_fc) {
        if (desc->in_h <= 0 || desc->in_w <= 0 || desc->conv_k <= 0 || desc->conv_s <= 0) return GATI_ERR_INVALID_ARG;
        if (desc->conv_k > desc->in_h || desc->conv_k > desc->in_w) return GATI_ERR_INVALID_ARG;
        if ((long)desc->in_h * desc->in_w != (long)desc->S) return GATI_ERR_INVALID_ARG;
        if (desc->H <= 0) return GATI_ERR_INVALID_ARG;
        if (desc->H > 64 || desc->conv_k > 15) return GATI_ERR_UNSUPPORTED;
        conv_oh = (desc->in_h - desc->conv_k) / desc->conv_s + 1;
        conv_ow = (desc->in_w - desc->conv_k) / desc->conv_s + 1;
        if ((long)desc->H * conv_oh * conv_ow > (1L << 20)) return GATI_ERR_UNSUPPORTED;
    }
    if (desc->C <= 0 || desc->S <= 0 || desc->K <= 0 || desc->max_rows <= 0) return GATI_ERR_INVALID_ARG;
    if (!pool_fc && desc->H <= 0) return GATI_ERR_INVALID_ARG;
    if (pool_fc) {
        if (desc->in_h <= 0 || desc->in_w <= 0 || desc->out_h <= 0 || desc->out_w <= 0) return GATI_ERR_INVALID_ARG;
        if (desc->out_h > desc->in_h || desc->out_w > desc->in_w) return GATI_ERR_INVALID_ARG;
        if ((long)desc->in_h * desc->in_w != (long)desc->S) return GATI_ERR_INVALID_ARG;
        if ((long)desc->C * desc->out_h * desc->out_w > (1L << 20)) return GATI_ERR_UNSUPPORTED;
    }
    if (desc->act_dtype != GATI_F32 && desc->act_dtype != GATI_BF16) return GATI_ERR_INVALID_ARG;
    if (desc->layout != GATI_LAYOUT_NCS && desc->layout != GATI_LAYOUT_NSC) return GATI_ERR_INVALID_ARG;
    if (desc->selector != GATI_SEL_LINEAR && desc->selector != GATI_SEL_SOFTMAX && desc->selector != GATI_SEL_HIDDEN)
        return GATI_ERR_INVALID_ARG;
    const bool sel_hidden = desc->selector == GATI_SEL_HIDDEN;
    if (sel_hidden && (desc->selector_hidden < 1 || desc->selector_hidden > 1024 || !w->Ws || !w->cs || !w->vs))
        return GATI_ERR_INVALID_ARG;
    const bool needs_ws = desc->selector == GATI_SEL_LINEAR;
    if (!w->W2 || !w->b2 || (needs_ws && !w->ws)) return GATI_ERR_INVALID_ARG;
    if (!pool_fc && (!w->W1 || !w->b1)) return GATI_ERR_INVALID_ARG;
    if (flat_fc && (long)desc->C * desc->S >= (1L << 31)) return GATI_ERR_UNSUPPORTED;
    if (!(desc->threshold == desc->threshold)) return GATI_ERR_INVALID_ARG;   // NaN
    // sizes whose padded products still fit the kernels' 32-bit tile arithmetic
    if (desc->C > (1 << 20) || desc->H > (1 << 20) || desc->K > (1 << 20) || desc->max_rows > (1 << 22))
        return GATI_ERR_UNSUPPORTED;
    const long F_l = pool_fc ? (long)desc->C * desc->out_h * desc->out_w
                   : conv_fc ? (long)desc->H * conv_oh * conv_ow : (flat_fc ? (long)desc->H : (long)desc->C);
    if ((long)desc->max_rows * (F_l + 64) >= (1L << 31)) return GATI_ERR_UNSUPPORTED;

    gati_cache* c = new (std::nothrow) gati_cache();
    if (!c) return GATI_ERR_OOM;
    c->desc = *desc;
    c->bf16 = desc->act_dtype == GATI_BF16;
    c->elem = c->bf16 ? 2 : 4;
    c->bs = w->bs;
    c->tau = desc->threshold;
    c->pool_fc = no_hidden_kernel;
    c->flat_fc = flat_fc;
    c->conv_fc = conv_fc;
    c->conv_oh = conv_oh; c->conv_ow = conv_ow;
    c->F = (int)F_l;
    // features are padded to whole k-step groups; a thousand or more of them (an output layer straight over pooled
    // or convolved features) to 256, so that each of the 4 waves of fc_kernel owns whole 128-byte lines of a row
    c->Cp = round_up(c->F, (no_hidden_kernel && c->F >= 1024) ? 256 : 64);
    c->Hp = no_hidden_kernel ? c->Cp : round_up(desc->H, 64);   // width of the layer that feeds the output FC
    c->fc2_nt = desc->K > 96 ? 2 : 1;
    c->Kp = round_up(desc->K, 32 * c->fc2_nt);
    c->rows_pad = round_up(desc->max_rows, 32);

    if (hipGetDevice(&c->device) != hipSuccess) { (void)hipGetLastError(); delete c; return GATI_ERR_DEVICE; }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0)
        c->num_cu = cus;
    else
        (void)hipGetLastError();
    c->pool_blocks_per_cu = 16;

    if (flat_fc && ((long)desc->C * desc->S) % 64 != 0) {
        c->flat_generic = true;
        c->variant = POOL_FC_FLAT_GENERIC;
    } else if (flat_fc) {
        const int k_step = c->bf16 ? 16 : 8;
        const long D = (long)desc->C * desc->S;
        c->flat_t = (desc->max_rows >= 256 && desc->H >= 256) ? 4 : (desc->max_rows >= 128 && desc->H >= 128) ? 2 : 1;
        if (c->flat_t == 4 && raise_flat_lds_limit(c->bf16) != hipSuccess) {
            (void)hipGetLastError(); delete c; return GATI_ERR_DEVICE;
        }
        c->flat_KS = (int)(D / k_step);
        c->Hb = round_up(desc->H, 64 * c->flat_t);
        c->rows_b = round_up(desc->max_rows, 64 * c->flat_t);
        c->flat_tiles_m = c->rows_b / (64 * c->flat_t);
        c->flat_tiles_n = c->Hb / (64 * c->flat_t);
        const int tiles = c->flat_tiles_m * c->flat_tiles_n;
        // enough workgroups for every CU, each with at least 16 k-steps; multiples of 8 keep the XCD mapping
        int splits = std::max(1, std::min(c->num_cu / tiles, c->flat_KS / 16));
        if (splits >= 8) splits = splits / 8 * 8;
        splits = std::min(splits, 64);
        c->flat_ks_per = round_up((c->flat_KS + splits - 1) / splits, 4);   // whole permutation blocks
        c->flat_splits = (c->flat_KS + c->flat_ks_per - 1) / c->flat_ks_per;
        c->variant = POOL_FC_FLAT;
    } else if (conv_fc) {
        plan_conv(c);
        // the LDS ring of conv_rows_kernel is above the 64 KB a kernel gets by default
        if (c->variant == POOL_CONV_ROWS &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(conv_rows_instance(c->rows_slot, c->rows_tpw)),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kRowsLdsBytes) != hipSuccess) {
            (void)hipGetLastError(); delete c; return GATI_ERR_DEVICE;
        }
    } else {
        plan_pool(c);
    }

    gati_status_t st = upload_weights(c, w);
    if (st == GATI_OK && c->variant == POOL_NCS_ADAPTIVE) {
        // window table of the tiled adaptive-pool kernel; window i of an axis covers
        // [floor(i*in/out), ceil((i+1)*in/out))
        try {
            const int OO = desc->out_h * desc->out_w;
            std::vector<AdaptiveWindow> win((size_t)c->gt * OO);
            for (int lc = 0; lc < c->gt; ++lc)
                for (int oy = 0; oy < desc->out_h; ++oy)
                    for (int ox = 0; ox < desc->out_w; ++ox) {
                        const int y0 = (oy * desc->in_h) / desc->out_h, y1 = ((oy + 1) * desc->in_h + desc->out_h - 1) / desc->out_h;
                        const int x0 = (ox * desc->in_w) / desc->out_w, x1 = ((ox + 1) * desc->in_w + desc->out_w - 1) / desc->out_w;
                        AdaptiveWindow& e = win[(size_t)lc * OO + oy * desc->out_w + ox];
                        e.start = lc * desc->S + y0 * desc->in_w + x0;
                        e.rows = y1 - y0; e.cols = x1 - x0; e.area = (float)((y1 - y0) * (x1 - x0));
                    }
            st = upload((void**)&c->ad_win, win.data(), win.size() * sizeof(AdaptiveWindow));
        } catch (const std::bad_alloc&) { st = GATI_ERR_OOM; }
    }
    if (st == GATI_OK) st = alloc_workspace(c);
    if (st == GATI_OK && hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); st = GATI_ERR_DEVICE; }
    if (st != GATI_OK) { free_all(c); delete c; return st; }
    *out = c;
    return GATI_OK;
}

gati_status_t gati_cache_destroy(gati_cache_t* c) {
    if (!c) return GATI_OK;
    if (c->forks > 0) return GATI_ERR_INVALID_ARG;      // its forks still use the weights
    if (c->owner) --c->owner->forks;
    free_all(c);
    delete c;
    return GATI_OK;
}

gati_status_t gati_cache_fork(gati_cache_t* src, gati_cache_t** out) {
    if (!src || !out) return GATI_ERR_INVALID_ARG;
    gati_cache* root = src->owner ? src->owner : src;
    if (!on_cache_device(root)) return GATI_ERR_DEVICE;
    gati_cache* c = new (std::nothrow) gati_cache(*root);   // plan, padded sizes and the owner's device pointers
    if (!c) return GATI_ERR_OOM;
    c->owner = root; c->forks = 0;
    c->p = nullptr; c->p16 = nullptr; c->h = nullptr; c->u_pool = nullptr; c->stats = nullptr;
    c->flat_partial = nullptr; c->sel_in = nullptr; c->sel_g = nullptr; c->zbuf = nullptr; c->conv_partial = nullptr;
    gati_status_t st = alloc_workspace(c);
    if (st == GATI_OK && hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); st = GATI_ERR_DEVICE; }
    if (st != GATI_OK) { free_all(c); delete c; return st; }
    ++root->forks;
    *out = c;
    return GATI_OK;
}

gati_status_t gati_cache_set_weights(gati_cache_t* c, const gati_cache_weights_t* w) {
    if (!c || !w || c->owner) return GATI_ERR_INVALID_ARG;       // weights change through the cache that owns them
    const bool pool_fc = c->desc.predictor == GATI_PRED_POOL_FC;
    const bool sel_hidden = c->desc.selector == GATI_SEL_HIDDEN;
    if (sel_hidden && (!w->Ws || !w->cs || !w->vs)) return GATI_ERR_INVALID_ARG;
    if (!w->W2 || !w->b2 || (c->desc.selector == GATI_SEL_LINEAR && !w->ws)) return GATI_ERR_INVALID_ARG;
    if (!pool_fc && (!w->W1 || !w->b1)) return GATI_ERR_INVALID_ARG;
    if (!(w->bs == w->bs)) return GATI_ERR_INVALID_ARG;
    if (!on_cache_device(c)) return GATI_ERR_DEVICE;
    // lookups already enqueued must finish with the old weights
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    const gati_status_t st = upload_weights(c, w);
    if (st != GATI_OK) return st;
    c->bs = w->bs;
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    return GATI_OK;
}

}  // extern "C"

namespace {
template <bool BF16>
hipError_t load_trainer_t(gati_cache* c, const TrainerView& v, hipStream_t st) {
    using elem_t = typename PackElem<BF16>::type;
    const gati_cache_desc_t& d = c->desc;
    const int K = d.K, F = c->F;
    const bool pool_fc = d.predictor == GATI_PRED_POOL_FC;
    auto blocks = [&](long total) { return (int)std::max<long>(1, std::min<long>((total + 255) / 256, (long)c->num_cu * 32)); };
    // first layer
    if (c->flat_fc && c->flat_generic) {
        const long cnt = (long)d.H * d.C * d.S;
        pack_plain_kernel<BF16><<<blocks(cnt), 256, 0, st>>>(v.W1, cnt, static_cast<elem_t*>(c->W1));
    } else if (c->flat_fc) {
        const long D = (long)d.C * d.S;
        pack_flat_kernel<BF16><<<blocks((long)c->Hb * D), 256, 0, st>>>(v.W1, D, d.H, c->Hb, static_cast<elem_t*>(c->W1));
    } else if (c->conv_fc) {
        if (c->variant == POOL_CONV_ROWS) {
            const long cnt = (long)(d.C / (16 / c->rows_slot)) * d.conv_s * 64 * 8;
            pack_conv_rows_kernel<<<blocks(cnt), 256, 0, st>>>(v.W1, d.H, d.C, d.conv_k, d.conv_s, c->rows_slot, cnt,
                                                              static_cast<__bf16*>(c->W1));
        } else {
            const int rows_p = round_up(d.H, 32);
            const int k_step = BF16 ? 16 : 8;
            const long kd = (long)((d.C + k_step - 1) / k_step) * conv_taps_padded(d.conv_k) * k_step;
            pack_conv_kernel<BF16><<<blocks(rows_p * kd), 256, 0, st>>>(v.W1, d.H, d.C, d.conv_k, rows_p, static_cast<elem_t*>(c->W1));
        }
        const long cnt = (long)d.H * d.C * d.conv_k * d.conv_k;
        const ColMap all{(int)cnt, 0, (int)cnt, 0, 0};
        pack_vector_kernel<BF16><<<blocks(cnt), 256, 0, st>>>(v.W1, cnt, all, c->W1plain);
    } else if (!pool_fc) {
        const ColMap m{d.C, 0, d.C, 0, 0};
        pack_fc_kernel<BF16><<<blocks((long)c->Hp * c->Cp), 256, 0, st>>>(v.W1, d.C, d.H, c->Hp, c->Cp, m, static_cast<elem_t*>(c->W1));
    }
    if (!pool_fc) {
        const ColMap m{d.H, 0, d.H, 0, 0};
        // one bias per hidden unit (Conv(k,s): per filter), zero up to the padded length
        pack_vector_kernel<false><<<blocks(c->Hp), 256, 0, st>>>(v.b1, c->Hp, m, c->b1);
    }
    // output layer: its inputs are the hidden layer or the features; Conv(k,s) hidden values change order
    const int Hcols = c->pool_fc ? F : d.H;
    const ColMap feat{Hcols, 0, Hcols, v.conv ? v.P : 0, v.conv ? v.H : 0};
    pack_fc_kernel<BF16><<<blocks((long)c->Kp * c->Hp), 256, 0, st>>>(v.W2, v.Hin, K, c->Kp, c->Hp, feat, static_cast<elem_t*>(c->W2));
    const ColMap km{K, 0, K, 0, 0};
    pack_vector_kernel<false><<<blocks(c->Kp), 256, 0, st>>>(v.b2, c->Kp, km, c->b2);
    if (d.selector == GATI_SEL_LINEAR) {
        const ColMap fm{F, 0, F, v.conv ? v.P : 0, v.conv ? v.H : 0};
        pack_vector_kernel<false><<<blocks(c->Cp), 256, 0, st>>>(v.ws, c->Cp, fm, c->ws_pool);
        pack_vector_kernel<false><<<blocks(c->Kp), 256, 0, st>>>(v.ws + F, c->Kp, km, c->ws_prob);
    } else if (d.selector == GATI_SEL_HIDDEN) {
        const ColMap wide{F, c->Cp - F, F + K, v.conv ? v.P : 0, v.conv ? v.H : 0};
        pack_fc_kernel<BF16><<<blocks((long)c->Hsp * c->Sin), 256, 0, st>>>(v.Ws, v.Sx, c->Hs, c->Hsp, c->Sin, wide,
                                                                              static_cast<elem_t*>(c->Ws));
        const ColMap hm{c->Hs, 0, c->Hs, 0, 0};
        pack_vector_kernel<false><<<blocks(c->Hsp), 256, 0, st>>>(v.cs, c->Hsp, hm, c->cs);
        pack_vector_kernel<false><<<blocks(c->Hsp), 256, 0, st>>>(v.vs, c->Hsp, hm, c->vs);
    }
    return hipGetLastError();
}
}  // namespace

extern "C" {

gati_status_t gati_cache_load_trainer(gati_cache_t* c, gati_trainer_t* t, void* stream) {
    if (!c || !t || c->owner) return GATI_ERR_INVALID_ARG;
    TrainerView v;
    trainer_view(t, &v);
    const gati_cache_desc_t& d = c->desc;
    if (!on_cache_device(c) || v.device != c->device) return GATI_ERR_DEVICE;
    // the trainer must hold the same networks as the cache
    bool same = v.K == d.K && v.Fsel == c->F;
    switch (d.predictor) {
    case GATI_PRED_GAP_MLP: same = same && !v.conv && !v.sel_hidden_feat && v.H == d.H && v.C == d.C; break;
    case GATI_PRED_POOL_FC: same = same && v.H == 0 && v.C == c->F; break;
    case GATI_PRED_FC_MLP: same = same && !v.conv && v.sel_hidden_feat && v.H == d.H && (long)v.C == (long)d.C * d.S; break;
    case GATI_PRED_CONV_FC:
        same = same && v.conv && v.H == d.H && v.Cin == d.C * d.conv_k * d.conv_k && v.P == c->conv_oh * c->conv_ow &&
               (long)v.C == (long)d.C * d.S;
        break;
    }
    switch (d.selector) {
    case GATI_SEL_LINEAR: same = same && !v.no_selector && v.Hs == 0; break;
    case GATI_SEL_HIDDEN: same = same && v.Hs == d.selector_hidden; break;
    case GATI_SEL_SOFTMAX: same = same && v.no_selector; break;
    }
    if (!same) return GATI_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const hipError_t e = c->bf16 ? load_trainer_t<true>(c, v, st) : load_trainer_t<false>(c, v, st);
    if (e != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    if (d.selector != GATI_SEL_SOFTMAX) {
        // the selector bias travels to the kernels as an argument: fetch the scalar once the stream has caught up
        float bs = 0.f;
        if (hipMemcpyAsync(&bs, v.bs, sizeof(float), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) {
            (void)hipGetLastError(); return GATI_ERR_DEVICE;
        }
        if (!(bs == bs)) return GATI_ERR_INVALID_ARG;
        c->bs = bs;
    }
    return GATI_OK;
}

gati_status_t gati_cache_set_selector(gati_cache_t* c, float bs, float threshold) {
    if (!c || c->owner || !(bs == bs) || !(threshold == threshold)) return GATI_ERR_INVALID_ARG;
    c->bs = bs;
    c->tau = threshold;
    c->desc.threshold = threshold;
    return GATI_OK;
}

gati_status_t gati_cache_pool(gati_cache_t* c, const void* act, const int32_t* row_index, int32_t n_max,
                              const int32_t* n_dev, float* pooled, void* stream) {
    if (!c || n_max < 0 || n_max > c->desc.max_rows) return GATI_ERR_INVALID_ARG;
    if (n_max == 0) return GATI_OK;
    if (!act || !pooled) return GATI_ERR_INVALID_ARG;
    const bool flat_mfma = c->flat_fc && !c->flat_generic;
    if (flat_mfma && ((reinterpret_cast<uintptr_t>(act) | reinterpret_cast<uintptr_t>(pooled)) & 15u) != 0)
        return GATI_ERR_UNSUPPORTED;
    if (flat_mfma && c->F % 4 != 0) return GATI_ERR_UNSUPPORTED;
    if (!on_cache_device(c)) return GATI_ERR_DEVICE;
    const hipError_t e = launch_pool(c, act, row_index, n_max, n_dev, pooled, nullptr, c->F, (hipStream_t)stream);
    return e == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}

namespace {
gati_status_t lookup_impl(gati_cache_t* c, const void* act, const int32_t* row_index, int32_t n_max,
                          const int32_t* n_dev, int32_t* pred_class, float* confidence, uint8_t* hit,
                          float* logits, const int32_t* ids_in, int32_t* ids_out, int32_t* n_miss,
                          hipStream_t st) {
    if (c->flat_fc && !c->flat_generic && (reinterpret_cast<uintptr_t>(act) & 15u) != 0) return GATI_ERR_UNSUPPORTED;
    hipError_t e = launch_pool(c, act, row_index, n_max, n_dev, c->p, c->p16, c->Cp, st);
    if (e != hipSuccess) return GATI_ERR_DEVICE;
    e = c->bf16 ? launch_head_t<true>(c, n_max, n_dev, pred_class, confidence, hit, logits, ids_in, ids_out, n_miss, st)
                : launch_head_t<false>(c, n_max, n_dev, pred_class, confidence, hit, logits, ids_in, ids_out, n_miss, st);
    return e == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}
}  // namespace

gati_status_t gati_cache_lookup(gati_cache_t* c, const void* act, const int32_t* row_index, int32_t n_max,
                                const int32_t* n_dev, int32_t* pred_class, float* confidence, uint8_t* hit,
                                float* logits, void* stream) {
    if (!c || n_max < 0 || n_max > c->desc.max_rows) return GATI_ERR_INVALID_ARG;
    if (n_max == 0) return GATI_OK;
    if (!act || !pred_class || !confidence || !hit) return GATI_ERR_INVALID_ARG;
    if (!on_cache_device(c)) return GATI_ERR_DEVICE;
    return lookup_impl(c, act, row_index, n_max, n_dev, pred_class, confidence, hit, logits, nullptr, nullptr,
                       nullptr, (hipStream_t)stream);
}

gati_status_t gati_cache_lookup_compact(gati_cache_t* c, const void* act, const int32_t* row_index,
                                        int32_t n_max, const int32_t* n_dev, int32_t* pred_class,
                                        float* confidence, uint8_t* hit, float* logits, const int32_t* ids_in,
                                        int32_t* ids_out, int32_t* n_miss_dev, void* stream) {
    if (!c || n_max < 0 || n_max > c->desc.max_rows || !n_miss_dev) return GATI_ERR_INVALID_ARG;
    if (n_max > 0 && (!act || !pred_class || !confidence || !hit || !ids_out)) return GATI_ERR_INVALID_ARG;
    if (ids_in && ids_in == ids_out) return GATI_ERR_INVALID_ARG;
    if (!on_cache_device(c)) return GATI_ERR_DEVICE;
    if (n_max == 0) {   // nothing to look up: the miss list is empty
        CompactArgs a;
        a.hit = nullptr; a.ids_in = nullptr; a.n_dev = n_dev; a.n_max = 0; a.ids_out = ids_out; a.n_miss = n_miss_dev;
        compact_misses_kernel<<<1, 1024, 0, (hipStream_t)stream>>>(a);
        return hipGetLastError() == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
    }
    return lookup_impl(c, act, row_index, n_max, n_dev, pred_class, confidence, hit, logits, ids_in, ids_out,
                       n_miss_dev, (hipStream_t)stream);
}

gati_status_t gati_compact_misses(gati_cache_t* c, const uint8_t* hit, const int32_t* ids_in, int32_t n_max,
                                  const int32_t* n_dev, int32_t* ids_out, int32_t* n_miss_dev, void* stream) {
    if (n_max < 0 || !n_miss_dev) return GATI_ERR_INVALID_ARG;
    if (c && n_max > c->desc.max_rows) return GATI_ERR_INVALID_ARG;
    if (n_max > 0 && (!hit || !ids_out)) return GATI_ERR_INVALID_ARG;
    if (ids_in && ids_in == ids_out) return GATI_ERR_INVALID_ARG;
    if (c && !on_cache_device(c)) return GATI_ERR_DEVICE;
    CompactArgs a;
    a.hit = hit; a.ids_in = ids_in; a.n_dev = n_dev; a.n_max = n_max; a.ids_out = ids_out; a.n_miss = n_miss_dev;
    int32_t* table = nullptr;
    if (n_max > kCompactSingleMax) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
        if (dev < 0 || dev >= kMaxDevices) return GATI_ERR_UNSUPPORTED;
        std::lock_guard<std::mutex> lock(g_compact_mu);
        if (!g_compact_ws[dev]) {
            void* p = nullptr;
            if (hipMalloc(&p, kCompactScratchWords * sizeof(int32_t)) != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_OOM; }
            g_compact_ws[dev] = static_cast<int32_t*>(p);
        }
        table = g_compact_ws[dev];
    }
    return launch_compact(a, table, (hipStream_t)stream) == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}

gati_status_t gati_compact_misses_static(gati_cache_t* c, const uint8_t* hit, const int32_t* ids_in, int32_t n_max,
                                         const int32_t* n_dev, int32_t* ids_out, int32_t* n_miss_dev, void* stream) {
    if (n_max < 0 || !n_miss_dev) return GATI_ERR_INVALID_ARG;
    if (c && n_max > c->desc.max_rows) return GATI_ERR_INVALID_ARG;
    if (n_max > GATI_COMPACT_STATIC_MAX_ROWS) return GATI_ERR_UNSUPPORTED;
    if (n_max > 0 && (!hit || !ids_out)) return GATI_ERR_INVALID_ARG;
    if (ids_in && ids_in == ids_out) return GATI_ERR_INVALID_ARG;
    if (c && !on_cache_device(c)) return GATI_ERR_DEVICE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    if (dev < 0 || dev >= kMaxDevices) return GATI_ERR_UNSUPPORTED;
    int32_t* table = nullptr;
    {
        // first call on this device: ask the runtime where this device's copy of the array lives
        std::lock_guard<std::mutex> lock(g_compact_mu);
        if (!g_compact_static[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
            g_compact_static[dev] = static_cast<int32_t*>(p);
        }
        table = g_compact_static[dev];
    }
    CompactArgs a;
    a.hit = hit; a.ids_in = ids_in; a.n_dev = n_dev; a.n_max = n_max; a.ids_out = ids_out; a.n_miss = n_miss_dev;
    return launch_compact(a, table, (hipStream_t)stream) == hipSuccess ? GATI_OK : GATI_ERR_DEVICE;
}

const char* gati_cache_pool_variant(const gati_cache_t* c) {
    if (!c) return "none";
    switch (c->variant) {
    case POOL_NCS_WAVE: return "ncs_wave";
    case POOL_NCS_SEG: return "ncs_seg";
    case POOL_NCS_SEGW: return "ncs_segw";
    case POOL_NSC_VEC: return "nsc_vec";
    case POOL_NSC_UNIT: return "nsc_unit";
    case POOL_NCS_ADAPTIVE: return "ncs_adaptive";
    case POOL_ADAPTIVE_GENERIC: return "adaptive_generic";
    case POOL_FC_FLAT: return "fc_flat";
    case POOL_FC_FLAT_GENERIC: return "fc_flat_generic";
    case POOL_CONV: return "conv_mfma";
    case POOL_CONV_GENERIC: return "conv_generic";
    case POOL_CONV_ROWS: return "conv_rows";
    default: return "generic";
    }
}

}  // extern "C"
