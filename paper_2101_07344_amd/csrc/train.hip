// C ABI of the retraining step (see include/gati.h): the trainer object (fp32 master weights in
// plain row-major layout + a workspace for max_rows samples) and the launch sequence of one SGD
// step.  gfx950 only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/gati.h"
#include "train_conv_kernels.h"
#include "train_kernels.h"
#include "trainer_view.h"

using namespace gati;

// What the trainer holds, by predictor (Section 3, table of predictor architectures):
//   pooling (global)   input p [n, C]           -> W1 [H, C]       -> h [n, H]      -> W2 [K, H];   selector reads [p ; q]
//   Pool(h)            input f [n, F]                                               -> W2 [K, F];   selector reads [f ; q]
//   FC(h)              input x [n, D]           -> W1 [H, D]       -> h [n, H]      -> W2 [K, H];   selector reads [h ; q]
//   Conv(k,s)          input x [n, C*ih*iw] -> windows Xc [n*P, C*k*k] -> W1 [Co, C*k*k] -> h [n*P, Co] = [n, P*Co]
//                                                                                   -> W2 [K, P*Co]; selector reads [h ; q]
// Conv(k,s) keeps its hidden values in [position][filter] order, which is what the product over windows
// writes; the caller's order is [filter][position], so the columns of W2, ws and Ws that belong to hidden
// values are permuted on the way in and out (every formula of the step is indifferent to that order).
struct gati_trainer {
    int C = 0, H = 0, K = 0, max_rows = 0;    // C: width of the caller's input rows; H: first layer's outputs (0: none)
    int Cin = 0;                              // reduction length of the first layer (C; C*k*k for Conv(k,s))
    int P = 1;                                // first-layer output rows per sample (Conv(k,s): oh*ow)
    int Hin = 0;                              // inputs of the output layer: P*H, or C without a first layer
    int Fsel = 0;                             // features the selector reads beside q: C (pooling predictors) or Hin
    bool sel_hidden_feat = false;             // the selector reads the hidden layer (FC(h), Conv(k,s))
    bool no_selector = false;                 // softmax-threshold mode: the predictor alone is trained
    int conv_k = 0, conv_s = 0, conv_c = 0, conv_ih = 0, conv_iw = 0, conv_oh = 0, conv_ow = 0;   // Conv(k,s) only
    int device = 0, num_cu = 256;
    float *W1 = nullptr, *b1 = nullptr, *W2 = nullptr, *b2 = nullptr, *ws = nullptr, *bs = nullptr;
    float *h = nullptr, *z = nullptr, *q = nullptr, *dh = nullptr, *du = nullptr, *lp = nullptr, *ls = nullptr;
    float* W1t = nullptr;      // Conv(k,s) on the maps: the filters as [C][k*k][8], rewritten at the start of a step
    float* Xc = nullptr;       // Conv(k,s) through the product over windows: gathered windows [max_rows*P][Cin]
    // Conv(k,s) on the maps themselves (train_conv_kernels.h) where the shape allows; fixed at creation
    struct ConvDirect {
        bool on = false;
        int f_wpc = 1, f_pp = 1, f_sg = 1, f_cpw = 1;    // forward: waves per channel, positions per lane, samples per workgroup, channels per wave and pass
        int g_wpc = 1, g_ns = 1, g_splits = 1;           // filter gradient: waves per channel, samples per pass, sample splits wanted
    } cd;
    float* part = nullptr;     // split-reduction slices of the largest product
    size_t part_floats = 0;
    // selector with a hidden layer: Hs units over input rows X = [features ; q] of stride Sx (Fsel + K rounded up
    // to 4, zero padded, so that rows stay 16-byte aligned); Ws is held with the same stride
    int Hs = 0, Sx = 0;
    float *Ws = nullptr, *cs = nullptr, *vs = nullptr, *X = nullptr, *g = nullptr, *dg = nullptr, *G = nullptr;
};

namespace {

constexpr int kMaxSlices = 16;

void free_all(gati_trainer* t) {
    void* ptrs[] = {t->W1, t->b1, t->W2, t->b2, t->ws, t->bs, t->h, t->z, t->q, t->dh, t->du, t->lp, t->ls, t->part,
                    t->Ws, t->cs, t->vs, t->X, t->g, t->dg, t->G, t->Xc, t->W1t};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
}

gati_status_t dev_alloc(float** dst, size_t floats, const float* host_src) {
    if (hipMalloc(reinterpret_cast<void**>(dst), std::max<size_t>(floats, 1) * sizeof(float)) != hipSuccess) {
        *dst = nullptr; (void)hipGetLastError(); return GATI_ERR_OOM;
    }
    if (host_src && floats &&
        hipMemcpy(*dst, host_src, floats * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError(); return GATI_ERR_DEVICE;
    }
    return GATI_OK;
}

// Slices of the reduction for an M x N product over Kd: enough workgroups for about two per
// compute unit, never more slices than stages.  Depends on the shape only.
int plan_slices(const gati_trainer* t, int M, int N, int Kd) {
    const long tiles = (long)((M + kGemmTile - 1) / kGemmTile) * ((N + kGemmTile - 1) / kGemmTile);
    const int stages = (Kd + kGemmK - 1) / kGemmK;
    long nz = (2L * t->num_cu + tiles - 1) / tiles;
    nz = std::min<long>(nz, std::max(1, stages / 2));       // at least two stages per slice
    nz = std::min<long>(nz, kMaxSlices);
    return (int)std::max<long>(nz, 1);
}

bool aligned16(const void* p, int ld) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && ld % 4 == 0; }

template <bool TA, bool TB, int EPI>
hipError_t launch_gemm(const gati_trainer* t, GemmArgs g, hipStream_t st) {
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    g.veca = aligned16(g.A, g.lda) ? 1 : 0;
    g.vecb = aligned16(g.B, g.ldb) ? 1 : 0;
    int nz = plan_slices(t, g.M, g.N, g.Kd);
    if ((size_t)nz * g.M * g.N > t->part_floats) nz = 1;
    g.part = t->part;
    const dim3 grid((g.N + kGemmTile - 1) / kGemmTile, (g.M + kGemmTile - 1) / kGemmTile, nz);
    train_gemm_kernel<TA, TB, EPI><<<grid, 256, 0, st>>>(g);
    if (nz > 1) {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const long total = (long)g.M * g.N;
        const int blocks = (int)std::min<long>((total + 255) / 256, (long)t->num_cu * 8);
        gemm_epilogue_kernel<EPI><<<blocks, 256, 0, st>>>(g, nz);
    }
    return hipGetLastError();
}

// Conv(k,s): column of hidden value (filter o, position p) in the caller's order and in the trainer's.
inline size_t col_caller(const gati_trainer* t, int o, int p) { return (size_t)o * t->P + p; }
inline size_t col_inner(const gati_trainer* t, int o, int p) { return (size_t)p * t->H + o; }

// Copy a [rows][Hin (+ tail)] matrix between the caller's column order and the trainer's (to_inner or
// back); columns past the hidden values (the class-probability part of selector weights) keep their place.
void permute_hidden_cols(const gati_trainer* t, const float* src, size_t lds, float* dst, size_t ldd, int rows, int tail,
                         bool to_inner) {
    for (int r = 0; r < rows; ++r) {
        const float* s = src + (size_t)r * lds;
        float* d = dst + (size_t)r * ldd;
        for (int o = 0; o < t->H; ++o)
            for (int p = 0; p < t->P; ++p) {
                if (to_inner) d[col_inner(t, o, p)] = s[col_caller(t, o, p)];
                else d[col_caller(t, o, p)] = s[col_inner(t, o, p)];
            }
        for (int k = 0; k < tail; ++k) d[t->Hin + k] = s[t->Hin + k];
    }
}

// Launch shapes of the direct Conv(k,s) kernels for maps of S values, P output positions, k x k taps, H filters.
gati_trainer::ConvDirect plan_conv_direct(int C, int S, int P, int k, int H, int num_cu) {
    gati_trainer::ConvDirect p;
    if ((k != 3 && k != 5) || H > kConvTrainFilters || S > kConvTrainXFloats || P > kConvTrainMaxP || P < 1) return p;
    // forward: the fewest lane slots that hold a map's positions; ties go to more channels per workgroup
    long best = -1;
    for (int wpc = 1; wpc <= 4; wpc *= 2) {
        if ((4 / wpc) * S > kConvTrainXFloats) continue;
        for (int pp = 1; pp <= 3; ++pp) {
            const long slots = 64L * wpc * pp;
            if (slots < P) continue;
            const long cost = slots * 8 + wpc;
            if (best < 0 || cost < best) { best = cost; p.f_wpc = wpc; p.f_pp = pp; }
            break;
        }
    }
    if (best < 0) return p;
    const int fcw = 4 / p.f_wpc, slots = 64 * p.f_wpc * p.f_pp;
    p.f_sg = std::max(1, std::min({slots / P, kConvTrainXFloats / (fcw * S), 64}));
    p.f_cpw = std::max(1, std::min({kConvTrainXFloats / (p.f_sg * fcw * S), 16,
                                    (C + fcw - 1) / fcw}));
    // filter gradient: as many channels per workgroup as the staged maps allow, then samples per pass
    const int gcw = 4 * S <= kConvTrainGXFloats ? 4 : 2 * S <= kConvTrainGXFloats ? 2 : 1;
    p.g_wpc = 4 / gcw;
    p.g_ns = std::max(1, std::min({kConvTrainGXFloats / (gcw * S), kConvTrainDFloats / (P * 8), 32}));
    const int groups = (C + gcw - 1) / gcw;
    p.g_splits = std::max(1, std::min((4 * num_cu + groups - 1) / groups, kMaxSlices));
    p.on = true;
    return p;
}

bool on_trainer_device(const gati_trainer* t) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == t->device;
}

}  // namespace

void gati::trainer_view(const gati_trainer* t, gati::TrainerView* v) {
    v->device = t->device; v->C = t->C; v->H = t->H; v->K = t->K; v->Cin = t->Cin; v->P = t->P; v->Hin = t->Hin;
    v->Fsel = t->Fsel; v->conv = t->conv_k > 0; v->sel_hidden_feat = t->sel_hidden_feat; v->no_selector = t->no_selector;
    v->Hs = t->Hs; v->Sx = t->Sx;
    v->W1 = t->W1; v->b1 = t->b1; v->W2 = t->W2; v->b2 = t->b2; v->ws = t->ws; v->bs = t->bs;
    v->Ws = t->Ws; v->cs = t->cs; v->vs = t->vs;
}

extern "C" {

gati_status_t gati_trainer_create(const gati_cache_desc_t* desc, const gati_cache_weights_t* w,
                                  gati_trainer_t** out) {
    if (!desc || !w || !out) return GATI_ERR_INVALID_ARG;
    if (desc->C <= 0 || desc->K <= 0 || desc->max_rows <= 0) return GATI_ERR_INVALID_ARG;
    if (desc->predictor != GATI_PRED_GAP_MLP && desc->predictor != GATI_PRED_POOL_FC &&
        desc->predictor != GATI_PRED_FC_MLP && desc->predictor != GATI_PRED_CONV_FC)
        return GATI_ERR_INVALID_ARG;
    // Pool(h): no hidden layer; the features are the C * out_h * out_w pooled windows
    const bool pool_fc = desc->predictor == GATI_PRED_POOL_FC;
    const bool flat_fc = desc->predictor == GATI_PRED_FC_MLP;
    const bool conv_fc = desc->predictor == GATI_PRED_CONV_FC;
    if (pool_fc ? (desc->out_h <= 0 || desc->out_w <= 0 || (long)desc->C * desc->out_h * desc->out_w > (1L << 24))
                : (desc->H <= 0 || !w->W1 || !w->b1))
        return GATI_ERR_INVALID_ARG;
    if (flat_fc && (desc->S <= 0 || (long)desc->C * desc->S >= (1L << 30))) return GATI_ERR_INVALID_ARG;
    int oh = 0, ow = 0;
    if (conv_fc) {
        if (desc->in_h <= 0 || desc->in_w <= 0 || desc->conv_k <= 0 || desc->conv_s <= 0 ||
            desc->conv_k > desc->in_h || desc->conv_k > desc->in_w || (long)desc->in_h * desc->in_w != (long)desc->S)
            return GATI_ERR_INVALID_ARG;
        oh = (desc->in_h - desc->conv_k) / desc->conv_s + 1;
        ow = (desc->in_w - desc->conv_k) / desc->conv_s + 1;
        if ((long)desc->C * desc->S >= (1L << 30) || (long)desc->H * oh * ow > (1L << 24) ||
            (long)desc->max_rows * oh * ow >= (1L << 31) / 64 * 64 || (long)desc->C * desc->conv_k * desc->conv_k >= (1L << 24))
            return GATI_ERR_UNSUPPORTED;
    }
    if (!w->W2 || !w->b2) return GATI_ERR_INVALID_ARG;
    if (desc->selector != GATI_SEL_LINEAR && desc->selector != GATI_SEL_HIDDEN && desc->selector != GATI_SEL_SOFTMAX)
        return GATI_ERR_INVALID_ARG;
    const bool hidden = desc->selector == GATI_SEL_HIDDEN;
    const bool no_selector = desc->selector == GATI_SEL_SOFTMAX;
    if (hidden ? (!w->Ws || !w->cs || !w->vs || desc->selector_hidden <= 0 || desc->selector_hidden > 4096)
               : (!no_selector && !w->ws))
        return GATI_ERR_INVALID_ARG;
    gati_trainer* t = new (std::nothrow) gati_trainer;
    if (!t) return GATI_ERR_OOM;
    t->C = pool_fc ? desc->C * desc->out_h * desc->out_w : (flat_fc || conv_fc) ? desc->C * desc->S : desc->C;
    t->H = pool_fc ? 0 : desc->H;                                         // 0: no hidden layer
    t->K = desc->K; t->max_rows = desc->max_rows;
    t->P = conv_fc ? oh * ow : 1;
    t->Cin = conv_fc ? desc->C * desc->conv_k * desc->conv_k : t->C;
    t->Hin = t->H ? t->P * t->H : t->C;
    t->sel_hidden_feat = flat_fc || conv_fc;
    t->Fsel = t->sel_hidden_feat ? t->Hin : t->C;
    t->no_selector = no_selector;
    if (conv_fc) {
        t->conv_k = desc->conv_k; t->conv_s = desc->conv_s; t->conv_c = desc->C;
        t->conv_ih = desc->in_h; t->conv_iw = desc->in_w; t->conv_oh = oh; t->conv_ow = ow;
    }
    if (hipGetDevice(&t->device) != hipSuccess) { (void)hipGetLastError(); delete t; return GATI_ERR_DEVICE; }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device) == hipSuccess && cus > 0)
        t->num_cu = cus;
    const size_t H = t->H, K = t->K, n = t->max_rows, Cin = t->Cin, Hin = t->Hin, P = t->P, F = t->Fsel;
    // the largest split product: slices x (M x N) over the products of a step
    t->Hs = hidden ? desc->selector_hidden : 0;
    t->Sx = hidden ? (int)((F + K + 3) / 4 * 4) : 0;
    const size_t Hs = t->Hs, Sx = t->Sx;
    if (conv_fc) {
        t->cd = plan_conv_direct(desc->C, desc->S, oh * ow, desc->conv_k, desc->H, t->num_cu);
        if (t->cd.on) {
            const bool ok =
                hipFuncSetAttribute(reinterpret_cast<const void*>(&train_conv_wgrad_kernel<3, 1>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kConvTrainGradLds) == hipSuccess &&
                hipFuncSetAttribute(reinterpret_cast<const void*>(&train_conv_wgrad_kernel<5, 2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kConvTrainGradLds) == hipSuccess;
            if (!ok) { (void)hipGetLastError(); delete t; return GATI_ERR_DEVICE; }
        }
    }
    // the direct Conv(k,s) kernels replace the two products over windows (and their slices)
    const size_t conv_part = t->cd.on ? (size_t)t->cd.g_splits * desc->C * kConvTrainFilters * desc->conv_k * desc->conv_k : 0;
    const size_t conv_bpart = t->cd.on ? (size_t)kMaxSlices * kConvTrainFilters : 0;   // bias gradient slices, behind the filters'

    const size_t mn[7] = {t->cd.on ? n * P * kConvTrainFilters : n * P * H, n * K, n * Hin, K * Hin, t->cd.on ? 0 : H * Cin, n * Hs, Hs * Sx};
    t->part_floats = 0;
    for (size_t v : mn) t->part_floats = std::max(t->part_floats, v * kMaxSlices);
    t->part_floats = std::min<size_t>(t->part_floats, (size_t)64 << 20);   // 256 MB at most; fewer slices beyond
    t->part_floats = std::max(t->part_floats, conv_part + conv_bpart);
    gati_status_t st = GATI_OK;
    auto take = [&](gati_status_t s) { if (st == GATI_OK) st = s; };
    take(dev_alloc(&t->W1, H * Cin, H ? w->W1 : nullptr));     // Conv(k,s): [Co][C][k][k] is [Co][C*k*k] as stored
    take(dev_alloc(&t->b1, H, H ? w->b1 : nullptr));
    take(dev_alloc(&t->b2, K, w->b2));
    take(dev_alloc(&t->bs, 1, &w->bs));
    take(dev_alloc(&t->h, n * Hin * (H ? 1 : 0), nullptr));
    take(dev_alloc(&t->z, n * K, nullptr));
    take(dev_alloc(&t->q, n * K, nullptr));
    take(dev_alloc(&t->dh, n * Hin * (H ? 1 : 0), nullptr));
    take(dev_alloc(&t->du, n, nullptr));
    take(dev_alloc(&t->lp, n, nullptr));
    take(dev_alloc(&t->ls, n, nullptr));
    take(dev_alloc(&t->part, t->part_floats, nullptr));
    if (conv_fc && !t->cd.on) take(dev_alloc(&t->Xc, n * P * Cin, nullptr));
    if (t->cd.on) take(dev_alloc(&t->W1t, (size_t)desc->C * desc->conv_k * desc->conv_k * kConvTrainFilters, nullptr));
    try {
        if (conv_fc) {
            std::vector<float> tmp(K * Hin);
            permute_hidden_cols(t, w->W2, Hin, tmp.data(), Hin, (int)K, 0, true);
            take(dev_alloc(&t->W2, K * Hin, tmp.data()));
            if (!hidden && !no_selector) {
                tmp.assign(F + K, 0.f);
                permute_hidden_cols(t, w->ws, F + K, tmp.data(), F + K, 1, (int)K, true);
                take(dev_alloc(&t->ws, F + K, tmp.data()));
            }
        } else {
            take(dev_alloc(&t->W2, K * Hin, w->W2));
            if (!hidden && !no_selector) take(dev_alloc(&t->ws, F + K, w->ws));
        }
        if (hidden) {
            // zero padded to the row stride Sx; the padding columns stay zero (their gradient is a product with zero)
            std::vector<float> wide(Hs * Sx, 0.f);
            if (conv_fc) permute_hidden_cols(t, w->Ws, F + K, wide.data(), Sx, (int)Hs, (int)K, true);
            else for (size_t j = 0; j < Hs; ++j) std::copy(w->Ws + j * (F + K), w->Ws + (j + 1) * (F + K), wide.begin() + j * Sx);
            take(dev_alloc(&t->Ws, Hs * Sx, wide.data()));
            take(dev_alloc(&t->cs, Hs, w->cs));
            take(dev_alloc(&t->vs, Hs, w->vs));
            take(dev_alloc(&t->X, n * Sx, nullptr));
            take(dev_alloc(&t->g, n * Hs, nullptr));
            take(dev_alloc(&t->dg, n * Hs, nullptr));
            take(dev_alloc(&t->G, n, nullptr));
            if (st == GATI_OK && hipMemset(t->X, 0, n * Sx * sizeof(float)) != hipSuccess) {
                (void)hipGetLastError(); st = GATI_ERR_DEVICE;
            }
        }
    } catch (const std::bad_alloc&) { take(GATI_ERR_OOM); }
    if (st != GATI_OK) { free_all(t); delete t; return st; }
    *out = t;
    return GATI_OK;
}

gati_status_t gati_trainer_destroy(gati_trainer_t* t) {
    if (!t) return GATI_OK;
    free_all(t);
    delete t;
    return GATI_OK;
}

gati_status_t gati_trainer_step(gati_trainer_t* t, const float* pooled, int32_t ld_pooled, int32_t n,
                                const int32_t* labels, const float* teacher, int32_t ld_teacher,
                                const gati_train_params_t* params, float* losses, void* stream) {
    if (!t || !params) return GATI_ERR_INVALID_ARG;
    if (n < 0 || n > t->max_rows) return GATI_ERR_INVALID_ARG;
    if (n == 0) return GATI_OK;
    if (!pooled || !labels || !teacher || ld_pooled < t->C || ld_teacher < t->K) return GATI_ERR_INVALID_ARG;
    if (!(params->alpha >= 0.0f && params->alpha <= 1.0f) || !(params->fp_weight >= 0.0f) ||
        !(params->lr >= 0.0f))
        return GATI_ERR_INVALID_ARG;
    if (!on_trainer_device(t)) return GATI_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int H = t->H, K = t->K, Cin = t->Cin, P = t->P, Hin = t->Hin;
    const float lr = params->lr;
    hipError_t e;
    GemmArgs g{};
    // first layer's operand rows: the caller's input, or the gathered windows of Conv(k,s)
    const float* a1 = pooled;
    int lda1 = ld_pooled;
    // the layer that feeds the output FC: h = relu(a1 W1^T + b1), or the features themselves (Pool(h))
    const float* hin = H ? t->h : pooled;
    const int ldh = H ? Hin : ld_pooled;
    // what the selector reads beside the class probabilities
    const float* sfeat = t->sel_hidden_feat ? t->h : pooled;
    const int ldsf = t->sel_hidden_feat ? Hin : ld_pooled, Fsel = t->Fsel;
    ConvTrainArgs ca{};
    if (t->cd.on) {
        ca.x = pooled; ca.ldx = ld_pooled; ca.n = n; ca.C = t->conv_c; ca.ih = t->conv_ih; ca.iw = t->conv_iw;
        ca.s = t->conv_s; ca.oh = t->conv_oh; ca.ow = t->conv_ow; ca.H = H; ca.W1 = t->W1; ca.W1t = t->W1t; ca.b1 = t->b1;
        ca.h = t->h; ca.dh = t->dh; ca.part = t->part; ca.lr = lr;
        ca.bpart = t->part + (size_t)t->cd.g_splits * t->conv_c * kConvTrainFilters * t->conv_k * t->conv_k;
        ca.wpc = t->cd.f_wpc; ca.sg = t->cd.f_sg; ca.cpw = t->cd.f_cpw;
        const int S = t->conv_ih * t->conv_iw;
        ca.vec = aligned16(pooled, ld_pooled) && ((4 / ca.wpc) * ca.cpw * S) % 4 == 0 && (t->conv_c * S) % 4 == 0;
        const int wt = t->conv_c * t->conv_k * t->conv_k * kConvTrainFilters;
        train_conv_pack_kernel<<<(wt + 255) / 256, 256, 0, st>>>(ca, t->conv_k * t->conv_k);
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
        const int nblk = (n + ca.sg - 1) / ca.sg;
        // enough workgroups for about sixteen per compute unit, whole passes each, within the slices' room
        const int passes = (t->conv_c + (4 / ca.wpc) * ca.cpw - 1) / ((4 / ca.wpc) * ca.cpw);
        const long room = (long)(t->part_floats / ((size_t)n * P * kConvTrainFilters));
        ca.csplit = (int)std::max<long>(1, std::min<long>({(16L * t->num_cu + nblk - 1) / nblk, 16, passes, room}));
        const dim3 blocks(nblk, ca.csplit);
        const int key = t->conv_k * 10 + t->cd.f_pp;
        switch (key) {
            case 31: train_conv_fwd_kernel<3, 1><<<blocks, 256, 0, st>>>(ca); break;
            case 32: train_conv_fwd_kernel<3, 2><<<blocks, 256, 0, st>>>(ca); break;
            case 33: train_conv_fwd_kernel<3, 3><<<blocks, 256, 0, st>>>(ca); break;
            case 51: train_conv_fwd_kernel<5, 1><<<blocks, 256, 0, st>>>(ca); break;
            case 52: train_conv_fwd_kernel<5, 2><<<blocks, 256, 0, st>>>(ca); break;
            default: train_conv_fwd_kernel<5, 3><<<blocks, 256, 0, st>>>(ca); break;
        }
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
        if (ca.csplit > 1) {
            const long hv = (long)n * P * H;
            train_conv_finish_kernel<<<(int)((hv + 255) / 256), 256, 0, st>>>(ca);
            if ((e = hipGetLastError()) != hipSuccess) goto fail;
        }
    } else if (t->Xc) {
        Im2colArgs ia;
        ia.x = pooled; ia.ldx = ld_pooled; ia.Xc = t->Xc; ia.n = n; ia.C = t->conv_c; ia.ih = t->conv_ih; ia.iw = t->conv_iw;
        ia.k = t->conv_k; ia.s = t->conv_s; ia.oh = t->conv_oh; ia.ow = t->conv_ow;
        const long total = (long)n * P * Cin;
        train_im2col_kernel<<<(int)std::min<long>((total + 255) / 256, (long)t->num_cu * 32), 256, 0, st>>>(ia);
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
        a1 = t->Xc; lda1 = Cin;
    }
    if (H && !t->cd.on) {
        g = GemmArgs{}; g.A = a1; g.lda = lda1; g.B = t->W1; g.ldb = Cin; g.M = n * P; g.N = H; g.Kd = Cin;
        g.out = t->h; g.ldo = H; g.bias = t->b1;
        if ((e = launch_gemm<false, true, EPI_BIAS_RELU>(t, g, st)) != hipSuccess) goto fail;
    }
    // z = h W2^T + b2
    g = GemmArgs{}; g.A = hin; g.lda = ldh; g.B = t->W2; g.ldb = Hin; g.M = n; g.N = K; g.Kd = Hin;
    g.out = t->z; g.ldo = K; g.bias = t->b2;
    if ((e = launch_gemm<false, true, EPI_BIAS>(t, g, st)) != hipSuccess) goto fail;
    {
        TrainRowArgs a;
        a.z = t->z; a.q = t->q; a.p = sfeat; a.ldp = ldsf; a.labels = labels; a.Y = teacher; a.ldy = ld_teacher;
        a.ws = t->ws; a.bs = t->bs; a.n = n; a.C = Fsel; a.K = K; a.alpha = params->alpha; a.fp_weight = params->fp_weight;
        a.du = t->du; a.lp = t->lp; a.ls = t->ls;
        a.X = t->X; a.ldx = t->Sx; a.G = t->G;      // null for the linear selector
        const int blocks = (n + 3) / 4;
        if (K <= 64) train_row_kernel<1><<<blocks, 256, 0, st>>>(a);
        else if (K <= 256) train_row_kernel<4><<<blocks, 256, 0, st>>>(a);
        else if (K <= 1024) train_row_kernel<16><<<blocks, 256, 0, st>>>(a);
        else train_row_kernel<0><<<blocks, 256, 0, st>>>(a);
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
    }
    if (t->Hs) {
        // g = relu(X Ws^T + cs), then score, loss and gradients per sample
        g = GemmArgs{}; g.A = t->X; g.lda = t->Sx; g.B = t->Ws; g.ldb = t->Sx; g.M = n; g.N = t->Hs; g.Kd = t->Sx;
        g.out = t->g; g.ldo = t->Hs; g.bias = t->cs;
        if ((e = launch_gemm<false, true, EPI_BIAS_RELU>(t, g, st)) != hipSuccess) goto fail;
        TrainSelHiddenArgs sh;
        sh.g = t->g; sh.dg = t->dg; sh.vs = t->vs; sh.bs = t->bs; sh.G = t->G; sh.n = n; sh.Hs = t->Hs;
        sh.fp_weight = params->fp_weight; sh.du = t->du; sh.ls = t->ls;
        train_selector_hidden_kernel<<<(n + 3) / 4, 256, 0, st>>>(sh);
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
        // Ws -= lr dg^T X
        g = GemmArgs{}; g.A = t->dg; g.lda = t->Hs; g.B = t->X; g.ldb = t->Sx; g.M = t->Hs; g.N = t->Sx; g.Kd = n;
        g.out = t->Ws; g.ldo = t->Sx; g.lr = lr;
        if ((e = launch_gemm<true, false, EPI_SGD>(t, g, st)) != hipSuccess) goto fail;
    }
    if (H) {
        // dh = (dz W2) where h > 0      (uses W2 before its update)
        g = GemmArgs{}; g.A = t->z; g.lda = K; g.B = t->W2; g.ldb = Hin; g.M = n; g.N = Hin; g.Kd = K;
        g.out = t->dh; g.ldo = Hin; g.mask = t->h;
        if ((e = launch_gemm<false, false, EPI_MASK>(t, g, st)) != hipSuccess) goto fail;
    }
    // W2 -= lr dz^T h
    g = GemmArgs{}; g.A = t->z; g.lda = K; g.B = hin; g.ldb = ldh; g.M = K; g.N = Hin; g.Kd = n;
    g.out = t->W2; g.ldo = Hin; g.lr = lr;
    if ((e = launch_gemm<true, false, EPI_SGD>(t, g, st)) != hipSuccess) goto fail;
    if (t->cd.on) {
        // W1 -= lr * (filter gradient over all samples and positions), split over the samples
        ca.wpc = t->cd.g_wpc; ca.ns = t->cd.g_ns;
        const int cw = 4 / ca.wpc;
        ca.vec = aligned16(pooled, ld_pooled) && (cw * t->conv_ih * t->conv_iw) % 4 == 0 &&
                 (t->conv_c * t->conv_ih * t->conv_iw) % 4 == 0 && H == kConvTrainFilters;
        int rps = (n + t->cd.g_splits - 1) / t->cd.g_splits;
        rps = (rps + ca.ns - 1) / ca.ns * ca.ns;
        ca.rows_per_split = rps; ca.splits = (n + rps - 1) / rps;
        const dim3 grid((t->conv_c + cw - 1) / cw, ca.splits);
        if (t->conv_k == 3) train_conv_wgrad_kernel<3, 1><<<grid, 256, kConvTrainGradLds, st>>>(ca);
        else train_conv_wgrad_kernel<5, 2><<<grid, 256, kConvTrainGradLds, st>>>(ca);
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
        const int kk2 = t->conv_k * t->conv_k;
        train_conv_update_kernel<<<(H * t->conv_c * kk2 + 255) / 256, 256, 0, st>>>(ca, kk2);
        if ((e = hipGetLastError()) != hipSuccess) goto fail;
    } else if (H) {
        // W1 -= lr dh^T a1      (dh as [n*P][H])
        g = GemmArgs{}; g.A = t->dh; g.lda = H; g.B = a1; g.ldb = lda1; g.M = H; g.N = Cin; g.Kd = n * P;
        g.out = t->W1; g.ldo = Cin; g.lr = lr;
        if ((e = launch_gemm<true, false, EPI_SGD>(t, g, st)) != hipSuccess) goto fail;
    }
    // biases and selector
    {
        ColsumArgs c;
        c.lr = lr;
        const ColsumJob none{t->z, K, 0, nullptr, t->b2, 0, 0};
        c.job[0] = ColsumJob{t->z, K, K, nullptr, t->b2, 0, n};
        c.job[1] = ColsumJob{t->dh, H, H, nullptr, t->b1, 0, n * P};     // dh as [n*P][H]
        if (t->cd.on) c.job[1] = none;                                   // done with the filters, from the same staged values
        if (t->Hs) {
            c.job[2] = ColsumJob{t->dg, t->Hs, t->Hs, nullptr, t->cs, 0, n};
            c.job[3] = ColsumJob{t->g, t->Hs, t->Hs, t->du, t->vs, 0, n};
        } else if (!t->no_selector) {
            c.job[2] = ColsumJob{sfeat, ldsf, Fsel, t->du, t->ws, 0, n};
            c.job[3] = ColsumJob{t->q, K, K, t->du, t->ws + Fsel, 0, n};
        } else {
            c.job[2] = c.job[3] = none;
        }
        int blocks = 0;
        for (int j = 0; j < 4; ++j) { c.job[j].first_block = blocks; blocks += (c.job[j].cols + 63) / 64; }
        train_colsums_kernel<<<blocks, 1024, 0, st>>>(c);
    }
    train_scalar_kernel<<<1, 256, 0, st>>>(t->du, t->lp, t->ls, n, lr, t->bs, losses);
    if ((e = hipGetLastError()) != hipSuccess) goto fail;
    return GATI_OK;
fail:
    (void)hipGetLastError();
    return GATI_ERR_DEVICE;
}

gati_status_t gati_trainer_get_weights(gati_trainer_t* t, float* W1, float* b1, float* W2, float* b2,
                                       float* ws, float* bs) {
    const bool has_ws = t && !t->Hs && !t->no_selector;
    if (!t || !W2 || !b2 || !bs || (has_ws && !ws) || (t->H && (!W1 || !b1))) return GATI_ERR_INVALID_ARG;
    if (!on_trainer_device(t)) return GATI_ERR_DEVICE;
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    const size_t H = t->H, K = t->K, Cin = t->Cin, Hin = t->Hin, F = t->Fsel;
    const bool permute = t->conv_k > 0;                  // Conv(k,s): hidden-value columns back to [filter][position]
    try {
        std::vector<float> w2(permute ? K * Hin : 0), wsel(permute && has_ws ? F + K : 0);
        struct { float* dst; const float* src; size_t n; } cp[] = {
            {W1, t->W1, H * Cin}, {b1, t->b1, H}, {permute ? w2.data() : W2, t->W2, K * Hin}, {b2, t->b2, K},
            {permute && has_ws ? wsel.data() : ws, t->ws, has_ws ? F + K : 0}, {bs, t->bs, 1}};
        for (auto& c : cp)
            if (c.n && hipMemcpy(c.dst, c.src, c.n * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) {
                (void)hipGetLastError(); return GATI_ERR_DEVICE;
            }
        if (permute) {
            permute_hidden_cols(t, w2.data(), Hin, W2, Hin, (int)K, 0, false);
            if (has_ws) permute_hidden_cols(t, wsel.data(), F + K, ws, F + K, 1, (int)K, false);
        }
    } catch (const std::bad_alloc&) { return GATI_ERR_OOM; }
    return GATI_OK;
}

gati_status_t gati_trainer_get_hidden_selector(gati_trainer_t* t, float* Ws, float* cs, float* vs) {
    if (!t || !Ws || !cs || !vs) return GATI_ERR_INVALID_ARG;
    if (!t->Hs) return GATI_ERR_UNSUPPORTED;
    if (!on_trainer_device(t)) return GATI_ERR_DEVICE;
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    const size_t cols = (size_t)t->Fsel + t->K, w = cols * sizeof(float);
    try {
        std::vector<float> tmp(t->conv_k ? (size_t)t->Hs * cols : 0);
        float* dst = t->conv_k ? tmp.data() : Ws;
        if (hipMemcpy2D(dst, w, t->Ws, (size_t)t->Sx * sizeof(float), w, t->Hs, hipMemcpyDeviceToHost) != hipSuccess ||
            hipMemcpy(cs, t->cs, (size_t)t->Hs * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess ||
            hipMemcpy(vs, t->vs, (size_t)t->Hs * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError(); return GATI_ERR_DEVICE;
        }
        if (t->conv_k) permute_hidden_cols(t, tmp.data(), cols, Ws, cols, t->Hs, t->K, false);
    } catch (const std::bad_alloc&) { return GATI_ERR_OOM; }
    return GATI_OK;
}

}  // extern "C"
