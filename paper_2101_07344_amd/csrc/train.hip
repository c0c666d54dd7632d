// C ABI of the retraining step (see include/gati.h): the trainer object (fp32 master weights in
// plain row-major layout + a workspace for max_rows samples) and the launch sequence of one SGD
// step.  gfx950 only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>

#include "../../include/gati.h"
#include "train_kernels.h"

using namespace gati;

struct gati_trainer {
    int C = 0, H = 0, K = 0, max_rows = 0;
    int device = 0, num_cu = 256;
    float *W1 = nullptr, *b1 = nullptr, *W2 = nullptr, *b2 = nullptr, *ws = nullptr, *bs = nullptr;
    float *h = nullptr, *z = nullptr, *q = nullptr, *dh = nullptr, *du = nullptr, *lp = nullptr, *ls = nullptr;
    float* part = nullptr;     // split-reduction slices of the largest product
    size_t part_floats = 0;
    // selector with a hidden layer: Hs units over input rows X = [p ; q] of stride Sx (C + K rounded up to 4,
    // zero padded, so that rows stay 16-byte aligned); Ws is held with the same stride
    int Hs = 0, Sx = 0;
    float *Ws = nullptr, *cs = nullptr, *vs = nullptr, *X = nullptr, *g = nullptr, *dg = nullptr, *G = nullptr;
};

namespace {

constexpr int kMaxSlices = 16;

void free_all(gati_trainer* t) {
    void* ptrs[] = {t->W1, t->b1, t->W2, t->b2, t->ws, t->bs, t->h, t->z, t->q, t->dh, t->du, t->lp, t->ls, t->part,
                    t->Ws, t->cs, t->vs, t->X, t->g, t->dg, t->G};
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

bool on_trainer_device(const gati_trainer* t) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == t->device;
}

}  // namespace

extern "C" {

gati_status_t gati_trainer_create(const gati_cache_desc_t* desc, const gati_cache_weights_t* w,
                                  gati_trainer_t** out) {
    if (!desc || !w || !out) return GATI_ERR_INVALID_ARG;
    if (desc->C <= 0 || desc->K <= 0 || desc->max_rows <= 0) return GATI_ERR_INVALID_ARG;
    if (desc->predictor != GATI_PRED_GAP_MLP && desc->predictor != GATI_PRED_POOL_FC) return GATI_ERR_UNSUPPORTED;
    // Pool(h): no hidden layer; the features are the C * out_h * out_w pooled windows
    const bool pool_fc = desc->predictor == GATI_PRED_POOL_FC;
    if (pool_fc ? (desc->out_h <= 0 || desc->out_w <= 0 || (long)desc->C * desc->out_h * desc->out_w > (1L << 24))
                : (desc->H <= 0 || !w->W1 || !w->b1))
        return GATI_ERR_INVALID_ARG;
    if (!w->W2 || !w->b2) return GATI_ERR_INVALID_ARG;
    if (desc->selector != GATI_SEL_LINEAR && desc->selector != GATI_SEL_HIDDEN) return GATI_ERR_UNSUPPORTED;
    const bool hidden = desc->selector == GATI_SEL_HIDDEN;
    if (hidden ? (!w->Ws || !w->cs || !w->vs || desc->selector_hidden <= 0 || desc->selector_hidden > 4096) : !w->ws)
        return GATI_ERR_INVALID_ARG;
    gati_trainer* t = new (std::nothrow) gati_trainer;
    if (!t) return GATI_ERR_OOM;
    t->C = pool_fc ? desc->C * desc->out_h * desc->out_w : desc->C;      // features per sample
    t->H = pool_fc ? 0 : desc->H;                                         // 0: no hidden layer
    t->K = desc->K; t->max_rows = desc->max_rows;
    if (hipGetDevice(&t->device) != hipSuccess) { (void)hipGetLastError(); delete t; return GATI_ERR_DEVICE; }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device) == hipSuccess && cus > 0)
        t->num_cu = cus;
    const size_t C = t->C, H = t->H, K = t->K, n = t->max_rows;
    // the largest split product: slices x (M x N) over the five products of a step
    t->Hs = hidden ? desc->selector_hidden : 0;
    t->Sx = hidden ? (int)((C + K + 3) / 4 * 4) : 0;
    const size_t Hs = t->Hs, Sx = t->Sx;
    const size_t mn[7] = {n * H, n * K, n * H, K * (H ? H : C), H * C, n * Hs, Hs * Sx};
    t->part_floats = 0;
    for (size_t v : mn) t->part_floats = std::max(t->part_floats, v * kMaxSlices);
    t->part_floats = std::min<size_t>(t->part_floats, (size_t)64 << 20);   // 256 MB at most; fewer slices beyond
    gati_status_t st = GATI_OK;
    auto take = [&](gati_status_t s) { if (st == GATI_OK) st = s; };
    take(dev_alloc(&t->W1, H * C, H ? w->W1 : nullptr));
    take(dev_alloc(&t->b1, H, H ? w->b1 : nullptr));
    take(dev_alloc(&t->W2, K * (H ? H : C), w->W2));
    take(dev_alloc(&t->b2, K, w->b2));
    if (!hidden) take(dev_alloc(&t->ws, C + K, w->ws));
    take(dev_alloc(&t->bs, 1, &w->bs));
    take(dev_alloc(&t->h, n * H, nullptr));
    take(dev_alloc(&t->z, n * K, nullptr));
    take(dev_alloc(&t->q, n * K, nullptr));
    take(dev_alloc(&t->dh, n * H, nullptr));
    take(dev_alloc(&t->du, n, nullptr));
    take(dev_alloc(&t->lp, n, nullptr));
    take(dev_alloc(&t->ls, n, nullptr));
    take(dev_alloc(&t->part, t->part_floats, nullptr));
    if (hidden) {
        take(dev_alloc(&t->Ws, Hs * Sx, nullptr));
        take(dev_alloc(&t->cs, Hs, w->cs));
        take(dev_alloc(&t->vs, Hs, w->vs));
        take(dev_alloc(&t->X, n * Sx, nullptr));
        take(dev_alloc(&t->g, n * Hs, nullptr));
        take(dev_alloc(&t->dg, n * Hs, nullptr));
        take(dev_alloc(&t->G, n, nullptr));
        // the padding columns of X and Ws are zero and stay zero (their gradient is a product with zero)
        if (st == GATI_OK && (hipMemset(t->X, 0, n * Sx * sizeof(float)) != hipSuccess ||
                              hipMemset(t->Ws, 0, Hs * Sx * sizeof(float)) != hipSuccess ||
                              hipMemcpy2D(t->Ws, Sx * sizeof(float), w->Ws, (C + K) * sizeof(float), (C + K) * sizeof(float), Hs,
                                          hipMemcpyHostToDevice) != hipSuccess)) {
            (void)hipGetLastError(); st = GATI_ERR_DEVICE;
        }
    }
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
    const int C = t->C, H = t->H, K = t->K;
    const float lr = params->lr;
    hipError_t e;
    GemmArgs g{};
    // the layer that feeds the output FC: h = relu(p W1^T + b1), or the features themselves (Pool(h))
    const float* hin = H ? t->h : pooled;
    const int ldh = H ? H : ld_pooled, Hin = H ? H : C;
    if (H) {
        g = GemmArgs{}; g.A = pooled; g.lda = ld_pooled; g.B = t->W1; g.ldb = C; g.M = n; g.N = H; g.Kd = C;
        g.out = t->h; g.ldo = H; g.bias = t->b1;
        if ((e = launch_gemm<false, true, EPI_BIAS_RELU>(t, g, st)) != hipSuccess) goto fail;
    }
    // z = h W2^T + b2
    g = GemmArgs{}; g.A = hin; g.lda = ldh; g.B = t->W2; g.ldb = Hin; g.M = n; g.N = K; g.Kd = Hin;
    g.out = t->z; g.ldo = K; g.bias = t->b2;
    if ((e = launch_gemm<false, true, EPI_BIAS>(t, g, st)) != hipSuccess) goto fail;
    {
        TrainRowArgs a;
        a.z = t->z; a.q = t->q; a.p = pooled; a.ldp = ld_pooled; a.labels = labels; a.Y = teacher; a.ldy = ld_teacher;
        a.ws = t->ws; a.bs = t->bs; a.n = n; a.C = C; a.K = K; a.alpha = params->alpha; a.fp_weight = params->fp_weight;
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
        g = GemmArgs{}; g.A = t->z; g.lda = K; g.B = t->W2; g.ldb = H; g.M = n; g.N = H; g.Kd = K;
        g.out = t->dh; g.ldo = H; g.mask = t->h;
        if ((e = launch_gemm<false, false, EPI_MASK>(t, g, st)) != hipSuccess) goto fail;
    }
    // W2 -= lr dz^T h
    g = GemmArgs{}; g.A = t->z; g.lda = K; g.B = hin; g.ldb = ldh; g.M = K; g.N = Hin; g.Kd = n;
    g.out = t->W2; g.ldo = Hin; g.lr = lr;
    if ((e = launch_gemm<true, false, EPI_SGD>(t, g, st)) != hipSuccess) goto fail;
    if (H) {
        // W1 -= lr dh^T p
        g = GemmArgs{}; g.A = t->dh; g.lda = H; g.B = pooled; g.ldb = ld_pooled; g.M = H; g.N = C; g.Kd = n;
        g.out = t->W1; g.ldo = C; g.lr = lr;
        if ((e = launch_gemm<true, false, EPI_SGD>(t, g, st)) != hipSuccess) goto fail;
    }
    // biases and selector
    {
        ColsumArgs c;
        c.n = n; c.lr = lr;
        c.job[0] = ColsumJob{t->z, K, K, nullptr, t->b2, 0};
        c.job[1] = ColsumJob{t->dh, H, H, nullptr, t->b1, 0};
        if (t->Hs) {
            c.job[2] = ColsumJob{t->dg, t->Hs, t->Hs, nullptr, t->cs, 0};
            c.job[3] = ColsumJob{t->g, t->Hs, t->Hs, t->du, t->vs, 0};
        } else {
            c.job[2] = ColsumJob{pooled, ld_pooled, C, t->du, t->ws, 0};
            c.job[3] = ColsumJob{t->q, K, K, t->du, t->ws + C, 0};
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
    if (!t || !W2 || !b2 || !bs || (!t->Hs && !ws) || (t->H && (!W1 || !b1))) return GATI_ERR_INVALID_ARG;
    if (!on_trainer_device(t)) return GATI_ERR_DEVICE;
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    const size_t C = t->C, H = t->H, K = t->K;
    struct { float* dst; const float* src; size_t n; } cp[] = {
        {W1, t->W1, H * C}, {b1, t->b1, H}, {W2, t->W2, K * (H ? H : C)}, {b2, t->b2, K}, {ws, t->ws, t->Hs ? 0 : C + K}, {bs, t->bs, 1}};
    for (auto& c : cp)
        if (c.n && hipMemcpy(c.dst, c.src, c.n * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError(); return GATI_ERR_DEVICE;
        }
    return GATI_OK;
}

gati_status_t gati_trainer_get_hidden_selector(gati_trainer_t* t, float* Ws, float* cs, float* vs) {
    if (!t || !Ws || !cs || !vs) return GATI_ERR_INVALID_ARG;
    if (!t->Hs) return GATI_ERR_UNSUPPORTED;
    if (!on_trainer_device(t)) return GATI_ERR_DEVICE;
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return GATI_ERR_DEVICE; }
    const size_t w = (size_t)(t->C + t->K) * sizeof(float);
    if (hipMemcpy2D(Ws, w, t->Ws, (size_t)t->Sx * sizeof(float), w, t->Hs, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(cs, t->cs, (size_t)t->Hs * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(vs, t->vs, (size_t)t->Hs * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError(); return GATI_ERR_DEVICE;
    }
    return GATI_OK;
}

}  // extern "C"
