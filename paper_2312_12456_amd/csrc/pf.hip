// libpf host side: contexts, layers, argument checking and kernel launches behind the C ABI
// declared in include/pf.h.  gfx950 only.
#include "../../include/pf.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "k_predict.h"
#include "k_sparse.h"

namespace {

constexpr int kMaxBatch = 8;
constexpr int kChunksCap = 128;         // upper bound of neuron chunks in the FC2 kernel
constexpr int kLdsMax = 160 * 1024;     // LDS per workgroup on gfx950
constexpr int kLdsDefault = 64 * 1024;  // what a kernel may use without opting in

}  // namespace

struct pf_ctx {
    int device = 0;
    int max_d = 0, max_ffn = 0, max_r = 0, max_batch = 0;
    int num_cu = 256;
    int down_chunks = 64;    // grid.y of the FC2 kernel
    int down_min_rows = 16;  // least neurons per chunk
    int up_grid_cap = 2048;
    int lds_budget = kLdsDefault;  // dynamic LDS a kernel of this context may request
    // scratch (device)
    float *t = nullptr;             // [max_batch][max_r] predictor hidden vector
    uint64_t *mask_words = nullptr; // [max_ffn / 64]
    int32_t *idx = nullptr;         // [max_ffn]
    int32_t *count = nullptr;       // [1]
    float *h = nullptr;             // [max_batch][max_ffn] FC1 outputs of the listed neurons
    float *partial = nullptr;       // [kChunksCap][max_batch][max_d]
    unsigned int *arrive = nullptr; // [tiles + 1] arrival counters (zero between launches)
    float *ybuf = nullptr;          // [max_batch][max_d] FFN output inside pf_stack_step
    hipStream_t capture_stream = nullptr;
    char err[512] = {0};
};

struct pf_layer {
    pf_ctx *ctx;
    pf_layer_desc desc;
    pf_layer_weights w;
    float thr_logit;
};

struct pf_plan {
    pf_ctx *ctx;
    hipGraph_t graph;
    hipGraphExec_t exec;
};

namespace {

pf_status fail(pf_ctx *ctx, pf_status s, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

#define PF_HIP(ctx, call)                                                                   \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail((ctx), e_ == hipErrorOutOfMemory ? PF_ENOMEM : PF_EHIP, "%s: %s",   \
                        #call, hipGetErrorString(e_));                                      \
    } while (0)

inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline int kpad_of(int k) { return cdiv(k, pf::kChunk) * pf::kChunk; }

// Largest batch tile whose staged activations ([tile][kpad] fp32) fit the LDS budget.
inline int batch_tile(const pf_ctx *ctx, int k, int B)
{
    int fit = ctx->lds_budget / (kpad_of(k) * 4);
    if (fit > kMaxBatch) fit = kMaxBatch;
    return fit < B ? fit : B;
}

// ---- template dispatch over the batch tile -------------------------------------------
#define PF_SWITCH_B(Bt, ...)                                                 \
    switch (Bt) {                                                            \
        case 1: { constexpr int BT = 1; __VA_ARGS__; } break;                \
        case 2: { constexpr int BT = 2; __VA_ARGS__; } break;                \
        case 3: { constexpr int BT = 3; __VA_ARGS__; } break;                \
        case 4: { constexpr int BT = 4; __VA_ARGS__; } break;                \
        case 5: { constexpr int BT = 5; __VA_ARGS__; } break;                \
        case 6: { constexpr int BT = 6; __VA_ARGS__; } break;                \
        case 7: { constexpr int BT = 7; __VA_ARGS__; } break;                \
        default: { constexpr int BT = 8; __VA_ARGS__; } break;               \
    }

template <typename K>
hipError_t allow_lds(K kernel)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax);
}

template <int B>
hipError_t allow_lds_for_batch()
{
    hipError_t e = allow_lds(pf::k_pred_hidden<B>);
    if (e == hipSuccess) e = allow_lds(pf::k_up<B, 0>);
    if (e == hipSuccess) e = allow_lds(pf::k_up<B, 1>);
    return e;
}

hipError_t allow_lds_all()
{
    hipError_t e = allow_lds_for_batch<1>();
    if (e == hipSuccess) e = allow_lds_for_batch<2>();
    if (e == hipSuccess) e = allow_lds_for_batch<3>();
    if (e == hipSuccess) e = allow_lds_for_batch<4>();
    if (e == hipSuccess) e = allow_lds_for_batch<5>();
    if (e == hipSuccess) e = allow_lds_for_batch<6>();
    if (e == hipSuccess) e = allow_lds_for_batch<7>();
    if (e == hipSuccess) e = allow_lds_for_batch<8>();
    return e;
}

pf_status check_batch(pf_ctx *ctx, const pf_layer *layer, const void *x, int B)
{
    if (!ctx) return PF_EINVAL;
    if (!layer || !x) return fail(ctx, PF_EINVAL, "null layer or input");
    if (layer->ctx != ctx) return fail(ctx, PF_EINVAL, "layer belongs to another context");
    if (B < 1 || B > ctx->max_batch)
        return fail(ctx, PF_EINVAL, "batch %d outside [1, %d]", B, ctx->max_batch);
    return PF_OK;
}

// ---- launches ------------------------------------------------------------------------
pf_status launch_predict(pf_ctx *ctx, const pf_layer *L, const float *x, int B, float *scores,
                         uint64_t *mask_words, bool fuse_compact, hipStream_t st)
{
    const pf_layer_desc &D = L->desc;
    if (!L->w.p1 || !L->w.p2) return fail(ctx, PF_EINVAL, "layer has no predictor weights");
    const __half *p1 = static_cast<const __half *>(L->w.p1);
    const __half *p2 = static_cast<const __half *>(L->w.p2);
    // hidden layer, in batch tiles that fit LDS
    const int tile = batch_tile(ctx, D.d, B);
    for (int b0 = 0; b0 < B; b0 += tile) {
        const int bt = (B - b0) < tile ? (B - b0) : tile;
        const size_t lds = (size_t)bt * kpad_of(D.d) * sizeof(float);
        const dim3 grid(cdiv(D.r, pf::kPredThreads / pf::kWave));
        PF_SWITCH_B(bt, hipLaunchKernelGGL(pf::k_pred_hidden<BT>, grid, dim3(pf::kPredThreads),
                                           lds, st, p1, x + (size_t)b0 * D.d,
                                           ctx->t + (size_t)b0 * D.r, D.d, D.r));
    }
    // output layer over the whole batch (its staged vector is only B * r floats)
    const size_t lds = (size_t)B * kpad_of(D.r) * sizeof(float);
    const dim3 grid(D.ffn / 64);
    unsigned int *arrive = ctx->arrive;  // slot 0: predictor arrival counter
    if (fuse_compact) {
        PF_SWITCH_B(B, hipLaunchKernelGGL((pf::k_pred_out<BT, true>), grid,
                                          dim3(pf::kPredOutThreads), lds, st, p2, L->w.p_bias,
                                          ctx->t, D.r, D.ffn, L->thr_logit, scores, mask_words,
                                          arrive, ctx->idx, ctx->count));
    } else {
        PF_SWITCH_B(B, hipLaunchKernelGGL((pf::k_pred_out<BT, false>), grid,
                                          dim3(pf::kPredOutThreads), lds, st, p2, L->w.p_bias,
                                          ctx->t, D.r, D.ffn, L->thr_logit, scores, mask_words,
                                          arrive, (int32_t *)nullptr, (int32_t *)nullptr));
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status launch_sparse(pf_ctx *ctx, const pf_layer *L, const float *x, int B,
                        const int32_t *idx, const int32_t *count, float *y, hipStream_t st)
{
    const pf_layer_desc &D = L->desc;
    const __half *w_up = static_cast<const __half *>(L->w.w_up);
    const __half *w_gate = static_cast<const __half *>(L->w.w_gate);
    const __half *w_down = static_cast<const __half *>(L->w.w_down);
    const int tile = batch_tile(ctx, D.d, B);
    int up_grid = cdiv(D.ffn, pf::kUpWaves);
    if (up_grid > ctx->up_grid_cap) up_grid = ctx->up_grid_cap;
    for (int b0 = 0; b0 < B; b0 += tile) {
        const int bt = (B - b0) < tile ? (B - b0) : tile;
        const size_t lds = (size_t)bt * kpad_of(D.d) * sizeof(float);
        if (D.act == PF_ACT_REGLU) {
            PF_SWITCH_B(bt, hipLaunchKernelGGL((pf::k_up<BT, 1>), dim3(up_grid),
                                               dim3(pf::kUpThreads), lds, st, w_up, w_gate,
                                               L->w.b_up, x + (size_t)b0 * D.d, idx, count,
                                               ctx->h + (size_t)b0 * D.ffn, D.d, D.ffn));
        } else {
            PF_SWITCH_B(bt, hipLaunchKernelGGL((pf::k_up<BT, 0>), dim3(up_grid),
                                               dim3(pf::kUpThreads), lds, st, w_up, w_gate,
                                               L->w.b_up, x + (size_t)b0 * D.d, idx, count,
                                               ctx->h + (size_t)b0 * D.ffn, D.d, D.ffn));
        }
    }
    const dim3 grid(cdiv(D.d, pf::kDownTile), ctx->down_chunks);
    PF_SWITCH_B(B, hipLaunchKernelGGL(pf::k_down<BT>, grid, dim3(pf::kDownThreads), 0, st, w_down,
                                      L->w.b_down, ctx->h, idx, count, ctx->partial,
                                      ctx->arrive + 1, y, D.d, D.ffn, ctx->down_min_rows));
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status launch_glue(pf_ctx *ctx, const float *x, const float *y, int d, int B, float *x_next,
                      hipStream_t st)
{
    hipLaunchKernelGGL(pf::k_glue, dim3(B), dim3(pf::kGlueThreads), 0, st, x, y, x_next, d);
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status stack_enqueue(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x, int B,
                        float *x_out, hipStream_t st)
{
    const float *cur = x;
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer *L = layers[l];
        pf_status s = launch_predict(ctx, L, cur, B, nullptr, ctx->mask_words, true, st);
        if (s != PF_OK) return s;
        s = launch_sparse(ctx, L, cur, B, ctx->idx, ctx->count, ctx->ybuf, st);
        if (s != PF_OK) return s;
        s = launch_glue(ctx, cur, ctx->ybuf, L->desc.d, B, x_out, st);
        if (s != PF_OK) return s;
        cur = x_out;
    }
    return PF_OK;
}

pf_status check_stack(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x, int B,
                      float *x_out)
{
    if (!ctx) return PF_EINVAL;
    if (!layers || !x || !x_out || n_layers < 1)
        return fail(ctx, PF_EINVAL, "null argument or empty stack");
    for (int l = 0; l < n_layers; ++l) {
        pf_status s = check_batch(ctx, layers[l], x, B);
        if (s != PF_OK) return s;
        if (layers[l]->desc.d != layers[0]->desc.d)
            return fail(ctx, PF_ESHAPE, "layer %d has d=%d, layer 0 has d=%d", l,
                        layers[l]->desc.d, layers[0]->desc.d);
        if (!layers[l]->w.p1) return fail(ctx, PF_EINVAL, "layer %d has no predictor", l);
    }
    return PF_OK;
}

}  // namespace

extern "C" {

pf_status pf_ctx_create(pf_ctx **out, int device, int max_d, int max_ffn, int max_r, int max_batch)
{
    if (!out) return PF_EINVAL;
    *out = nullptr;
    if (max_d < 1 || max_ffn < 1 || max_r < 1 || max_batch < 1 || max_batch > kMaxBatch || device < 0)
        return PF_EINVAL;
    if (max_ffn % 64 != 0 || max_d % 8 != 0 || max_r % 8 != 0) return PF_ESHAPE;
    // the staged hidden vector of the whole batch and one staged token must fit LDS
    if ((size_t)max_batch * kpad_of(max_r) * sizeof(float) > (size_t)kLdsDefault - 16 * 1024 ||
        (size_t)kpad_of(max_d) * sizeof(float) > (size_t)kLdsDefault)
        return PF_ESHAPE;
    pf_ctx *ctx = new (std::nothrow) pf_ctx();
    if (!ctx) return PF_ENOMEM;
    ctx->device = device;
    ctx->max_d = max_d;
    ctx->max_ffn = max_ffn;
    ctx->max_r = max_r;
    ctx->max_batch = max_batch;
    pf_status st = PF_OK;
    do {
        hipError_t e = hipSetDevice(device);
        if (e != hipSuccess) { st = PF_EHIP; break; }
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) { st = PF_EHIP; break; }
        if (prop.multiProcessorCount > 0) ctx->num_cu = prop.multiProcessorCount;
        const int tiles = cdiv(max_d, pf::kDownTile);
        int chunks = (4 * ctx->num_cu) / tiles;
        if (chunks < 1) chunks = 1;
        if (chunks > kChunksCap) chunks = kChunksCap;
        ctx->down_chunks = chunks;
        ctx->up_grid_cap = 8 * ctx->num_cu;
        if (const char *v = getenv("PF_DOWN_CHUNKS")) {
            int c = atoi(v);
            if (c >= 1 && c <= kChunksCap) ctx->down_chunks = c;
        }
        if (const char *v = getenv("PF_DOWN_MIN_ROWS")) {
            int c = atoi(v);
            if (c >= 1) ctx->down_min_rows = c;
        }
        if (const char *v = getenv("PF_UP_GRID")) {
            int c = atoi(v);
            if (c >= 1 && c <= 65535) ctx->up_grid_cap = c;
        }
        // larger staged batches need the opt-in LDS size; without it batches are tiled smaller
        if (prop.sharedMemPerBlock >= (size_t)kLdsMax || prop.maxSharedMemoryPerMultiProcessor >= (size_t)kLdsMax) {
            if (allow_lds_all() == hipSuccess)
                ctx->lds_budget = kLdsMax;
            else
                (void)hipGetLastError();
        }
#define PF_ALLOC(ptr, bytes)                                                  \
        e = hipMalloc(reinterpret_cast<void **>(&(ptr)), (bytes));            \
        if (e != hipSuccess) { st = e == hipErrorOutOfMemory ? PF_ENOMEM : PF_EHIP; break; }
        PF_ALLOC(ctx->t, (size_t)max_batch * max_r * sizeof(float));
        PF_ALLOC(ctx->mask_words, (size_t)(max_ffn / 64) * sizeof(uint64_t));
        PF_ALLOC(ctx->idx, (size_t)max_ffn * sizeof(int32_t));
        PF_ALLOC(ctx->count, 64);
        PF_ALLOC(ctx->h, (size_t)max_batch * max_ffn * sizeof(float));
        PF_ALLOC(ctx->partial, (size_t)kChunksCap * max_batch * max_d * sizeof(float));
        PF_ALLOC(ctx->arrive, (size_t)(tiles + 1) * sizeof(unsigned int));
        PF_ALLOC(ctx->ybuf, (size_t)max_batch * max_d * sizeof(float));
#undef PF_ALLOC
        e = hipMemset(ctx->arrive, 0, (size_t)(tiles + 1) * sizeof(unsigned int));
        if (e == hipSuccess) e = hipMemset(ctx->count, 0, 64);
        if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->capture_stream, hipStreamNonBlocking);
        if (e != hipSuccess) { st = PF_EHIP; break; }
    } while (0);
    if (st != PF_OK) {
        pf_ctx_destroy(ctx);
        return st;
    }
    *out = ctx;
    return PF_OK;
}

void pf_ctx_destroy(pf_ctx *ctx)
{
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    if (ctx->capture_stream) (void)hipStreamDestroy(ctx->capture_stream);
    (void)hipFree(ctx->t);
    (void)hipFree(ctx->mask_words);
    (void)hipFree(ctx->idx);
    (void)hipFree(ctx->count);
    (void)hipFree(ctx->h);
    (void)hipFree(ctx->partial);
    (void)hipFree(ctx->arrive);
    (void)hipFree(ctx->ybuf);
    delete ctx;
}

pf_status pf_layer_create(pf_ctx *ctx, const pf_layer_desc *desc, const pf_layer_weights *w,
                          pf_layer **out)
{
    if (!ctx) return PF_EINVAL;
    if (!out) return fail(ctx, PF_EINVAL, "out is null");
    *out = nullptr;
    if (!desc || !w) return fail(ctx, PF_EINVAL, "null descriptor or weights");
    if (desc->d < 1 || desc->ffn < 1 || desc->r < 1)
        return fail(ctx, PF_EINVAL, "non-positive size");
    if (!(desc->threshold > 0.f && desc->threshold < 1.f))
        return fail(ctx, PF_EINVAL, "threshold %g outside (0,1)", (double)desc->threshold);
    if (desc->act != PF_ACT_RELU && desc->act != PF_ACT_REGLU)
        return fail(ctx, PF_EUNSUPPORTED, "activation %d", desc->act);
    if (desc->wtype != PF_W_FP16 && desc->wtype != PF_W_INT4_G128)
        return fail(ctx, PF_EUNSUPPORTED, "weight type %d", desc->wtype);
    if (desc->ffn % 64 != 0) return fail(ctx, PF_ESHAPE, "ffn %d is not a multiple of 64", desc->ffn);
    if (desc->d % 8 != 0) return fail(ctx, PF_ESHAPE, "d %d is not a multiple of 8", desc->d);
    if (desc->r % 8 != 0) return fail(ctx, PF_ESHAPE, "r %d is not a multiple of 8", desc->r);
    if (desc->wtype == PF_W_INT4_G128 && desc->d % 128 != 0)
        return fail(ctx, PF_ESHAPE, "int4 needs d %% 128 == 0, got %d", desc->d);
    if (desc->d > ctx->max_d || desc->ffn > ctx->max_ffn || desc->r > ctx->max_r)
        return fail(ctx, PF_ESHAPE, "layer (d=%d, ffn=%d, r=%d) exceeds context (%d, %d, %d)",
                    desc->d, desc->ffn, desc->r, ctx->max_d, ctx->max_ffn, ctx->max_r);
    if (!w->w_up || !w->w_down) return fail(ctx, PF_EINVAL, "w_up / w_down is null");
    if (desc->act == PF_ACT_REGLU && !w->w_gate) return fail(ctx, PF_EINVAL, "gated layer without w_gate");
    if ((w->p1 == nullptr) != (w->p2 == nullptr))
        return fail(ctx, PF_EINVAL, "p1 and p2 must both be given or both be null");
    if (desc->wtype == PF_W_INT4_G128) {
        if (!w->s_up || !w->s_down || (desc->act == PF_ACT_REGLU && !w->s_gate))
            return fail(ctx, PF_EINVAL, "int4 layer without scales");
        return fail(ctx, PF_EUNSUPPORTED, "int4 weights are not built yet");
    }
    pf_layer *L = new (std::nothrow) pf_layer();
    if (!L) return fail(ctx, PF_ENOMEM, "host allocation failed");
    L->ctx = ctx;
    L->desc = *desc;
    L->w = *w;
    const double tau = (double)desc->threshold;
    L->thr_logit = (float)std::log(tau / (1.0 - tau));
    *out = L;
    return PF_OK;
}

void pf_layer_destroy(pf_layer *layer) { delete layer; }

pf_status pf_predict(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *scores,
                     uint64_t *mask_words, void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!mask_words) return fail(ctx, PF_EINVAL, "mask_words is null");
    return launch_predict(ctx, layer, x, B, scores, mask_words, false, static_cast<hipStream_t>(stream));
}

pf_status pf_compact(pf_ctx *ctx, const uint64_t *mask_words, int ffn, int32_t *idx, int32_t *count,
                     void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!mask_words || !idx || !count) return fail(ctx, PF_EINVAL, "null argument");
    if (ffn < 0) return fail(ctx, PF_EINVAL, "negative ffn");
    if (ffn % 64 != 0) return fail(ctx, PF_ESHAPE, "ffn %d is not a multiple of 64", ffn);
    hipLaunchKernelGGL(pf::k_compact, dim3(1), dim3(pf::kCompactThreads), 0,
                       static_cast<hipStream_t>(stream), mask_words, ffn / 64, idx, count);
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status pf_sparse_ffn(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, const int32_t *idx,
                        const int32_t *count, float *y, void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!idx || !count || !y) return fail(ctx, PF_EINVAL, "null argument");
    return launch_sparse(ctx, layer, x, B, idx, count, y, static_cast<hipStream_t>(stream));
}

pf_status pf_layer_step(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *y,
                        void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!y) return fail(ctx, PF_EINVAL, "y is null");
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = launch_predict(ctx, layer, x, B, nullptr, ctx->mask_words, true, st);
    if (s != PF_OK) return s;
    return launch_sparse(ctx, layer, x, B, ctx->idx, ctx->count, y, st);
}

pf_status pf_ctx_last_active(pf_ctx *ctx, const uint64_t **mask_words, const int32_t **idx,
                             const int32_t **count)
{
    if (!ctx) return PF_EINVAL;
    if (mask_words) *mask_words = ctx->mask_words;
    if (idx) *idx = ctx->idx;
    if (count) *count = ctx->count;
    return PF_OK;
}

pf_status pf_stack_glue(pf_ctx *ctx, const float *x, const float *y, int d, int B, float *x_next,
                        void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!x || !y || !x_next) return fail(ctx, PF_EINVAL, "null argument");
    if (d < 1 || B < 1) return fail(ctx, PF_EINVAL, "non-positive size");
    return launch_glue(ctx, x, y, d, B, x_next, static_cast<hipStream_t>(stream));
}

pf_status pf_stack_step(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x, int B,
                        float *x_out, void *stream)
{
    pf_status s = check_stack(ctx, layers, n_layers, x, B, x_out);
    if (s != PF_OK) return s;
    return stack_enqueue(ctx, layers, n_layers, x, B, x_out, static_cast<hipStream_t>(stream));
}

pf_status pf_plan_create(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x, int B,
                         float *x_out, void *stream, pf_plan **out)
{
    (void)stream;
    if (!ctx) return PF_EINVAL;
    if (!out) return fail(ctx, PF_EINVAL, "out is null");
    *out = nullptr;
    pf_status s = check_stack(ctx, layers, n_layers, x, B, x_out);
    if (s != PF_OK) return s;
    pf_plan *plan = new (std::nothrow) pf_plan();
    if (!plan) return fail(ctx, PF_ENOMEM, "host allocation failed");
    plan->ctx = ctx;
    plan->graph = nullptr;
    plan->exec = nullptr;
    hipStream_t cs = ctx->capture_stream;
    hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) {
        delete plan;
        return fail(ctx, PF_EHIP, "hipStreamBeginCapture: %s", hipGetErrorString(e));
    }
    s = stack_enqueue(ctx, layers, n_layers, x, B, x_out, cs);
    e = hipStreamEndCapture(cs, &plan->graph);
    if (s == PF_OK && e != hipSuccess) s = fail(ctx, PF_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
    if (s == PF_OK) {
        e = hipGraphInstantiate(&plan->exec, plan->graph, nullptr, nullptr, 0);
        if (e != hipSuccess) s = fail(ctx, PF_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e));
    }
    if (s != PF_OK) {
        pf_plan_destroy(plan);
        return s;
    }
    *out = plan;
    return PF_OK;
}

pf_status pf_plan_run(pf_plan *plan, void *stream)
{
    if (!plan || !plan->exec) return PF_EINVAL;
    PF_HIP(plan->ctx, hipGraphLaunch(plan->exec, static_cast<hipStream_t>(stream)));
    return PF_OK;
}

void pf_plan_destroy(pf_plan *plan)
{
    if (!plan) return;
    if (plan->exec) (void)hipGraphExecDestroy(plan->exec);
    if (plan->graph) (void)hipGraphDestroy(plan->graph);
    delete plan;
}

const char *pf_strerror(pf_status s)
{
    switch (s) {
        case PF_OK: return "ok";
        case PF_EINVAL: return "invalid argument";
        case PF_ESHAPE: return "unsupported shape";
        case PF_ENOMEM: return "out of memory";
        case PF_EHIP: return "HIP runtime error";
        case PF_EUNSUPPORTED: return "not supported";
    }
    return "unknown status";
}

const char *pf_last_error(const pf_ctx *ctx) { return ctx ? ctx->err : ""; }

const char *pf_version(void) { return "libpf 0.1 (gfx950)"; }

}  // extern "C"
