// libpf host side: contexts, layers, argument checking and kernel launches behind the C ABI
// declared in include/pf.h.  gfx950 only.
#include "../../include/pf.h"

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "k_predict.h"
#include "k_sparse.h"
#include "k_int4.h"
#include "k_mfma.h"
#include "k_fused.h"
#include "k_lookahead.h"

namespace {

constexpr int kMaxBatch = 8;
constexpr int kMaxFfn = 4096 * 64;      // the in-kernel bit select handles 4096 mask words
constexpr int kProfPairsCap = 32768;    // event pairs one profiling pass may record
constexpr int kLdsMax = 160 * 1024;     // LDS per workgroup on gfx950
constexpr int kLdsDefault = 64 * 1024;  // what a kernel may use without opting in

enum KernelId {
    K_PRED_HIDDEN = 0, K_PRED_OUT, K_COMPACT, K_UP, K_DOWN, K_GLUE, K_UP_MFMA, K_COMBINE, K_OUT_UP,
    K_DOWN_MASK, K_LA_UP_HIDDEN, K_LA_DOWN_OUT, K_NUM
};
static_assert(K_NUM <= 16, "pf_profile_end documents a capacity of 16 entries");
const char *const kKernelNames[K_NUM] = {"k_pred_hidden", "k_pred_out", "k_compact", "k_up",
                                         "k_down",        "k_glue",     "k_up_mfma",  "k_combine",
                                         "k_out_up",      "k_down_mask", "k_la_up_hidden",
                                         "k_la_down_out"};

}  // namespace

struct pf_ctx {
    int device = 0;
    int max_d = 0, max_ffn = 0, max_r = 0, max_batch = 0;
    int num_cu = 256;
    int up_grid_cap = 2048;
    int up_grid_cap_i4 = 512;
    int mfma_grid = 0;              // PF_OPT_MFMA_GRID: blocks of k_up_mfma (0 = from the CU count)
    // The hidden layer goes to the matrix cores only above this B * d: below it the vector kernel
    // with the glue fused in beats MFMA + a glue kernel of its own (measured: +1..3 % on the
    // stack at 4 x 4096 and 4 x 5120, -9 % and worse from 8 x 4096 on).
    int hidden_mfma_min_elems = 20480;
    int lds_budget = kLdsDefault;  // dynamic LDS a kernel of this context may request
    int down_split = 0;            // PF_OPT_DOWN_SPLIT: row groups of FC2 (0 = from the CU count)
    int mfma_min_batch = 4;        // FC1 goes to the matrix cores from this batch size on
    bool mfma_min_batch_forced = false;  // set through PF_OPT_MFMA_MIN_BATCH
    int fused = 1;                 // PF_OPT_FUSED: inner layers of a stack as three launches (0 never,
                                   // 1 where measured faster, 2 wherever possible)
    int seg_strided = 0;           // PF_OPT_SEG_STRIDED: strided segments (models stored hot-first)
    int la_form = 0;               // PF_OPT_LOOKAHEAD_FORM: 0 automatic, 1 two launches per layer,
                                   // 2 second stream, 3 one stream

    uint64_t *mask_trace = nullptr;  // caller's buffer for every layer's mask words (or null)
    int mask_trace_layers = 0;
    // scratch (device)
    float *t = nullptr;              // [max_batch][max_r] predictor hidden vector
    uint64_t *mask_words = nullptr;  // [max_ffn / 64]
    int32_t *idx = nullptr;          // [max_ffn]
    int32_t *count = nullptr;        // [1]
    int32_t *idx_all = nullptr;      // [max_ffn] 0, 1, 2, ...: the list of the dense path
    int32_t *count_all = nullptr;    // [1] = max_ffn (kernels clamp the count to the layer's ffn)
    const uint64_t *last_mask = nullptr;  // what the last layer step used
    const int32_t *last_idx = nullptr, *last_count = nullptr;
    float *h = nullptr;              // [max_ffn][h_stride(batch)] FC1 outputs, by list slot
    float *ypart = nullptr;          // [4][max_batch][max_d] FC2 output as partial sums
    float *xbuf[2] = {nullptr, nullptr};  // [max_batch][max_d] layer inputs inside pf_stack_step
    // fp16 hi + lo planes of the activations the matrix-core kernels read ([2][B][d] halfs each;
    // two buffers, used in turn); split_src = the fp32 array whose split xsplit[split_cur] holds,
    // valid within one entry-point call only (reset by check_batch)
    __half *xsplit[2] = {nullptr, nullptr};
    const float *split_src = nullptr;
    int split_cur = 0;
    bool split_off = false;  // set while kernels are enqueued on a second stream
    hipStream_t capture_stream = nullptr;
    // look-ahead mode: predictors on a stream of their own, masks double-buffered
    int lookahead = 0;
    hipStream_t side_stream = nullptr;
    uint64_t *mask_words2 = nullptr;        // [max_ffn / 64]
    std::vector<hipEvent_t> la_events;      // fork / join events, created on demand
    // per-kernel timing with HIP events (pf_profile_begin / pf_profile_end)
    bool prof_on = false;
    bool capturing = false;
    std::vector<hipEvent_t> prof_events;  // start/stop pairs, created on demand, reused
    std::vector<int> prof_kernel;         // kernel id of each recorded pair
    char err[512] = {0};
};

struct pf_layer {
    pf_ctx *ctx;
    pf_layer_desc desc;
    pf_layer_weights w;
    float thr_logit;
    const int32_t *table = nullptr;  // stored neuron -> original neuron (borrowed), or null
    int always_on = 0;               // stored neurons [0, always_on) are listed without prediction
    int32_t *adapt = nullptr;        // device: {dense flag for the next adaptive step, neurons
                                     // counted at the last one, mode of the last one}; owned
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
// Lower clamp of the up branch in the gated kernels: none for the ReLU-gated block, 0 for dReLU.
inline float up_floor_of(const pf_layer_desc &D) { return D.act == PF_ACT_DRELU ? 0.f : -INFINITY; }
inline float logit_of(float tau) { return (float)std::log((double)tau / (1.0 - (double)tau)); }
inline int kpad_of(int k) { return cdiv(k, pf::kChunk) * pf::kChunk; }

// Largest batch tile whose staged activations ([tile][kpad] fp32) plus `extra` bytes fit LDS.
inline int batch_tile(const pf_ctx *ctx, int k, int B, size_t extra)
{
    int fit = (int)(((size_t)ctx->lds_budget - extra) / ((size_t)kpad_of(k) * 4));
    if (fit > kMaxBatch) fit = kMaxBatch;
    if (fit < 1) fit = 1;
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

// The three-launch kernels exist for batch 1..3 only (fused_ok).
#define PF_SWITCH_B3(Bt, ...)                                                \
    switch (Bt) {                                                            \
        case 1: { constexpr int BT = 1; __VA_ARGS__; } break;                \
        case 2: { constexpr int BT = 2; __VA_ARGS__; } break;                \
        default: { constexpr int BT = 3; __VA_ARGS__; } break;               \
    }

// Opt a kernel in to the full 160 KB of LDS: dynamic limit = 160 KB minus its static LDS.
template <typename K>
hipError_t allow_lds(K kernel)
{
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(kernel));
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               kLdsMax - (int)attr.sharedSizeBytes);
}

template <int B>
hipError_t allow_lds_for_batch()
{
    hipError_t e = allow_lds(pf::k_pred_hidden<B, false>);
    if (e == hipSuccess && B == 1) e = allow_lds(pf::k_pred_hidden<1, true, 4>);
    if (e == hipSuccess) e = allow_lds(pf::k_pred_hidden<B, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_up<B, 0, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up<B, 1, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up<B, 0, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_up<B, 1, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_i4<B, 0, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_i4<B, 1, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_i4<B, 0, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_i4<B, 1, true>);
    if constexpr (B <= 3) {
        if (e == hipSuccess) e = allow_lds(pf::k_out_up<B, 0>);
        if (e == hipSuccess) e = allow_lds(pf::k_out_up<B, 1>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden<B, 0, false>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden<B, 0, true>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden<B, 1, false>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden<B, 1, true>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_down_out<B>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden_i4<B, 0>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden_i4<B, 1>);
        if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_i4<B>);
    }
    return e;
}

hipError_t allow_lds_mfma()
{
    hipError_t e = allow_lds(pf::k_up_mfma<0, false, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_mfma<0, true, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_mfma<1, false, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_mfma<1, true, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_mfma<0, true, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_up_mfma<1, true, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_rows_mfma<8, 512, 0, true>);
    if (e == hipSuccess) e = allow_lds(pf::k_rows_mfma<8, 512, 0, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_rows_mfma<64, 64, 1, false>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden_mfma<0>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_up_hidden_mfma<1>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_mfma<3>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_mfma<4>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_mfma<5>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_mfma<6>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_mfma<7>);
    if (e == hipSuccess) e = allow_lds(pf::k_la_down_out_mfma<8>);
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
    if (e == hipSuccess) e = allow_lds_mfma();
    return e;
}

pf_status check_batch(pf_ctx *ctx, const pf_layer *layer, const void *x, int B)
{
    if (ctx) ctx->split_src = nullptr;  // no split planes carry over from an earlier call
    if (!ctx) return PF_EINVAL;
    if (!layer || !x) return fail(ctx, PF_EINVAL, "null layer or input");
    if (layer->ctx != ctx) return fail(ctx, PF_EINVAL, "layer belongs to another context");
    if (B < 1 || B > ctx->max_batch)
        return fail(ctx, PF_EINVAL, "batch %d outside [1, %d]", B, ctx->max_batch);
    return PF_OK;
}

// While profiling is on, hands out a pair of events for one kernel launch; the launch then
// goes through hipExtLaunchKernelGGL, which stamps them with the kernel's own start and
// end times on its stream (nothing but the kernel lies between the two stamps).
struct ProfScope {
    hipEvent_t start = nullptr, stop = nullptr;
    ProfScope(pf_ctx *c, int kernel)
    {
        if (!c->prof_on || c->capturing || (int)c->prof_kernel.size() >= kProfPairsCap) return;
        const size_t pair = c->prof_kernel.size();
        while (c->prof_events.size() < 2 * (pair + 1)) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return;
            c->prof_events.push_back(e);
        }
        c->prof_kernel.push_back(kernel);
        start = c->prof_events[2 * pair];
        stop = c->prof_events[2 * pair + 1];
    }
};

#define PF_LAUNCH(ps, kernel, grid, block, lds, st, ...)                                          \
    do {                                                                                          \
        if ((ps).start)                                                                           \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, st, (ps).start, (ps).stop, 0,         \
                                  __VA_ARGS__);                                                   \
        else                                                                                      \
            hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                        \
    } while (0)

// ---- launches ------------------------------------------------------------------------
pf_status launch_glue(pf_ctx *ctx, const float *x, const float *y, int ny, int d, int B,
                      float *x_next, hipStream_t st, bool split = false);
const __half *split_of(const pf_ctx *ctx, const float *x);
pf_status ensure_split(pf_ctx *ctx, const float *x, int B, int d, hipStream_t st, const __half **xs);

// Batch size from which a layer's kernels run on the matrix cores: 4, and already 3 for rows
// longer than 4096 (measured at batch 3: OPT-30B shape 1 001 against 925 tokens/s, LLaMA-13B
// shape 1 439 against 1 409, but OPT-6.7B shape 2 557 against 3 042); PF_OPT_MFMA_MIN_BATCH
// overrides.
inline int mfma_from(const pf_ctx *ctx, const pf_layer_desc &D)
{
    if (ctx->mfma_min_batch_forced || ctx->mfma_min_batch <= 3) return ctx->mfma_min_batch;
    return D.d > 4096 ? 3 : ctx->mfma_min_batch;
}

// The predictor runs on the matrix cores from the same batch size on as FC1 (row length a
// multiple of 32, and the opt-in LDS size for its 64 KB of slots + static LDS).
inline bool pred_mfma(const pf_ctx *ctx, const pf_layer_desc &D, int K, int B)
{
    return B >= mfma_from(ctx, D) && K % 32 == 0 && ctx->lds_budget > kLdsDefault;
}

// Predictor hidden layer.  With glue_y the layer input is formed inside the kernel as
// norm(x + glue_y) and also written to x_new.
pf_status launch_hidden(pf_ctx *ctx, const pf_layer *L, const float *x, const float *glue_y,
                        int glue_ny, float *x_new, int B, hipStream_t st, const int32_t *skip = nullptr)
{
    const pf_layer_desc &D = L->desc;
    if (!L->w.p1 || !L->w.p2) return fail(ctx, PF_EINVAL, "layer has no predictor weights");
    const __half *p1 = static_cast<const __half *>(L->w.p1);
    if (pred_mfma(ctx, D, D.d, B) && (size_t)B * (size_t)D.d > (size_t)ctx->hidden_mfma_min_elems) {
        // a batch on the matrix cores; the glue, if any, as a kernel of its own in front
        if (glue_y) {
            pf_status s = launch_glue(ctx, x, glue_y, glue_ny, D.d, B, x_new, st, true);
            if (s != PF_OK) return s;
            x = x_new;
        }
        const __half *xs = nullptr;  // the activations as fp16 hi + lo planes where possible
        pf_status s = ensure_split(ctx, x, B, D.d, st, &xs);
        if (s != PF_OK) return s;
        ProfScope ps(ctx, K_PRED_HIDDEN);
        if (xs)
            PF_LAUNCH(ps, (pf::k_rows_mfma<8, 512, 0, true>), dim3(cdiv(D.r, 8)), dim3(pf::kMfmaThreads),
                      (size_t)pf::kMfmaWaves * pf::kRowsMfmaSlotBytes, st, p1, (const void *)xs, B, D.d, D.r,
                      (const float *)nullptr, 0.f, ctx->t, (uint64_t *)nullptr, 0, skip);
        else
            PF_LAUNCH(ps, (pf::k_rows_mfma<8, 512, 0, false>), dim3(cdiv(D.r, 8)), dim3(pf::kMfmaThreads),
                      (size_t)pf::kMfmaWaves * pf::kRowsMfmaSlotBytes, st, p1, (const void *)x, B, D.d, D.r,
                      (const float *)nullptr, 0.f, ctx->t, (uint64_t *)nullptr, 0, skip);
        PF_HIP(ctx, hipGetLastError());
        return PF_OK;
    }
    // hidden layer, in batch tiles that fit LDS
    if (glue_y && ctx->split_src == x_new) ctx->split_src = nullptr;  // x_new is rewritten as fp32 only
    const int tile = batch_tile(ctx, D.d, B, 1024);
    for (int b0 = 0; b0 < B; b0 += tile) {
        const int bt = (B - b0) < tile ? (B - b0) : tile;
        const size_t lds = ((size_t)bt * kpad_of(D.d) + pf::kStageScrap) * sizeof(float);
        const dim3 grid(cdiv(D.r, pf::kPredWaves));
        const size_t xo = (size_t)b0 * D.d;
        ProfScope ps(ctx, K_PRED_HIDDEN);
        if (glue_y && bt == 1 && kpad_of(D.d) <= 4096) {  // the whole glue in one round trip
            PF_LAUNCH(ps, (pf::k_pred_hidden<1, true, 4>), grid, dim3(pf::kPredThreads), lds, st, p1,
                      x + xo, glue_y + xo, glue_ny, B * D.d, x_new + xo, ctx->t + (size_t)b0 * D.r, D.d,
                      D.r, b0, skip);
        } else if (glue_y) {
            PF_SWITCH_B(bt, PF_LAUNCH(ps, (pf::k_pred_hidden<BT, true>), grid,
                                               dim3(pf::kPredThreads), lds, st, p1, x + xo,
                                               glue_y + xo, glue_ny, B * D.d, x_new + xo,
                                               ctx->t + (size_t)b0 * D.r, D.d, D.r, b0, skip));
        } else {
            PF_SWITCH_B(bt, PF_LAUNCH(ps, (pf::k_pred_hidden<BT, false>), grid,
                                               dim3(pf::kPredThreads), lds, st, p1, x + xo,
                                               (const float *)nullptr, 0, 0, (float *)nullptr,
                                               ctx->t + (size_t)b0 * D.r, D.d, D.r, b0, skip));
        }
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// Workgroups of the predictor's output layer: one per mask word past the always-on prefix; at
// least one, which then also marks the prefix (a layer whose neurons are all always on keeps
// its last word predicted).
inline int pred_out_words(const pf_layer *L) { return L->desc.ffn / 64 - L->always_on / 64; }

// Predictor: hidden layer, then output layer + ballot into mask words.
pf_status launch_predict(pf_ctx *ctx, const pf_layer *L, const float *x, const float *glue_y,
                         int glue_ny, float *x_new, int B, float *scores, uint64_t *mask_words,
                         hipStream_t st, const int32_t *skip = nullptr)
{
    pf_status s = launch_hidden(ctx, L, x, glue_y, glue_ny, x_new, B, st, skip);
    if (s != PF_OK) return s;
    const pf_layer_desc &D = L->desc;
    const __half *p2 = static_cast<const __half *>(L->w.p2);
    if (pred_mfma(ctx, D, D.r, B)) {
        ProfScope ps(ctx, K_PRED_OUT);
        PF_LAUNCH(ps, (pf::k_rows_mfma<64, 64, 1, false>), dim3(pred_out_words(L)), dim3(pf::kMfmaThreads),
                  (size_t)pf::kMfmaWaves * pf::kRowsMfmaSlotBytes, st, p2, (const void *)ctx->t, B, D.r,
                  D.ffn, L->w.p_bias, L->thr_logit, scores, mask_words, L->always_on / 64, skip);
        PF_HIP(ctx, hipGetLastError());
        return PF_OK;
    }
    // output layer over the whole batch (its staged vector is only B * r floats)
    const size_t lds = ((size_t)B * kpad_of(D.r) + pf::kStageScrap) * sizeof(float);
    const dim3 grid(pred_out_words(L));
    {
        ProfScope ps(ctx, K_PRED_OUT);
        PF_SWITCH_B(B, PF_LAUNCH(ps, pf::k_pred_out<BT>, grid, dim3(pf::kPredOutThreads), lds,
                                          st, p2, L->w.p_bias, ctx->t, D.r, D.ffn, L->thr_logit,
                                          scores, mask_words, L->always_on / 64, skip));
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// Row groups of FC2 (P): with `tiles` column tiles the launch has tiles * P workgroups, each
// over 1/P of the listed rows.  One round of workgroups (<= one per CU) costs 1/P; two
// workgroups share a CU at about 1.6 x the time of one while the batch is small enough for two
// to be resident (measured at 112 and 128 tiles; at batch 8 the second workgroup waits); more
// rounds cost a round each.  Ties go to the smaller P (fewer partial sums to add).
// two_per_cu = false: one round only (FC2 over segments, whose workgroups carry more state;
// measured at the OPT-30B and Falcon-40B shapes at batch 2: 776 against 752, 638 against 628).
inline int fc2_split(const pf_ctx *ctx, int tiles, int B, bool two_per_cu = true)
{
    if (ctx->down_split > 0) return ctx->down_split < pf::kDown2MaxSplit ? ctx->down_split : pf::kDown2MaxSplit;
    int best = 1;
    double best_cost = 1e30;
    for (int P = 1; P <= pf::kDown2MaxSplit; ++P) {
        const int blocks = tiles * P;
        double rounds;
        if (blocks <= ctx->num_cu)
            rounds = 1.0;
        else if (two_per_cu && B <= 4 && blocks <= 2 * ctx->num_cu)
            rounds = 1.6;
        else
            rounds = (double)cdiv(blocks, ctx->num_cu);
        const double cost = rounds / P;
        if (cost < best_cost - 1e-9) {
            best_cost = cost;
            best = P;
        }
    }
    return best;
}

inline int kpad_i4(int k) { return cdiv(k, pf::kI4Chunk) * pf::kI4Chunk; }

// Sparse FFN over int4 weights (same launch structure as the fp16 one below).
pf_status launch_sparse_i4(pf_ctx *ctx, const pf_layer *L, const float *x, int B,
                           const int32_t *idx_in, const int32_t *count_in,
                           const uint64_t *mask_words, float *y, int *ny_out, hipStream_t st)
{
    const pf_layer_desc &D = L->desc;
    const uint8_t *q_up = static_cast<const uint8_t *>(L->w.w_up);
    const uint8_t *q_gate = static_cast<const uint8_t *>(L->w.w_gate);
    const uint8_t *q_down = static_cast<const uint8_t *>(L->w.w_down);
    const __half *s_up = static_cast<const __half *>(L->w.s_up);
    const __half *s_gate = static_cast<const __half *>(L->w.s_gate);
    const __half *s_down = static_cast<const __half *>(L->w.s_down);
    const bool from_mask = mask_words != nullptr;
    const size_t extra = from_mask ? pf::up_mask_lds_bytes(D.ffn) : 0;
    const size_t per_tok = (size_t)kpad_i4(D.d) * sizeof(float);
    int tile = (int)(((size_t)ctx->lds_budget - extra - 1024) / per_tok);
    if (tile > kMaxBatch) tile = kMaxBatch;
    if (tile < 1) tile = 1;
    if (tile > B) tile = B;
    int up_grid = cdiv(D.ffn, pf::kUpI4Waves);
    if (up_grid > ctx->up_grid_cap_i4) up_grid = ctx->up_grid_cap_i4;
    const bool gated = D.act != PF_ACT_RELU;
    for (int b0 = 0; b0 < B; b0 += tile) {
        const int bt = (B - b0) < tile ? (B - b0) : tile;
        const size_t lds = (size_t)bt * per_tok + pf::kStageScrap * sizeof(float) + extra;
        const float *xb = x + (size_t)b0 * D.d;
        float *hb = ctx->h + b0;
        ProfScope ps(ctx, K_UP);
#define PF_UP4(ACT, FM)                                                                           \
    PF_SWITCH_B(bt, PF_LAUNCH(ps, (pf::k_up_i4<BT, ACT, FM>), dim3(up_grid),                      \
                              dim3(pf::kUpI4Threads), lds, st, q_up, s_up, q_gate, s_gate,        \
                              L->w.b_up, xb, idx_in, count_in, mask_words, ctx->idx, ctx->count,  \
                              hb, pf::h_stride(B), D.d, D.ffn, up_floor_of(D)))
        if (gated && from_mask) { PF_UP4(1, true); }
        else if (gated) { PF_UP4(1, false); }
        else if (from_mask) { PF_UP4(0, true); }
        else { PF_UP4(0, false); }
#undef PF_UP4
    }
    const int32_t *idx = from_mask ? ctx->idx : idx_in;
    const int32_t *count = from_mask ? ctx->count : count_in;
    const int tiles = cdiv(D.d, pf::kDown2I4Cols);
    const int P = fc2_split(ctx, tiles, B);
    float *part = (ny_out || P > 1) ? ctx->ypart : y;
    {
        ProfScope ps(ctx, K_DOWN);
        PF_SWITCH_B(B, PF_LAUNCH(ps, pf::k_down2_i4<BT>, dim3(tiles, P), dim3(pf::kDown2I4Threads),
                                 0, st, q_down, s_down, L->w.b_down, ctx->h, idx, count, part, D.d,
                                 D.ffn));
    }
    if (ny_out) {
        *ny_out = P;
    } else if (P > 1) {
        ProfScope ps(ctx, K_COMBINE);
        const int nel = B * D.d;
        PF_LAUNCH(ps, pf::k_combine, dim3(cdiv(nel, 1024)), dim3(256), 0, st,
                  (const float *)ctx->ypart, P, nel, y);
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// Sparse FFN.  Either an index list is given (idx_in, count_in) or mask words, from which
// the FC1 kernel derives the list itself and leaves it in ctx->idx / ctx->count.
// FC2's output goes to y when ny_out is null; otherwise it may be left as *ny_out partial sums
// in ctx->ypart ([ny][B][d]) for a consumer that adds them up itself.
pf_status launch_sparse(pf_ctx *ctx, const pf_layer *L, const float *x, int B,
                        const int32_t *idx_in, const int32_t *count_in,
                        const uint64_t *mask_words, float *y, int *ny_out, hipStream_t st)
{
    const pf_layer_desc &D = L->desc;
    if (D.wtype == PF_W_INT4_G128)
        return launch_sparse_i4(ctx, L, x, B, idx_in, count_in, mask_words, y, ny_out, st);
    const __half *w_up = static_cast<const __half *>(L->w.w_up);
    const __half *w_gate = static_cast<const __half *>(L->w.w_gate);
    const __half *w_down = static_cast<const __half *>(L->w.w_down);
    const bool from_mask = mask_words != nullptr;
    const size_t extra = from_mask ? pf::up_mask_lds_bytes(D.ffn) : 0;
    const int tile = batch_tile(ctx, D.d, B, extra + 1024);
    const bool gated = D.act != PF_ACT_RELU;
    int up_grid = cdiv(D.ffn, pf::kUpWaves);
    if (up_grid > ctx->up_grid_cap) up_grid = ctx->up_grid_cap;
    const size_t mfma_lds = pf::up_mfma_lds_bytes(D.ffn, from_mask, gated);
    const bool mfma = B >= mfma_from(ctx, D) && D.d % 32 == 0 && mfma_lds <= (size_t)ctx->lds_budget;
    if (mfma) {  // the whole batch in one launch: tokens are the N columns of the tile
        // one block per CU: a block's fixed cost (mask scan, bit select, tile reduction) is about
        // 7 us, so two rounds of smaller blocks lose more than their longer chunks gain
        const int grid = ctx->mfma_grid > 0 ? ctx->mfma_grid : ctx->num_cu;
        ProfScope ps(ctx, K_UP_MFMA);
        // the activations as split planes where this call has them already (the glue kernel or
        // the matrix-core hidden layer in front made them; only calls that predict get there),
        // else as fp32 values
        const __half *xs = from_mask ? split_of(ctx, x) : nullptr;
        const void *xop = xs ? (const void *)xs : (const void *)x;
#define PF_UPM(ACT, FM, XSV)                                                                          \
    PF_LAUNCH(ps, (pf::k_up_mfma<ACT, FM, XSV>), dim3(grid), dim3(pf::kMfmaThreads), mfma_lds, st, w_up, \
              w_gate, L->w.b_up, xop, B, idx_in, count_in, mask_words, ctx->idx, ctx->count, ctx->h,   \
              pf::h_stride(B), D.d, D.ffn, up_floor_of(D))
        if (xs && gated) { PF_UPM(1, true, true); }
        else if (xs) { PF_UPM(0, true, true); }
        else if (gated && from_mask) { PF_UPM(1, true, false); }
        else if (gated) { PF_UPM(1, false, false); }
        else if (from_mask) { PF_UPM(0, true, false); }
        else { PF_UPM(0, false, false); }
#undef PF_UPM
    }
    for (int b0 = 0; b0 < B && !mfma; b0 += tile) {
        const int bt = (B - b0) < tile ? (B - b0) : tile;
        const size_t lds = ((size_t)bt * kpad_of(D.d) + pf::kStageScrap) * sizeof(float) + extra;
        const float *xb = x + (size_t)b0 * D.d;
        float *hb = ctx->h + b0;
        ProfScope ps(ctx, K_UP);
#define PF_UP(ACT, FM)                                                                            \
    PF_SWITCH_B(bt, PF_LAUNCH(ps, (pf::k_up<BT, ACT, FM>), dim3(up_grid),                    \
                                       dim3(pf::kUpThreads), lds, st, w_up, w_gate, L->w.b_up, xb, \
                                       idx_in, count_in, mask_words, ctx->idx, ctx->count, hb,    \
                                       pf::h_stride(B), D.d, D.ffn, up_floor_of(D)))
        if (gated && from_mask) { PF_UP(1, true); }
        else if (gated) { PF_UP(1, false); }
        else if (from_mask) { PF_UP(0, true); }
        else { PF_UP(0, false); }
#undef PF_UP
    }
    const int32_t *idx = from_mask ? ctx->idx : idx_in;
    const int32_t *count = from_mask ? ctx->count : count_in;
    // row-split FC2: enough row groups per column tile to give every CU a workgroup
    const int tiles = cdiv(D.d, pf::kDown2Cols);
    const int P = fc2_split(ctx, tiles, B);
    float *part = (ny_out || P > 1) ? ctx->ypart : y;
    {
        ProfScope ps(ctx, K_DOWN);
        PF_SWITCH_B(B, PF_LAUNCH(ps, pf::k_down2<BT>, dim3(tiles, P), dim3(pf::kDown2Threads), 0,
                                 st, w_down, L->w.b_down, ctx->h, idx, count, part, D.d, D.ffn));
    }
    if (ny_out) {
        *ny_out = P;
    } else if (P > 1) {
        ProfScope ps(ctx, K_COMBINE);
        const int nel = B * D.d;
        PF_LAUNCH(ps, pf::k_combine, dim3(cdiv(nel, 1024)), dim3(256), 0, st,
                  (const float *)ctx->ypart, P, nel, y);
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// Whole layer step: predictor (two launches), FC1 with fused compaction, FC2.  x_in is the
// layer input as the later kernels see it: x itself, or x_new when the hidden kernel forms
// it (glue_y given).
pf_status launch_layer(pf_ctx *ctx, const pf_layer *L, const float *x, const float *glue_y,
                       int glue_ny, float *x_new, int B, float *y, int *ny_out, hipStream_t st)
{
    const float *x_in = glue_y ? x_new : x;
    pf_status s = launch_predict(ctx, L, x, glue_y, glue_ny, x_new, B, nullptr, ctx->mask_words, st);
    if (s != PF_OK) return s;
    ctx->last_mask = ctx->mask_words;
    ctx->last_idx = ctx->idx;
    ctx->last_count = ctx->count;
    return launch_sparse(ctx, L, x_in, B, nullptr, nullptr, ctx->mask_words, y, ny_out, st);
}

// Whether the three-launch form of the layer step applies: fp16 weights, the vector path
// (below the batch of the matrix-core kernels), and hidden vector + layer input of the whole
// batch fit LDS.
bool fused_ok(const pf_ctx *ctx, const pf_layer *L, int B)
{
    const pf_layer_desc &D = L->desc;
    if (!ctx->fused || D.wtype == PF_W_INT4_G128 || B >= mfma_from(ctx, D) || B > 3 ||
        pf::out_up_lds_bytes(B, D.r, D.d) + 1024 > (size_t)ctx->lds_budget)
        return false;
    if (ctx->fused > 1) return true;  // forced
    // Measured on the five benchmark shapes: the fused form wins by 8 - 20 % where the saved
    // kernel boundary weighs most (short rows, or three tokens, whose list-based kernels are
    // slow) and loses 1 - 7 % with long rows at batch 1, where FC1 and FC2 are long enough
    // for the uneven work per segment to cost more than the boundary.  (Three tokens with
    // long rows never get here: mfma_from sends them to the matrix cores.)
    const bool gated = D.act != PF_ACT_RELU;
    return B == 3 || D.d <= 4096 || (B == 2 && !gated);
}

// Layer step in three launches: hidden layer, output layer + FC1 per mask word, FC2 over the
// mask words.  Leaves the mask but no index list; FC2's output stays as *ny_out partial sums.
pf_status launch_layer_fused(pf_ctx *ctx, const pf_layer *L, const float *x, const float *glue_y,
                             int glue_ny, float *x_new, int B, int *ny_out, hipStream_t st)
{
    const float *x_in = glue_y ? x_new : x;
    pf_status s = launch_hidden(ctx, L, x, glue_y, glue_ny, x_new, B, st);
    if (s != PF_OK) return s;
    const pf_layer_desc &D = L->desc;
    const __half *p2 = static_cast<const __half *>(L->w.p2);
    const __half *w_up = static_cast<const __half *>(L->w.w_up);
    const __half *w_gate = static_cast<const __half *>(L->w.w_gate);
    const __half *w_down = static_cast<const __half *>(L->w.w_down);
    const bool gated = D.act != PF_ACT_RELU;
    const size_t lds = pf::out_up_lds_bytes(B, D.r, D.d);
    {
        ProfScope ps(ctx, K_OUT_UP);
#define PF_OU(ACT)                                                                                \
    PF_SWITCH_B3(B, PF_LAUNCH(ps, (pf::k_out_up<BT, ACT>), dim3(D.ffn / 64),                      \
                             dim3(pf::kPredOutThreads), lds, st, p2, L->w.p_bias,                 \
                             (const float *)ctx->t, w_up, w_gate, L->w.b_up, x_in, D.r, D.d,      \
                             D.ffn, pf::h_stride(B), L->thr_logit, ctx->seg_strided != 0,         \
                             ctx->mask_words2,                                                    \
                             reinterpret_cast<uint8_t *>(ctx->idx), ctx->h, up_floor_of(D), L->always_on))
        if (gated) { PF_OU(1); } else { PF_OU(0); }
#undef PF_OU
    }
    const int tiles = cdiv(D.d, pf::kDown2Cols);
    const int P = fc2_split(ctx, tiles, B, false);
    {
        ProfScope ps(ctx, K_DOWN_MASK);
        const bool multi = cdiv(D.ffn / 64, 8 * P) > pf::down2m_batch(B);
#define PF_DM(MULTI)                                                                              \
    PF_SWITCH_B3(B, PF_LAUNCH(ps, (pf::k_down2m<BT, MULTI>), dim3(tiles, P),                      \
                             dim3(pf::kDown2Threads), 0, st, w_down, L->w.b_down,                 \
                             (const float *)ctx->h, (const uint64_t *)ctx->mask_words2,           \
                             reinterpret_cast<const uint8_t *>(ctx->idx), ctx->ypart, D.d, D.ffn, \
                             ctx->seg_strided != 0))
        if (multi) { PF_DM(true); } else { PF_DM(false); }
#undef PF_DM
    }
    *ny_out = P;
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// split: also leave x_next as fp16 hi + lo planes for the matrix-core kernels (split_of(x_next)).
pf_status launch_glue(pf_ctx *ctx, const float *x, const float *y, int ny, int d, int B,
                      float *x_next, hipStream_t st, bool split)
{
    __half *xs = nullptr;
    if (split && d % 4 == 0 && ctx->xsplit[0] != nullptr && !ctx->split_off) {
        ctx->split_cur ^= 1;
        xs = ctx->xsplit[ctx->split_cur];
        ctx->split_src = x_next;
    } else if (ctx->split_src == x_next) {
        ctx->split_src = nullptr;  // its planes go stale
    }
    {
        ProfScope ps(ctx, K_GLUE);
        if (d <= pf::kGlueMaxD && d % 4 == 0)
            PF_LAUNCH(ps, pf::k_glue, dim3(B), dim3(pf::kGlueThreads), 0, st, x, y, ny, x_next, d, xs);
        else
            PF_LAUNCH(ps, pf::k_glue_long, dim3(B), dim3(pf::kGlueThreads), 0, st, x, y, ny, x_next, d, xs);
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// The split planes of x if this call has produced them already, else null.
const __half *split_of(const pf_ctx *ctx, const float *x)
{
    return (x != nullptr && !ctx->split_off && ctx->split_src == x) ? ctx->xsplit[ctx->split_cur] : nullptr;
}

// The split planes of x, produced by a small kernel if this call has not made them yet.
pf_status ensure_split(pf_ctx *ctx, const float *x, int B, int d, hipStream_t st, const __half **xs)
{
    *xs = split_of(ctx, x);
    if (*xs) return PF_OK;
    // no planes: a context without the buffers, an odd shape, or kernels being enqueued on a
    // second stream (the planes' bookkeeping follows one stream); the caller reads fp32 then
    if (!ctx->xsplit[0] || (B * d) % 4 != 0 || ctx->split_off) return PF_OK;
    ctx->split_cur ^= 1;
    __half *dst = ctx->xsplit[ctx->split_cur];
    const int n = B * d;
    {
        ProfScope ps(ctx, K_GLUE);
        PF_LAUNCH(ps, pf::k_split, dim3(cdiv(n, 1024)), dim3(256), 0, st, x, dst, n);
    }
    PF_HIP(ctx, hipGetLastError());
    ctx->split_src = x;
    *xs = dst;
    return PF_OK;
}

// Copies a layer's mask words to the caller's trace buffer in the caller-visible format.
// Segment words of the three-launch form with strided segments hold neuron p * G + g at bit p
// of word g; they are re-ballotted here.  grid = ffn / 64, block = 64.
__global__ __launch_bounds__(64) void k_trace_mask(const uint64_t *__restrict__ words, int nwords,
                                                   bool strided, uint64_t *__restrict__ out)
{
    const int w = blockIdx.x, lane = threadIdx.x;
    if (!strided) {
        if (lane == 0) out[w] = words[w];
        return;
    }
    const int n = w * 64 + lane;  // neuron: position n / nwords of segment n % nwords
    const uint64_t bit = (words[n % nwords] >> (n / nwords)) & 1ull;
    const uint64_t word = __ballot(bit != 0);
    if (lane == 0) out[w] = word;
}

pf_status trace_mask(pf_ctx *ctx, int l, const pf_layer *L, const uint64_t *words, bool strided,
                     hipStream_t st)
{
    if (!ctx->mask_trace || l >= ctx->mask_trace_layers) return PF_OK;
    const int nwords = L->desc.ffn / 64;
    hipLaunchKernelGGL(k_trace_mask, dim3(nwords), dim3(64), 0, st, words, nwords, strided,
                       ctx->mask_trace + (size_t)l * (size_t)(ctx->max_ffn / 64));
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

// One decode step of the stack.  The glue between layer l-1 and layer l runs inside layer
// l's hidden-layer kernel; only the glue after the last layer is a kernel of its own.
// Event number `i` of the look-ahead schedule (created on demand, reused by later calls).
hipEvent_t la_event(pf_ctx *ctx, size_t i)
{
    while (ctx->la_events.size() <= i) {
        hipEvent_t e = nullptr;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
        ctx->la_events.push_back(e);
    }
    return ctx->la_events[i];
}

// One decode step with look-ahead prediction at distance 1: the predictor of layer l reads
// the input of layer l-1 (layer 0 and 1: the stack's input) and runs on the side stream
// while the main stream is busy with the sparse kernels of layer l-1.  Masks alternate
// between two buffers; the glue is a kernel of its own on the main stream.
pf_status stack_enqueue_lookahead(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x,
                                  int B, float *x_out, hipStream_t st)
{
    hipStream_t side = ctx->side_stream;
    uint64_t *masks[2] = {ctx->mask_words, ctx->mask_words2};
    const int d = layers[0]->desc.d;
    // events: 0 = fork, 1 + l = mask of layer l ready, 1 + n_layers + l = input of layer l ready
    hipEvent_t fork = la_event(ctx, 0);
    if (!la_event(ctx, 2 * (size_t)n_layers + 1) || !fork) return fail(ctx, PF_EHIP, "hipEventCreate failed");
    auto ev_mask = [&](int l) { return ctx->la_events[1 + (size_t)l]; };
    auto ev_input = [&](int l) { return ctx->la_events[1 + (size_t)n_layers + (size_t)l]; };
    PF_HIP(ctx, hipEventRecord(fork, st));
    PF_HIP(ctx, hipStreamWaitEvent(side, fork, 0));
    auto predict_on_side = [&](int l, const float *seen) -> pf_status {
        ctx->split_off = true;  // the split planes' bookkeeping follows the main stream only
        pf_status s = launch_predict(ctx, layers[l], seen, nullptr, 0, nullptr, B, nullptr, masks[l & 1], side);
        ctx->split_off = false;
        if (s != PF_OK) return s;
        PF_HIP(ctx, hipEventRecord(ev_mask(l), side));
        return PF_OK;
    };
    pf_status s = predict_on_side(0, x);
    if (s == PF_OK && n_layers > 1) s = predict_on_side(1, x);
    if (s != PF_OK) return s;
    int ny = 1;
    const float *cur = x;
    for (int l = 0; l < n_layers; ++l) {
        PF_HIP(ctx, hipStreamWaitEvent(st, ev_mask(l), 0));
        ctx->last_mask = masks[l & 1];
        ctx->last_idx = ctx->idx;
        ctx->last_count = ctx->count;
        s = launch_sparse(ctx, layers[l], cur, B, nullptr, nullptr, masks[l & 1], nullptr, &ny, st);
        if (s == PF_OK) s = trace_mask(ctx, l, layers[l], masks[l & 1], false, st);
        if (s != PF_OK) return s;
        if (l + 1 < n_layers) {
            float *xn = ctx->xbuf[(l + 1) & 1];
            s = launch_glue(ctx, cur, ctx->ypart, ny, d, B, xn, st);
            if (s != PF_OK) return s;
            cur = xn;
            if (l + 2 < n_layers) {  // layer l+2 is predicted from the input of layer l+1
                PF_HIP(ctx, hipEventRecord(ev_input(l + 1), st));
                PF_HIP(ctx, hipStreamWaitEvent(side, ev_input(l + 1), 0));
                s = predict_on_side(l + 2, xn);
                if (s != PF_OK) return s;
            }
        }
    }
    return launch_glue(ctx, cur, ctx->ypart, ny, d, B, x_out, st);
}

// Look-ahead prediction on one stream: the predictor of layer l+2 follows the sparse kernels of
// layer l, and its hidden kernel forms the input of layer l+1 (the glue) on the way, so the
// launches are those of the default schedule with the masks taken one layer earlier.
pf_status stack_enqueue_lookahead_serial(pf_ctx *ctx, pf_layer *const *layers, int n_layers,
                                         const float *x, int B, float *x_out, hipStream_t st)
{
    uint64_t *masks[2] = {ctx->mask_words, ctx->mask_words2};
    const int d = layers[0]->desc.d;
    pf_status s = launch_predict(ctx, layers[0], x, nullptr, 0, nullptr, B, nullptr, masks[0], st);
    if (s == PF_OK && n_layers > 1)
        s = launch_predict(ctx, layers[1], x, nullptr, 0, nullptr, B, nullptr, masks[1], st);
    if (s != PF_OK) return s;
    int ny = 1;
    const float *cur = x;
    for (int l = 0; l < n_layers; ++l) {
        ctx->last_mask = masks[l & 1];
        ctx->last_idx = ctx->idx;
        ctx->last_count = ctx->count;
        s = launch_sparse(ctx, layers[l], cur, B, nullptr, nullptr, masks[l & 1], nullptr, &ny, st);
        if (s == PF_OK) s = trace_mask(ctx, l, layers[l], masks[l & 1], false, st);
        if (s != PF_OK) return s;
        if (l + 1 < n_layers) {
            float *xn = ctx->xbuf[(l + 1) & 1];
            if (l + 2 < n_layers)  // its mask takes the buffer layer l has just finished with
                s = launch_predict(ctx, layers[l + 2], cur, ctx->ypart, ny, xn, B, nullptr, masks[l & 1], st);
            else
                s = launch_glue(ctx, cur, ctx->ypart, ny, d, B, xn, st);
            if (s != PF_OK) return s;
            cur = xn;
        }
    }
    return launch_glue(ctx, cur, ctx->ypart, ny, d, B, x_out, st);
}

// Whether a stack can run look-ahead prediction in the two-launch form (k_lookahead.h): fp16
// weights and the vector path (batch below the matrix-core kernels', at most 3), whole batch
// staged at once.
bool la_merged_ok(const pf_ctx *ctx, pf_layer *const *layers, int n_layers, int B)
{
    if (B > 3) return false;
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer_desc &D = layers[l]->desc;
        if (D.wtype != PF_W_FP16 || B >= mfma_from(ctx, D)) return false;
        if (batch_tile(ctx, D.d, B, pf::up_mask_lds_bytes(D.ffn) + 1024) < B) return false;
    }
    return true;
}

// One decode step with look-ahead prediction, two launches per layer: [hidden layer of
// predictor l+1 | FC1 of layer l], then [FC2 of layer l | output layer of predictor l+1].
// The glue runs inside the first launch of the next layer; masks alternate between two buffers.
pf_status stack_enqueue_lookahead_merged(pf_ctx *ctx, pf_layer *const *layers, int n_layers,
                                         const float *x, int B, float *x_out, hipStream_t st)
{
    uint64_t *masks[2] = {ctx->mask_words, ctx->mask_words2};
    const int d = layers[0]->desc.d;
    // the list of layer 0 comes from its own input
    pf_status s = launch_predict(ctx, layers[0], x, nullptr, 0, nullptr, B, nullptr, masks[0], st);
    if (s != PF_OK) return s;
    int ny = 1;
    const float *cur = x;  // what the first launch of layer l reads: x_0, or the input of layer l-1
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer *L = layers[l];
        const pf_layer *N = l + 1 < n_layers ? layers[l + 1] : nullptr;  // whose predictor rides along
        const pf_layer_desc &D = L->desc;
        const bool gated = D.act != PF_ACT_RELU;
        const bool glue = l > 0;
        float *xn = glue ? ctx->xbuf[l & 1] : nullptr;
        if (glue && ctx->split_src == xn) ctx->split_src = nullptr;  // rewritten as fp32 only
        const int n_hid = N ? cdiv(N->desc.r, pf::kPredWaves) : 0;
        int n_up = cdiv(D.ffn, pf::kUpWaves);
        // Measured on the benchmark shapes (batch 1..3): the roles with the dependent chains
        // (FC1, FC2) take the low block numbers, FC1 gets two workgroups per CU (every one of
        // them forms the glue, so surplus workgroups cost cache reads), and FC2 leaves two
        // partial sums instead of four (fewer CUs gather, but the output layer's stream keeps
        // the others busy, and the next launch reads 3 instead of 5 vectors per workgroup).
        if (n_up > 2 * ctx->num_cu) n_up = 2 * ctx->num_cu;
        const size_t lds1 = ((size_t)B * kpad_of(D.d) + pf::kStageScrap) * sizeof(float) +
                            pf::up_mask_lds_bytes(D.ffn);
        {
            ProfScope ps(ctx, K_LA_UP_HIDDEN);
#define PF_LA1(ACT, GLUE)                                                                          \
    PF_SWITCH_B3(B, PF_LAUNCH(ps, (pf::k_la_up_hidden<BT, ACT, GLUE>), dim3(n_hid + n_up),          \
                              dim3(pf::kUpThreads), lds1, st, n_hid,                                \
                              static_cast<const __half *>(N ? N->w.p1 : nullptr), ctx->t,           \
                              N ? N->desc.r : 0, static_cast<const __half *>(L->w.w_up),            \
                              static_cast<const __half *>(L->w.w_gate), L->w.b_up, cur,             \
                              (const float *)ctx->ypart, ny, B * d, xn,                             \
                              (const uint64_t *)masks[l & 1], ctx->idx, ctx->count, ctx->h,         \
                              pf::h_stride(B), D.d, D.ffn, up_floor_of(D), true))
            if (gated && glue) { PF_LA1(1, true); }
            else if (gated) { PF_LA1(1, false); }
            else if (glue) { PF_LA1(0, true); }
            else { PF_LA1(0, false); }
#undef PF_LA1
        }
        if (glue) cur = xn;
        ctx->last_mask = masks[l & 1];
        ctx->last_idx = ctx->idx;
        ctx->last_count = ctx->count;
        const int tiles = cdiv(D.d, pf::kDown2Cols);
        int P = ctx->down_split > 0 ? ctx->down_split : ctx->num_cu / tiles;
        if (P < 1) P = 1;
        if (ctx->down_split == 0 && P > 2) P = 2;
        // a single row group where the output layer beside it streams long enough to cover it
        // (measured: OPT-30B shape, 88 MB, +2 % at batch 1 and +4 % at batch 2; Falcon-40B shape,
        // 67 MB, even; OPT-6.7B shape, 34 MB, -10 %): the next launch then reads one vector less
        if (ctx->down_split == 0 && N && (size_t)2 * N->desc.ffn * N->desc.r >= (size_t)80000000) P = 1;
        if (P > pf::kDown2MaxSplit) P = pf::kDown2MaxSplit;
        const int n_out = N ? (N->desc.ffn - N->always_on) / pf::kLaOutNeurons : 0;
        const size_t lds2 = N ? ((size_t)B * kpad_of(N->desc.r) + pf::kStageScrap) * sizeof(float) : 0;
        {
            ProfScope ps(ctx, K_LA_DOWN_OUT);
            PF_SWITCH_B3(B, PF_LAUNCH(ps, (pf::k_la_down_out<BT>), dim3(tiles * P + n_out),
                                      dim3(pf::kDown2Threads), lds2, st, tiles, P,
                                      static_cast<const __half *>(L->w.w_down), L->w.b_down,
                                      (const float *)ctx->h, (const int32_t *)ctx->idx,
                                      (const int32_t *)ctx->count, ctx->ypart, D.d, D.ffn,
                                      static_cast<const __half *>(N ? N->w.p2 : nullptr),
                                      N ? N->w.p_bias : nullptr, (const float *)ctx->t,
                                      N ? N->desc.r : 0, N ? N->desc.ffn : 0, N ? N->thr_logit : 0.f,
                                      masks[(l + 1) & 1], N ? N->always_on / 64 : 0, false));
        }
        ny = P;
        PF_HIP(ctx, hipGetLastError());
        s = trace_mask(ctx, l, L, masks[l & 1], false, st);
        if (s != PF_OK) return s;
    }
    return launch_glue(ctx, cur, ctx->ypart, ny, d, B, x_out, st);
}

// Whether a stack can run look-ahead prediction in the two-launch form of the matrix-core
// kernels: fp16 layers whose FC1 and predictor run on the matrix cores at this batch.  (Gated
// layers take the whole LDS of a CU per FC1 workgroup: the hidden-layer role then follows FC1
// on the CUs instead of sharing them, and still saves the launch boundary.)
bool la_merged_mfma_ok(const pf_ctx *ctx, pf_layer *const *layers, int n_layers, int B)
{
    if (B < 3 || ctx->lds_budget <= kLdsDefault || !ctx->xsplit[0]) return false;
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer_desc &D = layers[l]->desc;
        if (D.wtype != PF_W_FP16 || B < mfma_from(ctx, D)) return false;
        if (D.d % 32 != 0 || D.r % 32 != 0) return false;
        if (pf::up_mfma_lds_bytes(D.ffn, true, D.act != PF_ACT_RELU) > (size_t)ctx->lds_budget) return false;
    }
    return true;
}

// One decode step with look-ahead prediction on the matrix cores: glue, then [FC1 of layer l |
// hidden layer of predictor l+1], then [FC2 of layer l | output layer of predictor l+1].
pf_status stack_enqueue_lookahead_merged_mfma(pf_ctx *ctx, pf_layer *const *layers, int n_layers,
                                              const float *x, int B, float *x_out, hipStream_t st)
{
    uint64_t *masks[2] = {ctx->mask_words, ctx->mask_words2};
    const int d = layers[0]->desc.d;
    pf_status s = launch_predict(ctx, layers[0], x, nullptr, 0, nullptr, B, nullptr, masks[0], st);
    if (s != PF_OK) return s;
    int ny = 1;
    const float *cur = x;
    const size_t slots = (size_t)pf::kMfmaWaves * pf::kRowsMfmaSlotBytes;
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer *L = layers[l];
        const pf_layer *N = l + 1 < n_layers ? layers[l + 1] : nullptr;
        const pf_layer_desc &D = L->desc;
        if (l > 0) {  // the matrix-core kernels read the layer input from memory
            float *xn = ctx->xbuf[l & 1];
            s = launch_glue(ctx, cur, ctx->ypart, ny, d, B, xn, st, true);
            if (s != PF_OK) return s;
            cur = xn;
        }
        const __half *xs = nullptr;  // both roles of the first launch read the split planes
        s = ensure_split(ctx, cur, B, d, st, &xs);
        if (s != PF_OK) return s;
        const int n_hid = N ? cdiv(N->desc.r, 8) : 0;
        const int n_up = ctx->mfma_grid > 0 ? ctx->mfma_grid : ctx->num_cu;
        const bool gated = D.act != PF_ACT_RELU;
        size_t lds1 = pf::up_mfma_lds_bytes(D.ffn, true, gated);
        if (lds1 < slots) lds1 = slots;
        {
            ProfScope ps(ctx, K_LA_UP_HIDDEN);
#define PF_LA1M(ACT)                                                                                   \
    PF_LAUNCH(ps, (pf::k_la_up_hidden_mfma<ACT>), dim3(n_up + n_hid), dim3(pf::kMfmaThreads), lds1, st, \
              n_hid, static_cast<const __half *>(N ? N->w.p1 : nullptr), ctx->t, N ? N->desc.r : 0,    \
              static_cast<const __half *>(L->w.w_up), static_cast<const __half *>(L->w.w_gate),        \
              L->w.b_up, (const void *)xs, B, (const uint64_t *)masks[l & 1], ctx->idx, ctx->count,    \
              ctx->h,                                                                                  \
              pf::h_stride(B), D.d, D.ffn, up_floor_of(D))
            if (gated)
                PF_LA1M(1);
            else
                PF_LA1M(0);
#undef PF_LA1M
        }
        ctx->last_mask = masks[l & 1];
        ctx->last_idx = ctx->idx;
        ctx->last_count = ctx->count;
        const int tiles = cdiv(D.d, pf::kDown2Cols);
        // one round of FC2 workgroups here: the output-layer role fills the CUs beside them
        // (measured: a second FC2 workgroup per CU costs this launch 4 %)
        int P = ctx->down_split > 0 ? ctx->down_split : ctx->num_cu / tiles;
        if (P < 1) P = 1;
        if (P > pf::kDown2MaxSplit) P = pf::kDown2MaxSplit;
        const int n_out = N ? (N->desc.ffn - N->always_on) / 64 : 0;
        {
            ProfScope ps(ctx, K_LA_DOWN_OUT);
#define PF_LA2M(BB)                                                                               \
    PF_LAUNCH(ps, (pf::k_la_down_out_mfma<BB>), dim3(tiles * P + n_out), dim3(pf::kMfmaThreads), slots, \
              st, tiles, P, static_cast<const __half *>(L->w.w_down), L->w.b_down,                \
              (const float *)ctx->h, (const int32_t *)ctx->idx, (const int32_t *)ctx->count,      \
              ctx->ypart, D.d, D.ffn, static_cast<const __half *>(N ? N->w.p2 : nullptr),         \
              N ? N->w.p_bias : nullptr, (const float *)ctx->t, N ? N->desc.r : 0,                \
              N ? N->desc.ffn : 0, N ? N->thr_logit : 0.f, masks[(l + 1) & 1],                    \
              N ? N->always_on / 64 : 0)
            switch (B) {
                case 3: PF_LA2M(3); break;
                case 4: PF_LA2M(4); break;
                case 5: PF_LA2M(5); break;
                case 6: PF_LA2M(6); break;
                case 7: PF_LA2M(7); break;
                default: PF_LA2M(8); break;
            }
#undef PF_LA2M
        }
        ny = P;
        PF_HIP(ctx, hipGetLastError());
        s = trace_mask(ctx, l, L, masks[l & 1], false, st);
        if (s != PF_OK) return s;
    }
    return launch_glue(ctx, cur, ctx->ypart, ny, d, B, x_out, st);
}

// Whether a stack can run look-ahead prediction in the two-launch form of the int4 kernels:
// int4 layers at a batch of at most 3 whose staged input fits LDS in one piece.
bool la_merged_i4_ok(const pf_ctx *ctx, pf_layer *const *layers, int n_layers, int B)
{
    if (B > 3) return false;
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer_desc &D = layers[l]->desc;
        if (D.wtype != PF_W_INT4_G128) return false;
        const size_t lds = ((size_t)B * kpad_i4(D.d) + pf::kStageScrap) * sizeof(float) + pf::up_mask_lds_bytes(D.ffn);
        if (lds > (size_t)ctx->lds_budget) return false;
    }
    return true;
}

// One decode step with look-ahead prediction over int4 layers: glue, then [FC1 of layer l |
// hidden layer of predictor l+1], then [FC2 of layer l | output layer of predictor l+1].
pf_status stack_enqueue_lookahead_merged_i4(pf_ctx *ctx, pf_layer *const *layers, int n_layers,
                                            const float *x, int B, float *x_out, hipStream_t st)
{
    uint64_t *masks[2] = {ctx->mask_words, ctx->mask_words2};
    const int d = layers[0]->desc.d;
    pf_status s = launch_predict(ctx, layers[0], x, nullptr, 0, nullptr, B, nullptr, masks[0], st);
    if (s != PF_OK) return s;
    int ny = 1;
    const float *cur = x;
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer *L = layers[l];
        const pf_layer *N = l + 1 < n_layers ? layers[l + 1] : nullptr;
        const pf_layer_desc &D = L->desc;
        if (l > 0) {  // the int4 FC1 reads the layer input from memory
            float *xn = ctx->xbuf[l & 1];
            s = launch_glue(ctx, cur, ctx->ypart, ny, d, B, xn, st);
            if (s != PF_OK) return s;
            cur = xn;
        }
        const bool gated = D.act != PF_ACT_RELU;
        const int n_hid = N ? cdiv(N->desc.r, pf::kUpI4Waves) : 0;
        int n_up = cdiv(D.ffn, pf::kUpI4Waves);
        if (n_up > ctx->up_grid_cap_i4) n_up = ctx->up_grid_cap_i4;
        size_t lds1 = ((size_t)B * kpad_i4(D.d) + pf::kStageScrap) * sizeof(float) + pf::up_mask_lds_bytes(D.ffn);
        const size_t lds_hid = ((size_t)B * kpad_of(D.d) + pf::kStageScrap) * sizeof(float);
        if (lds1 < lds_hid) lds1 = lds_hid;
        {
            ProfScope ps(ctx, K_LA_UP_HIDDEN);
#define PF_LA1I(ACT)                                                                                  \
    PF_SWITCH_B3(B, PF_LAUNCH(ps, (pf::k_la_up_hidden_i4<BT, ACT>), dim3(n_up + n_hid),               \
                              dim3(pf::kUpI4Threads), lds1, st, n_hid,                                \
                              static_cast<const __half *>(N ? N->w.p1 : nullptr), ctx->t,             \
                              N ? N->desc.r : 0, static_cast<const uint8_t *>(L->w.w_up),             \
                              static_cast<const __half *>(L->w.s_up),                                 \
                              static_cast<const uint8_t *>(L->w.w_gate),                              \
                              static_cast<const __half *>(L->w.s_gate), L->w.b_up, cur,               \
                              (const uint64_t *)masks[l & 1], ctx->idx, ctx->count, ctx->h,           \
                              pf::h_stride(B), D.d, D.ffn, up_floor_of(D)))
            if (gated) { PF_LA1I(1); }
            else { PF_LA1I(0); }
#undef PF_LA1I
        }
        ctx->last_mask = masks[l & 1];
        ctx->last_idx = ctx->idx;
        ctx->last_count = ctx->count;
        const int tiles = cdiv(D.d, pf::kDown2I4Cols);
        const int P = fc2_split(ctx, tiles, B);
        const int n_out = N ? (N->desc.ffn - N->always_on) / pf::kLaOutNeurons : 0;
        const size_t lds2 = N ? ((size_t)B * kpad_of(N->desc.r) + pf::kStageScrap) * sizeof(float) : 0;
        {
            ProfScope ps(ctx, K_LA_DOWN_OUT);
            PF_SWITCH_B3(B, PF_LAUNCH(ps, (pf::k_la_down_out_i4<BT>), dim3(tiles * P + n_out),
                                      dim3(pf::kDown2I4Threads), lds2, st, tiles, P,
                                      static_cast<const uint8_t *>(L->w.w_down),
                                      static_cast<const __half *>(L->w.s_down), L->w.b_down,
                                      (const float *)ctx->h, (const int32_t *)ctx->idx,
                                      (const int32_t *)ctx->count, ctx->ypart, D.d, D.ffn,
                                      static_cast<const __half *>(N ? N->w.p2 : nullptr),
                                      N ? N->w.p_bias : nullptr, (const float *)ctx->t,
                                      N ? N->desc.r : 0, N ? N->desc.ffn : 0, N ? N->thr_logit : 0.f,
                                      masks[(l + 1) & 1], N ? N->always_on / 64 : 0));
        }
        ny = P;
        PF_HIP(ctx, hipGetLastError());
        s = trace_mask(ctx, l, L, masks[l & 1], false, st);
        if (s != PF_OK) return s;
    }
    return launch_glue(ctx, cur, ctx->ypart, ny, d, B, x_out, st);
}

pf_status stack_enqueue(pf_ctx *ctx, pf_layer *const *layers, int n_layers, const float *x, int B,
                        float *x_out, hipStream_t st)
{
    if (ctx->lookahead) {
        // form 0: two launches per layer where that applies; otherwise (matrix-core batches,
        // int4) the predictors on a second stream for ReLU layers, where that measured 2 - 14 %
        // faster than the default schedule (the predictor is the larger share of a two-matrix
        // layer), and on one stream for gated layers, where the second stream measured 3 - 7 %
        // slower (FC1 on the matrix cores leaves no room beside it) and one stream costs what
        // the default schedule costs
        int form = ctx->la_form;
        if ((form == 0 || form == 1) && la_merged_ok(ctx, layers, n_layers, B))
            return stack_enqueue_lookahead_merged(ctx, layers, n_layers, x, B, x_out, st);
        if ((form == 0 || form == 1) && la_merged_mfma_ok(ctx, layers, n_layers, B))
            return stack_enqueue_lookahead_merged_mfma(ctx, layers, n_layers, x, B, x_out, st);
        if ((form == 0 || form == 1) && la_merged_i4_ok(ctx, layers, n_layers, B))
            return stack_enqueue_lookahead_merged_i4(ctx, layers, n_layers, x, B, x_out, st);
        if (form == 0 || form == 1) form = layers[0]->desc.act == PF_ACT_RELU ? 2 : 3;
        return form == 2 ? stack_enqueue_lookahead(ctx, layers, n_layers, x, B, x_out, st)
                         : stack_enqueue_lookahead_serial(ctx, layers, n_layers, x, B, x_out, st);
    }
    int ny = 1;            // partial sums FC2 left in ctx->ypart
    const float *cur = x;  // input of the layer being enqueued (raw input of the previous one
                           // until the hidden kernel has formed it)
    for (int l = 0; l < n_layers; ++l) {
        const pf_layer *L = layers[l];
        pf_status s;
        // the last layer always builds its index list (pf_ctx_last_active, pf_count_activations)
        const bool fused = l + 1 < n_layers && fused_ok(ctx, L, B);
        const float *gy = l == 0 ? nullptr : ctx->ypart;
        float *xn = l == 0 ? nullptr : ctx->xbuf[l & 1];
        if (fused)
            s = launch_layer_fused(ctx, L, cur, gy, ny, xn, B, &ny, st);
        else
            s = launch_layer(ctx, L, cur, gy, l == 0 ? 0 : ny, xn, B, nullptr, &ny, st);
        if (l > 0) cur = xn;
        if (s == PF_OK)
            s = fused ? trace_mask(ctx, l, L, ctx->mask_words2, ctx->seg_strided != 0, st)
                      : trace_mask(ctx, l, L, ctx->mask_words, false, st);
        if (s != PF_OK) return s;
    }
    return launch_glue(ctx, cur, ctx->ypart, ny, layers[0]->desc.d, B, x_out, st);
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

// Launch-shape defaults that follow from the device (CU count, LDS opt-in); shared by every
// way a context comes into being.  The device must be current.
hipError_t init_device_limits(pf_ctx *ctx, int device)
{
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) return e;
    if (prop.multiProcessorCount > 0) ctx->num_cu = prop.multiProcessorCount;
    ctx->up_grid_cap = 8 * ctx->num_cu;
    ctx->up_grid_cap_i4 = 2 * ctx->num_cu;
    ctx->mfma_grid = 0;  // 0: from the CU count
    // larger staged batches need the opt-in LDS size; without it batches are tiled smaller
    if (prop.sharedMemPerBlock >= (size_t)kLdsMax ||
        prop.maxSharedMemoryPerMultiProcessor >= (size_t)kLdsMax) {
        if (allow_lds_all() == hipSuccess)
            ctx->lds_budget = kLdsMax - 4096;  // room for the kernels' small static LDS
        else
            (void)hipGetLastError();
    }
    return hipSuccess;
}

// Descriptor and weight pointers of a layer against the limits of the context that will run it.
pf_status check_layer(pf_ctx *ctx, const pf_layer_desc *desc, const pf_layer_weights *w)
{
    if (!desc || !w) return fail(ctx, PF_EINVAL, "null descriptor or weights");
    if (desc->d < 1 || desc->ffn < 1 || desc->r < 1)
        return fail(ctx, PF_EINVAL, "non-positive size");
    if (!(desc->threshold > 0.f && desc->threshold < 1.f))
        return fail(ctx, PF_EINVAL, "threshold %g outside (0,1)", (double)desc->threshold);
    if (desc->act != PF_ACT_RELU && desc->act != PF_ACT_REGLU && desc->act != PF_ACT_DRELU)
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
    // kernels address a matrix through a 32-bit buffer descriptor
    if ((uint64_t)desc->ffn * desc->d * 2 >= (1ull << 32) || (uint64_t)desc->ffn * desc->r * 2 >= (1ull << 32))
        return fail(ctx, PF_ESHAPE, "a weight matrix of 4 GiB or more is not supported");
    if (!w->w_up || !w->w_down) return fail(ctx, PF_EINVAL, "w_up / w_down is null");
    if (desc->act != PF_ACT_RELU && !w->w_gate) return fail(ctx, PF_EINVAL, "gated layer without w_gate");
    if ((w->p1 == nullptr) != (w->p2 == nullptr))
        return fail(ctx, PF_EINVAL, "p1 and p2 must both be given or both be null");
    if (desc->wtype == PF_W_INT4_G128) {
        if (!w->s_up || !w->s_down || (desc->act != PF_ACT_RELU && !w->s_gate))
            return fail(ctx, PF_EINVAL, "int4 layer without scales");
    }
    return PF_OK;
}

__global__ void k_iota(int32_t *idx, int n, int32_t *count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) idx[i] = i;
    if (i == 0) *count = n;
}

// counts[id(idx[j])] += 1 for j < *count, id = the layer's neuron table (stored -> original
// number) or the identity: every neuron is listed at most once and the table is a permutation
__global__ void k_count_activations(const int32_t *__restrict__ idx, const int32_t *__restrict__ count_p,
                                    int ffn, const int32_t *__restrict__ table,
                                    uint32_t *__restrict__ counts)
{
    const int n = min(max(*count_p, 0), ffn);
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
        int i = idx[j];
        if ((unsigned)i < (unsigned)ffn && table) i = table[i];
        if ((unsigned)i < (unsigned)ffn) counts[i] += 1u;
    }
}

// After an adaptive layer step: the density seen at this step decides the mode of the next.
// A sparse step saw the predicted list (its count); a dense step computed every neuron, so it
// counts the neurons whose FC1 output is non-zero for some token -- the exact active set.
// state = {dense flag, count, mode of this step}.  One workgroup.
__global__ __launch_bounds__(1024) void k_adapt_update(int32_t *__restrict__ state,
                                                       const int32_t *__restrict__ count_p,
                                                       const float *__restrict__ h, int hs, int B,
                                                       int ffn, int threshold_count)
{
    __shared__ int part[16];
    const int dense = state[0];
    int n = min(max(*count_p, 0), ffn);
    if (dense) {  // uniform
        int mine = 0;
        for (int j = threadIdx.x; j < ffn; j += 1024) {
            bool nz = false;
            for (int b = 0; b < B; ++b) nz = nz || h[(size_t)j * hs + b] != 0.f;
            mine += nz ? 1 : 0;
        }
        for (int o = 32; o >= 1; o >>= 1) mine += __shfl_xor(mine, o, 64);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mine;
        __syncthreads();
        n = 0;
        for (int k = 0; k < 16; ++k) n += part[k];
    }
    if (threadIdx.x == 0) {
        state[1] = n;
        state[2] = dense;
        state[0] = n >= threshold_count ? 1 : 0;
    }
}

__global__ void k_zero_words(uint64_t *__restrict__ words, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) words[i] = 0ull;
}

// Mask words in the original neuron numbering from a list in stored numbering: bit
// table[idx[j]] is set for j < *count.  Setting bits commutes, so the atomic OR leaves the
// same words whatever the order.
__global__ void k_scatter_original(const int32_t *__restrict__ idx, const int32_t *__restrict__ count_p,
                                   int ffn, const int32_t *__restrict__ table,
                                   uint32_t *__restrict__ words32)
{
    const int n = min(max(*count_p, 0), ffn);
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n; j += gridDim.x * blockDim.x) {
        int i = idx[j];
        if ((unsigned)i < (unsigned)ffn && table) i = table[i];
        if ((unsigned)i < (unsigned)ffn) atomicOr(&words32[i >> 5], 1u << (i & 31));
    }
}


// ---- layer step for callers that cannot allocate -----------------------------------------
// Scratch of pf_layer_step_noalloc: a fixed device array instead of a context's allocations.
// Pieces (each a multiple of 256 bytes): hidden vector t, mask words, index list, count, FC1
// outputs h, FC2 partial sums.
constexpr int kNaMaxD = 8192, kNaMaxFfn = 32768, kNaMaxR = 2048, kNaMaxBatch = 4;
constexpr size_t kNaOffT = 0;
constexpr size_t kNaOffMask = kNaOffT + (size_t)kNaMaxBatch * kNaMaxR * sizeof(float);
constexpr size_t kNaOffIdx = kNaOffMask + (size_t)(kNaMaxFfn / 64) * sizeof(uint64_t);
constexpr size_t kNaOffCount = kNaOffIdx + (size_t)kNaMaxFfn * sizeof(int32_t);
constexpr size_t kNaOffH = kNaOffCount + 256;
constexpr size_t kNaOffYpart = kNaOffH + (size_t)pf::h_stride(kNaMaxBatch) * kNaMaxFfn * sizeof(float);
constexpr size_t kNaScratchBytes =
    kNaOffYpart + (size_t)pf::kDown2MaxSplit * kNaMaxBatch * kNaMaxD * sizeof(float);
static_assert(kNaOffMask % 256 == 0 && kNaOffIdx % 256 == 0 && kNaOffCount % 256 == 0 &&
                  kNaOffH % 256 == 0 && kNaOffYpart % 256 == 0,
              "scratch pieces keep the array's alignment");

static __device__ __align__(256) unsigned char scratch[kNaScratchBytes];  // about 1.2 MB per GPU

constexpr int kNaMaxDevices = 64;
struct NoAllocState {
    bool ready = false;
    pf_ctx ctx;  // a context whose scratch pointers lie inside this device's copy of `scratch`
};
NoAllocState g_noalloc[kNaMaxDevices];
std::mutex g_noalloc_mutex;

// First call on a device: the device address of its copy of `scratch` (the array's name is
// only a host-side handle) and the launch limits of the device.  Nothing is allocated.
pf_status noalloc_state(int device, pf_ctx **out)
{
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    NoAllocState &S = g_noalloc[device];
    if (!S.ready) {
        unsigned char *ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return PF_EHIP;
        pf_ctx &c = S.ctx;
        c.device = device;
        c.max_d = kNaMaxD;
        c.max_ffn = kNaMaxFfn;
        c.max_r = kNaMaxR;
        c.max_batch = kNaMaxBatch;
        if (init_device_limits(&c, device) != hipSuccess) return PF_EHIP;
        c.t = reinterpret_cast<float *>(ptr + kNaOffT);
        c.mask_words = reinterpret_cast<uint64_t *>(ptr + kNaOffMask);
        c.idx = reinterpret_cast<int32_t *>(ptr + kNaOffIdx);
        c.count = reinterpret_cast<int32_t *>(ptr + kNaOffCount);
        c.h = reinterpret_cast<float *>(ptr + kNaOffH);
        c.ypart = reinterpret_cast<float *>(ptr + kNaOffYpart);
        S.ready = true;
    }
    *out = &S.ctx;
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
    if (max_ffn % 64 != 0 || max_d % 8 != 0 || max_r % 8 != 0 || max_ffn > kMaxFfn) return PF_ESHAPE;
    // the staged hidden vector of the whole batch, and one staged token (padded to an int4
    // chunk) next to the mask words of the widest layer, must fit LDS
    if ((size_t)max_batch * kpad_of(max_r) * sizeof(float) > (size_t)kLdsDefault - 2048 ||
        (size_t)kpad_i4(max_d) * sizeof(float) + pf::up_mask_lds_bytes(max_ffn) + 1024 >
            (size_t)kLdsMax)
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
        e = init_device_limits(ctx, device);
        if (e != hipSuccess) { st = PF_EHIP; break; }
        if ((size_t)kpad_i4(max_d) * sizeof(float) + pf::up_mask_lds_bytes(max_ffn) + 1024 >
            (size_t)ctx->lds_budget) {
            st = PF_ESHAPE;
            break;
        }
#define PF_ALLOC(ptr, bytes)                                                  \
        e = hipMalloc(reinterpret_cast<void **>(&(ptr)), (bytes));            \
        if (e != hipSuccess) { st = e == hipErrorOutOfMemory ? PF_ENOMEM : PF_EHIP; break; }
        PF_ALLOC(ctx->t, (size_t)max_batch * max_r * sizeof(float));
        PF_ALLOC(ctx->mask_words, (size_t)(max_ffn / 64) * sizeof(uint64_t));
        PF_ALLOC(ctx->idx, (size_t)max_ffn * sizeof(int32_t));
        PF_ALLOC(ctx->count, 64);
        PF_ALLOC(ctx->idx_all, (size_t)max_ffn * sizeof(int32_t));
        PF_ALLOC(ctx->mask_words2, (size_t)(max_ffn / 64) * sizeof(uint64_t));
        PF_ALLOC(ctx->count_all, 64);
        PF_ALLOC(ctx->h, (size_t)pf::h_stride(max_batch) * max_ffn * sizeof(float));
        PF_ALLOC(ctx->ypart, (size_t)pf::kDown2MaxSplit * max_batch * max_d * sizeof(float));
        PF_ALLOC(ctx->xbuf[0], (size_t)max_batch * max_d * sizeof(float));
        PF_ALLOC(ctx->xbuf[1], (size_t)max_batch * max_d * sizeof(float));
        PF_ALLOC(ctx->xsplit[0], (size_t)2 * max_batch * max_d * sizeof(__half));
        PF_ALLOC(ctx->xsplit[1], (size_t)2 * max_batch * max_d * sizeof(__half));
#undef PF_ALLOC
        e = hipMemset(ctx->count, 0, 64);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(k_iota, dim3(cdiv(max_ffn, 256)), dim3(256), 0, 0, ctx->idx_all, max_ffn,
                               ctx->count_all);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->capture_stream, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->side_stream, hipStreamNonBlocking);
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
    for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
    (void)hipFree(ctx->t);
    (void)hipFree(ctx->mask_words);
    (void)hipFree(ctx->idx);
    (void)hipFree(ctx->count);
    (void)hipFree(ctx->idx_all);
    (void)hipFree(ctx->mask_words2);
    if (ctx->side_stream) (void)hipStreamDestroy(ctx->side_stream);
    for (hipEvent_t e : ctx->la_events) (void)hipEventDestroy(e);
    (void)hipFree(ctx->count_all);
    (void)hipFree(ctx->h);
    (void)hipFree(ctx->ypart);
    (void)hipFree(ctx->xsplit[0]);
    (void)hipFree(ctx->xsplit[1]);
    (void)hipFree(ctx->xbuf[0]);
    (void)hipFree(ctx->xbuf[1]);
    delete ctx;
}

pf_status pf_layer_create(pf_ctx *ctx, const pf_layer_desc *desc, const pf_layer_weights *w,
                          pf_layer **out)
{
    if (!ctx) return PF_EINVAL;
    if (!out) return fail(ctx, PF_EINVAL, "out is null");
    *out = nullptr;
    const pf_status chk = check_layer(ctx, desc, w);
    if (chk != PF_OK) return chk;
    pf_layer *L = new (std::nothrow) pf_layer();
    if (!L) return fail(ctx, PF_ENOMEM, "host allocation failed");
    L->ctx = ctx;
    L->desc = *desc;
    L->w = *w;
    L->thr_logit = logit_of(desc->threshold);
    // the few words of device state of pf_layer_step_adaptive
    hipError_t e = hipSetDevice(ctx->device);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&L->adapt), 256);
    if (e == hipSuccess) e = hipMemset(L->adapt, 0, 256);
    if (e != hipSuccess) {
        (void)hipFree(L->adapt);
        delete L;
        return fail(ctx, e == hipErrorOutOfMemory ? PF_ENOMEM : PF_EHIP, "layer state: %s",
                    hipGetErrorString(e));
    }
    *out = L;
    return PF_OK;
}

void pf_layer_destroy(pf_layer *layer)
{
    if (!layer) return;
    (void)hipFree(layer->adapt);
    delete layer;
}

pf_status pf_predict(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *scores,
                     uint64_t *mask_words, void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!mask_words) return fail(ctx, PF_EINVAL, "mask_words is null");
    return launch_predict(ctx, layer, x, nullptr, 0, nullptr, B, scores, mask_words,
                          static_cast<hipStream_t>(stream));
}

pf_status pf_compact(pf_ctx *ctx, const uint64_t *mask_words, int ffn, int32_t *idx, int32_t *count,
                     void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!mask_words || !idx || !count) return fail(ctx, PF_EINVAL, "null argument");
    if (ffn < 0) return fail(ctx, PF_EINVAL, "negative ffn");
    if (ffn % 64 != 0) return fail(ctx, PF_ESHAPE, "ffn %d is not a multiple of 64", ffn);
    {
        ProfScope ps(ctx, K_COMPACT);
        PF_LAUNCH(ps, pf::k_compact, dim3(1), dim3(pf::kCompactThreads), 0,
                  static_cast<hipStream_t>(stream), mask_words, ffn / 64, idx, count);
    }
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status pf_sparse_ffn(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, const int32_t *idx,
                        const int32_t *count, float *y, void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!idx || !count || !y) return fail(ctx, PF_EINVAL, "null argument");
    return launch_sparse(ctx, layer, x, B, idx, count, nullptr, y, nullptr,
                         static_cast<hipStream_t>(stream));
}

pf_status pf_layer_step(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *y,
                        void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!y) return fail(ctx, PF_EINVAL, "y is null");
    if (!layer->w.p1) return fail(ctx, PF_EINVAL, "layer has no predictor weights");
    return launch_layer(ctx, layer, x, nullptr, 0, nullptr, B, y, nullptr,
                        static_cast<hipStream_t>(stream));
}

pf_status pf_layer_step_noalloc(const pf_layer_desc *desc, const pf_layer_weights *w, const float *x,
                                int B, float *y, void *stream)
{
    if (!desc || !w || !x || !y) return PF_EINVAL;
    if (desc->d > kNaMaxD || desc->ffn > kNaMaxFfn || desc->r > kNaMaxR || B > kNaMaxBatch)
        return PF_ELIMIT;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return PF_EHIP;
    if (device < 0 || device >= kNaMaxDevices) return PF_ELIMIT;
    pf_ctx *ctx = nullptr;
    pf_status s = noalloc_state(device, &ctx);
    if (s != PF_OK) return s;
    s = check_layer(ctx, desc, w);
    if (s != PF_OK) return s;
    if (!w->p1) return PF_EINVAL;
    pf_layer L;  // on the stack: the kernels take the weight pointers, not the handle
    L.ctx = ctx;
    L.desc = *desc;
    L.w = *w;
    L.thr_logit = logit_of(desc->threshold);
    s = check_batch(ctx, &L, x, B);
    if (s != PF_OK) return s;
    return launch_layer(ctx, &L, x, nullptr, 0, nullptr, B, y, nullptr, static_cast<hipStream_t>(stream));
}

pf_status pf_dense_ffn(pf_ctx *ctx, const pf_layer *layer, const float *x, int B, float *y,
                       void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!y) return fail(ctx, PF_EINVAL, "y is null");
    ctx->last_mask = nullptr;
    ctx->last_idx = ctx->idx_all;
    ctx->last_count = ctx->count_all;
    return launch_sparse(ctx, layer, x, B, ctx->idx_all, ctx->count_all, nullptr, y, nullptr,
                         static_cast<hipStream_t>(stream));
}

pf_status pf_layer_step_auto(pf_ctx *ctx, const pf_layer *layer, const float *x, int B,
                             float density_hint, float crossover, float *y, void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!(crossover > 0.f && crossover <= 1.f) || !(density_hint >= 0.f))
        return fail(ctx, PF_EINVAL, "crossover %g outside (0, 1] or negative density hint %g",
                    (double)crossover, (double)density_hint);
    if (density_hint >= crossover) return pf_dense_ffn(ctx, layer, x, B, y, stream);
    return pf_layer_step(ctx, layer, x, B, y, stream);
}

pf_status pf_layer_step_adaptive(pf_ctx *ctx, pf_layer *layer, const float *x, int B, float crossover,
                                 float *y, void *stream)
{
    pf_status s = check_batch(ctx, layer, x, B);
    if (s != PF_OK) return s;
    if (!y) return fail(ctx, PF_EINVAL, "y is null");
    if (!layer->w.p1) return fail(ctx, PF_EINVAL, "layer has no predictor weights");
    if (!(crossover > 0.f && crossover <= 1.f))
        return fail(ctx, PF_EINVAL, "crossover %g outside (0, 1]", (double)crossover);
    if (!layer->adapt) return fail(ctx, PF_EINVAL, "layer has no adaptive state");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const pf_layer_desc &D = layer->desc;
    // predictor kernels return at once, and mark every neuron, when the layer's flag is set
    s = launch_predict(ctx, layer, x, nullptr, 0, nullptr, B, nullptr, ctx->mask_words, st, layer->adapt);
    if (s != PF_OK) return s;
    ctx->last_mask = ctx->mask_words;
    ctx->last_idx = ctx->idx;
    ctx->last_count = ctx->count;
    s = launch_sparse(ctx, layer, x, B, nullptr, nullptr, ctx->mask_words, y, nullptr, st);
    if (s != PF_OK) return s;
    int thr = (int)std::ceil((double)crossover * (double)D.ffn);
    if (thr < 1) thr = 1;
    hipLaunchKernelGGL(k_adapt_update, dim3(1), dim3(1024), 0, st, layer->adapt,
                       (const int32_t *)ctx->count, (const float *)ctx->h, pf::h_stride(B), B, D.ffn, thr);
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status pf_layer_adaptive_state(pf_layer *layer, int32_t *host_state, int reset)
{
    if (!layer || !layer->adapt) return PF_EINVAL;
    pf_ctx *ctx = layer->ctx;
    PF_HIP(ctx, hipDeviceSynchronize());
    if (host_state) PF_HIP(ctx, hipMemcpy(host_state, layer->adapt, 3 * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (reset) PF_HIP(ctx, hipMemset(layer->adapt, 0, 256));
    return PF_OK;
}

pf_status pf_count_activations(pf_ctx *ctx, const pf_layer *layer, uint32_t *counts, void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!layer || !counts) return fail(ctx, PF_EINVAL, "null argument");
    if (layer->ctx != ctx) return fail(ctx, PF_EINVAL, "layer belongs to another context");
    if (!ctx->last_idx) return fail(ctx, PF_EINVAL, "no layer step has run on this context");
    hipLaunchKernelGGL(k_count_activations, dim3(64), dim3(256), 0, static_cast<hipStream_t>(stream),
                       ctx->last_idx, ctx->last_count, layer->desc.ffn, layer->table, counts);
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status pf_layer_set_neuron_table(pf_layer *layer, const int32_t *stored_to_original, int always_on)
{
    if (!layer) return PF_EINVAL;
    pf_ctx *ctx = layer->ctx;
    if (always_on < 0 || always_on % 64 != 0 || always_on > layer->desc.ffn - 64)
        return fail(ctx, PF_EINVAL, "always_on %d: a multiple of 64 in [0, ffn - 64]", always_on);
    layer->table = stored_to_original;
    layer->always_on = always_on;
    return PF_OK;
}

pf_status pf_layer_active_original(pf_ctx *ctx, const pf_layer *layer, uint64_t *mask_words,
                                   int32_t *idx, int32_t *count, void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!layer || !mask_words || !idx || !count) return fail(ctx, PF_EINVAL, "null argument");
    if (layer->ctx != ctx) return fail(ctx, PF_EINVAL, "layer belongs to another context");
    if (!ctx->last_idx) return fail(ctx, PF_EINVAL, "no layer step has run on this context");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nwords = layer->desc.ffn / 64;
    hipLaunchKernelGGL(k_zero_words, dim3(cdiv(nwords, 256)), dim3(256), 0, st, mask_words, nwords);
    hipLaunchKernelGGL(k_scatter_original, dim3(64), dim3(256), 0, st, ctx->last_idx, ctx->last_count,
                       layer->desc.ffn, layer->table, reinterpret_cast<uint32_t *>(mask_words));
    hipLaunchKernelGGL(pf::k_compact, dim3(1), dim3(pf::kCompactThreads), 0, st,
                       (const uint64_t *)mask_words, nwords, idx, count);
    PF_HIP(ctx, hipGetLastError());
    return PF_OK;
}

pf_status pf_ctx_last_active(pf_ctx *ctx, const uint64_t **mask_words, const int32_t **idx,
                             const int32_t **count)
{
    if (!ctx) return PF_EINVAL;
    if (mask_words) *mask_words = ctx->last_idx ? ctx->last_mask : ctx->mask_words;
    if (idx) *idx = ctx->last_idx ? ctx->last_idx : ctx->idx;
    if (count) *count = ctx->last_count ? ctx->last_count : ctx->count;
    return PF_OK;
}

pf_status pf_stack_glue(pf_ctx *ctx, const float *x, const float *y, int d, int B, float *x_next,
                        void *stream)
{
    if (!ctx) return PF_EINVAL;
    if (!x || !y || !x_next) return fail(ctx, PF_EINVAL, "null argument");
    if (d < 1 || B < 1) return fail(ctx, PF_EINVAL, "non-positive size");
    return launch_glue(ctx, x, y, 1, d, B, x_next, static_cast<hipStream_t>(stream));
}

pf_status pf_ctx_set_lookahead(pf_ctx *ctx, int distance)
{
    if (!ctx) return PF_EINVAL;
    if (distance != 0 && distance != 1) return fail(ctx, PF_EINVAL, "look-ahead distance %d: 0 or 1", distance);
    ctx->lookahead = distance;
    return PF_OK;
}

pf_status pf_ctx_set_option(pf_ctx *ctx, int key, int value)
{
    if (!ctx) return PF_EINVAL;
    switch (key) {
        case PF_OPT_FUSED:
            if (value < 0 || value > 2) break;
            ctx->fused = value;
            return PF_OK;
        case PF_OPT_SEG_STRIDED:
            if (value < 0 || value > 1) break;
            ctx->seg_strided = value;
            return PF_OK;
        case PF_OPT_MFMA_MIN_BATCH:
            if (value < 0) break;
            ctx->mfma_min_batch = value > 0 ? value : 4;
            ctx->mfma_min_batch_forced = value > 0;
            return PF_OK;
        case PF_OPT_HIDDEN_MFMA_MIN_ELEMS:
            if (value < 0) break;
            ctx->hidden_mfma_min_elems = value;
            return PF_OK;
        case PF_OPT_UP_GRID:
            if (value < 0 || value > 65535) break;
            ctx->up_grid_cap = value > 0 ? value : 8 * ctx->num_cu;
            ctx->up_grid_cap_i4 = value > 0 ? value : 2 * ctx->num_cu;
            return PF_OK;
        case PF_OPT_MFMA_GRID:
            if (value < 0 || value > 65535) break;
            ctx->mfma_grid = value;
            return PF_OK;
        case PF_OPT_DOWN_SPLIT:
            if (value < 0 || value > pf::kDown2MaxSplit) break;
            ctx->down_split = value;
            return PF_OK;
        case PF_OPT_LOOKAHEAD_FORM:
            if (value < 0 || value > 3) break;
            ctx->la_form = value;
            return PF_OK;

        default:
            return fail(ctx, PF_EINVAL, "unknown option %d", key);
    }
    return fail(ctx, PF_EINVAL, "option %d: value %d out of range", key, value);
}

pf_status pf_ctx_get_option(const pf_ctx *ctx, int key, int *value)
{
    if (!ctx || !value) return PF_EINVAL;
    switch (key) {
        case PF_OPT_FUSED: *value = ctx->fused; break;
        case PF_OPT_SEG_STRIDED: *value = ctx->seg_strided; break;
        case PF_OPT_MFMA_MIN_BATCH: *value = ctx->mfma_min_batch_forced ? ctx->mfma_min_batch : 0; break;
        case PF_OPT_HIDDEN_MFMA_MIN_ELEMS: *value = ctx->hidden_mfma_min_elems; break;
        case PF_OPT_UP_GRID: *value = ctx->up_grid_cap; break;
        case PF_OPT_MFMA_GRID: *value = ctx->mfma_grid; break;
        case PF_OPT_DOWN_SPLIT: *value = ctx->down_split; break;
        case PF_OPT_LOOKAHEAD_FORM: *value = ctx->la_form; break;
        default: return PF_EINVAL;
    }
    return PF_OK;
}

pf_status pf_ctx_set_mask_trace(pf_ctx *ctx, uint64_t *trace, int n_layers_capacity)
{
    if (!ctx) return PF_EINVAL;
    if (trace && n_layers_capacity < 1) return fail(ctx, PF_EINVAL, "trace buffer without capacity");
    ctx->mask_trace = trace;
    ctx->mask_trace_layers = trace ? n_layers_capacity : 0;
    return PF_OK;
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
    ctx->capturing = true;
    s = stack_enqueue(ctx, layers, n_layers, x, B, x_out, cs);
    ctx->capturing = false;
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

pf_status pf_profile_begin(pf_ctx *ctx)
{
    if (!ctx) return PF_EINVAL;
    ctx->prof_kernel.clear();
    ctx->prof_on = true;
    return PF_OK;
}

pf_status pf_profile_end(pf_ctx *ctx, pf_kernel_stat *stats, int capacity, int *n_out)
{
    if (!ctx) return PF_EINVAL;
    if (!stats || !n_out || capacity < K_NUM)
        return fail(ctx, PF_EINVAL, "stats needs %d entries", (int)K_NUM);
    ctx->prof_on = false;
    for (int k = 0; k < K_NUM; ++k) {
        stats[k].name = kKernelNames[k];
        stats[k].launches = 0;
        stats[k].total_ms = 0.0;
    }
    *n_out = K_NUM;
    for (size_t p = 0; p < ctx->prof_kernel.size(); ++p) {
        PF_HIP(ctx, hipEventSynchronize(ctx->prof_events[2 * p + 1]));
        float ms = 0.f;
        PF_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_events[2 * p], ctx->prof_events[2 * p + 1]));
        pf_kernel_stat &st = stats[ctx->prof_kernel[p]];
        st.launches += 1;
        st.total_ms += (double)ms;
    }
    ctx->prof_kernel.clear();
    return PF_OK;
}

#ifdef PF_TRACE
// Tuning builds only: device buffer of [4 kernels][4096 blocks][8] 64-bit stamps, or NULL.
pf_status pf_debug_set_trace(unsigned long long *device_buffer)
{
    return hipMemcpyToSymbol(HIP_SYMBOL(pf::g_pf_trace), &device_buffer, sizeof(device_buffer)) ==
                   hipSuccess
               ? PF_OK
               : PF_EHIP;
}
#endif

const char *pf_strerror(pf_status s)
{
    switch (s) {
        case PF_OK: return "ok";
        case PF_EINVAL: return "invalid argument";
        case PF_ESHAPE: return "unsupported shape";
        case PF_ENOMEM: return "out of memory";
        case PF_EHIP: return "HIP runtime error";
        case PF_EUNSUPPORTED: return "not supported";
        case PF_ELIMIT: return "size beyond the fixed limits of the no-allocation entry point";
    }
    return "unknown status";
}

const char *pf_last_error(const pf_ctx *ctx) { return ctx ? ctx->err : ""; }

const char *pf_version(void) { return "libpf 0.2 (gfx950)"; }

}  // extern "C"
