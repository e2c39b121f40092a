// Look-ahead prediction with the overlap realised inside the launches (PowerInfer Sec. 2.1: the
// activations of a layer can be predicted from an earlier layer's input).  With the active set
// of layer l+1 taken from its predictor applied to the INPUT of layer l, the predictor of the
// next layer and the sparse kernels of this layer are independent, and a layer becomes two
// launches whose block ranges play two roles each:
//   k_la_up_hidden : blocks [0, n_hid)   hidden layer of predictor l+1 on x_l     (k_predict.h)
//                    blocks [n_hid, ..)  FC1 of layer l over mask_l                (k_sparse.h)
//   k_la_down_out  : blocks [0, n_fc2)   FC2 of layer l over the list FC1 left     (k_sparse.h)
//                    blocks [n_fc2, ..)  output layer of predictor l+1 -> mask_l+1 (k_predict.h)
// The dense predictor rows stream while the dependent chains of the sparse kernels (mask scan,
// list, gathered rows) wait on memory, in the same launch: nothing is gained from a second
// stream on this part (graph branches replay one after the other), but workgroups of two roles
// share the CUs.  Inside a stack both roles of the first launch form the layer input from the
// previous layer's input and FC2 partial sums themselves (GLUE); FC1's first block stores it.
// The role bodies are the stand-alone kernels' own.  Three families: the vector kernels (fp16,
// batch <= 3; below), the matrix-core kernels (fp16, larger batches) and the int4 kernels
// (further down; those two read a layer input that a glue kernel in front has formed).
#pragma once
#include "dev_util.h"
#include "k_predict.h"
#include "k_sparse.h"
#include "k_mfma.h"
#include "k_int4.h"

namespace pf {

static_assert(kUpThreads == kPredThreads, "both roles of the first launch use the same block size");

// grid = n_hid + n_up, block = 256.  Dynamic LDS: staged input [B][dpad] + scrap + mask scan.
template <int B, int ACT, bool GLUE>
__global__ __launch_bounds__(kUpThreads) void k_la_up_hidden(
    int n_hid, const __half *__restrict__ p1, float *__restrict__ t, int r,
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const float *__restrict__ x, const float *__restrict__ yp, int ny,
    int ypstride, float *__restrict__ x_new, const uint64_t *__restrict__ mask_words,
    int32_t *__restrict__ idx_out, int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d,
    int ffn, float up_floor, bool up_first)
{
    extern __shared__ float xs[];
    __shared__ uint32_t wave_tot[kUpWaves];
    __shared__ float ss_w[kUpWaves][B];
    // up_first: FC1's blocks take the low block numbers (dispatched first)
    const int n_up = (int)gridDim.x - n_hid;
    const int bid = (int)blockIdx.x;
    const bool is_hid = up_first ? bid >= n_up : bid < n_hid;
    if (is_hid) {  // uniform over the block
        pred_hidden_body<B, GLUE, (B >= 2 ? 1 : 4)>(xs, ss_w, up_first ? bid - n_up : bid, false, p1, x, yp,
                                                    ny, ypstride, x_new, t, d, r, 0);
    } else {
        const int ub = up_first ? bid : bid - n_hid;
        up_body<B, ACT, true, GLUE>(xs, wave_tot, ss_w, ub, n_up, ub == 0, w_up, w_gate, b_up, x, nullptr,
                                    nullptr, mask_words, idx_out, count_out, h, hs, d, ffn, up_floor,
                                    yp, ny, ypstride, x_new);
    }
}

constexpr int kLaOutNeurons = 32;                      // output-layer role: 32 neurons per block,
static_assert(kLaOutNeurons * 16 == kDown2Threads,     // 16 threads per neuron = FC2's block size
              "both roles of the second launch use the same block size");

// grid = tiles * P + ffn_next / 32, block = 512.  Dynamic LDS: staged hidden vector [B][rpad].
template <int B>
__global__ __launch_bounds__(kDown2Threads) void k_la_down_out(
    int tiles, int P, const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const int32_t *__restrict__ idx, const int32_t *__restrict__ count_p,
    float *__restrict__ part, int d, int ffn, const __half *__restrict__ p2,
    const float *__restrict__ p_bias, const float *__restrict__ t, int r, int ffn_next, float thr_logit,
    uint64_t *__restrict__ mask_next, int first_word, bool out_first)
{
    extern __shared__ float ts[];
    __shared__ float red[kDown2Waves][B][kDown2Cols];
    __shared__ float logit_s[B][kLaOutNeurons];
    const int bid = (int)blockIdx.x, n_fc2 = tiles * P, n_out = (int)gridDim.x - n_fc2;
    const bool is_fc2 = out_first ? bid >= n_out : bid < n_fc2;
    if (is_fc2) {  // uniform over the block
        const int fb = out_first ? bid - n_out : bid;
        down2_body<B>(red, fb % tiles, fb / tiles, P, w_down, b_down, h, idx, count_p, part, d, ffn);
    } else {
        pred_out_body<B, kLaOutNeurons>(ts, logit_s, out_first ? bid : bid - n_fc2, p2, p_bias, t, r,
                                        ffn_next, thr_logit, nullptr, mask_next, first_word);
    }
}

// ---------------------------------------------------------------------------------------
// The same two launches for batches on the matrix cores (batch >= 4, or 3 with long rows),
// from the matrix-core kernels' bodies.  These read the layer input from memory, as split
// fp16 planes, so a glue kernel of its own (or k_split for the first layer) runs in front of
// the first launch.  Ungated layers: two workgroups of
// either role fit a CU.  The gated FC1 needs 128 KB of LDS per workgroup, so there a CU holds
// one workgroup at a time and the hidden-layer role follows FC1 rather than sharing the CUs.
static_assert(kMfmaThreads == kDown2Threads, "all roles of these launches use 512 threads");

// grid = n_up + n_hid, block = 512: [FC1 of layer l on the matrix cores | hidden layer of
// predictor l+1 on the matrix cores].  Dynamic LDS: FC1's mask scan + slots (>= the hidden
// layer's 64 KB of slots).
template <int ACT>
__global__ __launch_bounds__(kMfmaThreads) void k_la_up_hidden_mfma(
    int n_hid, const __half *__restrict__ p1, float *__restrict__ t, int r,
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const void *__restrict__ xs, int B,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor)
{
    extern __shared__ uint64_t dyn_lds64[];
    __shared__ uint32_t wave_tot[kMfmaWaves];
    __shared__ int irow[32];
    __shared__ float brow[32];
    __shared__ float logit_s[16][16];
    const int n_up = (int)gridDim.x - n_hid, bid = (int)blockIdx.x;
    if (bid < n_up) {  // uniform over the block
        up_mfma_body<ACT, true, true>(dyn_lds64, wave_tot, irow, brow, bid, n_up, w_up, w_gate, b_up, xs, B,
                                      nullptr, nullptr, mask_words, idx_out, count_out, h, hs, d, ffn, up_floor);
    } else {
        rows_mfma_body<8, 512, 0, true>(dyn_lds64, logit_s, bid - n_up, p1, xs, B, d, r, nullptr, 0.f, t, nullptr,
                                        0);
    }
}

// grid = tiles * P + (ffn_next - always-on prefix) / 64, block = 512: [FC2 of layer l | output
// layer of predictor l+1 on the matrix cores].  Dynamic LDS: the output layer's 64 KB of slots;
// FC2's cross-wave sums live in the same region (a workgroup plays one role), so that two
// workgroups fit a CU.
template <int B>
__global__ __launch_bounds__(kMfmaThreads) void k_la_down_out_mfma(
    int tiles, int P, const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const int32_t *__restrict__ idx, const int32_t *__restrict__ count_p,
    float *__restrict__ part, int d, int ffn, const __half *__restrict__ p2,
    const float *__restrict__ p_bias, const float *__restrict__ t, int r, int ffn_next, float thr_logit,
    uint64_t *__restrict__ mask_next, int first_word)
{
    extern __shared__ uint64_t dyn_lds64[];
    __shared__ float logit_s[16][64];
    static_assert(sizeof(float) * kDown2Waves * B * kDown2Cols <= (size_t)kMfmaWaves * kRowsMfmaSlotBytes,
                  "FC2's sums fit the slots");
    const int bid = (int)blockIdx.x, n_fc2 = tiles * P;
    if (bid < n_fc2) {  // uniform over the block
        down2_body<B>(reinterpret_cast<float(*)[B][kDown2Cols]>(dyn_lds64), bid % tiles, bid / tiles, P, w_down,
                      b_down, h, idx, count_p, part, d, ffn);
    } else {
        rows_mfma_body<64, 64, 1, false>(dyn_lds64, logit_s, bid - n_fc2, p2, t, B, r, ffn_next, p_bias, thr_logit,
                                         nullptr, mask_next, first_word);
    }
}

// ---------------------------------------------------------------------------------------
// The same two launches over int4 weights (the predictor stays fp16).  FC1's int4 kernel reads
// the layer input from memory, so a glue kernel of its own runs in front of the first launch.
static_assert(kUpI4Threads == kDown2I4Threads && kDown2I4Threads == kDown2Threads, "512 threads in all roles");

// grid = n_up + n_hid, block = 512: [FC1 of layer l over int4 rows | hidden layer of predictor
// l+1, 8 rows per block].  Dynamic LDS: FC1's staged input + scrap + mask scan (>= the hidden
// layer's staged input).
template <int B, int ACT>
__global__ __launch_bounds__(kUpI4Threads) void k_la_up_hidden_i4(
    int n_hid, const __half *__restrict__ p1, float *__restrict__ t, int r,
    const uint8_t *__restrict__ q_up, const __half *__restrict__ s_up,
    const uint8_t *__restrict__ q_gate, const __half *__restrict__ s_gate,
    const float *__restrict__ b_up, const float *__restrict__ x,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor)
{
    extern __shared__ float xs[];
    __shared__ uint32_t wave_tot[kUpI4Waves];
    __shared__ float ss_w[kUpI4Waves][B];
    const int n_up = (int)gridDim.x - n_hid, bid = (int)blockIdx.x;
    if (bid < n_up) {  // uniform over the block
        up_i4_body<B, ACT, true>(xs, wave_tot, bid, n_up, q_up, s_up, q_gate, s_gate, b_up, x, nullptr, nullptr,
                                 mask_words, idx_out, count_out, h, hs, d, ffn, up_floor);
    } else {
        pred_hidden_body<B, false, 1, kUpI4Threads>(xs, ss_w, bid - n_up, false, p1, x, nullptr, 0, 0, nullptr, t,
                                                    d, r, 0);
    }
}

// grid = tiles * P + (ffn_next - always-on prefix) / 32, block = 512: [FC2 of layer l over int4
// rows | output layer of predictor l+1].  Dynamic LDS: staged hidden vector [B][rpad].
template <int B>
__global__ __launch_bounds__(kDown2I4Threads) void k_la_down_out_i4(
    int tiles, int P, const uint8_t *__restrict__ q_down, const __half *__restrict__ s_down,
    const float *__restrict__ b_down, const float *__restrict__ h, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_p, float *__restrict__ part, int d, int ffn,
    const __half *__restrict__ p2, const float *__restrict__ p_bias, const float *__restrict__ t, int r,
    int ffn_next, float thr_logit, uint64_t *__restrict__ mask_next, int first_word)
{
    extern __shared__ float ts[];
    __shared__ float red[kDown2I4Waves][B][kDown2I4Cols];
    __shared__ float logit_s[B][kLaOutNeurons];
    const int bid = (int)blockIdx.x, n_fc2 = tiles * P;
    if (bid < n_fc2) {  // uniform over the block
        down2_i4_body<B>(red, bid % tiles, tiles, bid / tiles, P, q_down, s_down, b_down, h, idx, count_p, part,
                         d, ffn);
    } else {
        pred_out_body<B, kLaOutNeurons>(ts, logit_s, bid - n_fc2, p2, p_bias, t, r, ffn_next, thr_logit, nullptr,
                                        mask_next, first_word);
    }
}

}  // namespace pf
