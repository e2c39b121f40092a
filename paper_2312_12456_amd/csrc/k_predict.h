// Activation predictor (PowerInfer Sec. 5.1: input layer, one hidden layer, output layer)
// and active-index compaction.
//   hidden : t[b][m]     = ReLU(p1[m] . x[b])                          r rows of d fp16
//   output : logit[b][i] = p2[i] . t[b] + p_bias[i]                     ffn rows of r fp16
//            bit i of the mask = any_b(logit[b][i] > logit(threshold))  (wave ballot)
//   compact: idx[] = ascending positions of the set bits, count = popcount
// Both GEMVs are HBM-bound streams of fp16 rows: one wave per row, 16-byte loads per
// lane, activations staged once per workgroup in LDS, fp32 accumulation, DPP reduction.
#pragma once
#include "dev_util.h"

namespace pf {

constexpr int kPredThreads = 256;  // 4 waves per workgroup

// ---------------------------------------------------------------------------------------
// Hidden layer.  grid = ceil(r / 4); wave w of block g owns row 4g + w.
template <int B>
__global__ __launch_bounds__(kPredThreads) void k_pred_hidden(const __half *__restrict__ p1,
                                                              const float *__restrict__ x,
                                                              float *__restrict__ t, int d, int r)
{
    extern __shared__ float xs[];
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nch = (d + kChunk - 1) / kChunk, kpad = nch * kChunk;
    const int m = blockIdx.x * (kPredThreads / kWave) + wave;
    const bool live = m < r;
    const __half *row = p1 + (size_t)(live ? m : 0) * d;

    WGroup<U> g;
    load_group<U>(g, row, live ? d : 0, 0, lane);  // in flight while x is staged
    stage_vector<B>(xs, x, d, kpad);
    __syncthreads();

    float acc[B];
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = 0.f;
    fma_group<B, U>(g, xs, kpad, 0, nch, lane, acc);
    for (int it0 = U; it0 < nch; it0 += U) {
        load_group<U>(g, row, live ? d : 0, it0, lane);
        fma_group<B, U>(g, xs, kpad, it0, nch, lane, acc);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const float s = wave_sum(acc[b]);
        if (live && lane == 0) t[(size_t)b * r + m] = fmaxf(s, 0.f);
    }
}

// ---------------------------------------------------------------------------------------
// Compaction of mask words into an ascending index list, by one workgroup of NT threads.
// Pass 1: per-word popcount and a block-wide exclusive prefix (wave scan + LDS).
// Pass 2: one wave per word; lane l owns bit l, its rank inside the word is the popcount
//         of the lower bits (what a ballot + mbcnt pair would give for a live predicate).
template <int NT>
struct CompactLds {
    uint64_t word[NT];
    uint32_t pre[NT];
    uint32_t wave_tot[NT / kWave];
};

template <int NT>
__device__ __forceinline__ void compact_block(const uint64_t *mask_words, int nwords,
                                              int32_t *__restrict__ idx, int32_t *__restrict__ count,
                                              CompactLds<NT> &s)
{
    constexpr int NW = NT / kWave;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t carry = 0;
    for (int w0 = 0; w0 < nwords; w0 += NT) {
        const int w = w0 + tid;
        const uint64_t word = w < nwords ? mask_words[w] : 0ull;
        const uint32_t pc = (uint32_t)__popcll(word);
        uint32_t inc = pc;  // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = (uint32_t)__shfl_up((int)inc, o, 64);
            if (lane >= o) inc += up;
        }
        if (lane == 63) s.wave_tot[wave] = inc;
        s.word[tid] = word;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            const uint32_t v = s.wave_tot[k];
            if (k < wave) before += v;
            total += v;
        }
        s.pre[tid] = carry + before + inc - pc;
        __syncthreads();
        const int nhere = min(NT, nwords - w0);
        for (int q = wave; q < nhere; q += NW) {
            const uint64_t wq = s.word[q];
            const uint32_t base = s.pre[q];
            const uint64_t below = wq & ((1ull << lane) - 1ull);
            if ((wq >> lane) & 1ull) idx[base + (uint32_t)__popcll(below)] = (w0 + q) * 64 + lane;
        }
        carry += total;
        __syncthreads();
    }
    if (tid == 0) *count = (int32_t)carry;
}

constexpr int kCompactThreads = 1024;

__global__ __launch_bounds__(kCompactThreads) void k_compact(const uint64_t *__restrict__ mask_words,
                                                             int nwords, int32_t *__restrict__ idx,
                                                             int32_t *__restrict__ count)
{
    __shared__ CompactLds<kCompactThreads> lds;
    compact_block<kCompactThreads>(mask_words, nwords, idx, count, lds);
}

// ---------------------------------------------------------------------------------------
// Output layer + threshold + ballot.  grid = ffn / 64; block g (16 waves) owns neurons
// 64g .. 64g+63, wave w of it rows 4w .. 4w+3, all in flight at once.  With FUSE the last block to
// finish (device-scope arrival counter) also compacts the mask words, which saves a
// launch on the layer-step path.
constexpr int kPredOutThreads = 1024;

template <int B, bool FUSE>
__global__ __launch_bounds__(kPredOutThreads) void k_pred_out(
    const __half *__restrict__ p2, const float *__restrict__ p_bias, const float *__restrict__ t,
    int r, int ffn, float thr_logit, float *__restrict__ scores, uint64_t *__restrict__ mask_words,
    unsigned int *__restrict__ arrive, int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    extern __shared__ float ts[];          // [B][kpad] staged hidden vector
    __shared__ float logit_s[B][64];
    __shared__ CompactLds<kPredOutThreads> clds;
    __shared__ int is_last;
    // 16 waves per block leave 128 VGPRs per lane: fewer loads in flight at larger batch
    constexpr int U = (B <= 2) ? 4 : 2, R = 4, ROWS = 64 / (kPredOutThreads / kWave);
    static_assert(ROWS == R, "one round of R rows per wave");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nch = (r + kChunk - 1) / kChunk, kpad = nch * kChunk;
    const int n0 = blockIdx.x * 64 + wave * ROWS;

    WGroup<U> g[R];
#pragma unroll
    for (int q = 0; q < R; ++q) load_group<U>(g[q], p2 + (size_t)(n0 + q) * r, r, 0, lane);
    stage_vector<B>(ts, t, r, kpad);
    __syncthreads();

    for (int q0 = 0; q0 < ROWS; q0 += R) {
        float acc[R][B];
#pragma unroll
        for (int q = 0; q < R; ++q) {
#pragma unroll
            for (int b = 0; b < B; ++b) acc[q][b] = 0.f;
            fma_group<B, U>(g[q], ts, kpad, 0, nch, lane, acc[q]);
        }
        for (int it0 = U; it0 < nch; it0 += U) {
#pragma unroll
            for (int q = 0; q < R; ++q)
                load_group<U>(g[q], p2 + (size_t)(n0 + q0 + q) * r, r, it0, lane);
#pragma unroll
            for (int q = 0; q < R; ++q) fma_group<B, U>(g[q], ts, kpad, it0, nch, lane, acc[q]);
        }
        if (q0 + R < ROWS) {  // next four rows go in flight before the reductions
#pragma unroll
            for (int q = 0; q < R; ++q)
                load_group<U>(g[q], p2 + (size_t)(n0 + q0 + R + q) * r, r, 0, lane);
        }
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int i = n0 + q0 + q;
            const float pb = p_bias ? p_bias[i] : 0.f;
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const float s = wave_sum(acc[q][b]) + pb;
                if (lane == 0) logit_s[b][wave * ROWS + q0 + q] = s;
            }
        }
    }
    __syncthreads();

    if (scores != nullptr) {
        for (int e = threadIdx.x; e < B * 64; e += kPredOutThreads) {
            const int b = e >> 6, q = e & 63;
            scores[(size_t)b * ffn + blockIdx.x * 64 + q] = 1.f / (1.f + __expf(-logit_s[b][q]));
        }
    }
    if (wave == 0) {
        bool on = false;
#pragma unroll
        for (int b = 0; b < B; ++b) on = on || (logit_s[b][lane] > thr_logit);
        const uint64_t word = __ballot(on);
        if (lane == 0) mask_words[blockIdx.x] = word;
    }

    if (FUSE) {
        __threadfence();  // the mask word is visible device-wide before the arrival
        if (threadIdx.x == 0) {
            const unsigned int prev = atomicAdd(arrive, 1u);
            is_last = (prev == gridDim.x - 1);
            if (is_last) *arrive = 0u;  // ready for the next launch
        }
        __syncthreads();
        if (is_last) {
            __threadfence();
            compact_block<kPredOutThreads>(mask_words, ffn / 64, idx, count, clds);
        }
    }
}

}  // namespace pf
