// EXPERIMENTAL, off unless PF_FUSED=1 (measured slower than the four-launch step on the
// OPT-6.7B shape: 18.5 + 12.8 us against 8.6 + 7.0 + 8.8 us; kept because it is parity-clean
// and the balance may differ at other shapes).
// The layer step as three launches instead of four (PowerInfer Sec. 5.1 + 5.4):
//   k_pred_hidden            t = ReLU(p1 . x)                                   (k_predict.h)
//   k_pred_out_up            logits, threshold and ballot for 64 neurons, then FC1 for the
//                            neurons of that very mask word that came out active
//   k_down_mask              FC2 over the active set, each workgroup deriving the ascending
//                            list from the mask words itself
// A workgroup that has just balloted its own 64 predictions does not need anyone else's to
// run FC1 on them, so predictor output layer and FC1 share a launch -- the closest this
// design comes to the paper's "every thread block checks its own neurons" (Sec. 5.4) -- and
// FC1 results are stored by neuron id (h[b][i]).  The compaction moves into the FC2 kernel:
// popcount prefix of the mask words in LDS, then every lane finds the neuron of its list
// slot by binary search.  One kernel boundary, one launch ramp and one trip through memory
// for the index list are saved per layer.
#pragma once
#include "dev_util.h"
#include "k_predict.h"
#include "k_sparse.h"

namespace pf {

constexpr int kOutUpThreads = 1024;
constexpr int kOutUpWaves = kOutUpThreads / kWave;

// LDS floats of the fused kernel: staged hidden vector and staged layer input, each with scrap.
inline size_t out_up_lds_bytes(int B, int r, int d)
{
    const size_t rpad = (size_t)((r + kChunk - 1) / kChunk) * kChunk;
    const size_t dpad = (size_t)((d + kChunk - 1) / kChunk) * kChunk;
    return ((size_t)B * rpad + kStageScrap + (size_t)B * dpad + kStageScrap) * sizeof(float);
}

// grid = ffn / 64, block = 1024 (16 waves).  Wave w computes the logits of neurons
// 64g + 4w .. 4w+3; wave 0 ballots the word; then wave a takes the a-th set bit of the word
// (a, a+16, ... if more than 16 are set) and computes that neuron's FC1 output.
template <int B, int ACT>
__global__ __launch_bounds__(kOutUpThreads) void k_pred_out_up(
    const __half *__restrict__ p2, const float *__restrict__ p_bias, const float *__restrict__ t,
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const float *__restrict__ x, int r, int d, int ffn,
    float thr_logit, uint64_t *__restrict__ mask_words, float *__restrict__ h)
{
    extern __shared__ float lds[];
    __shared__ float logit_s[B][64];
    __shared__ uint64_t word_s;
    constexpr int UP = (B <= 2) ? 4 : 2;  // predictor chunks in flight per row
    constexpr int R = 64 / kOutUpWaves;   // predictor rows per wave
    constexpr int U = 8;                  // FC1 chunks in flight per row
    constexpr bool GATED = (ACT == 1);
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int nchr = (r + kChunk - 1) / kChunk, rpad = nchr * kChunk;
    const int nchd = (d + kChunk - 1) / kChunk, dpad = nchd * kChunk;
    float *ts = lds;
    float *xs = lds + (size_t)B * rpad + kStageScrap;
    const int n0 = blockIdx.x * 64 + wave * R;

    PF_TSTAMP(4, 0);
    // activations first (they land first), then this wave's four predictor rows
    Staged<B, 1> st_t, st_x;
    stage_issue<B, 1>(st_t, t, r);
    stage_issue<B, 1>(st_x, x, d);
    rsrc_t rows[R];
#pragma unroll
    for (int q = 0; q < R; ++q) rows[q] = row_rsrc(p2, n0 + q, r, true);
#ifndef PF_FUSED_PRE
#define PF_FUSED_PRE 0  // predictor rows whose loads are issued before the block barrier
#endif
    WGroup<UP> g[R];
#pragma unroll
    for (int q = 0; q < PF_FUSED_PRE; ++q) load_group<UP>(g[q], rows[q], 0, lane);
    stage_commit<B, 1>(st_t, ts, t, r, rpad);
    stage_commit<B, 1>(st_x, xs, x, d, dpad);
    __syncthreads();
#pragma unroll
    for (int q = PF_FUSED_PRE; q < R; ++q) load_group<UP>(g[q], rows[q], 0, lane);
    PF_TSTAMP(4, 1);

    {
        float acc[R][B];
#pragma unroll
        for (int q = 0; q < R; ++q) {
#pragma unroll
            for (int b = 0; b < B; ++b) acc[q][b] = 0.f;
            fma_group<B, UP>(g[q], ts, rpad, 0, nchr, lane, acc[q]);
        }
        for (int it0 = UP; it0 < nchr; it0 += UP) {
#pragma unroll
            for (int q = 0; q < R; ++q) load_group<UP>(g[q], rows[q], it0, lane);
#pragma unroll
            for (int q = 0; q < R; ++q) fma_group<B, UP>(g[q], ts, rpad, it0, nchr, lane, acc[q]);
        }
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const float pb = p_bias ? p_bias[n0 + q] : 0.f;
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const float s = wave_sum(acc[q][b]) + pb;
                if (lane == 0) logit_s[b][wave * R + q] = s;
            }
        }
    }
    __syncthreads();
    if (wave == 0) {
        bool on = false;
#pragma unroll
        for (int b = 0; b < B; ++b) on = on || (logit_s[b][lane] > thr_logit);
        const uint64_t word = __ballot(on);
        if (lane == 0) {
            mask_words[blockIdx.x] = word;
            word_s = word;
        }
    }
    __syncthreads();

    PF_TSTAMP(4, 2);
    // FC1 for the set bits of this block's own word
    const uint64_t word = word_s;
    const int nact = __popcll(word);
    const uint64_t below = word & ((1ull << lane) - 1ull);
    const bool mybit = (word >> lane) & 1ull;
    const int myrank = __popcll(below);
    for (int a = wave; a < nact; a += kOutUpWaves) {  // wave-uniform
        const int pos = (int)__builtin_ctzll(__ballot(mybit && myrank == a));
        const int i = blockIdx.x * 64 + pos;
        const rsrc_t ru = row_rsrc(w_up, i, d, true);
        const rsrc_t rg = row_rsrc(GATED ? w_gate : w_up, i, d, true);
        float au[B], ag[B];
#pragma unroll
        for (int b = 0; b < B; ++b) au[b] = ag[b] = 0.f;
        for (int it0 = 0; it0 < nchd; it0 += U) {
            WGroup<U> gu, gg;
            load_group<U>(gu, ru, it0, lane);
            if (GATED) load_group<U>(gg, rg, it0, lane);
            fma_group<B, U>(gu, xs, dpad, it0, nchd, lane, au);
            if (GATED) fma_group<B, U>(gg, xs, dpad, it0, nchd, lane, ag);
        }
        const float bias = b_up ? b_up[i] : 0.f;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float v;
            if (GATED) {
                const float gsum = wave_sum(ag[b]) + bias;
                const float usum = wave_sum(au[b]);
                v = fmaxf(gsum, 0.f) * usum;
            } else {
                v = fmaxf(wave_sum(au[b]) + bias, 0.f);
            }
            if (lane == 0) h[(size_t)b * ffn + i] = v;
        }
    }
    PF_TSTAMP(4, 3);
}

// LDS of the FC2 kernel beyond its reduction buffer: mask words and their popcount prefix.
inline size_t down_mask_lds_bytes(int ffn)
{
    const size_t nwords = (size_t)ffn / 64;
    return nwords * sizeof(uint64_t) + (nwords + 1) * sizeof(uint32_t) + 64;
}

// Neuron ids of U list slots per lane (slot j[u], or -1 when j[u] >= total): binary search of
// the prefix for the word, then of the word for the bit.  The U searches advance in
// lockstep so that their LDS reads overlap instead of queueing one behind the other.
template <int U>
__device__ __forceinline__ void select_set_bits_lane(const uint64_t *words_lds,
                                                     const uint32_t *pre_lds, int nwords,
                                                     int top_step, int total, const int (&j)[U],
                                                     int (&out)[U])
{
    int lo[U];
#pragma unroll
    for (int u = 0; u < U; ++u) lo[u] = 0;
    for (int step = top_step; step >= 1; step >>= 1) {
        uint32_t p[U];
#pragma unroll
        for (int u = 0; u < U; ++u) p[u] = pre_lds[min(lo[u] + step, nwords)];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (lo[u] + step < nwords && p[u] <= (uint32_t)j[u]) lo[u] += step;
    }
    uint64_t w[U];
    uint32_t rank[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        w[u] = words_lds[lo[u]];
        rank[u] = (uint32_t)j[u] - pre_lds[lo[u]];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int pos = 0;
#pragma unroll
        for (int width = 32; width >= 1; width >>= 1) {
            const uint32_t c = (uint32_t)__popcll(w[u] & ((1ull << width) - 1ull));
            if (rank[u] >= c) {  // the bit lies in the upper half
                rank[u] -= c;
                w[u] >>= width;
                pos += width;
            }
        }
        out[u] = j[u] < total ? lo[u] * 64 + pos : -1;
    }
}

// FC2 over the active set given as mask words; h is indexed by neuron id.  Same tiling as
// k_down (16 columns per block, the whole list per block, XCD-aware tile numbering).
// Block 0 also writes the ascending index list and the count for the caller.
template <int B>
__global__ __launch_bounds__(kDownThreads) void k_down_mask(
    const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const uint64_t *__restrict__ mask_words,
    int32_t *__restrict__ idx_out, int32_t *__restrict__ count_out, float *__restrict__ y, int d,
    int ffn, int ntiles)
{
    constexpr int U = (B <= 2) ? PF_DOWN_U : 4;
    constexpr int STEP = kDownRowsPerLoad * U;
    extern __shared__ uint64_t dyn_lds64[];
    __shared__ float red[kDownWaves][B][kDownCols];
    __shared__ uint32_t wave_tot[kDownWaves];
    const int per_xcd = (ntiles + 7) >> 3;
    const int tile = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (tile >= ntiles) return;  // uniform over the block
    const int nwords = ffn / 64;
    uint64_t *words_lds = dyn_lds64;
    uint32_t *pre_lds = reinterpret_cast<uint32_t *>(words_lds + nwords);
    PF_TSTAMP(5, 0);
    const int n = (int)mask_prefix<kDownThreads>(mask_words, nwords, words_lds, pre_lds, wave_tot);
    if (blockIdx.x == 0 && threadIdx.x == 0) *count_out = n;
    PF_TSTAMP(5, 1);
    int top_step = 1;
    while (top_step * 2 < nwords) top_step *= 2;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5;
    const int rlane = wave * 32 + (lane & 31);
    const int col = tile * kDownCols + half * 8;
    const bool colok = col < d;
    const rsrc_t wd = make_rsrc(w_down, (uint32_t)ffn * (uint32_t)d * 2u);
    const rsrc_t hr = make_rsrc(h, (uint32_t)B * (uint32_t)ffn * 4u);

    float acc[B][8];
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;

    for (int j0 = 0; j0 < n; j0 += STEP) {
        uint4 w[U];
        float hv[U][B];
        int iv[U];
        int jj[U];
#pragma unroll
        for (int u = 0; u < U; ++u) jj[u] = j0 + u * kDownRowsPerLoad + rlane;
        select_set_bits_lane<U>(words_lds, pre_lds, nwords, top_step, n, jj, iv);
        PF_TSTAMP(5, 2);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = iv[u] >= 0;
            w[u] = ld16_stream(wd, (ok && colok) ? ((uint32_t)iv[u] * (uint32_t)d + (uint32_t)col) * 2u
                                                 : kOobOffset);
#pragma unroll
            for (int b = 0; b < B; ++b)
                hv[u][b] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                    hr, ok ? (int)(((uint32_t)b * (uint32_t)ffn + (uint32_t)iv[u]) * 4u) : (int)kOobOffset, 0, 0));
            if (blockIdx.x == 0 && half == 0 && ok) idx_out[j0 + u * kDownRowsPerLoad + rlane] = iv[u];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float f0 = h_lo(w[u].x), f1 = h_hi(w[u].x), f2 = h_lo(w[u].y), f3 = h_hi(w[u].y);
            const float f4 = h_lo(w[u].z), f5 = h_hi(w[u].z), f6 = h_lo(w[u].w), f7 = h_hi(w[u].w);
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const float s = hv[u][b];
                acc[b][0] = fmaf(s, f0, acc[b][0]);
                acc[b][1] = fmaf(s, f1, acc[b][1]);
                acc[b][2] = fmaf(s, f2, acc[b][2]);
                acc[b][3] = fmaf(s, f3, acc[b][3]);
                acc[b][4] = fmaf(s, f4, acc[b][4]);
                acc[b][5] = fmaf(s, f5, acc[b][5]);
                acc[b][6] = fmaf(s, f6, acc[b][6]);
                acc[b][7] = fmaf(s, f7, acc[b][7]);
            }
        }
    }

#pragma unroll
    for (int b = 0; b < B; ++b) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[b][e];
            v += dpp_f32<0xB1>(v);
            v += dpp_f32<0x4E>(v);
            v += dpp_f32<0x141>(v);
            v += dpp_f32<0x140>(v);
            v += __shfl_xor(v, 16, 64);
            if ((lane & 31) == 0) red[wave][b][half * 8 + e] = v;
        }
    }
    __syncthreads();
    if (threadIdx.x < B * kDownCols) {
        const int b = threadIdx.x / kDownCols, c = threadIdx.x % kDownCols;
        const int oc = tile * kDownCols + c;
        if (oc < d) {
            float s = b_down ? b_down[oc] : 0.f;
#pragma unroll
            for (int wv = 0; wv < kDownWaves; ++wv) s += red[wv][b][c];
            y[(size_t)b * d + oc] = s;
        }
    }
    PF_TSTAMP(5, 3);
}

}  // namespace pf
