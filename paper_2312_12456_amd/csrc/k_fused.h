// The layer step as three launches instead of four (PowerInfer Sec. 5.1 + 5.4):
//   k_pred_hidden   t = ReLU(p1 . x)                                            (k_predict.h)
//   k_out_up        logits, threshold and ballot for 64 neurons, then FC1 for those of the 64
//                   that came out active
//   k_down2m        FC2 over the active neurons, segment by segment
// A workgroup that has just balloted its own 64 predictions needs nobody else's to run FC1 on
// them -- the paper's "every thread block checks its own neurons" (Sec. 5.4) applied where it
// costs nothing: the block is there anyway, for the predictor.  No global index list is built.
// Block g of k_out_up leaves a SEGMENT: seg_words[g] = its 64 decisions as a bit word,
// a byte table with the positions (0 .. 63) of its active neurons, h[64 g + a][token] = the
// FC1 output of its a-th active neuron.  FC2 deals whole segments to its waves.  One kernel
// boundary, one launch ramp, the mask scan and the trip of the index list through memory are
// saved per layer.
// Work per workgroup follows the number of active neurons per segment (see seg_neuron for
// the two ways of forming segments).  The bit words are internal; the caller-visible mask
// format is produced by k_pred_out only.
#pragma once
#include "dev_util.h"
#include "k_predict.h"
#include "k_sparse.h"

namespace pf {

// LDS bytes of k_out_up: staged hidden vector [B][rpad] and staged layer input [B][dpad].
inline size_t out_up_lds_bytes(int B, int r, int d)
{
    const size_t rpad = (size_t)((r + kChunk - 1) / kChunk) * kChunk;
    const size_t dpad = (size_t)((d + kChunk - 1) / kChunk) * kChunk;
    return (size_t)B * (rpad + dpad) * sizeof(float);
}

// Neuron at position p (0 .. 63) of segment g when there are G segments.  Contiguous
// (64 g + p) keeps a segment's weight rows within a few pages, which is worth 3 - 6 % of a
// decode step; strided (p G + g) spreads neighbouring hot neurons over all segments and is
// meant for models stored hot-first, where contiguous segments would leave FC1 to a few
// workgroups.
__device__ __forceinline__ int seg_neuron(int p, int g, int G, bool strided)
{
    return strided ? p * G + g : g * 64 + p;
}

// Byte of a segment's position table that holds entry a (the a-th active neuron of the
// segment): entries a, a + 8, a + 16, a + 24 share a dword, so that row slot a % 8 of an FC2
// wave gets the positions of its first four rounds with one 4-byte load.
__host__ __device__ constexpr int seg_pos_byte(int a)
{
    return (a >= 32 ? 32 : 0) + (a & 7) * 4 + ((a >> 3) & 3);
}

// grid = ffn / 64, block = 1024 (16 waves).  Wave w computes the logits of the block's
// neurons number 4 w .. 4 w + 3; every wave then ballots the word for itself and takes the set
// bits number w, w + 16, ... of it.
template <int B, int ACT>
__global__ __launch_bounds__(kPredOutThreads) void k_out_up(
    const __half *__restrict__ p2, const float *__restrict__ p_bias, const float *__restrict__ t,
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const float *__restrict__ x, int r, int d, int ffn, int hs,
    float thr_logit, bool strided, uint64_t *__restrict__ seg_words,
    uint8_t *__restrict__ seg_pos, float *__restrict__ h, float up_floor, int always_on)
{
    extern __shared__ float ts[];  // [B][rpad] hidden vector, then [B][dpad] layer input
    static_assert(kPredOutNeurons == 64, "one mask word per block");
    __shared__ float logit_s[B][64];
    constexpr int NW = kPredOutThreads / kWave;
    constexpr int UP = (B <= 2) ? 4 : 2, R = 64 / NW;
    constexpr int U = 8;
    constexpr bool GATED = (ACT == 1);
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int nchr = (r + kChunk - 1) / kChunk, rpad = nchr * kChunk;
    const int nchd = (d + kChunk - 1) / kChunk, dpad = nchd * kChunk;
    float *xs = ts + (size_t)B * rpad;
    const int G = gridDim.x, g0 = blockIdx.x;
    rsrc_t rows[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {  // neurons below always_on are taken without reading their rows
        const int nq = seg_neuron(wave * R + q, g0, G, strided);
        rows[q] = row_rsrc(p2, nq, r, nq >= always_on);
    }

    PF_TSTAMP(4, 0);
    // a segment of the always-on prefix: no predictor rows are read, every neuron is taken
    const bool all_on = !strided && g0 * 64 + 63 < always_on;  // uniform over the block
    if (all_on) {
        stage_dma<B>(xs, x, d, dpad);
        __syncthreads();
    } else {
    stage_dma<B>(ts, t, r, rpad);
    constexpr int PRE = 2;  // rows whose loads are issued before the block barrier
    WGroup<UP> g[R];
#pragma unroll
    for (int q = 0; q < PRE; ++q) load_group<UP>(g[q], rows[q], 0, lane);
    __syncthreads();
    // the layer input is not needed before the second barrier: fetched behind the first
    stage_dma<B>(xs, x, d, dpad);
#pragma unroll
    for (int q = PRE; q < R; ++q) load_group<UP>(g[q], rows[q], 0, lane);
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
            const float pb = p_bias ? p_bias[seg_neuron(wave * R + q, g0, G, strided)] : 0.f;
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const float s = wave_sum(acc[q][b]) + pb;
                if (lane == 0) logit_s[b][wave * R + q] = s;
            }
        }
    }
    __syncthreads();
    }
    PF_TSTAMP(4, 2);

    bool on = seg_neuron(lane, g0, G, strided) < always_on;
    if (!all_on) {
#pragma unroll
        for (int b = 0; b < B; ++b) on = on || (logit_s[b][lane] > thr_logit);
    }
    const uint64_t word = __ballot(on);
    const int myrank = __popcll(word & ((1ull << lane) - 1ull));
    if (wave == 0) {
        if (lane == 0) seg_words[blockIdx.x] = word;
        if (on) seg_pos[blockIdx.x * 64 + seg_pos_byte(myrank)] = (uint8_t)lane;
    }
    const int nact = __popcll(word);
    int a = wave;
    if (a >= nact) {  // wave-uniform; no block-level synchronisation below
        PF_TSTAMP_MAX(4, 5);
        return;
    }

    // position of set bit number `a` of the word (wave-uniform)
    auto neuron_of = [&](int rank) -> int {
        const uint64_t hit = __ballot(on && myrank == rank);
        return seg_neuron((int)__builtin_ctzll(hit), g0, G, strided);
    };
    int i = wave_uniform(neuron_of(a));
    rsrc_t ru = row_rsrc(w_up, i, d, true), rg = row_rsrc(GATED ? w_gate : w_up, i, d, true);
    WGroup<U> gu, gg;
    load_group<U>(gu, ru, 0, lane);
    if (GATED) load_group<U>(gg, rg, 0, lane);
    PF_TSTAMP(4, 3);
    while (true) {
        float au[B], ag[B];
#pragma unroll
        for (int b = 0; b < B; ++b) au[b] = ag[b] = 0.f;
        fma_group<B, U>(gu, xs, dpad, 0, nchd, lane, au);
        if (GATED) fma_group<B, U>(gg, xs, dpad, 0, nchd, lane, ag);
        for (int it0 = U; it0 < nchd; it0 += U) {
            load_group<U>(gu, ru, it0, lane);
            if (GATED) load_group<U>(gg, rg, it0, lane);
            fma_group<B, U>(gu, xs, dpad, it0, nchd, lane, au);
            if (GATED) fma_group<B, U>(gg, xs, dpad, it0, nchd, lane, ag);
        }
        const int icur = i, acur = a;
        a += NW;
        const bool more = a < nact;
        if (more) {  // next row in flight before this row's reductions
            i = wave_uniform(neuron_of(a));
            ru = row_rsrc(w_up, i, d, true);
            rg = row_rsrc(GATED ? w_gate : w_up, i, d, true);
            load_group<U>(gu, ru, 0, lane);
            if (GATED) load_group<U>(gg, rg, 0, lane);
        }
        const float bias = b_up != nullptr ? b_up[icur] : 0.f;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float v;
            if (GATED) {
                const float gsum = wave_sum(ag[b]) + bias;
                const float usum = wave_sum(au[b]);
                v = fmaxf(gsum, 0.f) * fmaxf(usum, up_floor);
            } else {
                v = fmaxf(wave_sum(au[b]) + bias, 0.f);
            }
            if (lane == 0) h[((size_t)blockIdx.x * 64 + acur) * hs + b] = v;
        }
        if (!more) break;
    }
    PF_TSTAMP(4, 4);
    PF_TSTAMP_MAX(4, 5);
}

// FC2 over the segments k_out_up leaves (popcount(seg_words[w]) valid entries in segment w:
// seg_pos[64 w + seg_pos_byte(a)] = position p of entry a, neuron id = p * nwords + w;
// h[64 w + a] = its FC1 output).  Tiling of k_down2 (64 columns x one of P row groups per
// workgroup, P partial sums left for the consumer), but whole SEGMENTS are dealt to the waves:
// segment (8 j + wave) P + g is wave `wave`'s j-th, and its 8 row slots take entries
// s, s + 8, ... of it.  Words come through the scalar unit, so which rounds a segment needs
// is a scalar branch; positions and FC1 outputs of a round are 4-byte loads issued together
// with nothing between them and the weight rows but one trip to memory.
// Segments of a wave that k_down2m keeps in flight together.
constexpr __host__ __device__ int down2m_batch(int B) { return B <= 2 ? 8 : 4; }

// MULTI: a wave has more than one batch of segments; the next batch's words, positions and
// FC1 outputs are then requested behind the current batch's rows.
template <int B, bool MULTI>
__global__ __launch_bounds__(kDown2Threads) void k_down2m(
    const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const uint64_t *__restrict__ seg_words,
    const uint8_t *__restrict__ seg_pos, float *__restrict__ part, int d, int ffn, bool strided)
{
    constexpr int S = down2m_batch(B);
    constexpr int HS = h_stride(B);
    __shared__ float red[kDown2Waves][B][kDown2Cols];
    const int P = gridDim.y, g = blockIdx.y, tile = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int cl = lane & 7;   // which 16 bytes of the row's 128-byte line
    const int sl = lane >> 3;  // row slot of this lane inside the wave
    const int col = tile * kDown2Cols + cl * 8;
    const bool colok = col < d;
    const int nwords = ffn / 64;
    const rsrc_t wd = make_rsrc(w_down, (uint32_t)ffn * (uint32_t)d * 2u);
    const rsrc_t pr = make_rsrc(seg_pos, (uint32_t)ffn);
    const rsrc_t hr = make_rsrc(h, (uint32_t)ffn * (uint32_t)HS * 4u);

    PF_TSTAMP(5, 0);
    constexpr int BP = B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : 8;
    float acc[BP * 8];
#pragma unroll
    for (int f = 0; f < BP * 8; ++f) acc[f] = 0.f;

    auto load_h = [&](int slot, float (&hv)[B]) {  // the HS floats of one slot
        float t[HS];
        if (HS == 1) {
            t[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(hr, slot * 4, 0, 0));
        } else if (HS == 2) {
            typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
            const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(hr, slot * 8, 0, 0);
            t[0] = __uint_as_float(v.x);
            t[HS > 1 ? 1 : 0] = __uint_as_float(v.y);
        } else {
#pragma unroll
            for (int k = 0; k < HS / 4; ++k) {
                const float4 v = ld16_f32(hr, (uint32_t)(slot * HS + 4 * k) * 4u);
                t[(4 * k) % HS] = v.x;
                t[(4 * k + 1) % HS] = v.y;
                t[(4 * k + 2) % HS] = v.z;
                t[(4 * k + 3) % HS] = v.w;
            }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) hv[b] = t[b];
    };
    auto load_row = [&](uint32_t posbyte, int w, bool ok) -> uint4 {
        const uint32_t id = (uint32_t)seg_neuron((int)posbyte, w, nwords, strided);
        return ld16_stream(wd, (ok && colok) ? (id * (uint32_t)d + (uint32_t)col) * 2u : kOobOffset);
    };
    auto fma_row = [&](const uint4 &wt, const float (&hv)[B], bool ok) {
        const float f0 = h_lo(wt.x), f1 = h_hi(wt.x), f2 = h_lo(wt.y), f3 = h_hi(wt.y);
        const float f4 = h_lo(wt.z), f5 = h_hi(wt.z), f6 = h_lo(wt.w), f7 = h_hi(wt.w);
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float s = ok ? hv[b] : 0.f;  // slots past the count hold stale values
            acc[8 * b + 0] = fmaf(s, f0, acc[8 * b + 0]);
            acc[8 * b + 1] = fmaf(s, f1, acc[8 * b + 1]);
            acc[8 * b + 2] = fmaf(s, f2, acc[8 * b + 2]);
            acc[8 * b + 3] = fmaf(s, f3, acc[8 * b + 3]);
            acc[8 * b + 4] = fmaf(s, f4, acc[8 * b + 4]);
            acc[8 * b + 5] = fmaf(s, f5, acc[8 * b + 5]);
            acc[8 * b + 6] = fmaf(s, f6, acc[8 * b + 6]);
            acc[8 * b + 7] = fmaf(s, f7, acc[8 * b + 7]);
        }
    };

    const int nj = (nwords + 8 * P - 1) / (8 * P);  // segments per wave (uniform over the grid)
    const int nbatch = (nj + S - 1) / S;
    const int sb = (nj + nbatch - 1) / nbatch;      // segments per batch, evened out (<= S)
    // words (through the scalar unit), positions and first-round FC1 outputs of a batch
    auto fetch_meta = [&](int j0, int (&wseg)[S], int (&cnt)[S], uint32_t (&pos)[S], float (&h0)[S][B]) {
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const int w = ((j0 + u) * 8 + wave) * P + g;
            wseg[u] = min(w, nwords - 1);
            const uint64_t word = seg_words[wseg[u]];
            const int c = __popc(__builtin_amdgcn_readfirstlane((int)(uint32_t)word)) +
                          __popc(__builtin_amdgcn_readfirstlane((int)(uint32_t)(word >> 32)));
            cnt[u] = (w < nwords && u < sb && j0 + u < nj) ? c : 0;
        }
#pragma unroll
        for (int u = 0; u < S; ++u) {
            pos[u] = __builtin_amdgcn_raw_buffer_load_b32(pr, wseg[u] * 64 + sl * 4, 0, 0);
            load_h(wseg[u] * 64 + sl, h0[u]);
        }
    };
    int wseg[S], cnt[S];  // scalar registers
    uint32_t pos[S];
    float h0[S][B];
    fetch_meta(0, wseg, cnt, pos, h0);
    PF_TSTAMP(5, 1);
    for (int j0 = 0; j0 < nj; j0 += sb) {
        float h1[S][B];
        uint4 r0[S], r1[S];
#pragma unroll
        for (int u = 0; u < S; ++u) r0[u] = load_row(pos[u] & 0xffu, wseg[u], sl < cnt[u]);
#pragma unroll
        for (int u = 0; u < S; ++u)
            if (cnt[u] > 8) {  // scalar
                r1[u] = load_row((pos[u] >> 8) & 0xffu, wseg[u], 8 + sl < cnt[u]);
                load_h(wseg[u] * 64 + 8 + sl, h1[u]);
            }
        int wsegn[S], cntn[S];
        uint32_t posn[S];
        float h0n[S][B];
        // (past the last batch the indices are clamped and the counts zero: no branch, so the
        // compiler keeps exact counts of the loads in flight)
        if constexpr (MULTI) fetch_meta(j0 + sb, wsegn, cntn, posn, h0n);
#pragma unroll
        for (int u = 0; u < S; ++u) fma_row(r0[u], h0[u], sl < cnt[u]);
#pragma unroll
        for (int u = 0; u < S; ++u)
            if (cnt[u] > 8) fma_row(r1[u], h1[u], 8 + sl < cnt[u]);
        // further rounds (more than 16 active neurons in a segment), one round at a time
        int maxc = 0;
#pragma unroll
        for (int u = 0; u < S; ++u) maxc = max(maxc, cnt[u]);
        for (int r = 2; 8 * r < maxc; ++r) {
#pragma unroll
            for (int u = 0; u < S; ++u)
                if (cnt[u] > 8 * r) {
                    if (r == 4)
                        pos[u] = __builtin_amdgcn_raw_buffer_load_b32(pr, wseg[u] * 64 + 32 + sl * 4, 0, 0);
                    r0[u] = load_row((pos[u] >> (8 * (r & 3))) & 0xffu, wseg[u], 8 * r + sl < cnt[u]);
                    load_h(wseg[u] * 64 + 8 * r + sl, h0[u]);
                }
#pragma unroll
            for (int u = 0; u < S; ++u)
                if (cnt[u] > 8 * r) fma_row(r0[u], h0[u], 8 * r + sl < cnt[u]);
        }
        if (j0 == 0) PF_TSTAMP(5, 2);
        if constexpr (MULTI) {
#pragma unroll
            for (int u = 0; u < S; ++u) {
                wseg[u] = wsegn[u];
                cnt[u] = cntn[u];
                pos[u] = posn[u];
#pragma unroll
                for (int b = 0; b < B; ++b) h0[u][b] = h0n[u][b];
            }
        }
    }
    PF_TSTAMP(5, 3);

    butterfly_halve<32, BP * 4>(acc, lane);
    butterfly_halve<16, BP * 2>(acc, lane);
    butterfly_halve<8, BP>(acc, lane);
    {
        const int slot = ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
#pragma unroll
        for (int k = 0; k < BP; ++k) {
            const int f = BP * slot + k, b = f >> 3, e = f & 7;
            if (b < B) red[wave][b][cl * 8 + e] = acc[k];
        }
    }
    __syncthreads();
    if (threadIdx.x < B * kDown2Cols) {
        const int b = threadIdx.x / kDown2Cols, c = threadIdx.x % kDown2Cols;
        const int oc = tile * kDown2Cols + c;
        if (oc < d) {
            float s = (g == 0 && b_down) ? b_down[oc] : 0.f;
#pragma unroll
            for (int wv = 0; wv < kDown2Waves; ++wv) s += red[wv][b][c];
            part[((size_t)g * B + b) * d + oc] = s;
        }
    }
    PF_TSTAMP(5, 4);
}

}  // namespace pf
