// Activation predictor (PowerInfer Sec. 5.1: input layer, one hidden layer, output layer)
// and active-index compaction.
//   hidden : t[b][m]     = ReLU(p1[m] . x[b])                          r rows of d fp16
//   output : logit[b][i] = p2[i] . t[b] + p_bias[i]                     ffn rows of r fp16
//            bit i of the mask = any_b(logit[b][i] > logit(threshold))  (wave ballot)
//   compact: idx[] = ascending positions of the set bits, count = popcount
// Both GEMVs are HBM-bound streams of fp16 rows: one wave per row, 16-byte loads per
// lane, activations staged once per workgroup in LDS, fp32 accumulation, DPP reduction.
// No kernel here uses device-scope fences: data crosses workgroups only at kernel ends.
#pragma once
#include "dev_util.h"

namespace pf {

constexpr int kPredThreads = 256;  // 4 waves per workgroup
constexpr int kGlueMaxParts = 4;   // FC2 may hand its output over as up to 4 partial sums
constexpr int kPredWaves = kPredThreads / kWave;

// ---------------------------------------------------------------------------------------
// One pass of the stack glue inside a consumer kernel: S strides of NT * 4 elements of
// v = sign * (x_prev + sum of FC2's partial sums), for B tokens.  glue_issue puts the loads in
// flight (x and up to kGlueMaxParts partial sums per element, partials added in the fixed
// order 0 .. ny-1), glue_commit adds them up, accumulates ||v||^2 per token into ss and
// stores v in the staged-activation layout of dev_util.h (scrap slot for strides past the
// vector).  The caller reduces ss over the block and applies sqrt(d / ss) to its dot products.
template <int B, int S>
struct GluePass {
    float4 va[S][B], vc[S][B], vp[S][B][kGlueMaxParts - 1];
};

template <int B, int S, int NT>
__device__ __forceinline__ void glue_issue(GluePass<B, S> &gp, rsrc_t xr, rsrc_t yr, uint32_t pbytes,
                                           int ny, int d, int e0)
{
    constexpr int step = NT * 4;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int e = e0 + s * step;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const uint32_t off = e < d ? (uint32_t)(b * d + e) * 4u : kOobOffset;
            gp.va[s][b] = ld16_f32(xr, off);
            gp.vc[s][b] = ld16_f32(yr, off);
#pragma unroll
            for (int p = 1; p < kGlueMaxParts; ++p)  // partial sums of FC2, in order
                gp.vp[s][b][p - 1] = ld16_f32(yr, (e < d && p < ny) ? off + (uint32_t)p * pbytes : kOobOffset);
        }
    }
}

template <int B, int S, int NT>
__device__ __forceinline__ void glue_commit(const GluePass<B, S> &gp, float *__restrict__ xs, int kpad,
                                            int b0, int e0, float (&ss)[B])
{
    constexpr int step = NT * 4;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int e = e0 + s * step;
#pragma unroll
        for (int b = 0; b < B; ++b) {  // strides past the vector hold zeros: scrap slot
            const float4 a = gp.va[s][b];
            float4 c = gp.vc[s][b];
#pragma unroll
            for (int p = 1; p < kGlueMaxParts; ++p) {
                const float4 q = gp.vp[s][b][p - 1];
                c = make_float4(c.x + q.x, c.y + q.y, c.z + q.z, c.w + q.w);
            }
            const float4 v = glue_signed(make_float4(a.x + c.x, a.y + c.y, a.z + c.z, a.w + c.w),
                                         (uint32_t)b0 + (uint32_t)b, (uint32_t)e);
            ss[b] = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss[b]))));
            *reinterpret_cast<float4 *>(xs + (e < kpad ? b * kpad + lds_slot(e) : B * kpad)) = v;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Hidden layer.  grid = ceil(r / 4); wave w of block g owns row 4g + w.
// With GLUE the input of the layer is formed on the fly from the previous layer's input and
// FFN output, x = (xp + yp) * sqrt(d) / ||xp + yp||_2 per token (the stack's residual +
// scale-only RMS norm): every block stages v = xp + yp, reduces ||v||^2 itself and applies
// the scale to its dot products; block 0 also writes x for the kernels that follow.
// yp may arrive as ny <= 4 partial sums, ypstride floats apart (row-split FC2): they are
// added in the fixed order 0 .. ny-1.  b0 = batch row of the first token this launch handles
// (the glue's sign pattern depends on the row).
// GS = strides of 1024 elements whose glue loads (x and up to 4 partial sums each) a thread
// issues together: 4 covers d <= 4096 in a single round trip, at 80 registers.
// The body takes the block's number explicitly (bid) so that a launch can run it in a range of
// its blocks beside another role; write_x: this block also writes x for the kernels that follow.
// NT = threads of the launch (a block owns NT / 64 rows).
template <int B, bool GLUE, int GS, int NT = kPredThreads>
__device__ __forceinline__ void pred_hidden_body(float *xs, float (*ss_w)[B], const int bid, const bool write_x,
                                                 const __half *__restrict__ p1,
                                                 const float *__restrict__ x,
                                                 const float *__restrict__ yp, int ny,
                                                 int ypstride, float *__restrict__ x_new,
                                                 float *__restrict__ t, int d, int r, int b0)
{
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int nch = (d + kChunk - 1) / kChunk, kpad = nch * kChunk;
    const int m = bid * (NT / kWave) + wave;
    const bool live = m < r;
    const rsrc_t row = row_rsrc(p1, live ? m : 0, d, live);

    PF_TSTAMP(0, 0);
    if (!GLUE) stage_dma<B>(xs, x, d, kpad);
    WGroup<U> g;
    float scale[B];
    if (GLUE) {
        float ss[B];
#pragma unroll
        for (int b = 0; b < B; ++b) ss[b] = 0.f;
        constexpr int S = GS;  // strides whose loads are issued together
        constexpr int step = NT * 4;
        bool issued = false;
        const rsrc_t xr = make_rsrc(x, (uint32_t)B * (uint32_t)d * 4u);
        const uint32_t pbytes = (uint32_t)ypstride * 4u;  // distance between partials
        const rsrc_t yr = make_rsrc(yp, (uint32_t)(ny - 1) * pbytes + (uint32_t)B * (uint32_t)d * 4u);
        for (int e0 = threadIdx.x * 4; e0 < kpad; e0 += step * S) {
            GluePass<B, S> gp;
            glue_issue<B, S, NT>(gp, xr, yr, pbytes, ny, d, e0);
            // the row's own loads queue up behind the first pass of activations
            if (!issued) {
                load_group<U>(g, row, 0, lane);
                issued = true;
            }
            glue_commit<B, S, NT>(gp, xs, kpad, b0, e0, ss);
        }
        if (!issued) load_group<U>(g, row, 0, lane);  // threads past a short vector
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float s = wave_sum(ss[b]);
            if (lane == 0) ss_w[wave][b] = s;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float tot = 0.f;
#pragma unroll
            for (int k = 0; k < NT / kWave; ++k) tot += ss_w[k][b];
            scale[b] = tot > 0.f ? sqrtf((float)d / tot) : 0.f;
        }
        if (write_x) {
            for (int e = threadIdx.x * 4; e < d; e += NT * 4) {
#pragma unroll
                for (int b = 0; b < B; ++b) {
                    const float4 v = *reinterpret_cast<const float4 *>(xs + b * kpad + lds_slot(e));
                    *reinterpret_cast<float4 *>(x_new + (size_t)b * d + e) =
                        make_float4(v.x * scale[b], v.y * scale[b], v.z * scale[b], v.w * scale[b]);
                }
            }
        }
    } else {
        load_group<U>(g, row, 0, lane);
        __syncthreads();
#pragma unroll
        for (int b = 0; b < B; ++b) scale[b] = 1.f;
    }

    PF_TSTAMP(0, 1);
    float acc[B];
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = 0.f;
    fma_group<B, U>(g, xs, kpad, 0, nch, lane, acc);
    for (int it0 = U; it0 < nch; it0 += U) {
        load_group<U>(g, row, it0, lane);
        fma_group<B, U>(g, xs, kpad, it0, nch, lane, acc);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const float s = wave_sum(acc[b]) * scale[b];
        if (live && lane == 0) t[(size_t)b * r + m] = fmaxf(s, 0.f);
    }
    PF_TSTAMP(0, 2);
}

template <int B, bool GLUE, int GS = (B >= 2 ? 1 : 2)>
__global__ __launch_bounds__(kPredThreads) void k_pred_hidden(const __half *__restrict__ p1,
                                                              const float *__restrict__ x,
                                                              const float *__restrict__ yp, int ny,
                                                              int ypstride,
                                                              float *__restrict__ x_new,
                                                              float *__restrict__ t, int d, int r,
                                                              int b0, const int32_t *__restrict__ skip)
{
    extern __shared__ float xs[];
    __shared__ float ss_w[kPredWaves][B];
    // adaptive layer step: a set flag means this step runs dense and needs no prediction
    if (skip != nullptr && *skip != 0) return;
    pred_hidden_body<B, GLUE, GS>(xs, ss_w, (int)blockIdx.x, blockIdx.x == 0, p1, x, yp, ny, ypstride,
                                  x_new, t, d, r, b0);
}

// ---------------------------------------------------------------------------------------
// Output layer + threshold + ballot.  grid = (ffn - 64 first_word) / NB; block g owns the NB
// neurons from 64 first_word + NB*g on (NB = 16, 32 or 64: a quarter, half or whole mask word), wave w of it rows
// 4w .. 4w+3, all in flight at once; wave 0 turns the NB decisions into its piece of the
// mask word with a ballot.
constexpr int kPredOutNeurons = 64;
constexpr int kPredOutThreads = kPredOutNeurons * 16;
static_assert(kPredOutNeurons == 16 || kPredOutNeurons == 32 || kPredOutNeurons == 64, "mask piece");
template <int NB> struct MaskPiece { typedef uint64_t type; };
template <> struct MaskPiece<32> { typedef uint32_t type; };
template <> struct MaskPiece<16> { typedef uint16_t type; };

// Writes "always on" for the first `words` mask words (and score 1 for their neurons): the
// neurons of an always-on prefix are not evaluated by the predictor's output layer at all.
// Called by one workgroup of the output-layer kernels.
template <int B>
__device__ __forceinline__ void mark_always_on(int words, int ffn, float *__restrict__ scores,
                                               uint64_t *__restrict__ mask_words)
{
    for (int w = threadIdx.x; w < words; w += blockDim.x) mask_words[w] = ~0ull;
    if (scores != nullptr)
        for (int e = threadIdx.x; e < B * words * 64; e += blockDim.x)
            scores[(size_t)(e / (words * 64)) * ffn + e % (words * 64)] = 1.f;
}

// Body for a block of NB neurons (NB * 16 threads: 4 rows per wave); bid = which NB neurons.
// The launch covers the neurons from 64 * first_word on; its first block marks the words below.
template <int B, int NB>
__device__ __forceinline__ void pred_out_body(float *ts, float (*logit_s)[NB], const int bid0,
                                              const __half *__restrict__ p2,
                                              const float *__restrict__ p_bias,
                                              const float *__restrict__ t, int r, int ffn,
                                              float thr_logit, float *__restrict__ scores,
                                              uint64_t *__restrict__ mask_words, const int first_word)
{
    constexpr int NT = NB * 16;
    const int bid = bid0 + first_word * (64 / NB);
    if (bid0 == 0 && first_word > 0) mark_always_on<B>(first_word, ffn, scores, mask_words);
    // 16 waves per block leave 128 VGPRs per lane: fewer loads in flight at larger batch
    constexpr int U = (B <= 2) ? 4 : 2, R = NB / (NT / kWave);
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int nch = (r + kChunk - 1) / kChunk, kpad = nch * kChunk;
    const int n0 = bid * NB + wave * R;
    rsrc_t rows[R];
#pragma unroll
    for (int q = 0; q < R; ++q) rows[q] = row_rsrc(p2, n0 + q, r, true);

    PF_TSTAMP(1, 0);
    stage_dma<B>(ts, t, r, kpad);
    constexpr int PRE = 2;  // rows whose loads are issued before the block barrier
    WGroup<U> g[R];
#pragma unroll
    for (int q = 0; q < PRE; ++q) load_group<U>(g[q], rows[q], 0, lane);
    __syncthreads();
#pragma unroll
    for (int q = PRE; q < R; ++q) load_group<U>(g[q], rows[q], 0, lane);
    PF_TSTAMP(1, 1);

    float acc[R][B];
#pragma unroll
    for (int q = 0; q < R; ++q) {
#pragma unroll
        for (int b = 0; b < B; ++b) acc[q][b] = 0.f;
        fma_group<B, U>(g[q], ts, kpad, 0, nch, lane, acc[q]);
    }
    for (int it0 = U; it0 < nch; it0 += U) {
#pragma unroll
        for (int q = 0; q < R; ++q) load_group<U>(g[q], rows[q], it0, lane);
#pragma unroll
        for (int q = 0; q < R; ++q) fma_group<B, U>(g[q], ts, kpad, it0, nch, lane, acc[q]);
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
    __syncthreads();

    if (scores != nullptr) {
        for (int e = threadIdx.x; e < B * NB; e += NT) {
            const int b = e / NB, q = e % NB;
            scores[(size_t)b * ffn + bid * NB + q] = 1.f / (1.f + __expf(-logit_s[b][q]));
        }
    }
    if (wave == 0) {
        bool on = false;
#pragma unroll
        for (int b = 0; b < B; ++b) on = on || (lane < NB && logit_s[b][lane % NB] > thr_logit);
        const uint64_t word = __ballot(on);
        typedef typename MaskPiece<NB>::type piece_t;  // little endian: piece g of the words
        if (lane == 0) reinterpret_cast<piece_t *>(mask_words)[bid] = (piece_t)word;
    }
    PF_TSTAMP(1, 2);
}

template <int B>
__global__ __launch_bounds__(kPredOutThreads) void k_pred_out(
    const __half *__restrict__ p2, const float *__restrict__ p_bias, const float *__restrict__ t,
    int r, int ffn, float thr_logit, float *__restrict__ scores, uint64_t *__restrict__ mask_words,
    int first_word, const int32_t *__restrict__ skip)
{
    extern __shared__ float ts[];  // [B][kpad] staged hidden vector
    __shared__ float logit_s[B][kPredOutNeurons];
    // adaptive layer step: a set flag means this step runs dense -- every neuron is marked
    if (skip != nullptr && *skip != 0) {
        if (threadIdx.x == 0) mask_words[first_word + (int)blockIdx.x] = ~0ull;
        if (blockIdx.x == 0 && first_word > 0) mark_always_on<B>(first_word, ffn, nullptr, mask_words);
        return;
    }
    pred_out_body<B, kPredOutNeurons>(ts, logit_s, (int)blockIdx.x, p2, p_bias, t, r, ffn, thr_logit,
                                      scores, mask_words, first_word);
}

// ---------------------------------------------------------------------------------------
// Block-wide exclusive prefix of the popcounts of mask words: pre[w] = set bits in words
// [0, w) for w in [0, nwords]; the words are kept in LDS beside it.  Returns pre[nwords].
// Thread t scans the contiguous words [t*per, (t+1)*per); wave scan + LDS across waves.
template <int NT>
__device__ __forceinline__ uint32_t mask_prefix(const uint64_t *__restrict__ mask_words, int nwords,
                                                uint64_t *words_lds, uint32_t *pre_lds,
                                                uint32_t *wave_tot /* [NT / 64] */)
{
    constexpr int NW = NT / kWave;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (nwords + NT - 1) / NT;
    const int w0 = tid * per, w1 = min(nwords, w0 + per);
    uint32_t mine = 0;
    for (int w = w0; w < w1; ++w) {
        const uint64_t word = mask_words[w];
        words_lds[w] = word;
        mine += (uint32_t)__popcll(word);
    }
    uint32_t inc = mine;  // inclusive scan inside the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)inc, o, 64);
        if (lane >= o) inc += up;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const uint32_t v = wave_tot[k];
        if (k < wave) before += v;
        total += v;
    }
    uint32_t run = before + inc - mine;
    for (int w = w0; w < w1; ++w) {
        pre_lds[w] = run;
        run += (uint32_t)__popcll(words_lds[w]);
    }
    if (tid == NT - 1) pre_lds[nwords] = total;
    __syncthreads();
    return total;
}

// Position of the j-th set bit (j < total) given the prefix above; all 64 lanes of a wave
// call it with the same j and get the same answer.  Two ballots find the word (coarse
// stride, then within the stride; nwords <= 4096), a third the bit inside the word.
__device__ __forceinline__ int select_set_bit(const uint64_t *words_lds, const uint32_t *pre_lds,
                                              int nwords, uint32_t j, int lane)
{
    const int step = (nwords + 63) >> 6;
    const int wc = min(lane * step, nwords);
    const int coarse = __popcll(__ballot(lane * step < nwords && pre_lds[wc] <= j)) - 1;
    const int wf = coarse * step + lane;
    const bool ok = lane < step && wf < nwords && pre_lds[min(wf, nwords)] <= j;
    const int w = coarse * step + __popcll(__ballot(ok)) - 1;
    const uint64_t word = words_lds[w];
    const uint32_t rank = j - pre_lds[w];
    const uint64_t below = word & ((1ull << lane) - 1ull);
    const uint64_t hit = __ballot(((word >> lane) & 1ull) && (uint32_t)__popcll(below) == rank);
    return w * 64 + (int)__builtin_ctzll(hit);
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

// ---------------------------------------------------------------------------------------
// Stand-alone compaction of mask words into an ascending index list, by one workgroup.
// Per pass of NT words: popcount prefix as above, then one wave per word; lane l owns
// bit l and its rank inside the word is the popcount of the lower bits (what a ballot +
// mbcnt pair gives for a live predicate).
constexpr int kCompactThreads = 1024;

__global__ __launch_bounds__(kCompactThreads) void k_compact(const uint64_t *__restrict__ mask_words,
                                                             int nwords, int32_t *__restrict__ idx,
                                                             int32_t *__restrict__ count)
{
    constexpr int NT = kCompactThreads, NW = NT / kWave;
    __shared__ uint64_t words_lds[NT];
    __shared__ uint32_t pre_lds[NT + 1];
    __shared__ uint32_t wave_tot[NW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t carry = 0;
    for (int w0 = 0; w0 < nwords; w0 += NT) {
        const int nhere = min(NT, nwords - w0);
        const uint32_t total = mask_prefix<NT>(mask_words + w0, nhere, words_lds, pre_lds, wave_tot);
        for (int q = wave; q < nhere; q += NW) {
            const uint64_t wq = words_lds[q];
            const uint64_t below = wq & ((1ull << lane) - 1ull);
            if ((wq >> lane) & 1ull)
                idx[carry + pre_lds[q] + (uint32_t)__popcll(below)] = (w0 + q) * 64 + lane;
        }
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) *count = (int32_t)carry;
}

}  // namespace pf
