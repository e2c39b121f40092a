// Neuron-aware sparse FFN over the active neurons (PowerInfer Sec. 5.4; the FFN block
// itself is Sec. 2.1, Fig. "bg-mlp"): only the FC1 / gate rows and FC2 columns of the listed
// neurons are read.  All three matrices are neuron-major [ffn][d] fp16, so one neuron is one
// contiguous run of 2d bytes (a multiple of 128 B at every model width used).
//   k_up   : h[b][j] = act(row idx[j] . x[b] + bias)           one wave per listed neuron
//   k_down2: y[b][:] = b_down + sum_j h[b][j] * FC2^T[idx[j]]  64 columns x every P-th slot per workgroup
// The number of listed neurons is read from device memory; grids are fixed.  No kernel
// uses device-scope fences or atomics: every sum has one owner and a fixed order.
#pragma once
#include "dev_util.h"
#include "k_predict.h"

namespace pf {

constexpr int kUpThreads = 256;
constexpr int kUpWaves = kUpThreads / kWave;

// LDS bytes the up kernel needs beyond the staged activations when it compacts itself.
inline size_t up_mask_lds_bytes(int ffn)
{
    const size_t nwords = (size_t)ffn / 64;
    return nwords * sizeof(uint64_t) + (nwords + 1) * sizeof(uint32_t) + 64;
}

// ---------------------------------------------------------------------------------------
// grid = any; waves stride over the list.  x is staged once per workgroup in LDS while the
// first row of every wave is already in flight.
// FROM_MASK: the list is not given; every workgroup derives it from the predictor's mask
// words (popcount prefix in LDS, then each wave selects its j-th set bit), writes the
// entries it owns to idx_out and block 0 writes the count -- the compaction fused into its
// consumer, so the layer step needs no separate compaction launch.
// Gated forms (ACT == 1): h = ReLU(gate . x + bias) * max(up . x, up_floor); up_floor is
// -infinity for the plain ReLU-gated block and 0 for dReLU (ReLU on both branches).
// GLUE (only with FROM_MASK, inside a stack): the layer input is formed in the kernel from the
// previous layer's input and FC2 partial sums, like the predictor's hidden kernel does, and
// applied as a scale on the dot products; the block with write_x set stores it for later kernels.
// The body takes its block number and the number of blocks of its role explicitly, so that a
// launch can run it in a range of its blocks beside another role.
template <int B, int ACT, bool FROM_MASK, bool GLUE>
__device__ __forceinline__ void up_body(
    float *xs, uint32_t *wave_tot, float (*ss_w)[B], const int bid, const int nblocks, const bool write_x,
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const float *__restrict__ x,
    const int32_t *__restrict__ idx_in, const int32_t *__restrict__ count_in,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor,
    const float *__restrict__ yp, int ny, int ypstride, float *__restrict__ x_new)
{
    constexpr int U = 8;
    constexpr bool GATED = (ACT == 1);
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int nch = (d + kChunk - 1) / kChunk, kpad = nch * kChunk;
    const int stride = nblocks * kUpWaves;
    const int nwords = ffn / 64;
    uint64_t *words_lds = reinterpret_cast<uint64_t *>(xs + (size_t)B * kpad + kStageScrap);
    uint32_t *pre_lds = reinterpret_cast<uint32_t *>(words_lds + nwords);

    PF_TSTAMP(2, 0);
    // Through registers rather than straight to LDS: a global -> LDS copy has to be waited
    // for at the first barrier of the mask scan, the register copy only at the commit
    // (measured: 3 % of the stack's time at batch 1, more at larger batches).
    constexpr int SS = (B >= 4) ? 1 : 4 / B;
    Staged<B, SS> st;
    // glue: strides of 1024 elements whose loads are in flight together (all of d <= 4096 at
    // batch 1, as in the hidden kernel)
    constexpr int GS = GLUE ? (B >= 2 ? 1 : 4) : 1;
    GluePass<B, GS> gp;
    const rsrc_t xr = make_rsrc(x, (uint32_t)B * (uint32_t)d * 4u);
    const uint32_t pbytes = (uint32_t)ypstride * 4u;
    const rsrc_t yr = make_rsrc(yp, GLUE ? (uint32_t)(ny - 1) * pbytes + (uint32_t)B * (uint32_t)d * 4u : 0u);
    if (GLUE)
        glue_issue<B, GS, kUpThreads>(gp, xr, yr, pbytes, ny, d, threadIdx.x * 4);
    else
        stage_issue<B, SS>(st, x, d);  // in flight during the mask scan; lands before any weight
    int n;
    if (FROM_MASK) {
        n = (int)mask_prefix<kUpThreads>(mask_words, nwords, words_lds, pre_lds, wave_tot);
        if (bid == 0 && threadIdx.x == 0) *count_out = n;
    } else {
        n = min(max(*count_in, 0), ffn);
    }
    if (bid * kUpWaves >= n && !(GLUE && write_x)) return;  // uniform over the block
    PF_TSTAMP(2, 1);

    auto neuron_of = [&](int j) -> int {
        if (FROM_MASK) {
            const int i = select_set_bit(words_lds, pre_lds, nwords, (uint32_t)j, lane);
            if (lane == 0) idx_out[j] = i;
            return i;
        }
        return idx_in[j];
    };

    int j = bid * kUpWaves + wave;
    int i = 0;
    bool valid = false;
    if (j < n) {
        i = wave_uniform(neuron_of(j));
        valid = (unsigned)i < (unsigned)ffn;
        if (!valid) i = 0;
    }
    PF_TSTAMP(2, 5);
    WGroup<U> gu, gg;
    rsrc_t ru = row_rsrc(w_up, i, d, valid), rg = row_rsrc(GATED ? w_gate : w_up, i, d, valid);
    load_group<U>(gu, ru, 0, lane);
    if (GATED) load_group<U>(gg, rg, 0, lane);

    PF_TSTAMP(2, 2);
    float scale[B];
    if (GLUE) {
        float ss[B];
#pragma unroll
        for (int b = 0; b < B; ++b) ss[b] = 0.f;
        glue_commit<B, GS, kUpThreads>(gp, xs, kpad, 0, threadIdx.x * 4, ss);
        for (int e0 = threadIdx.x * 4 + kUpThreads * 4 * GS; e0 < kpad; e0 += kUpThreads * 4 * GS) {
            glue_issue<B, GS, kUpThreads>(gp, xr, yr, pbytes, ny, d, e0);
            glue_commit<B, GS, kUpThreads>(gp, xs, kpad, 0, e0, ss);
        }
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
            for (int k = 0; k < kUpWaves; ++k) tot += ss_w[k][b];
            scale[b] = tot > 0.f ? sqrtf((float)d / tot) : 0.f;
        }
        if (write_x) {
            for (int e = threadIdx.x * 4; e < d; e += kUpThreads * 4) {
#pragma unroll
                for (int b = 0; b < B; ++b) {
                    const float4 v = *reinterpret_cast<const float4 *>(xs + b * kpad + lds_slot(e));
                    *reinterpret_cast<float4 *>(x_new + (size_t)b * d + e) =
                        make_float4(v.x * scale[b], v.y * scale[b], v.z * scale[b], v.w * scale[b]);
                }
            }
        }
    } else {
        stage_commit<B, SS>(st, xs, x, d, kpad);
        __syncthreads();
#pragma unroll
        for (int b = 0; b < B; ++b) scale[b] = 1.f;
    }
    PF_TSTAMP(2, 3);

    while (j < n) {  // wave-uniform; no block-level synchronisation inside
        float au[B], ag[B];
#pragma unroll
        for (int b = 0; b < B; ++b) au[b] = ag[b] = 0.f;
        fma_group<B, U>(gu, xs, kpad, 0, nch, lane, au);
        if (GATED) fma_group<B, U>(gg, xs, kpad, 0, nch, lane, ag);
        for (int it0 = U; it0 < nch; it0 += U) {
            load_group<U>(gu, ru, it0, lane);
            if (GATED) load_group<U>(gg, rg, it0, lane);
            fma_group<B, U>(gu, xs, kpad, it0, nch, lane, au);
            if (GATED) fma_group<B, U>(gg, xs, kpad, it0, nch, lane, ag);
        }
        const int jcur = j, icur = i;
        const bool vcur = valid;
        j += stride;
        if (j < n) {  // next row in flight before this row's reductions
            i = wave_uniform(neuron_of(j));
            valid = (unsigned)i < (unsigned)ffn;
            if (!valid) i = 0;
            ru = row_rsrc(w_up, i, d, valid);
            rg = row_rsrc(GATED ? w_gate : w_up, i, d, valid);
            load_group<U>(gu, ru, 0, lane);
            if (GATED) load_group<U>(gg, rg, 0, lane);
        }
        const float bias = (b_up != nullptr && vcur) ? b_up[icur] : 0.f;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float v;
            if (GATED) {
                const float gsum = (GLUE ? wave_sum(ag[b]) * scale[b] : wave_sum(ag[b])) + bias;
                const float usum = GLUE ? wave_sum(au[b]) * scale[b] : wave_sum(au[b]);
                v = fmaxf(gsum, 0.f) * fmaxf(usum, up_floor);
            } else {
                v = fmaxf((GLUE ? wave_sum(au[b]) * scale[b] : wave_sum(au[b])) + bias, 0.f);
            }
            if (lane == 0) h[(size_t)jcur * hs + b] = vcur ? v : 0.f;
        }
    }
    PF_TSTAMP(2, 4);
}

template <int B, int ACT, bool FROM_MASK>
__global__ __launch_bounds__(kUpThreads) void k_up(
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const float *__restrict__ x,
    const int32_t *__restrict__ idx_in, const int32_t *__restrict__ count_in,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor)
{
    extern __shared__ float xs[];
    __shared__ uint32_t wave_tot[kUpWaves];
    up_body<B, ACT, FROM_MASK, false>(xs, wave_tot, nullptr, (int)blockIdx.x, (int)gridDim.x, false, w_up,
                                      w_gate, b_up, x, idx_in, count_in, mask_words, idx_out, count_out,
                                      h, hs, d, ffn, up_floor, nullptr, 1, 0, nullptr);
}

// ---------------------------------------------------------------------------------------
// FC2 over the listed neurons, row-split.  The vector memory path of a CU handles gathered
// rows at a few nanoseconds per distinct 128-byte line, so a tiling in which every workgroup
// walks the whole list over a narrow column strip is bound by k lines per CU, not by HBM
// (measured: 16-column strips took 8.7 us where this form takes 5.6 us at d = 4096, k = 1300).
// Here a workgroup owns 64 output columns (one full line per row: 8 lanes x 16 bytes) and
// only every P-th list slot (slot = P * row + g for row group g), so a CU touches
// k * d / (64 * CUs) lines.  idx and h loads of the first pass are issued before the count
// has arrived (both arrays have capacity ffn), so they overlap with it.  The P
// partial sums of a column tile are NOT combined here: partial g goes to part[g][b][d]
// (group 0 adds b_down) and the consumer adds the P partials in the fixed order
// g = 0 .. P-1 -- the next layer's predictor kernel inside a stack, k_combine otherwise.
// grid = (d / 64 tiles, P), block = 512: 64 list slots per load of the block.
constexpr int kDown2Threads = 512;
constexpr int kDown2Waves = kDown2Threads / kWave;
constexpr int kDown2Cols = 64;
constexpr int kDown2RowsPerLoad = kDown2Threads / 8;
constexpr int kDown2MaxSplit = 4;

template <int B>
__device__ __forceinline__ void down2_body(
    float (*red)[B][kDown2Cols], const int tile, const int g, const int P,
    const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_p, float *__restrict__ part, int d, int ffn)
{
    constexpr int U = (B <= 2) ? 8 : 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cl = lane & 7;                      // which 16 bytes of the row's 128-byte line
    const int rslot = wave * 8 + (lane >> 3);     // row slot of this lane inside a load
    const int col = tile * kDown2Cols + cl * 8;
    const bool colok = col < d;
    const rsrc_t wd = make_rsrc(w_down, (uint32_t)ffn * (uint32_t)d * 2u);

    PF_TSTAMP(3, 0);
    // token b, column e of this lane -> acc[8 b + e]; padded to a power of two tokens for the
    // halving butterfly of the epilogue
    constexpr int BP = B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : 8;
    float acc[BP * 8];
#pragma unroll
    for (int f = 0; f < BP * 8; ++f) acc[f] = 0.f;

    int n = 0;
    bool have_n = false;
    for (int r0 = 0; r0 == 0 || r0 * P < n; r0 += kDown2RowsPerLoad * U) {
        uint4 w[U];
        float hv[U][B];
        int iv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {  // loads that depend on the slot number only
            const int jc = min((r0 + u * kDown2RowsPerLoad + rslot) * P + g, ffn - 1);
            iv[u] = idx[jc];
            load_h_slot<B>(h, jc, hv[u]);
        }
        if (!have_n) {
            n = min(max(*count_p, 0), ffn);
            have_n = true;
            PF_TSTAMP(3, 1);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jj = (r0 + u * kDown2RowsPerLoad + rslot) * P + g;
            const bool ok = jj < n && (unsigned)iv[u] < (unsigned)ffn;
            w[u] = ld16_stream(wd, (ok && colok) ? ((uint32_t)iv[u] * (uint32_t)d + (uint32_t)col) * 2u
                                                 : kOobOffset);
#pragma unroll
            for (int b = 0; b < B; ++b) hv[u][b] = ok ? hv[u][b] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float f0 = h_lo(w[u].x), f1 = h_hi(w[u].x), f2 = h_lo(w[u].y), f3 = h_hi(w[u].y);
            const float f4 = h_lo(w[u].z), f5 = h_hi(w[u].z), f6 = h_lo(w[u].w), f7 = h_hi(w[u].w);
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const float s = hv[u][b];
                acc[8 * b + 0] = fmaf(s, f0, acc[8 * b + 0]);
                acc[8 * b + 1] = fmaf(s, f1, acc[8 * b + 1]);
                acc[8 * b + 2] = fmaf(s, f2, acc[8 * b + 2]);
                acc[8 * b + 3] = fmaf(s, f3, acc[8 * b + 3]);
                acc[8 * b + 4] = fmaf(s, f4, acc[8 * b + 4]);
                acc[8 * b + 5] = fmaf(s, f5, acc[8 * b + 5]);
                acc[8 * b + 6] = fmaf(s, f6, acc[8 * b + 6]);
                acc[8 * b + 7] = fmaf(s, f7, acc[8 * b + 7]);
            }
        }
        if (r0 == 0) PF_TSTAMP(3, 2);
    }
    PF_TSTAMP(3, 3);

    // sum the 8 row slots of the wave (lane bits 5, 4, 3) with a halving butterfly: a lane ends
    // with BP of its 8 BP values, flat indices [BP * slot, BP * (slot + 1)); then the 8 waves
    // through LDS
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
    PF_TSTAMP(3, 4);
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
    PF_TSTAMP(3, 5);
}

template <int B>
__global__ __launch_bounds__(kDown2Threads) void k_down2(
    const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_p, float *__restrict__ part, int d, int ffn)
{
    __shared__ float red[kDown2Waves][B][kDown2Cols];
    down2_body<B>(red, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y, w_down, b_down, h, idx, count_p,
                  part, d, ffn);
}

// y[b][c] = sum of the P partials in order (for callers that need FC2's output itself).
__global__ __launch_bounds__(256) void k_combine(const float *__restrict__ part, int P, int n,
                                                 float *__restrict__ y)
{
    const int e = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= n) return;
    float4 s = *reinterpret_cast<const float4 *>(part + e);
    for (int p = 1; p < P; ++p) {
        const float4 v = *reinterpret_cast<const float4 *>(part + (size_t)p * n + e);
        s.x += v.x;
        s.y += v.y;
        s.z += v.z;
        s.w += v.w;
    }
    *reinterpret_cast<float4 *>(y + e) = s;
}

// ---------------------------------------------------------------------------------------
// Stack glue: x_next[b] = sign(b, .) * (x[b] + y[b]) * sqrt(d) / ||x[b] + y[b]||_2.  grid = B.
constexpr int kGlueThreads = 1024;

// Four consecutive values as fp16 hi + lo at element `at` of the hi plane and of the lo plane
// `plane` halfs behind it.
__device__ __forceinline__ void store_split4(__half *xs, size_t plane, size_t at, const float4 &o)
{
    _Float16 hi[4], lo[4];
    split_f32(o.x, hi[0], lo[0]);
    split_f32(o.y, hi[1], lo[1]);
    split_f32(o.z, hi[2], lo[2]);
    split_f32(o.w, hi[3], lo[3]);
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
    *reinterpret_cast<half4_t *>(reinterpret_cast<_Float16 *>(xs) + at) = (half4_t){hi[0], hi[1], hi[2], hi[3]};
    *reinterpret_cast<half4_t *>(reinterpret_cast<_Float16 *>(xs) + plane + at) =
        (half4_t){lo[0], lo[1], lo[2], lo[3]};
}

// x_next may alias x: every element is read and written by the same thread.
// y may come as ny partial sums [ny][B][d] (see k_down2): they are added in order.
// d <= kGlueMaxD: a thread keeps its (up to 4) float4 sums in registers, so every load of the
// kernel is issued before the first one is waited for -- one round trip, then the block
// reduction, then the stores.
constexpr int kGlueMaxD = kGlueThreads * 4 * 4;

// xs_next (may be null): the same values split into fp16 hi and lo planes, [B][d] each, lo
// plane B * d halfs behind the hi plane (the operand format of the matrix-core kernels).
__global__ __launch_bounds__(kGlueThreads) void k_glue(const float *x, const float *__restrict__ y,
                                                       int ny, float *x_next, int d, __half *xs_next)
{
    __shared__ float wsum[kGlueThreads / kWave];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t pbytes = (uint32_t)gridDim.x * (uint32_t)d * 4u;  // between partial sums
    const rsrc_t xr = make_rsrc(x + (size_t)b * d, (uint32_t)d * 4u);
    const rsrc_t yr = make_rsrc(y + (size_t)b * d, (uint32_t)(ny - 1) * pbytes + (uint32_t)d * 4u);
    float4 v[4], p[4][kGlueMaxParts];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (i * kGlueThreads + (int)threadIdx.x) * 4;
        const uint32_t off = e < d ? (uint32_t)e * 4u : kOobOffset;
        v[i] = ld16_f32(xr, off);
#pragma unroll
        for (int q = 0; q < kGlueMaxParts; ++q)
            p[i][q] = ld16_f32(yr, (e < d && q < ny) ? off + (uint32_t)q * pbytes : kOobOffset);
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float4 t = p[i][0];
#pragma unroll
        for (int q = 1; q < kGlueMaxParts; ++q)
            t = make_float4(t.x + p[i][q].x, t.y + p[i][q].y, t.z + p[i][q].z, t.w + p[i][q].w);
        v[i] = glue_signed(make_float4(v[i].x + t.x, v[i].y + t.y, v[i].z + t.z, v[i].w + t.w), (uint32_t)b,
                           (uint32_t)((i * kGlueThreads + (int)threadIdx.x) * 4));
        ss = fmaf(v[i].x, v[i].x, fmaf(v[i].y, v[i].y, fmaf(v[i].z, v[i].z, fmaf(v[i].w, v[i].w, ss))));
    }
    ss = wave_sum(ss);
    if (lane == 0) wsum[wave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < kGlueThreads / kWave; ++k) tot += wsum[k];
    const float scale = tot > 0.f ? sqrtf((float)d / tot) : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = (i * kGlueThreads + (int)threadIdx.x) * 4;
        if (e < d) {
            const float4 o = make_float4(v[i].x * scale, v[i].y * scale, v[i].z * scale, v[i].w * scale);
            *reinterpret_cast<float4 *>(x_next + (size_t)b * d + e) = o;
            if (xs_next != nullptr) store_split4(xs_next, (size_t)gridDim.x * d, (size_t)b * d + e, o);
        }
    }
}

// The same for any d (two passes over the inputs).
__global__ __launch_bounds__(kGlueThreads) void k_glue_long(const float *x, const float *__restrict__ y,
                                                            int ny, float *x_next, int d, __half *xs_next)
{
    __shared__ float wsum[kGlueThreads / kWave];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t pstride = (size_t)gridDim.x * d;
    const float *xb = x + (size_t)b * d, *yb = y + (size_t)b * d;
    auto ysum = [&](int c) {
        float t = yb[c];
        for (int p = 1; p < ny; ++p) t += yb[p * pstride + c];
        return t;
    };
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += kGlueThreads) {
        const float v = xb[c] + ysum(c);
        ss = fmaf(v, v, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) wsum[wave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < kGlueThreads / kWave; ++k) tot += wsum[k];
    const float scale = tot > 0.f ? sqrtf((float)d / tot) : 0.f;
    for (int c = threadIdx.x; c < d; c += kGlueThreads) {
        const float v = (xb[c] + ysum(c)) * scale;
        const float o = __uint_as_float(__float_as_uint(v) ^ glue_sign_bit((uint32_t)b, (uint32_t)c));
        x_next[(size_t)b * d + c] = o;
        if (xs_next != nullptr) {
            _Float16 hi, lo;
            split_f32(o, hi, lo);
            reinterpret_cast<_Float16 *>(xs_next)[(size_t)b * d + c] = hi;
            reinterpret_cast<_Float16 *>(xs_next)[(size_t)gridDim.x * d + (size_t)b * d + c] = lo;
        }
    }
}

// The split planes of a caller's activations x[n] (n = B * d, a multiple of 4): xs[0 .. n) hi,
// xs[n .. 2n) lo.  grid = ceil(n / 1024), block = 256.
__global__ __launch_bounds__(256) void k_split(const float *__restrict__ x, __half *__restrict__ xs, int n)
{
    const int e = ((int)blockIdx.x * 256 + (int)threadIdx.x) * 4;
    if (e < n) store_split4(xs, (size_t)n, (size_t)e, *reinterpret_cast<const float4 *>(x + e));
}

}  // namespace pf
