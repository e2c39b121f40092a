// Neuron-aware sparse FFN over a compacted index list (PowerInfer Sec. 5.4; the FFN block
// itself is Sec. 2.1, Fig. "bg-mlp"): only the FC1 / gate rows and FC2 columns of the listed
// neurons are read.  All three matrices are neuron-major [ffn][d] fp16, so one neuron is one
// contiguous run of 2d bytes (a multiple of 128 B at every model width used).
//   k_up   : h[b][j] = act(row idx[j] . x[b] + bias)           one wave per listed neuron
//   k_down : y[b][:] = b_down + sum_j h[b][j] * FC2^T[idx[j]]  d-tiles x neuron-chunks, then a
//            deterministic combine of the chunk partials by the last workgroup of each tile
// The number of listed neurons is read from device memory; grids are fixed.
#pragma once
#include "dev_util.h"

namespace pf {

constexpr int kUpThreads = 256;
constexpr int kUpWaves = kUpThreads / kWave;

// ---------------------------------------------------------------------------------------
// grid = any; waves stride over the list.  x is staged once per workgroup in LDS while the
// first row of every wave is already in flight.
template <int B, int ACT>
__global__ __launch_bounds__(kUpThreads) void k_up(const __half *__restrict__ w_up,
                                                   const __half *__restrict__ w_gate,
                                                   const float *__restrict__ b_up,
                                                   const float *__restrict__ x,
                                                   const int32_t *__restrict__ idx,
                                                   const int32_t *__restrict__ count_p,
                                                   float *__restrict__ h, int d, int ffn)
{
    extern __shared__ float xs[];
    constexpr int U = 8;
    constexpr bool GATED = (ACT == 1);
    const int n = min(max(*count_p, 0), ffn);
    if ((int)blockIdx.x * kUpWaves >= n) return;  // uniform over the block
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int nch = (d + kChunk - 1) / kChunk, kpad = nch * kChunk;
    const int stride = gridDim.x * kUpWaves;

    int j = blockIdx.x * kUpWaves + wave;
    int i = 0;
    bool valid = false;
    if (j < n) {
        i = idx[j];
        valid = (unsigned)i < (unsigned)ffn;
        if (!valid) i = 0;
    }
    WGroup<U> gu, gg;
    load_group<U>(gu, w_up + (size_t)i * d, valid ? d : 0, 0, lane);
    if (GATED) load_group<U>(gg, w_gate + (size_t)i * d, valid ? d : 0, 0, lane);

    stage_vector<B>(xs, x, d, kpad);
    __syncthreads();

    while (j < n) {  // wave-uniform; no block-level synchronisation inside
        float au[B], ag[B];
#pragma unroll
        for (int b = 0; b < B; ++b) au[b] = ag[b] = 0.f;
        fma_group<B, U>(gu, xs, kpad, 0, nch, lane, au);
        if (GATED) fma_group<B, U>(gg, xs, kpad, 0, nch, lane, ag);
        for (int it0 = U; it0 < nch; it0 += U) {
            load_group<U>(gu, w_up + (size_t)i * d, valid ? d : 0, it0, lane);
            if (GATED) load_group<U>(gg, w_gate + (size_t)i * d, valid ? d : 0, it0, lane);
            fma_group<B, U>(gu, xs, kpad, it0, nch, lane, au);
            if (GATED) fma_group<B, U>(gg, xs, kpad, it0, nch, lane, ag);
        }
        const int jcur = j, icur = i;
        const bool vcur = valid;
        j += stride;
        if (j < n) {  // next row in flight before this row's reductions
            i = idx[j];
            valid = (unsigned)i < (unsigned)ffn;
            if (!valid) i = 0;
            load_group<U>(gu, w_up + (size_t)i * d, valid ? d : 0, 0, lane);
            if (GATED) load_group<U>(gg, w_gate + (size_t)i * d, valid ? d : 0, 0, lane);
        }
        const float bias = (b_up != nullptr && vcur) ? b_up[icur] : 0.f;
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
            if (lane == 0) h[(size_t)b * ffn + jcur] = vcur ? v : 0.f;
        }
    }
}

// ---------------------------------------------------------------------------------------
constexpr int kDownThreads = 256;
constexpr int kDownWaves = kDownThreads / kWave;
constexpr int kDownTile = 512;  // columns per workgroup: 8 per lane, one 16-byte load per row

// grid = (ceil(d / 512), max_chunks).  The listed neurons are cut into `eff` equal chunks
// (eff derived from the device-side count, at least min_rows neurons each); block (tx, c)
// sums chunk c over column tile tx.  Within a block wave w takes rows w, w+4, ... of the
// chunk, U at a time; waves are combined in LDS in wave order, the block's partial goes
// to `partial[c][b][d]`, and the last block to arrive on a tile (device-scope counter) adds
// the partials in chunk order plus b_down into y.  The order of every sum is fixed.
template <int B>
__global__ __launch_bounds__(kDownThreads) void k_down(
    const __half *__restrict__ w_down, const float *__restrict__ b_down,
    const float *__restrict__ h, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_p, float *__restrict__ partial,
    unsigned int *__restrict__ tile_arrive, float *__restrict__ y, int d, int ffn, int min_rows)
{
    constexpr int U = 8;
    __shared__ float red[kDownWaves - 1][B][kDownTile];
    __shared__ int is_last;
    const int n = min(max(*count_p, 0), ffn);
    const int eff = min(max((n + min_rows - 1) / min_rows, 1), (int)gridDim.y);
    const int chunk = blockIdx.y;
    if (chunk >= eff) return;  // uniform over the block
    const int rows_per = (n + eff - 1) / eff;
    const int j0 = chunk * rows_per, j1 = min(n, j0 + rows_per);
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int col = blockIdx.x * kDownTile + lane * 8;
    const bool colok = col < d;

    float acc[B][8];
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;

    for (int j = j0 + wave; j < j1; j += kDownWaves * U) {
        uint4 w[U];
        float hv[U][B];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jj = j + u * kDownWaves;
            bool ok = jj < j1;
            int i = ok ? idx[jj] : 0;
            ok = ok && (unsigned)i < (unsigned)ffn;
            if (ok && colok)
                w[u] = ld16_stream(w_down + (size_t)i * d + col);
            else
                w[u] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int b = 0; b < B; ++b) hv[u][b] = ok ? h[(size_t)b * ffn + jj] : 0.f;
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

    // combine the waves of this block in wave order
    if (wave > 0) {
#pragma unroll
        for (int b = 0; b < B; ++b) {
            *reinterpret_cast<float4 *>(&red[wave - 1][b][lane * 8]) =
                make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
            *reinterpret_cast<float4 *>(&red[wave - 1][b][lane * 8 + 4]) =
                make_float4(acc[b][4], acc[b][5], acc[b][6], acc[b][7]);
        }
    }
    __syncthreads();
    if (wave == 0 && colok) {
#pragma unroll
        for (int b = 0; b < B; ++b) {
#pragma unroll
            for (int wv = 0; wv < kDownWaves - 1; ++wv) {
                const float4 a = *reinterpret_cast<const float4 *>(&red[wv][b][lane * 8]);
                const float4 c = *reinterpret_cast<const float4 *>(&red[wv][b][lane * 8 + 4]);
                acc[b][0] += a.x; acc[b][1] += a.y; acc[b][2] += a.z; acc[b][3] += a.w;
                acc[b][4] += c.x; acc[b][5] += c.y; acc[b][6] += c.z; acc[b][7] += c.w;
            }
            float *dst = partial + ((size_t)chunk * B + b) * d + col;
            *reinterpret_cast<float4 *>(dst) = make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
            *reinterpret_cast<float4 *>(dst + 4) =
                make_float4(acc[b][4], acc[b][5], acc[b][6], acc[b][7]);
        }
    }

    // arrival on this column tile; the last block combines the chunk partials
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int prev = atomicAdd(&tile_arrive[blockIdx.x], 1u);
        is_last = (prev == (unsigned int)eff - 1u);
        if (is_last) tile_arrive[blockIdx.x] = 0u;  // ready for the next launch
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    const int c0 = blockIdx.x * kDownTile + threadIdx.x * 2;
    if (c0 < d) {
        const float2 bias = b_down ? *reinterpret_cast<const float2 *>(b_down + c0)
                                   : make_float2(0.f, 0.f);
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float2 s = bias;
            for (int c = 0; c < eff; ++c) {
                const float2 p = *reinterpret_cast<const float2 *>(
                    partial + ((size_t)c * B + b) * d + c0);
                s.x += p.x;
                s.y += p.y;
            }
            *reinterpret_cast<float2 *>(y + (size_t)b * d + c0) = s;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Stack glue: x_next[b] = (x[b] + y[b]) * sqrt(d) / ||x[b] + y[b]||_2.  grid = B.
constexpr int kGlueThreads = 1024;

// x_next may alias x: every element is read and written by the same thread.
__global__ __launch_bounds__(kGlueThreads) void k_glue(const float *x, const float *__restrict__ y,
                                                       float *x_next, int d)
{
    __shared__ float wsum[kGlueThreads / kWave];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *xb = x + (size_t)b * d, *yb = y + (size_t)b * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += kGlueThreads) {
        const float v = xb[c] + yb[c];
        ss = fmaf(v, v, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) wsum[wave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < kGlueThreads / kWave; ++k) tot += wsum[k];
    const float scale = tot > 0.f ? sqrtf((float)d / tot) : 0.f;
    for (int c = threadIdx.x; c < d; c += kGlueThreads) x_next[(size_t)b * d + c] = (xb[c] + yb[c]) * scale;
}

}  // namespace pf
