// FC1 over the listed neurons for a batch of tokens as a matrix-core contraction
// (PowerInfer Sec. 8.2, batching: the active set is the union over the batch, so the gathered
// rows form a dense [k x d] block that multiplies [d x B]).  At batch 1 the row-sparse GEMV is
// pure HBM streaming; from a few tokens on, B FMAs per weight make the vector ALUs the
// limiter before HBM saturates, and v_mfma_f32_16x16x32_f16 does the same work in 1/8 of
// the issue slots.  M = 16 gathered rows, N = 16 batch columns (tokens >= B read as zero),
// K = 32 elements of d per instruction.
// Operand layout (verified on the device): lane l supplies A[row l%16][8 halfs from k = 8*(l/16)]
// and B[same 8 k][col l%16]; it receives C[rows 4*(l/16) .. +3][col l%16].
// Activations stay fp32-exact: x is split into fp16 hi + fp16 lo (x = hi + lo to 2^-21) and
// each step issues two MFMAs.
#pragma once
#include "dev_util.h"
#include "k_predict.h"

namespace pf {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4v_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaThreads = 512;
constexpr int kMfmaWaves = kMfmaThreads / kWave;  // the waves of a block split K between them
constexpr int kMfmaRows = 16;                     // list slots per block pass: one MFMA tile
constexpr int kMfmaKU = 8;                        // K steps (of 32) whose loads are in flight together

union Half8Bits {
    uint4 u;
    half8_t h;
};

// Split 8 fp32 values into fp16 hi (rounded) and fp16 lo (residual) vectors.
__device__ __forceinline__ void split_hi_lo(const float4 &a, const float4 &b, half8_t &hi, half8_t &lo)
{
    const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const _Float16 h = (_Float16)v[e];
        hi[e] = h;
        lo[e] = (_Float16)(v[e] - (float)h);
    }
}

// grid = any; blocks stride over passes of 16 list slots; the 8 waves of a block each take
// an eighth of the K steps of the same 16 rows (so that a pass has 8 x 16 rows x 512 bytes
// in flight instead of one wave walking d alone) and their C tiles are added in LDS in
// wave order.  d % 32 == 0, B <= 16.
template <int ACT, bool FROM_MASK>
__global__ __launch_bounds__(kMfmaThreads) void k_up_mfma(
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const float *__restrict__ x, int B,
    const int32_t *__restrict__ idx_in, const int32_t *__restrict__ count_in,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int d, int ffn)
{
    extern __shared__ uint64_t dyn_lds64[];
    __shared__ uint32_t wave_tot[kMfmaWaves];
    __shared__ float ctile[kMfmaWaves][2][256];  // per wave: C of up, C of gate (16 x 16 each)
    __shared__ int irow[16];
    constexpr bool GATED = (ACT == 1);
    constexpr int KU = kMfmaKU;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row16 = lane & 15, kg = lane >> 4;
    const int nwords = ffn / 64;
    uint64_t *words_lds = dyn_lds64;
    uint32_t *pre_lds = reinterpret_cast<uint32_t *>(words_lds + (FROM_MASK ? nwords : 0));

    PF_TSTAMP(2, 0);
    int n;
    int top_step = 1;
    if (FROM_MASK) {
        n = (int)mask_prefix<kMfmaThreads>(mask_words, nwords, words_lds, pre_lds, wave_tot);
        if (blockIdx.x == 0 && threadIdx.x == 0) *count_out = n;
        while (top_step * 2 < nwords) top_step *= 2;
    } else {
        n = min(max(*count_in, 0), ffn);
    }
    const rsrc_t wu = make_rsrc(w_up, (uint32_t)ffn * (uint32_t)d * 2u);
    const rsrc_t wg = make_rsrc(GATED ? w_gate : w_up, (uint32_t)ffn * (uint32_t)d * 2u);
    const rsrc_t xr = make_rsrc(x, (uint32_t)B * (uint32_t)d * 4u);
    const uint32_t xoff = row16 < B ? ((uint32_t)row16 * (uint32_t)d + (uint32_t)kg * 8u) * 4u : kOobOffset;
    const int nsteps = d / 32;
    const int per_wave = (nsteps + kMfmaWaves - 1) / kMfmaWaves;
    const int s_begin = wave * per_wave, s_end = min(nsteps, s_begin + per_wave);
    const int npass = (n + kMfmaRows - 1) / kMfmaRows;
    PF_TSTAMP(2, 1);

    for (int pass = blockIdx.x; pass < npass; pass += gridDim.x) {
        // the A-operand row of this lane: list slot -> neuron id
        const int jr[1] = {pass * kMfmaRows + row16};
        int ir[1];
        if (FROM_MASK) {
            select_set_bits_lane<1>(words_lds, pre_lds, nwords, top_step, n, jr, ir);
        } else {
            ir[0] = jr[0] < n ? idx_in[jr[0]] : -1;
            if ((unsigned)ir[0] >= (unsigned)ffn) ir[0] = -1;
        }
        const uint32_t aoff = ir[0] >= 0 ? ((uint32_t)ir[0] * (uint32_t)d + (uint32_t)kg * 8u) * 2u : kOobOffset;
        if (wave == 0 && kg == 0) {
            irow[row16] = ir[0];
            if (FROM_MASK && ir[0] >= 0) idx_out[jr[0]] = ir[0];
        }

        if (pass == (int)blockIdx.x) PF_TSTAMP(2, 2);
        float4v_t cu = {0.f, 0.f, 0.f, 0.f}, cg = {0.f, 0.f, 0.f, 0.f};
        for (int s0 = s_begin; s0 < s_end; s0 += KU) {
            Half8Bits au[KU], ag[KU];
            float4 xa[KU], xb[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const bool live = s0 + u < s_end;
                const uint32_t kb = (uint32_t)(s0 + u) * 32u;  // element offset of this K step
                const uint32_t o = live && aoff != kOobOffset ? aoff + kb * 2u : kOobOffset;
                au[u].u = ld16_stream(wu, o);
                if (GATED) ag[u].u = ld16_stream(wg, o);
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const bool live = s0 + u < s_end;
                const uint32_t kb = (uint32_t)(s0 + u) * 32u;
                xa[u] = ld16_f32(xr, live && xoff != kOobOffset ? xoff + kb * 4u : kOobOffset);
                xb[u] = ld16_f32(xr, live && xoff != kOobOffset ? xoff + kb * 4u + 16u : kOobOffset);
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                half8_t hi, lo;
                split_hi_lo(xa[u], xb[u], hi, lo);
                cu = __builtin_amdgcn_mfma_f32_16x16x32_f16(au[u].h, hi, cu, 0, 0, 0);
                cu = __builtin_amdgcn_mfma_f32_16x16x32_f16(au[u].h, lo, cu, 0, 0, 0);
                if (GATED) {
                    cg = __builtin_amdgcn_mfma_f32_16x16x32_f16(ag[u].h, hi, cg, 0, 0, 0);
                    cg = __builtin_amdgcn_mfma_f32_16x16x32_f16(ag[u].h, lo, cg, 0, 0, 0);
                }
            }
        }
        if (pass == (int)blockIdx.x) PF_TSTAMP(2, 3);
        // this lane holds C[row 4*kg + e][col row16] of its K slice
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            ctile[wave][0][(kg * 4 + e) * 16 + row16] = cu[e];
            if (GATED) ctile[wave][1][(kg * 4 + e) * 16 + row16] = cg[e];
        }
        __syncthreads();
        if (threadIdx.x < 256) {
            const int row = threadIdx.x >> 4, colb = threadIdx.x & 15;
            float su = 0.f, sg = 0.f;
#pragma unroll
            for (int wv = 0; wv < kMfmaWaves; ++wv) {
                su += ctile[wv][0][threadIdx.x];
                if (GATED) sg += ctile[wv][1][threadIdx.x];
            }
            const int i = irow[row];
            const int j = pass * kMfmaRows + row;
            const float bias = (b_up != nullptr && i >= 0) ? b_up[i] : 0.f;
            const float v = GATED ? fmaxf(sg + bias, 0.f) * su : fmaxf(su + bias, 0.f);
            if (colb < B && j < n) h[(size_t)colb * ffn + j] = i >= 0 ? v : 0.f;
        }
        __syncthreads();
        if (pass == (int)blockIdx.x) PF_TSTAMP(2, 4);
    }
    PF_TSTAMP(2, 5);
}

}  // namespace pf
