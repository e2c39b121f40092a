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
#include "k_fused.h"

namespace pf {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4v_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaThreads = 256;
constexpr int kMfmaWaves = kMfmaThreads / kWave;
constexpr int kMfmaRT = 2;                    // 16-row tiles per wave pass
constexpr int kMfmaRows = 16 * kMfmaRT;       // list slots per wave pass
constexpr int kMfmaKU = 4;                    // K steps (of 32) whose loads are in flight together

union Half8Bits {
    uint4 u;
    half8_t h;
};

// Split 8 fp32 values into fp16 hi (truncated) and fp16 lo (residual) vectors.
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

// grid = any; waves stride over passes of 32 list slots.  d % 32 == 0, B <= 16.
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
    constexpr bool GATED = (ACT == 1);
    constexpr int RT = kMfmaRT, KU = kMfmaKU;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row16 = lane & 15, kg = lane >> 4;
    const int nwords = ffn / 64;
    uint64_t *words_lds = dyn_lds64;
    uint32_t *pre_lds = reinterpret_cast<uint32_t *>(words_lds + (FROM_MASK ? nwords : 0));

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
    const int npass = (n + kMfmaRows - 1) / kMfmaRows;

    for (int pass = blockIdx.x * kMfmaWaves + wave; pass < npass; pass += gridDim.x * kMfmaWaves) {
        // the A-operand row of this lane in each tile: list slot -> neuron id
        int jr[RT], ir[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) jr[r] = pass * kMfmaRows + r * 16 + row16;
        if (FROM_MASK) {
            select_set_bits_lane<RT>(words_lds, pre_lds, nwords, top_step, n, jr, ir);
        } else {
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                ir[r] = jr[r] < n ? idx_in[jr[r]] : -1;
                if ((unsigned)ir[r] >= (unsigned)ffn) ir[r] = -1;
            }
        }
        uint32_t aoff[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            aoff[r] = ir[r] >= 0 ? ((uint32_t)ir[r] * (uint32_t)d + (uint32_t)kg * 8u) * 2u : kOobOffset;
            if (FROM_MASK && kg == 0 && ir[r] >= 0) idx_out[jr[r]] = ir[r];
        }

        float4v_t cu[RT], cg[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            cu[r] = (float4v_t){0.f, 0.f, 0.f, 0.f};
            cg[r] = (float4v_t){0.f, 0.f, 0.f, 0.f};
        }
        for (int s0 = 0; s0 < nsteps; s0 += KU) {
            Half8Bits au[KU][RT], ag[KU][RT];
            float4 xa[KU], xb[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const bool live = s0 + u < nsteps;
                const uint32_t kb = (uint32_t)(s0 + u) * 32u;  // element offset of this K step
                xa[u] = ld16_f32(xr, live && xoff != kOobOffset ? xoff + kb * 4u : kOobOffset);
                xb[u] = ld16_f32(xr, live && xoff != kOobOffset ? xoff + kb * 4u + 16u : kOobOffset);
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const uint32_t o = live && aoff[r] != kOobOffset ? aoff[r] + kb * 2u : kOobOffset;
                    au[u][r].u = ld16_stream(wu, o);
                    if (GATED) ag[u][r].u = ld16_stream(wg, o);
                }
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                half8_t hi, lo;
                split_hi_lo(xa[u], xb[u], hi, lo);
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    cu[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(au[u][r].h, hi, cu[r], 0, 0, 0);
                    cu[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(au[u][r].h, lo, cu[r], 0, 0, 0);
                    if (GATED) {
                        cg[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ag[u][r].h, hi, cg[r], 0, 0, 0);
                        cg[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ag[u][r].h, lo, cg[r], 0, 0, 0);
                    }
                }
            }
        }
        // C[row 4*kg + e][col row16]: the token is this lane's column, the neuron comes from
        // the lane that owned that A row
#pragma unroll
        for (int r = 0; r < RT; ++r) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = kg * 4 + e;
                const int i = __shfl(ir[r], row, 64);
                const int j = pass * kMfmaRows + r * 16 + row;
                const float bias = (b_up != nullptr && i >= 0) ? b_up[i] : 0.f;
                float v;
                if (GATED)
                    v = fmaxf(cg[r][e] + bias, 0.f) * cu[r][e];
                else
                    v = fmaxf(cu[r][e] + bias, 0.f);
                if (row16 < B && j < n) h[(size_t)row16 * ffn + j] = i >= 0 ? v : 0.f;
            }
        }
    }
}

}  // namespace pf
