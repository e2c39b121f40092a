// Sparse FFN kernels for int4 weights (PowerInfer Sec. 8.1: "FP16 and INT4 quantized
// parameters, intermediate activations in FP32"), dequantised in the kernel.
// Format (the paper does not fix one): unsigned nibble u, value = scale * (u - 8), one fp16
// scale per 128 consecutive elements of a neuron's row; element 2j is the low nibble of
// byte j.  A 16-byte load therefore carries 32 consecutive elements of a row, all inside
// one scale group, and dword k of it holds elements 8k .. 8k+7 in nibble order.
//   sum_e scale * (u_e - 8) * x_e = scale * (sum_e u_e * x_e  -  8 * sum_e x_e)
// so the inner loop multiplies raw nibbles (byte-to-float converts) and the offset and the
// scale are applied once per 32 elements.
#pragma once
#include "dev_util.h"
#include "k_predict.h"

namespace pf {

constexpr int kI4Epl = 32;                // elements per lane per 16-byte load
constexpr int kI4Chunk = 64 * kI4Epl;     // elements a wave covers per load: 2048
constexpr int kI4Group = 128;             // elements per scale

__device__ __forceinline__ float half_bits_to_float(unsigned short bits)
{
    return __half2float(__ushort_as_half(bits));
}

// The eight nibbles of a dword as floats, in element order.
__device__ __forceinline__ void nibbles8(uint32_t dw, float (&f)[8])
{
    const uint32_t lo = dw & 0x0f0f0f0fu, hi = (dw >> 4) & 0x0f0f0f0fu;
    f[0] = (float)(lo & 0xffu);
    f[1] = (float)(hi & 0xffu);
    f[2] = (float)((lo >> 8) & 0xffu);
    f[3] = (float)((hi >> 8) & 0xffu);
    f[4] = (float)((lo >> 16) & 0xffu);
    f[5] = (float)((hi >> 16) & 0xffu);
    f[6] = (float)(lo >> 24);
    f[7] = (float)(hi >> 24);
}

// acc[b] += scale * dot(32 dequantised weights of one load, staged activations of token b);
// xs_lane = staged image + chunk * 2048 + lane * 4 (eight planes of 256 floats per chunk).
template <int B>
__device__ __forceinline__ void fma_i4(const uint4 &w, float scale, const float *__restrict__ xs_lane,
                                       int kpad, float (&acc)[B])
{
    const uint32_t dws[4] = {w.x, w.y, w.z, w.w};
    float t[B], sx[B];
#pragma unroll
    for (int b = 0; b < B; ++b) t[b] = sx[b] = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float f[8];
        nibbles8(dws[k], f);
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float4 xa = *reinterpret_cast<const float4 *>(xs_lane + b * kpad + (2 * k) * 256);
            const float4 xb = *reinterpret_cast<const float4 *>(xs_lane + b * kpad + (2 * k + 1) * 256);
            t[b] = fmaf(f[0], xa.x, fmaf(f[1], xa.y, fmaf(f[2], xa.z, fmaf(f[3], xa.w, t[b]))));
            t[b] = fmaf(f[4], xb.x, fmaf(f[5], xb.y, fmaf(f[6], xb.z, fmaf(f[7], xb.w, t[b]))));
            sx[b] += ((xa.x + xa.y) + (xa.z + xa.w)) + ((xb.x + xb.y) + (xb.z + xb.w));
        }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) acc[b] = fmaf(scale, t[b] - 8.f * sx[b], acc[b]);
}

struct I4Row {
    rsrc_t q, s;  // packed nibbles [d/2 bytes] and scales [d/128 fp16] of one neuron
};

__device__ __forceinline__ I4Row i4_row(const uint8_t *q, const __half *s, int i, int d, bool valid)
{
    I4Row r;
    r.q = make_rsrc(q + (size_t)i * (d / 2), valid ? (uint32_t)d / 2u : 0u);
    r.s = make_rsrc(s + (size_t)i * (d / kI4Group), valid ? (uint32_t)(d / kI4Group) * 2u : 0u);
    return r;
}

template <int U>
struct I4Group {
    uint4 w[U];
    unsigned short sc[U];
};

template <int U>
__device__ __forceinline__ void i4_load_group(I4Group<U> &g, const I4Row &row, int it0, int lane)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t chunk = (uint32_t)(it0 + u);
        g.w[u] = ld16_stream(row.q, chunk * (kI4Chunk / 2) + (uint32_t)lane * 16u);
        g.sc[u] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(
            row.s, (int)((chunk * (kI4Chunk / kI4Group) + (uint32_t)(lane >> 2)) * 2u), 0, 0);
    }
}

template <int B, int U>
__device__ __forceinline__ void i4_fma_group(const I4Group<U> &g, const float *__restrict__ xs, int kpad,
                                             int it0, int nch, int lane, float (&acc)[B])
{
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (it0 + u < nch)
            fma_i4<B>(g.w[u], half_bits_to_float(g.sc[u]), xs + (it0 + u) * kI4Chunk + lane * 4, kpad, acc);
}

constexpr int kUpI4Threads = 512;  // rows are long (d up to 12288): fewer, larger workgroups
                                   // stage x less often (measured best at 512 x 2 per CU)
constexpr int kUpI4Waves = kUpI4Threads / kWave;

// FC1 (and gate) over listed neurons, int4 weights: the structure of k_up with 2048-element
// chunks.  With FROM_MASK the list is derived from the mask words inside the kernel.
// The body takes its block number and the number of blocks of its role explicitly, so that a
// launch can run it in a range of its blocks beside another role.
template <int B, int ACT, bool FROM_MASK>
__device__ __forceinline__ void up_i4_body(
    float *xs, uint32_t *wave_tot, const int bid, const int nblocks,
    const uint8_t *__restrict__ q_up, const __half *__restrict__ s_up,
    const uint8_t *__restrict__ q_gate, const __half *__restrict__ s_gate,
    const float *__restrict__ b_up, const float *__restrict__ x,
    const int32_t *__restrict__ idx_in, const int32_t *__restrict__ count_in,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor)
{
    constexpr int U = 2;
    constexpr bool GATED = (ACT == 1);
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int nch = (d + kI4Chunk - 1) / kI4Chunk, kpad = nch * kI4Chunk;
    const int stride = nblocks * kUpI4Waves;
    const int nwords = ffn / 64;
    uint64_t *words_lds = reinterpret_cast<uint64_t *>(xs + (size_t)B * kpad + kStageScrap);
    uint32_t *pre_lds = reinterpret_cast<uint32_t *>(words_lds + nwords);

    constexpr int SS = (B >= 4) ? 1 : 4 / B;
    Staged<B, SS> st;
    stage_issue<B, SS>(st, x, d);
    int n;
    if (FROM_MASK) {
        n = (int)mask_prefix<kUpI4Threads>(mask_words, nwords, words_lds, pre_lds, wave_tot);
        if (bid == 0 && threadIdx.x == 0) *count_out = n;
    } else {
        n = min(max(*count_in, 0), ffn);
    }
    if (bid * kUpI4Waves >= n) return;  // uniform over the block

    auto neuron_of = [&](int j) -> int {
        if (FROM_MASK) {
            const int i = select_set_bit(words_lds, pre_lds, nwords, (uint32_t)j, lane);
            if (lane == 0) idx_out[j] = i;
            return i;
        }
        return idx_in[j];
    };

    int j = bid * kUpI4Waves + wave;
    int i = 0;
    bool valid = false;
    if (j < n) {
        i = wave_uniform(neuron_of(j));
        valid = (unsigned)i < (unsigned)ffn;
        if (!valid) i = 0;
    }
    I4Row ru = i4_row(q_up, s_up, i, d, valid);
    I4Row rg = i4_row(GATED ? q_gate : q_up, GATED ? s_gate : s_up, i, d, valid);
    I4Group<U> gu, gg;
    i4_load_group<U>(gu, ru, 0, lane);
    if (GATED) i4_load_group<U>(gg, rg, 0, lane);

    stage_commit<B, SS, kI4Epl>(st, xs, x, d, kpad);
    __syncthreads();

    while (j < n) {  // wave-uniform; no block-level synchronisation inside
        float au[B], ag[B];
#pragma unroll
        for (int b = 0; b < B; ++b) au[b] = ag[b] = 0.f;
        i4_fma_group<B, U>(gu, xs, kpad, 0, nch, lane, au);
        if (GATED) i4_fma_group<B, U>(gg, xs, kpad, 0, nch, lane, ag);
        for (int it0 = U; it0 < nch; it0 += U) {
            i4_load_group<U>(gu, ru, it0, lane);
            if (GATED) i4_load_group<U>(gg, rg, it0, lane);
            i4_fma_group<B, U>(gu, xs, kpad, it0, nch, lane, au);
            if (GATED) i4_fma_group<B, U>(gg, xs, kpad, it0, nch, lane, ag);
        }
        const int jcur = j, icur = i;
        const bool vcur = valid;
        j += stride;
        if (j < n) {  // next row in flight before this row's reductions
            i = wave_uniform(neuron_of(j));
            valid = (unsigned)i < (unsigned)ffn;
            if (!valid) i = 0;
            ru = i4_row(q_up, s_up, i, d, valid);
            rg = i4_row(GATED ? q_gate : q_up, GATED ? s_gate : s_up, i, d, valid);
            i4_load_group<U>(gu, ru, 0, lane);
            if (GATED) i4_load_group<U>(gg, rg, 0, lane);
        }
        const float bias = (b_up != nullptr && vcur) ? b_up[icur] : 0.f;
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
            if (lane == 0) h[(size_t)jcur * hs + b] = vcur ? v : 0.f;
        }
    }
}

template <int B, int ACT, bool FROM_MASK>
__global__ __launch_bounds__(kUpI4Threads) void k_up_i4(
    const uint8_t *__restrict__ q_up, const __half *__restrict__ s_up,
    const uint8_t *__restrict__ q_gate, const __half *__restrict__ s_gate,
    const float *__restrict__ b_up, const float *__restrict__ x,
    const int32_t *__restrict__ idx_in, const int32_t *__restrict__ count_in,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor)
{
    extern __shared__ float xs[];
    __shared__ uint32_t wave_tot[kUpI4Waves];
    up_i4_body<B, ACT, FROM_MASK>(xs, wave_tot, (int)blockIdx.x, (int)gridDim.x, q_up, s_up, q_gate, s_gate, b_up,
                                  x, idx_in, count_in, mask_words, idx_out, count_out, h, hs, d, ffn, up_floor);
}

// ---------------------------------------------------------------------------------------
// FC2 over listed neurons, int4 weights, row-split like k_down2: a workgroup owns 256 output
// columns = one full 128-byte line of nibbles per row (8 lanes x 16 bytes, 32 columns per
// lane) and every P-th list slot; partial g goes to part[g][b][d], group 0 adds b_down, the
// consumer adds the partials in order.  A lane's 32 accumulators are summed over the 8 row
// slots of its wave by a halving butterfly (a lane gives away half of its values at every
// exchange), then over waves in LDS.  grid = (d / 256, P), block = 512.
constexpr int kDown2I4Threads = 512;
constexpr int kDown2I4Waves = kDown2I4Threads / kWave;
constexpr int kDown2I4Cols = 256;
constexpr int kDown2I4RowsPerLoad = kDown2I4Threads / 8;

// Body: bx = the block's number among the nt column tiles of row group g (of P).
template <int B>
__device__ __forceinline__ void down2_i4_body(
    float (*red)[B][kDown2I4Cols], const int bx, const int nt, const int g, const int P,
    const uint8_t *__restrict__ q_down, const __half *__restrict__ s_down,
    const float *__restrict__ b_down, const float *__restrict__ h,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count_p, float *__restrict__ part,
    int d, int ffn)
{
    constexpr int U = (B <= 2) ? 4 : 2;
    // Workgroups go to the 8 XCDs round-robin by their linear number, and every XCD has an L2
    // of its own.  A row's scales (2 bytes per 128 columns, 192 bytes per row at d = 12288) are
    // shared by all column tiles, so with tile = blockIdx.x every XCD fetched every listed
    // row's scale lines (measured: FC2 read 1.33 x its algorithmic bytes).  Giving an XCD a
    // contiguous run of tiles makes it touch one piece of them only.
    const int tile = (nt % 8 == 0) ? (bx % 8) * (nt / 8) + bx / 8 : bx;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cl = lane & 7;                   // which 16 bytes (32 columns) of the row's line
    const int rslot = wave * 8 + (lane >> 3);  // row slot of this lane inside a load
    const int col = tile * kDown2I4Cols + cl * 32;
    const bool colok = col < d;
    const int ngroups = d / kI4Group;
    const rsrc_t wq = make_rsrc(q_down, (uint32_t)ffn * (uint32_t)(d / 2));
    const rsrc_t ws = make_rsrc(s_down, (uint32_t)ffn * (uint32_t)ngroups * 2u);

    PF_TSTAMP(3, 0);
    float acc[B][32], wsum[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        wsum[b] = 0.f;
#pragma unroll
        for (int c = 0; c < 32; ++c) acc[b][c] = 0.f;
    }

    int n = 0;
    bool have_n = false;
    for (int r0 = 0; r0 == 0 || r0 * P < n; r0 += kDown2I4RowsPerLoad * U) {
        int iv[U];
        float hv[U][B];
#pragma unroll
        for (int u = 0; u < U; ++u) {  // loads that depend on the slot number only
            const int jc = min((r0 + u * kDown2I4RowsPerLoad + rslot) * P + g, ffn - 1);
            iv[u] = idx[jc];
            load_h_slot<B>(h, jc, hv[u]);
        }
        if (!have_n) {
            n = min(max(*count_p, 0), ffn);
            have_n = true;
            PF_TSTAMP(3, 1);
        }
        uint4 w[U];
        unsigned short sc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jj = (r0 + u * kDown2I4RowsPerLoad + rslot) * P + g;
            const bool ok = jj < n && (unsigned)iv[u] < (unsigned)ffn && colok;
            w[u] = ld16_stream(wq, ok ? (uint32_t)iv[u] * (uint32_t)(d / 2) + (uint32_t)col / 2u : kOobOffset);
            sc[u] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(
                ws, ok ? (int)(((uint32_t)iv[u] * (uint32_t)ngroups + (uint32_t)col / kI4Group) * 2u)
                       : (int)kOobOffset, 0, 0);
#pragma unroll
            for (int b = 0; b < B; ++b) hv[u][b] = ok ? hv[u][b] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float scale = half_bits_to_float(sc[u]);
            const uint32_t dws[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
            float hs[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                hs[b] = hv[u][b] * scale;
                wsum[b] += hs[b];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float f[8];
                nibbles8(dws[k], f);
#pragma unroll
                for (int b = 0; b < B; ++b)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[b][8 * k + e] = fmaf(hs[b], f[e], acc[b][8 * k + e]);
            }
        }
        if (r0 == 0) PF_TSTAMP(3, 2);
    }
    PF_TSTAMP(3, 3);

#pragma unroll
    for (int b = 0; b < B; ++b) {
#pragma unroll
        for (int c = 0; c < 32; ++c) acc[b][c] = fmaf(-8.f, wsum[b], acc[b][c]);
        // halving butterfly over the 8 row slots of the wave (lane bits 5, 4, 3): a lane ends
        // with 4 of its 32 columns, summed over the 8 rows
        butterfly_halve<32, 16>(acc[b], lane);
        butterfly_halve<16, 8>(acc[b], lane);
        butterfly_halve<8, 4>(acc[b], lane);
        const int sub = ((lane >> 5) & 1) * 16 + ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4;
        *reinterpret_cast<float4 *>(&red[wave][b][cl * 32 + sub]) =
            make_float4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
    }
    __syncthreads();
    PF_TSTAMP(3, 4);
    for (int e = threadIdx.x; e < B * kDown2I4Cols; e += kDown2I4Threads) {
        const int b = e / kDown2I4Cols, c = e % kDown2I4Cols;
        const int oc = tile * kDown2I4Cols + c;
        if (oc < d) {
            float s = (g == 0 && b_down) ? b_down[oc] : 0.f;
#pragma unroll
            for (int wv = 0; wv < kDown2I4Waves; ++wv) s += red[wv][b][c];
            part[((size_t)g * B + b) * d + oc] = s;
        }
    }
    PF_TSTAMP(3, 5);
}

template <int B>
__global__ __launch_bounds__(kDown2I4Threads) void k_down2_i4(
    const uint8_t *__restrict__ q_down, const __half *__restrict__ s_down,
    const float *__restrict__ b_down, const float *__restrict__ h,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count_p, float *__restrict__ part,
    int d, int ffn)
{
    __shared__ float red[kDown2I4Waves][B][kDown2I4Cols];
    down2_i4_body<B>(red, (int)blockIdx.x, (int)gridDim.x, (int)blockIdx.y, (int)gridDim.y, q_down, s_down,
                     b_down, h, idx, count_p, part, d, ffn);
}

}  // namespace pf
