// Device helpers shared by the kernels: wave64 reductions, 16-byte weight loads,
// fp16 -> fp32 fused multiply-adds, and the LDS layout of staged activations.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pf {

constexpr int kWave = 64;      // CDNA wavefront width
constexpr int kChunk = 512;    // elements of a row one wave covers per 16-byte load (64 lanes x 8 fp16)

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the 64 lanes of a wave; every lane receives the total.
// Four DPP steps sum within each row of 16 lanes, four lane reads join the rows.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);  // row_half_mirror
    v += dpp_f32<0x140>(v);  // row_mirror
    float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (a + b) + (c + d);
}

// 16-byte streaming load (weights are read once per token: no reuse to keep in cache).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ int wave_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// A group of U 16-byte weight loads of one row, kept in registers.
template <int U>
struct WGroup {
    uint4 w[U];
};

// Issue the loads of chunks it0 .. it0+U-1 of a row of K fp16 values (lanes past the end get zeros).
template <int U>
__device__ __forceinline__ void load_group(WGroup<U> &g, const __half *__restrict__ row, int K,
                                           int it0, int lane)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = (it0 + u) * kChunk + lane * 8;
        if (c < K)
            g.w[u] = ld16_stream(row + c);
        else
            g.w[u] = make_uint4(0u, 0u, 0u, 0u);
    }
}

__device__ __forceinline__ float h_lo(uint32_t p)
{
    return __half2float(__ushort_as_half((unsigned short)(p & 0xffffu)));
}
__device__ __forceinline__ float h_hi(uint32_t p)
{
    return __half2float(__ushort_as_half((unsigned short)(p >> 16)));
}

// acc += dot(8 fp16 weights in w, 8 fp32 activations in xa|xb)
__device__ __forceinline__ float dot8(const uint4 &w, const float4 &xa, const float4 &xb, float acc)
{
    acc = fmaf(h_lo(w.x), xa.x, acc);
    acc = fmaf(h_hi(w.x), xa.y, acc);
    acc = fmaf(h_lo(w.y), xa.z, acc);
    acc = fmaf(h_hi(w.y), xa.w, acc);
    acc = fmaf(h_lo(w.z), xb.x, acc);
    acc = fmaf(h_hi(w.z), xb.y, acc);
    acc = fmaf(h_lo(w.w), xb.z, acc);
    acc = fmaf(h_hi(w.w), xb.w, acc);
    return acc;
}

// Activations staged in LDS, one token = kpad floats (kpad = chunks * 512).  Within a
// chunk the two float4 halves a lane needs are split into two 1 KB planes so that both
// ds_read_b128 of a wave are unit-stride (no bank conflicts):
//   element e of the vector -> chunk*512 + ((e & 7) >> 2) * 256 + ((e & 511) >> 3) * 4 + (e & 3)
__device__ __forceinline__ int lds_slot(int e)
{
    return (e & ~511) + (((e & 7) >> 2) << 8) + (((e & 511) >> 3) << 2) + (e & 3);
}

// Cooperative copy of v[B][K] (global fp32) into the LDS layout above, zero padded to kpad.
// K % 4 == 0.  All threads of the block call it; the caller synchronises afterwards.
template <int B>
__device__ __forceinline__ void stage_vector(float *__restrict__ xs, const float *__restrict__ v,
                                             int K, int kpad)
{
    for (int e = threadIdx.x * 4; e < kpad; e += blockDim.x * 4) {
#pragma unroll
        for (int b = 0; b < B; ++b) {
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < K) val = *reinterpret_cast<const float4 *>(v + (size_t)b * K + e);
            *reinterpret_cast<float4 *>(xs + b * kpad + lds_slot(e)) = val;
        }
    }
}

// acc[b] += dot(chunks it0..it0+U-1 of a row (already in g), staged activations of token b)
template <int B, int U>
__device__ __forceinline__ void fma_group(const WGroup<U> &g, const float *__restrict__ xs,
                                          int kpad, int it0, int nch, int lane, float (&acc)[B])
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (it0 + u < nch) {
            const float *base = xs + (it0 + u) * kChunk + lane * 4;
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const float4 xa = *reinterpret_cast<const float4 *>(base + b * kpad);
                const float4 xb = *reinterpret_cast<const float4 *>(base + b * kpad + 256);
                acc[b] = dot8(g.w[u], xa, xb, acc[b]);
            }
        }
    }
}

}  // namespace pf
