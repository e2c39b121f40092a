// Device helpers shared by the kernels: wave64 reductions, 16-byte weight loads,
// fp16 -> fp32 fused multiply-adds, and the LDS layout of staged activations.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pf {

constexpr int kWave = 64;      // CDNA wavefront width
constexpr int kChunk = 512;    // elements of a row one wave covers per 16-byte load (64 lanes x 8 fp16)

// FC1 outputs are kept slot-major, h[list slot][token] with this many floats per slot, so that
// FC2 fetches all tokens of a slot with one or two vector loads.
constexpr __host__ __device__ int h_stride(int B) { return B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : 8; }

// The hs floats of slot j (hs = 1, 2, 4 or 8) into hv[0 .. B).
template <int B>
__device__ __forceinline__ void load_h_slot(const float *__restrict__ h, int j, float (&hv)[B])
{
    constexpr int HS = h_stride(B);
    const float *p = h + (size_t)j * HS;
    float t[HS];
    if (HS == 1) {
        t[0] = p[0];
    } else if (HS == 2) {
        const float2 a = *reinterpret_cast<const float2 *>(p);
        t[0] = a.x;
        t[HS > 1 ? 1 : 0] = a.y;
    } else {
#pragma unroll
        for (int q = 0; q < HS / 4; ++q) {
            const float4 a = *reinterpret_cast<const float4 *>(p + 4 * q);
            t[(4 * q + 0) % HS] = a.x;
            t[(4 * q + 1) % HS] = a.y;
            t[(4 * q + 2) % HS] = a.z;
            t[(4 * q + 3) % HS] = a.w;
        }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) hv[b] = t[b];
}

// Phase timestamps for kernel tuning, compiled in only with -DPF_TRACE: thread 0 of a block
// stores the 100 MHz wall clock at a few program points into a host-provided buffer.
#ifdef PF_TRACE
__constant__ unsigned long long *g_pf_trace = nullptr;  // [slot][4096 blocks][8 stamps]
#define PF_TSTAMP(slot, k)                                                                   \
    do {                                                                                     \
        if (threadIdx.x == 0 && g_pf_trace && blockIdx.x < 4096)                             \
            g_pf_trace[((size_t)(slot) * 4096 + blockIdx.x) * 8 + (k)] = wall_clock64();     \
    } while (0)
// latest time any wave of the block passes this point (lane 0 of every wave)
#define PF_TSTAMP_MAX(slot, k)                                                               \
    do {                                                                                     \
        if ((threadIdx.x & 63) == 0 && g_pf_trace && blockIdx.x < 4096)                      \
            atomicMax(&g_pf_trace[((size_t)(slot) * 4096 + blockIdx.x) * 8 + (k)],           \
                      (unsigned long long)wall_clock64());                                   \
    } while (0)
#else
#define PF_TSTAMP(slot, k) \
    do {                   \
    } while (0)
#define PF_TSTAMP_MAX(slot, k) \
    do {                       \
    } while (0)
#endif

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

// One exchange of a halving butterfly over lane bit D (8, 16 or 32): of its 2 * NV values a
// lane keeps the
// lower NV (bit clear) or the upper NV (bit set), adds the partner's copies of the same
// columns and gives the rest away.  D and NV are compile-time so the values stay in
// registers under fixed names.
template <int D, int NV, int N>
__device__ __forceinline__ void butterfly_halve(float (&a)[N], int lane)
{
    const bool upper = (lane & D) != 0;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const float send = upper ? a[k] : a[k + NV];
        const float keep = upper ? a[k + NV] : a[k];
        const float got = (D == 8) ? dpp_f32<0x128>(send)  // row_ror:8 = lane ^ 8 in a row of 16
                                   : __shfl_xor(send, D, 64);
        a[k] = keep + got;
    }
}

// Sign bit (0 or 0x80000000) the stack glue gives column c of batch row b: none for row 0,
// otherwise the top bit of a fixed integer mix of (b, c).  It decorrelates the rows of a
// batch, which the always-active neurons would otherwise align within a few layers.
__device__ __forceinline__ uint32_t glue_sign_bit(uint32_t b, uint32_t c)
{
    if (b == 0) return 0u;
    uint32_t h = b * 0x9E3779B1u + c * 0x85EBCA77u + 0x165667B1u;
    h ^= h >> 15;
    h *= 0x2C1B3C6Du;
    h ^= h >> 12;
    h *= 0x297A2D39u;
    h ^= h >> 15;
    return h & 0x80000000u;
}

__device__ __forceinline__ float4 glue_signed(float4 v, uint32_t b, uint32_t c0)
{
    return make_float4(__uint_as_float(__float_as_uint(v.x) ^ glue_sign_bit(b, c0)),
                       __uint_as_float(__float_as_uint(v.y) ^ glue_sign_bit(b, c0 + 1)),
                       __uint_as_float(__float_as_uint(v.z) ^ glue_sign_bit(b, c0 + 2)),
                       __uint_as_float(__float_as_uint(v.w) ^ glue_sign_bit(b, c0 + 3)));
}

// Buffer resources: every weight and activation load goes through a raw buffer descriptor
// (base, byte size) held in scalar registers.  Lanes whose offset lies past the end get
// zeros from the hardware, so loads need no branches -- which also lets the compiler count
// outstanding loads exactly and start the FMAs on the first chunk while later ones are
// still in flight.  Sizes are 32-bit: a matrix must stay below 4 GiB.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr uint32_t kOobOffset = 0xfffffff0u;  // an offset past any buffer: the load returns 0

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// 16-byte streaming load (weights are read once per token: no reuse to keep in cache).
__device__ __forceinline__ uint4 ld16_stream(rsrc_t r, uint32_t byte_off)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 2);  // nt
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte load of fp32 activations (shared by many workgroups: keep it cacheable).
__device__ __forceinline__ float4 ld16_f32(rsrc_t r, uint32_t byte_off)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
    // (element-wise __builtin_bit_cast on the vector's components is miscompiled into a
    // splat of the first dword by this toolchain; __uint_as_float is not)
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z),
                       __uint_as_float(v.w));
}

// 16-byte cacheable load, raw bits.
__device__ __forceinline__ uint4 ld16_cached(rsrc_t r, uint32_t byte_off)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// fp32 -> fp16 hi (rounded) + fp16 lo (residual): v = hi + lo to 2^-21 |v|.  The matrix-core
// kernels multiply fp16 weights by both halves, so activations stay fp32-exact.
__device__ __forceinline__ void split_f32(float v, _Float16 &hi, _Float16 &lo)
{
    hi = (_Float16)v;
    lo = (_Float16)(v - (float)hi);
}

__device__ __forceinline__ int wave_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Descriptor of row `i` (wave-uniform) of a neuron-major fp16 matrix with rows of K values;
// an invalid row gets an empty buffer, i.e. reads as zeros.
__device__ __forceinline__ rsrc_t row_rsrc(const __half *base, int i, int K, bool valid)
{
    return make_rsrc(base + (size_t)i * K, valid ? (uint32_t)K * 2u : 0u);
}

// A group of U 16-byte weight loads of one row, kept in registers.
template <int U>
struct WGroup {
    uint4 w[U];
};

// Issue the loads of chunks it0 .. it0+U-1 of a row (lanes and chunks past the end get zeros).
template <int U>
__device__ __forceinline__ void load_group(WGroup<U> &g, rsrc_t row, int it0, int lane)
{
#pragma unroll
    for (int u = 0; u < U; ++u)
        g.w[u] = ld16_stream(row, (uint32_t)((it0 + u) * kChunk + lane * 8) * 2u);
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

// The same idea for a lane that consumes EPL consecutive elements per 16-byte weight load
// (8 for fp16, 32 for int4): a chunk is 64 * EPL elements, split into EPL / 4 planes of 256
// floats, plane p holding float4 number p of every lane.
template <int EPL>
__device__ __forceinline__ int lds_slot_epl(int e)
{
    constexpr int W = 64 * EPL;
    const int r = e & (W - 1), q = r & (EPL - 1);
    return (e & ~(W - 1)) + ((q >> 2) << 8) + ((r / EPL) << 2) + (q & 3);
}

// Cooperative copy of v[B][K] (global fp32) into the LDS layout above, zero padded to kpad,
// in two phases so that the caller can put other work between them: stage_issue puts the
// global loads of the first pass in flight (S strides x B tokens per thread, kept in
// registers), stage_commit writes them to LDS and, for vectors longer than one pass, copies
// the rest.  Vector memory returns in issue order, so issuing these few loads BEFORE the
// weight loads lets the workgroup pass its barrier as soon as the activations are in, and
// the FMAs then consume weight chunks as they arrive.  K % 4 == 0.  All threads of the
// block call both; the caller synchronises after stage_commit.  S = strides per pass.
// The LDS image is followed by 4 floats of scrap: a thread whose stride lies past the vector
// writes there, so the commit has no branch the compiler could sink the loads into.
constexpr int kStageScrap = 4;

template <int B, int S>
struct Staged {
    float4 val[S][B];
};

template <int B, int S>
__device__ __forceinline__ void stage_issue(Staged<B, S> &st, const float *__restrict__ v, int K)
{
    const rsrc_t r = make_rsrc(v, (uint32_t)B * (uint32_t)K * 4u);
    const int step = blockDim.x * 4;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int e = threadIdx.x * 4 + s * step;
#pragma unroll
        for (int b = 0; b < B; ++b)
            st.val[s][b] = ld16_f32(r, e < K ? (uint32_t)(b * K + e) * 4u : kOobOffset);
    }
}

template <int B, int S, int EPL = 8>
__device__ __forceinline__ void stage_commit(const Staged<B, S> &st, float *__restrict__ xs,
                                             const float *__restrict__ v, int K, int kpad)
{
    const int step = blockDim.x * 4;
    const int scrap = B * kpad;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int e = threadIdx.x * 4 + s * step;
#pragma unroll
        for (int b = 0; b < B; ++b)
            *reinterpret_cast<float4 *>(xs + (e < kpad ? b * kpad + lds_slot_epl<EPL>(e) : scrap)) =
                st.val[s][b];
    }
    const rsrc_t r = make_rsrc(v, (uint32_t)B * (uint32_t)K * 4u);
    for (int e0 = threadIdx.x * 4 + S * step; e0 < kpad; e0 += step * S) {  // longer vectors
        float4 val[S][B];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int e = e0 + s * step;
#pragma unroll
            for (int b = 0; b < B; ++b)
                val[s][b] = ld16_f32(r, e < K ? (uint32_t)(b * K + e) * 4u : kOobOffset);
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int e = e0 + s * step;
#pragma unroll
            for (int b = 0; b < B; ++b)
                *reinterpret_cast<float4 *>(xs + (e < kpad ? b * kpad + lds_slot_epl<EPL>(e) : scrap)) =
                    val[s][b];
        }
    }
}

// The same LDS image written by global -> LDS loads that bypass the registers
// (buffer_load_dwordx4 ... lds): a wave instruction moves 64 x 16 bytes to 1 KB of contiguous
// LDS, and plane p of a chunk is exactly float4 number p of every lane, so one instruction
// fills one plane.  Nothing is held in registers, so the whole image of any length and batch
// is in flight at once (the register form needs one round trip per pass of a long vector).
// Offsets past the vector read as zeros, which pads the image.  The caller synchronises
// the block before reading xs.
typedef __attribute__((address_space(3))) void *lds_ptr_t;

template <int B, int EPL = 8>
__device__ __forceinline__ void stage_dma(float *__restrict__ xs, const float *__restrict__ v, int K,
                                          int kpad)
{
    constexpr int W = 64 * EPL, PL = EPL / 4;  // chunk width, planes per chunk
    const rsrc_t r = make_rsrc(v, (uint32_t)B * (uint32_t)K * 4u);
    const int lane = threadIdx.x & 63;
    const int wave = wave_uniform(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
    const int nplanes = (kpad / W) * PL;  // per token; plane q lies at float offset 256 * q
    for (int q = wave; q < B * nplanes; q += nwaves) {
        const int b = q / nplanes, pq = q - b * nplanes;
        const int e = (pq / PL) * W + lane * EPL + 4 * (pq % PL);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            r, (lds_ptr_t)(xs + (size_t)b * kpad + (size_t)pq * 256), 16,
            e < K ? (int)((uint32_t)(b * K + e) * 4u) : (int)kOobOffset, 0, 0, 0);
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
