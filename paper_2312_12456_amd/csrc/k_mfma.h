// FC1 over the listed neurons for a batch of tokens as a matrix-core contraction
// (PowerInfer Sec. 8.2, batching: the active set is the union over the batch, so the gathered
// rows form a dense [k x d] block that multiplies [d x B]).  At batch 1 the row-sparse GEMV is
// pure HBM streaming; from a few tokens on, B FMAs and B LDS reads per weight make the vector
// path the limiter before HBM saturates, and v_mfma_f32_16x16x32_f16 does the same work in a
// fraction of the issue slots.  M = 16 gathered rows, N = 16 batch columns (tokens >= B read
// as zero), K = 32 elements of d per instruction.
// Operand layout (verified on the device): lane l supplies A[row l%16][8 halfs from k = 8*(l/16)]
// and B[same 8 k][col l%16]; it receives C[rows 4*(l/16) .. +3][col l%16].
// Activations stay fp32-exact: x is split into fp16 hi + fp16 lo (x = hi + lo to 2^-21) and
// each step issues two MFMAs.
//
// Weights do not go to the registers in operand order: a load in which each quarter-wave
// touches 16 different rows costs the memory pipeline 16 line look-ups for 256 bytes.
// Instead they go global -> LDS (buffer_load ... lds) in instructions that read 512
// contiguous bytes of each of two rows, and the A operands are read back from LDS.
#pragma once
#include "dev_util.h"
#include "k_predict.h"

namespace pf {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4v_t __attribute__((ext_vector_type(4)));

constexpr int kMfmaThreads = 512;
constexpr int kMfmaWaves = kMfmaThreads / kWave;  // the waves of a block split K between them
// LDS image of one chunk of one matrix in a wave's slot: R rows x KC halfs = 8 KB, for
// R = 32 rows (two MFMA tiles) x 128 elements or R = 16 rows x 256 elements.  The fewer rows a
// block has, the longer its chunks: the bytes in flight per wave stay the same.
constexpr int kMfmaSlotBytes = 8192;

// dynamic LDS of k_up_mfma: [mask words | prefix] when compacting itself, then one slot per
// wave and matrix
inline size_t up_mfma_mask_bytes(int ffn, bool from_mask)
{
    if (!from_mask) return 0;
    const size_t nwords = (size_t)ffn / 64;
    return ((nwords * 8 + (nwords + 1) * 4 + 63) / 64) * 64;
}
inline size_t up_mfma_lds_bytes(int ffn, bool from_mask, bool gated)
{
    return up_mfma_mask_bytes(ffn, from_mask) + (size_t)kMfmaWaves * (gated ? 2 : 1) * kMfmaSlotBytes;
}

union Half8Bits {
    uint4 u;
    half8_t h;
};

// The B operand (activations) of one K step for a lane: 8 consecutive elements of its token,
// as loaded.  From fp32 activations: elements 0-3 and 4-7, split into fp16 hi (rounded) + lo
// (residual) when used.  From split planes (XS; written by the glue kernels or k_split): the 8
// hi halfs and the 8 lo halfs, used as they are -- the split then costs the matrix-core
// kernels nothing (it was 40 vector operations per K step in every workgroup).
struct XRaw {
    uint4 a, b;
};

// elem = index of the lane's first element in [B][K] (ok: the lane has a token and k < K);
// plane_bytes = distance between the hi and lo planes.
template <bool XS>
__device__ __forceinline__ XRaw load_xraw(rsrc_t xr, uint32_t elem, bool ok, uint32_t plane_bytes)
{
    XRaw r;
    if (XS) {
        r.a = ld16_cached(xr, ok ? elem * 2u : kOobOffset);
        r.b = ld16_cached(xr, ok ? elem * 2u + plane_bytes : kOobOffset);
    } else {
        r.a = ld16_cached(xr, ok ? elem * 4u : kOobOffset);
        r.b = ld16_cached(xr, ok ? elem * 4u + 16u : kOobOffset);
    }
    return r;
}

template <bool XS>
__device__ __forceinline__ void finish_x(const XRaw &r, half8_t &hi, half8_t &lo)
{
    if (XS) {
        Half8Bits h, l;
        h.u = r.a;
        l.u = r.b;
        hi = h.h;
        lo = l.h;
    } else {
        const float v[8] = {__uint_as_float(r.a.x), __uint_as_float(r.a.y), __uint_as_float(r.a.z),
                            __uint_as_float(r.a.w), __uint_as_float(r.b.x), __uint_as_float(r.b.y),
                            __uint_as_float(r.b.z), __uint_as_float(r.b.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            _Float16 h, l;
            split_f32(v[e], h, l);
            hi[e] = h;
            lo[e] = l;
        }
    }
}

// Put chunk `c` (KC = 4096 / R elements) of the R rows of a pass in flight towards `slot`.  One
// instruction moves 1 KB: 2 KC bytes (whole lines) of each of 512 / KC rows.  Row r stores
// 16-byte piece p at position p ^ (r & 7), so that the 8 rows a group of 8 lanes reads together
// (same piece) fall into 8 different 16-byte bank groups.  rowoff[i] = byte offset of this
// lane's row of instruction i in the matrix (kOobOffset: no row).
template <int R>
__device__ __forceinline__ void mfma_issue_chunk(rsrc_t w, char *slot, const uint32_t (&rowoff)[8],
                                                 int c, int d, int lane)
{
    constexpr int KC = kMfmaSlotBytes / 2 / R;
    constexpr int RPI = 512 / KC, LPR = 64 / RPI;  // rows per instruction, lanes per row
    const int rin = lane / LPR, p = lane % LPR;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int piece = p ^ ((RPI * i + rin) & 7);
        const int k = c * KC + piece * 8;
        const uint32_t off = (k < d && rowoff[i] != kOobOffset) ? rowoff[i] + (uint32_t)k * 2u : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(w, (lds_ptr_t)(slot + i * 1024), 16, (int)off, 0, 0, 0);
    }
}

// What the passes of a block need from the kernel around them.
struct UpMfmaArgs {
    rsrc_t wu, wg, xr;
    const float *b_up;
    const int32_t *idx_in;
    int32_t *idx_out;
    float *h;
    const uint64_t *words_lds;
    const uint32_t *pre_lds;
    char *slots;
    int *irow;
    float *brow;
    int B, hs, d, ffn, n, nwords, top_step, j_begin, j_end;
    float up_floor;  // gated forms: lower clamp of the up branch (-infinity, or 0 for dReLU)
};

// The list slots [j_begin, j_end) of a block in passes of R rows (R / 16 MFMA tiles).
template <int R, int ACT, bool FROM_MASK, bool XS>
__device__ __forceinline__ void up_mfma_passes(const UpMfmaArgs &a)
{
    constexpr bool GATED = (ACT == 1);
    constexpr int NM = GATED ? 2 : 1;
    constexpr int T = R / 16;                      // tiles per pass
    constexpr int KC = kMfmaSlotBytes / 2 / R;     // elements of d per chunk
    constexpr int STEPS = KC / 32;                 // MFMA K steps per chunk
    constexpr int RPI = 512 / KC, LPR = 64 / RPI;
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int row16 = lane & 15, kg = lane >> 4;
    char *slot = a.slots + (size_t)wave * NM * kMfmaSlotBytes;  // this wave's: up, then gate
    const int d = a.d, n = a.n;
    const bool xlane = row16 < a.B;  // this lane supplies a token's B operands
    const uint32_t xelem = (uint32_t)row16 * (uint32_t)d + (uint32_t)kg * 8u;
    const uint32_t xplane = (uint32_t)a.B * (uint32_t)d * 2u;
    const int nchunks = (d + KC - 1) / KC;

    for (int j0 = a.j_begin; j0 < a.j_end; j0 += R) {
        // list slot -> neuron id for the rows whose A operands this lane supplies (one per tile)
        int jr[T], ir[T];
#pragma unroll
        for (int t = 0; t < T; ++t) jr[t] = j0 + 16 * t + row16 < a.j_end ? j0 + 16 * t + row16 : n;
        if (FROM_MASK) {
            select_set_bits_lane<T>(a.words_lds, a.pre_lds, a.nwords, a.top_step, n, jr, ir);
        } else {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                ir[t] = jr[t] < n ? a.idx_in[jr[t]] : -1;
                if ((unsigned)ir[t] >= (unsigned)a.ffn) ir[t] = -1;
            }
        }
        // the rows' biases are fetched here and parked in LDS only after the chunk loop, so that
        // wave 0 does not wait for them before it puts its first chunk in flight
        float bpre[T];
#pragma unroll
        for (int t = 0; t < T; ++t) bpre[t] = 0.f;
        if (wave == 0 && kg == 0) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                a.irow[16 * t + row16] = ir[t];
                if (a.b_up != nullptr && ir[t] >= 0) bpre[t] = a.b_up[ir[t]];
                if (FROM_MASK && ir[t] >= 0) a.idx_out[jr[t]] = ir[t];
            }
        }
        // byte offsets of the rows this lane fetches: instruction i -> row RPI * i + lane / LPR
        uint32_t rowoff[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = RPI * i + lane / LPR;
            int id = -1;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int v = __shfl(ir[t], row & 15, 64);
                if ((row >> 4) == t) id = v;
            }
            rowoff[i] = id >= 0 ? (uint32_t)id * (uint32_t)d * 2u : kOobOffset;
        }
        if (j0 == a.j_begin) PF_TSTAMP(2, 2);

        float4v_t cu[T], cg[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            cu[t] = (float4v_t){0.f, 0.f, 0.f, 0.f};
            cg[t] = (float4v_t){0.f, 0.f, 0.f, 0.f};
        }
        const int ntile = min(T, (a.j_end - j0 + 15) >> 4);  // block-uniform: tiles with rows
        int c = wave;
        if (c < nchunks) {
            mfma_issue_chunk<R>(a.wu, slot, rowoff, c, d, lane);
            if (GATED) mfma_issue_chunk<R>(a.wg, slot + kMfmaSlotBytes, rowoff, c, d, lane);
        }
        while (c < nchunks) {  // wave-uniform
            XRaw xv[STEPS];
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const int k = c * KC + s * 32;
                xv[s] = load_xraw<XS>(a.xr, xelem + (uint32_t)k, xlane && k < d, xplane);
            }
            Half8Bits au[T][STEPS], ag[T][STEPS];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if (t >= ntile) break;
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    const int row = 16 * t + row16;
                    const int at = row * (KC * 2) + ((4 * s + kg) ^ (row & 7)) * 16;
                    au[t][s].u = *reinterpret_cast<const uint4 *>(slot + at);
                    if (GATED) ag[t][s].u = *reinterpret_cast<const uint4 *>(slot + kMfmaSlotBytes + at);
                }
            }
            const int cn = c + kMfmaWaves;
            if (cn < nchunks) {  // refill the slot once its contents are in the registers
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
                mfma_issue_chunk<R>(a.wu, slot, rowoff, cn, d, lane);
                if (GATED) mfma_issue_chunk<R>(a.wg, slot + kMfmaSlotBytes, rowoff, cn, d, lane);
            }
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                half8_t hi, lo;
                finish_x<XS>(xv[s], hi, lo);
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    if (t >= ntile) break;
                    cu[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(au[t][s].h, hi, cu[t], 0, 0, 0);
                    cu[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(au[t][s].h, lo, cu[t], 0, 0, 0);
                    if (GATED) {
                        cg[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ag[t][s].h, hi, cg[t], 0, 0, 0);
                        cg[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ag[t][s].h, lo, cg[t], 0, 0, 0);
                    }
                }
            }
            c = cn;
        }
        if (j0 == a.j_begin) PF_TSTAMP(2, 3);
        // this lane holds C[row 4*kg + e][col row16] of its chunks, per tile; the wave's slot
        // is free now: [tile][up | gate][256]
        float *ctile = reinterpret_cast<float *>(slot);
        if (wave == 0 && kg == 0) {
#pragma unroll
            for (int t = 0; t < T; ++t) a.brow[16 * t + row16] = bpre[t];
        }
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ctile[(t * 2) * 256 + (kg * 4 + e) * 16 + row16] = cu[t][e];
                if (GATED) ctile[(t * 2 + 1) * 256 + (kg * 4 + e) * 16 + row16] = cg[t][e];
            }
        __syncthreads();
        if ((int)threadIdx.x < T * 256) {
            const int t = threadIdx.x >> 8, e = threadIdx.x & 255;
            const int row = 16 * t + (e >> 4), colb = e & 15;
            float su = 0.f, sg = 0.f;
#pragma unroll
            for (int wv = 0; wv < kMfmaWaves; ++wv) {
                const float *ct = reinterpret_cast<const float *>(a.slots + (size_t)wv * NM * kMfmaSlotBytes);
                su += ct[(t * 2) * 256 + e];
                if (GATED) sg += ct[(t * 2 + 1) * 256 + e];
            }
            const int i = a.irow[row];
            const int j = j0 + row;
            const float bias = a.brow[row];  // fetched when the row was selected
            const float v = GATED ? fmaxf(sg + bias, 0.f) * fmaxf(su, a.up_floor) : fmaxf(su + bias, 0.f);
            if (colb < a.B && j < a.j_end) a.h[(size_t)j * a.hs + colb] = i >= 0 ? v : 0.f;
        }
        __syncthreads();
        if (j0 == a.j_begin) PF_TSTAMP(2, 4);
    }
}

// grid = G blocks; block b owns the list slots [b * rpb, (b + 1) * rpb), rpb = ceil(n / G): an
// even share of the rows for every block (with whole tiles dealt round-robin the CUs that get
// one tile more than the others set the kernel's time).  A share of at most 16 rows is done
// as one 16-row tile with 256-element chunks, a larger one in passes of 32 rows (two tiles)
// with 128-element chunks.  The 8 waves of a block take the chunks round-robin (wave w:
// chunks w, w + 8, ...) for the same rows and their C tiles are added in LDS in wave order.
// d % 32 == 0, B <= 16.
// The body takes its block number and the number of blocks of its role explicitly, so that a
// launch can run it in a range of its blocks beside another role.  Its pointer parameters carry
// no restrict qualifier on purpose: a wave reads back from LDS what its own global -> LDS loads
// wrote, and the wait between the two is the compiler's, which places it only while it takes
// the two accesses to alias.  Inlining a function with restrict parameters tags its accesses
// with no-alias scopes, and with those the waits were dropped (wrong sums on the device).
// XS: x points at the split planes of the activations (see XRaw) instead of fp32 values.
template <int ACT, bool FROM_MASK, bool XS>
__device__ __forceinline__ void up_mfma_body(
    uint64_t *dyn_lds64, uint32_t *wave_tot, int *irow, float *brow, const int bid, const int nblocks,
    const __half *w_up, const __half *w_gate,
    const float *b_up, const void *x, int B,
    const int32_t *idx_in, const int32_t *count_in,
    const uint64_t *mask_words, int32_t *idx_out,
    int32_t *count_out, float *h, int hs, int d, int ffn, float up_floor)
{
    constexpr bool GATED = (ACT == 1);
    const int nwords = ffn / 64;
    uint64_t *words_lds = dyn_lds64;
    uint32_t *pre_lds = reinterpret_cast<uint32_t *>(words_lds + (FROM_MASK ? nwords : 0));
    const size_t mask_bytes =
        FROM_MASK ? (((size_t)nwords * 8 + ((size_t)nwords + 1) * 4 + 63) / 64) * 64 : 0;

    PF_TSTAMP(2, 0);
    int n;
    int top_step = 1;
    if (FROM_MASK) {
        n = (int)mask_prefix<kMfmaThreads>(mask_words, nwords, words_lds, pre_lds, wave_tot);
        if (bid == 0 && threadIdx.x == 0) *count_out = n;
        while (top_step * 2 < nwords) top_step *= 2;
    } else {
        n = min(max(*count_in, 0), ffn);
    }
    UpMfmaArgs a;
    a.wu = make_rsrc(w_up, (uint32_t)ffn * (uint32_t)d * 2u);
    a.wg = make_rsrc(GATED ? w_gate : w_up, (uint32_t)ffn * (uint32_t)d * 2u);
    a.xr = make_rsrc(x, (uint32_t)B * (uint32_t)d * 4u);
    a.b_up = b_up;
    a.idx_in = idx_in;
    a.idx_out = idx_out;
    a.h = h;
    a.words_lds = words_lds;
    a.pre_lds = pre_lds;
    a.slots = reinterpret_cast<char *>(dyn_lds64) + mask_bytes;
    a.irow = irow;
    a.brow = brow;
    a.B = B;
    a.hs = hs;
    a.d = d;
    a.ffn = ffn;
    a.n = n;
    a.nwords = nwords;
    a.top_step = top_step;
    a.up_floor = up_floor;
    const int rpb = (n + nblocks - 1) / nblocks;
    a.j_begin = min(n, bid * rpb);
    a.j_end = min(n, a.j_begin + rpb);
    PF_TSTAMP(2, 1);
    if (rpb <= 16)
        up_mfma_passes<16, ACT, FROM_MASK, XS>(a);
    else
        up_mfma_passes<32, ACT, FROM_MASK, XS>(a);
    PF_TSTAMP(2, 5);
}

template <int ACT, bool FROM_MASK, bool XS>
__global__ __launch_bounds__(kMfmaThreads) void k_up_mfma(
    const __half *__restrict__ w_up, const __half *__restrict__ w_gate,
    const float *__restrict__ b_up, const void *__restrict__ x, int B,
    const int32_t *__restrict__ idx_in, const int32_t *__restrict__ count_in,
    const uint64_t *__restrict__ mask_words, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out, float *__restrict__ h, int hs, int d, int ffn, float up_floor)
{
    extern __shared__ uint64_t dyn_lds64[];
    __shared__ uint32_t wave_tot[kMfmaWaves];
    __shared__ int irow[32];
    __shared__ float brow[32];
    up_mfma_body<ACT, FROM_MASK, XS>(dyn_lds64, wave_tot, irow, brow, (int)blockIdx.x, (int)gridDim.x, w_up, w_gate,
                                 b_up, x, B, idx_in, count_in, mask_words, idx_out, count_out, h, hs, d,
                                 ffn, up_floor);
}

// ---------------------------------------------------------------------------------------
// The predictor's two layers for a batch on the matrix cores (PowerInfer Sec. 5.1): dense
// rows, so no list and no row gather.  Block b owns rows [R b, R (b + 1)); its 8 waves take
// the chunks of KC elements of the row length K round-robin, each through its own 8 KB LDS
// slot of R rows x KC halfs filled by global -> LDS loads that read 2 KC bytes of each of
// 512 / KC rows per instruction (whole lines).  Row r keeps 16-byte piece p at position
// p ^ (r & 7): the 8 rows a group of 8 lanes reads together (same piece) then fall into 8
// different bank groups.  v[B][K] are the activations (fp32, split into fp16 hi + lo).
//   EPI 0 (hidden layer, R = 8, KC = 512: few rows, so few and long chunks; rows 8..15 of
//          the MFMA tile are zeros):               out[b][row] = ReLU(sum)          out = t
//   EPI 1 (output layer, R = 64 = one mask word, KC = 64): logit = sum + p_bias[row];
//          scores[b][row] = sigmoid(logit) if asked; bit `row` of mask word b = any_b(logit > thr)
constexpr int kRowsMfmaSlotBytes = 8192;  // R rows x 2 KC bytes

template <int R, int KC>
__device__ __forceinline__ void rows_mfma_issue(rsrc_t w, char *slot, uint32_t row0_off, uint32_t row_bytes,
                                                int nrows_left, int c, int K, int lane)
{
    constexpr int RPI = 512 / KC;  // rows per instruction
    constexpr int LPR = 64 / RPI;  // lanes (16-byte pieces) per row
    constexpr int NI = R / RPI;    // instructions per chunk
    const int rin = lane / LPR, p = lane % LPR;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = RPI * i + rin;
        const int piece = p ^ (row & 7);
        const int k = c * KC + piece * 8;
        const uint32_t off = (k < K && row < nrows_left) ? row0_off + (uint32_t)row * row_bytes + (uint32_t)k * 2u
                                                         : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(w, (lds_ptr_t)(slot + i * 1024), 16, (int)off, 0, 0, 0);
    }
}

// Body: bid0 = the block's number within its role, logit_s = [16][16 * tiles] floats of LDS.
// No restrict qualifiers, for the same reason as in up_mfma_body.
// XS: v points at the split planes of the activations (see XRaw) instead of fp32 values.
template <int R, int KC, int EPI, bool XS>
__device__ __forceinline__ void rows_mfma_body(
    uint64_t *dyn_lds64, float (*logit_s)[16 * ((R + 15) / 16)], const int bid0,
    const __half *w, const void *v, int B, int K, int nrows,
    const float *p_bias, float thr_logit, float *out,
    uint64_t *mask_words, int first_word)
{
    constexpr int T = (R + 15) / 16;  // MFMA tiles per block
    static_assert(R * KC * 2 == kRowsMfmaSlotBytes, "slot size");
    static_assert(EPI == 0 || R == 64, "the output layer writes one mask word per block");
    constexpr int STEPS = KC / 32;                // MFMA K steps per chunk
    constexpr int SB = STEPS < 4 ? STEPS : 4;     // ... of which this many share a round of loads
    const int lane = threadIdx.x & 63, wave = wave_uniform(threadIdx.x >> 6);
    const int row16 = lane & 15, kg = lane >> 4;
    char *slots = reinterpret_cast<char *>(dyn_lds64);
    char *slot = slots + (size_t)wave * kRowsMfmaSlotBytes;
    // EPI 1: the launch covers the rows from 64 * first_word on (always-on prefix skipped)
    const int blk = bid0 + (EPI == 1 ? first_word : 0);
    const int r0 = blk * R;
    const int nleft = nrows - r0;  // rows of this block that exist (>= 1)
    if (EPI == 1 && bid0 == 0 && first_word > 0) {
        for (int w = threadIdx.x; w < first_word; w += kMfmaThreads) mask_words[w] = ~0ull;
        if (out != nullptr)
            for (int e = threadIdx.x; e < B * first_word * 64; e += kMfmaThreads)
                out[(size_t)(e / (first_word * 64)) * nrows + e % (first_word * 64)] = 1.f;
    }
    const rsrc_t wr = make_rsrc(w, (uint32_t)nrows * (uint32_t)K * 2u);
    const rsrc_t vr = make_rsrc(v, (uint32_t)B * (uint32_t)K * 4u);
    const uint32_t row_bytes = (uint32_t)K * 2u, row0_off = (uint32_t)r0 * row_bytes;
    const bool vlane = row16 < B;  // this lane supplies a token's B operands
    const uint32_t velem = (uint32_t)row16 * (uint32_t)K + (uint32_t)kg * 8u;
    const uint32_t vplane = (uint32_t)B * (uint32_t)K * 2u;
    const int nchunks = (K + KC - 1) / KC;

    PF_TSTAMP(EPI, 0);
    float4v_t acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = (float4v_t){0.f, 0.f, 0.f, 0.f};
    // activations of sub-block j (SB K steps) of chunk ch into one of two register buffers: they
    // are fetched one sub-block ahead of their use, so that their L2 round trip overlaps the
    // matrix work of the sub-block before
    constexpr int NSB = STEPS / SB;
    XRaw xv[2][SB];
    auto load_x = [&](int ch, int j, XRaw (&px)[SB]) {
#pragma unroll
        for (int s = 0; s < SB; ++s) {
            const int k = ch * KC + (j * SB + s) * 32;
            px[s] = load_xraw<XS>(vr, velem + (uint32_t)k, vlane && k < K, vplane);
        }
    };
    int c = wave;
    if (c < nchunks) {
        rows_mfma_issue<R, KC>(wr, slot, row0_off, row_bytes, nleft, c, K, lane);
        load_x(c, 0, xv[0]);
    }
    // output layer: the biases of the rows this thread finishes, fetched behind the first chunk
    // (read only after the chunk loop: their latency is off the block's tail)
    constexpr int NE = (T * 256 + kMfmaThreads - 1) / kMfmaThreads;
    float bias_pre[NE];
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        const int e = (int)threadIdx.x + i * kMfmaThreads;
        const int row = (e >> 8) * 16 + ((e >> 4) & 15);
        bias_pre[i] = (EPI == 1 && p_bias != nullptr && e < T * 256) ? p_bias[r0 + row] : 0.f;
    }
    while (c < nchunks) {  // wave-uniform
        const int cn = c + kMfmaWaves;
#pragma unroll
        for (int j = 0; j < NSB; ++j) {
            const int cur = j & 1, nxt = cur ^ 1;
            Half8Bits a[T][SB];
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int s = 0; s < SB; ++s) {
                    const int row = 16 * t + row16;
                    a[t][s].u = make_uint4(0u, 0u, 0u, 0u);
                    if (R >= 16 || row < R)
                        a[t][s].u = *reinterpret_cast<const uint4 *>(
                            slot + row * (KC * 2) + ((4 * (j * SB + s) + kg) ^ (row & 7)) * 16);
                }
            if (j + 1 < NSB) {
                load_x(c, j + 1, xv[nxt]);
            } else if (cn < nchunks) {  // last sub-block: refill the slot, fetch the next chunk's x
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the slot is all in registers
                rows_mfma_issue<R, KC>(wr, slot, row0_off, row_bytes, nleft, cn, K, lane);
                load_x(cn, 0, xv[nxt]);
            }
#pragma unroll
            for (int s = 0; s < SB; ++s) {
                half8_t hi, lo;
                finish_x<XS>(xv[cur][s], hi, lo);
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[t][s].h, hi, acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[t][s].h, lo, acc[t], 0, 0, 0);
                }
            }
        }
        if (NSB & 1) {  // the next chunk starts from buffer 0 again
#pragma unroll
            for (int s = 0; s < SB; ++s) xv[0][s] = xv[1][s];
        }
        c = cn;
    }
    PF_TSTAMP(EPI, 1);
    // this lane holds C[tile t][row 4*kg + e][col row16] of its chunks; the slot is free now
    float *ctile = reinterpret_cast<float *>(slot);
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) ctile[t * 256 + (kg * 4 + e) * 16 + row16] = acc[t][e];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        const int e = (int)threadIdx.x + i * kMfmaThreads;
        if (e >= T * 256) break;
        const int row = (e >> 8) * 16 + ((e >> 4) & 15), col = e & 15;
        float sum = 0.f;
#pragma unroll
        for (int wv = 0; wv < kMfmaWaves; ++wv)
            sum += reinterpret_cast<const float *>(slots + (size_t)wv * kRowsMfmaSlotBytes)[e];
        if (EPI == 0) {
            if (col < B && row < R && row < nleft) out[(size_t)col * nrows + r0 + row] = fmaxf(sum, 0.f);
        } else {
            const float lg = sum + bias_pre[i];
            logit_s[col][row] = lg;
            if (out != nullptr && col < B) out[(size_t)col * nrows + r0 + row] = 1.f / (1.f + __expf(-lg));
        }
    }
    if (EPI == 1) {
        __syncthreads();
        if (wave == 0) {
            bool on = false;
            for (int b = 0; b < B; ++b) on = on || logit_s[b][lane] > thr_logit;
            const uint64_t word = __ballot(on);
            if (lane == 0) mask_words[blk] = word;
        }
    }
    PF_TSTAMP(EPI, 2);
}

template <int R, int KC, int EPI, bool XS>
__global__ __launch_bounds__(kMfmaThreads) void k_rows_mfma(
    const __half *__restrict__ w, const void *__restrict__ v, int B, int K, int nrows,
    const float *__restrict__ p_bias, float thr_logit, float *__restrict__ out,
    uint64_t *__restrict__ mask_words, int first_word, const int32_t *__restrict__ skip)
{
    extern __shared__ uint64_t dyn_lds64[];
    constexpr int T = (R + 15) / 16;
    __shared__ float logit_s[16][16 * T];
    // adaptive layer step: a set flag means this step runs dense (no prediction; all marked)
    if (skip != nullptr && *skip != 0) {
        if (EPI == 1) {
            if (threadIdx.x == 0) mask_words[first_word + (int)blockIdx.x] = ~0ull;
            if (blockIdx.x == 0)
                for (int w = threadIdx.x; w < first_word; w += kMfmaThreads) mask_words[w] = ~0ull;
        }
        return;
    }
    rows_mfma_body<R, KC, EPI, XS>(dyn_lds64, logit_s, (int)blockIdx.x, w, v, B, K, nrows, p_bias, thr_logit,
                               out, mask_words, first_word);
}

}  // namespace pf
