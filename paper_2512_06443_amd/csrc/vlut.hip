// Vector-LUT ternary x INT8 mpGeMM for MI355X (gfx950): kernels and C ABI.
//
// Data layout in LDS (one "slot" = one 81-row table whose rows are 256 bytes):
//   a 256-byte row is 16 slices of 16 bytes; slice l belongs to LDS banks 4l..4l+3,
//   so 16 lanes that each read "their" slice of 16 different rows never conflict.
//   A slice holds 8 INT16 table entries (8 tokens) of ONE sub-table.  With
//   J = 1,2,4,8,16 sub-tables interleaved per row, a slot serves J sub-tables x
//   (128/J) tokens: slice l = j * (16/J) + t  (j = sub-table selector, t = 8-token chunk).
//   Lane (grp = lane/16, l = lane%16) of a wave looks up row idx of slice l for
//   output row 4*rowgroup + grp, so one ds_read_b128 serves 4 output rows x 128
//   (sub-table, token) pairs; the J partial sums of a token are added across lanes
//   once, after the K loop.
//
// Paper references: Alg. 1 (lookup/accumulate and Precompute), Eq. 1-2, Sec. 3.3
// (token-contiguous tables, tile-contiguous packed weights), Sec. 3.4 (tiling,
// streamed precompute-lookup, INT16->INT32 hierarchy, block size 64), Sec. 4
// (topological precompute).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "vlut.h"

namespace {

typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i32x4 lds_i32x4;
typedef __attribute__((address_space(3))) int lds_i32;

constexpr int kRows = 81;                    // 3^4 rows per sub-table
constexpr int kRowBytes = 256;               // LDS bytes per table row (16 slices x 16 B)
constexpr int kSlotBytes = kRows * kRowBytes;  // 20736
constexpr int kStageSlots = 4;               // slots resident per stage (one weight dword = 4 lookups)
constexpr int kTableBytes = kStageSlots * kSlotBytes;  // 82944
constexpr int kLdsBytes = kTableBytes + 128 * 4;    // + the output scales of the tile's tokens
// Fused quantisation: behind the tables and the scales, 16 x 8 partial absmax values, then the INT8 codes of the
// tile's 8 tokens for the workgroup's K range.  A stage (64 k-groups) is 8 blocks (slot of the stage x activation
// row pair) of 16 sub-tables x 16 bytes, pitched 288 bytes so that both the quantiser's dword stores and the build
// waves' 16-byte reads are free of bank conflicts.
constexpr int kFusedRedBase = kLdsBytes;
constexpr int kFusedAqBase = kFusedRedBase + 16 * 8 * 4;
constexpr int kFusedBlockPitch = 288;
constexpr int kFusedStageBytes = 8 * kFusedBlockPitch;           // 2304
constexpr int kFusedMaxLds = 160 * 1024;
constexpr int kFusedMaxStages = (kFusedMaxLds - kFusedAqBase) / kFusedStageBytes;   // 34 stages = 8704 values of K
constexpr int kWaves = 16;                   // waves per workgroup
constexpr int kThreads = kWaves * 64;
constexpr unsigned kZeroIdx4 = 0x28282828u;  // four copies of index 40 (the all-zero pattern)
constexpr int kMaxDim = 1 << 24;
constexpr int kBlockLookups = 64;            // INT16 block size B for g = 4 (Sec. 3.4)

struct LookupParams {
    const uint8_t* packed;
    const int8_t* a_q;
    const float* a_scale;
    const float* w_rows;      // per-output-row weight scales (stacked matrices) or null: w_scale for all rows
    const int16_t* lut;
    float* y;
    int32_t* acc;
    int32_t* ws;
    float w_scale;
    int M, K, N, G, KCn, RGtotal, ldy;
    int Jlog, S, tiles_m, tiles_n, RGW, stages_total, stages_per_split, total_tiles, per_xcd;
    int aligned8;
    // a_q may be a range of activation rows of a longer tensor: Ka = rows per token chunk of that tensor (0: K)
    int Ka;
    // partial-sum mode (mixed packing): write INT32 sums to ws slots slot0 + ks also when K is not split
    int partial, slot0;
    // fused quantisation (MODE kFusedQuant): fp32 activations [N][ldx] instead of a_q / a_scale
    const float* x;
    float* a_scale_out;       // optional: the token scales, written by the workgroups of the first row tile
    int64_t ldx;
    int x_vec;                // rows can be read as float4
};

__device__ __forceinline__ unsigned lds_base_of(void* p) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (unsigned)(__attribute__((address_space(3))) char*)p;
#else
    (void)p;
    return 0u;   // host pass of the single-source compile; never executed
#endif
}

// addr is a byte address inside LDS; OFF16 is a compile-time offset in units of 16 bytes, kept apart so that it
// lands in the instruction's immediate offset field instead of costing a VALU add.
template <int OFF16>
__device__ __forceinline__ i32x4 lds_read128(unsigned addr) {
    return ((const lds_i32x4*)addr)[OFF16];
}
template <int OFF16>
__device__ __forceinline__ void lds_write128(unsigned addr, i32x4 v) {
    ((lds_i32x4*)addr)[OFF16] = v;
}

// Value of x held by the lane whose index differs in bit MASK (1, 2, 4 or 8), inside each row of 16 lanes: data
// parallel primitives (no LDS traffic).  row_ror:8 swaps the halves of a row; for 4 the two directions are written
// under complementary bank masks; 2 and 1 are quad permutes.
template <int MASK>
__device__ __forceinline__ int lane_xor16(int x) {
    if (MASK == 8) return __builtin_amdgcn_update_dpp(0, x, 0x128, 0xF, 0xF, false);
    if (MASK == 4) {
        int t = __builtin_amdgcn_update_dpp(0, x, 0x104, 0xF, 0x5, false);   // lanes 0-3, 8-11 <- lane + 4
        return __builtin_amdgcn_update_dpp(t, x, 0x114, 0xF, 0xA, false);     // lanes 4-7, 12-15 <- lane - 4
    }
    if (MASK == 2) return __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false);
    return __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false);
}
// Value of lane l ^ 7 (row_half_mirror reverses each group of 8 lanes): a one-instruction partner whose bit 2 differs.
__device__ __forceinline__ int lane_xor7(int x) { return __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false); }

// 16 sub-tables per table row: the 16 lanes of a group hold 16 partial sums of the same 8 tokens (packed INT16 block
// sums, plus INT32 sums of earlier blocks when WIDE).  Reduce-scatter with partners l^8, l^7, l^2, l^1 (each a
// single DPP operand): lane l ends with the total of token l >> 1.  The first exchange moves packed INT16 pairs and
// widens while adding.
template <bool WIDE>
__device__ __forceinline__ int reduce16(const s16x2 (&a16)[4], const int (&a32)[8], int l) {
    const bool hi3 = (l & 8) != 0, hi2 = (l & 4) != 0, hi1 = (l & 2) != 0;
    int w[4];
    if constexpr (!WIDE) {
        const int a0 = __builtin_bit_cast(int, a16[0]), a1 = __builtin_bit_cast(int, a16[1]);
        const int a2 = __builtin_bit_cast(int, a16[2]), a3 = __builtin_bit_cast(int, a16[3]);
        const s16x2 kA = __builtin_bit_cast(s16x2, hi3 ? a2 : a0), kB = __builtin_bit_cast(s16x2, hi3 ? a3 : a1);
        const s16x2 rA = __builtin_bit_cast(s16x2, lane_xor16<8>(hi3 ? a0 : a2));
        const s16x2 rB = __builtin_bit_cast(s16x2, lane_xor16<8>(hi3 ? a1 : a3));
        w[0] = (int)kA.x + (int)rA.x;
        w[1] = (int)kA.y + (int)rA.y;
        w[2] = (int)kB.x + (int)rB.x;
        w[3] = (int)kB.y + (int)rB.y;
    } else {
        int v[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[2 * q] = (int)a16[q].x + a32[2 * q];
            v[2 * q + 1] = (int)a16[q].y + a32[2 * q + 1];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (hi3 ? v[e + 4] : v[e]) + lane_xor16<8>(hi3 ? v[e] : v[e + 4]);
    }
    const int x0 = (hi2 ? w[2] : w[0]) + lane_xor7(hi2 ? w[0] : w[2]);
    const int x1 = (hi2 ? w[3] : w[1]) + lane_xor7(hi2 ? w[1] : w[3]);
    const int y1 = (hi1 ? x1 : x0) + lane_xor16<2>(hi1 ? x0 : x1);
    return y1 + lane_xor16<1>(y1);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding global load
// and store of the wave (vmcnt(0)), which would expose the latency of the weight and activation prefetches at
// every stage; here a wave only has to finish its own LDS reads/writes before it signals the barrier.
__device__ __forceinline__ void wg_barrier_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ s16x2 as_s16x2(int v) { return __builtin_bit_cast(s16x2, v); }
__device__ __forceinline__ int as_int(s16x2 v) { return __builtin_bit_cast(int, v); }

// Two INT8 values (bytes 2h and 2h+1 of x) -> sign-extended packed INT16 pair.
__device__ __forceinline__ s16x2 unpack_pair(unsigned x, int h) {
    unsigned sel = h ? 0x070c060cu : 0x050c040cu;   // {0, byte, 0, byte}: value in the high byte of each half
    s16x2 v = as_s16x2((int)__builtin_amdgcn_perm(x, 0u, sel));
    return v >> (short)8;                            // arithmetic shift per half
}

// ---------------------------------------------------------------------------------------------
// Offline packing (Sec. 3.3): one thread per packed byte, including the padding bytes.
// ---------------------------------------------------------------------------------------------
__device__ int g_pack_error;

template <int GW>   // GW = weights per byte: 4 (2.00 bits per weight) or 5 (1.60)
__global__ void pack_kernel(const int8_t* __restrict__ w, int M, int64_t ldw, int G, int KCn, int RGtotal,
                            uint8_t* __restrict__ packed) {
    size_t total = (size_t)RGtotal * KCn * 64;
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i >= total) return;
    int b = (int)(i & 15);
    int r = (int)((i >> 4) & 3);
    size_t tile = i >> 6;
    int kc = (int)(tile % KCn);
    int rg = (int)(tile / KCn);
    int m = rg * 4 + r;
    int kg = kc * 16 + b;
    unsigned v = GW == 4 ? 40u : 121u;      // the all-zero pattern: every digit 1
    if (m < M && kg < G) {
        const int8_t* p = w + (size_t)m * (size_t)ldw + (size_t)kg * GW;
        bool ok = true;
        v = 0;
#pragma unroll
        for (int j = 0; j < GW; ++j) {      // first weight = most significant base-3 digit
            const int wj = p[j];
            ok = ok && wj >= -1 && wj <= 1;
            v = v * 3u + (unsigned)(wj + 1);
        }
        if (!ok) atomicOr(&g_pack_error, 1);
    }
    packed[i] = (uint8_t)v;
}

// ---------------------------------------------------------------------------------------------
// Activation quantisation + transposition (Sec. 3.4 first paragraph, Sec. 3.3).
// One workgroup handles one chunk of 8 consecutive tokens over all K.  A wave reads 8 consecutive float4 of each
// of the 8 tokens per pass (lane = token + 8 * quad): 128 contiguous bytes per token.  The four codes a lane makes
// (4 consecutive k of one token) are transposed inside its quad of lanes, so that every lane leaves with one dword
// of the chunk's [K][8] block (4 tokens of one k) and a wave's LDS store is 256 contiguous bytes, free of bank
// conflicts; the block is contiguous in the token-chunked layout and leaves with 16-byte stores.
//   NV  float4 values per thread kept in registers between the absmax pass and the rounding pass
//       (0: x is read twice, for large K)
//   VEC true when rows can be read as float4 (x and ldx 16-byte aligned)
// ---------------------------------------------------------------------------------------------
constexpr int kQuantThreads = 1024;
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Absmax quantiser of one token row, decided in fp32: inv = 127 / amax (IEEE division, 0 for an all-zero row),
// code = clamp(rint(x * inv), -127, 127) with ties to even.
// Four values at once, code of v[c] in byte c.  |v * inv| <= 127 (1 + 2^-23) for finite rows, so the rounded value r
// is an integer of [-127, 127], r + 128 is exact and fits a byte: one saturating float -> byte conversion per value
// writes it in place, and flipping the top bits afterwards subtracts the 128 again.  The lower clamp stays as an
// instruction (an overflowing inv = 127 / amax for rows below 4e-37 can make r = -inf); the upper one is the
// conversion's saturation.
__device__ __forceinline__ unsigned quant_codes4(const f32x4 v, float inv) {
    unsigned d = 0u;
    d = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(v.x * inv), -127.0f) + 128.0f, 0u, d);
    d = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(v.y * inv), -127.0f) + 128.0f, 1u, d);
    d = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(v.z * inv), -127.0f) + 128.0f, 2u, d);
    d = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(v.w * inv), -127.0f) + 128.0f, 3u, d);
    return d ^ 0x80808080u;
}
// The lane holds the codes of k = 4q .. 4q+3 of token `tok` (byte c = k offset c); the four lanes of a quad hold
// four consecutive tokens of the same q.  Returns, for the lane with tok % 4 == c, the codes of those four tokens
// at k = 4q + c (byte e = token 4*(tok/4) + e).
__device__ __forceinline__ unsigned quad_transpose_codes(unsigned d, int tok) {
    const unsigned d0 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)d, 0x00, 0xF, 0xF, false);
    const unsigned d1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)d, 0x55, 0xF, 0xF, false);
    const unsigned d2 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)d, 0xAA, 0xF, 0xF, false);
    const unsigned d3 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)d, 0xFF, 0xF, 0xF, false);
    const unsigned c = (unsigned)tok & 3u;
    const unsigned lo = __builtin_amdgcn_perm(d1, d0, 0x0c0c0000u | ((4u + c) << 8) | c);
    const unsigned hi = __builtin_amdgcn_perm(d3, d2, 0x00000c0cu | ((4u + c) << 24) | (c << 16));
    return lo | hi;
}

template <int NV, bool VEC>
__global__ void __launch_bounds__(kQuantThreads) quantize_kernel(const float* __restrict__ x, int N, int K, int64_t ldx,
                                                                 int8_t* __restrict__ a_q, float* __restrict__ a_scale) {
    extern __shared__ __attribute__((aligned(16))) unsigned char q_lds[];   // [K][8] codes
    __shared__ float red[kQuantThreads / 64][8];
    __shared__ float s_inv[8];
    const int chunk = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int t = lane & 7;                    // token of the chunk
    const int kq = wave * 8 + (lane >> 3);     // this thread handles k = 4*(kq + 128*i) .. +3
    const int n = chunk * 8 + t;
    const bool live = n < N;
    const float* row = x + (size_t)(live ? n : 0) * ldx;
    const int nquad = K >> 2;                  // K % 4 == 0

    auto load4 = [&](int qi) -> f32x4 {
        if (VEC) return *(const f32x4*)(row + 4 * (size_t)qi);
        return f32x4{row[4 * (size_t)qi], row[4 * (size_t)qi + 1], row[4 * (size_t)qi + 2], row[4 * (size_t)qi + 3]};
    };

    f32x4 xv[NV > 0 ? NV : 1];
    float amax = 0.0f;
    if (NV > 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int qi = kq + 128 * i;
            xv[i] = (live && qi < nquad) ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            amax = fmaxf(fmaxf(amax, fmaxf(fabsf(xv[i].x), fabsf(xv[i].y))), fmaxf(fabsf(xv[i].z), fabsf(xv[i].w)));
        }
    } else {
        // eight loads in flight per thread and pass (a plain loop would wait for every load in turn)
        for (int q0 = 0; q0 < nquad; q0 += 128 * 8) {
            f32x4 tv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int qi = q0 + kq + 128 * i;
                tv[i] = (live && qi < nquad) ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                amax = fmaxf(fmaxf(amax, fmaxf(fabsf(tv[i].x), fabsf(tv[i].y))), fmaxf(fabsf(tv[i].z), fabsf(tv[i].w)));
        }
    }
    for (int off = 32; off >= 8; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));   // lanes of the same token
    if (lane < 8) red[wave][lane] = amax;
    __syncthreads();
    if (tid < 8) {
        float v = 0.0f;
        for (int w = 0; w < kQuantThreads / 64; ++w) v = fmaxf(v, red[w][tid]);
        // IEEE-correct fp32 divisions (the default for HIP); no reciprocal approximation.
        s_inv[tid] = (v > 0.0f) ? 127.0f / v : 0.0f;
        if (chunk * 8 + tid < N) a_scale[chunk * 8 + tid] = v / 127.0f;
    }
    __syncthreads();
    const float inv = s_inv[t];
    // The quad transpose uses all four lanes of a quad; they share qi, so the bounds test is uniform per quad.
    auto emit = [&](int qi, const f32x4 v) {       // tokens past N: x = 0 -> code 0
        const unsigned e = quad_transpose_codes(quant_codes4(v, inv), t);
        if (qi < nquad) *(unsigned*)(q_lds + (size_t)qi * 32 + (t & 3) * 8 + (t >> 2) * 4) = e;
    };
    if (NV > 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) emit(kq + 128 * i, xv[i]);
    } else {
        // every lane runs the same number of passes (the quad exchange needs its partner lanes)
        for (int q0 = 0; q0 < nquad; q0 += 128 * 8) {
            f32x4 tv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int qi = q0 + kq + 128 * i;
                tv[i] = (live && qi < nquad) ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) emit(q0 + kq + 128 * i, tv[i]);
        }
    }
    __syncthreads();
    i32x4* dst = (i32x4*)(a_q + (size_t)chunk * K * 8);
    const i32x4* src = (const i32x4*)q_lds;
    for (int i = tid; i < K / 2; i += kQuantThreads) dst[i] = src[i];   // 16 bytes = 2 k-rows of 8 codes
}

// The same quantiser with one workgroup (256 threads) per token, for long rows or many tokens: the chunk kernel above
// lets one CU pull 8 whole rows twice, which takes 20 us at K = 8640, while here every CU reads one row once.  The
// price is the store: a token owns one byte in every 8 of its chunk's [K][8] block, so the codes leave as single
// bytes (distinct bytes written by different workgroups: no race).  Tokens past N (padding of the last chunk) are
// written as zeros.  Blocks are numbered so that the 8 tokens of a chunk sit 8 blocks apart (same XCD under
// round-robin dispatch, so their partial lines meet in one L2); this is a matter of speed only.
//   NV  float4 values per thread kept in registers between the two passes (0: x is read twice)
constexpr int kTokThreads = 256;

template <int NV, bool VEC>
__global__ void __launch_bounds__(kTokThreads) quantize_token_kernel(const float* __restrict__ x, int N, int K, int64_t ldx,
                                                                     int8_t* __restrict__ a_q,
                                                                     float* __restrict__ a_scale, int chunks) {
    __shared__ float red[kTokThreads / 64];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int chunk = (b >> 6) * 8 + (b & 7);
    const int t = (b >> 3) & 7;
    if (chunk >= chunks) return;
    const int n = chunk * 8 + t;
    const bool live = n < N;
    const float* row = x + (size_t)(live ? n : 0) * ldx;
    const int nquad = K >> 2;
    auto load4 = [&](int qi) -> f32x4 {
        const float* src = row + 4 * (size_t)qi;
        if (VEC) return *(const f32x4*)src;
        return f32x4{src[0], src[1], src[2], src[3]};
    };
    auto absmax4 = [](float m, const f32x4 v) {
        return fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    };
    constexpr int NB = NV > 0 ? NV : 8;            // loads in flight per thread and pass
    f32x4 xv[NB];
    float amax = 0.0f;
    if (live) {
        for (int q0 = 0; q0 < (NV > 0 ? 1 : nquad); q0 += kTokThreads * NB) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int qi = q0 + tid + kTokThreads * i;
                xv[i] = qi < nquad ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) amax = absmax4(amax, xv[i]);
        }
    }
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < kTokThreads / 64; ++w) v = fmaxf(v, red[w]);
    const float inv = (v > 0.0f) ? 127.0f / v : 0.0f;      // IEEE divisions
    if (tid == 0 && live) a_scale[n] = v / 127.0f;
    int8_t* dst = a_q + (size_t)chunk * K * 8 + t;
    auto store4 = [&](int qi, unsigned d) {
        int8_t* o = dst + (size_t)qi * 32;
        o[0] = (int8_t)(d & 0xffu);
        o[8] = (int8_t)((d >> 8) & 0xffu);
        o[16] = (int8_t)((d >> 16) & 0xffu);
        o[24] = (int8_t)(d >> 24);
    };
    for (int q0 = 0; q0 < (NV > 0 ? 1 : nquad); q0 += kTokThreads * NB) {
        if (NV == 0 && live) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int qi = q0 + tid + kTokThreads * i;
                xv[i] = qi < nquad ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int qi = q0 + tid + kTokThreads * i;
            if (qi < nquad) store4(qi, live ? quant_codes4(xv[i], inv) : 0u);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Whole table in global memory (Alg. 1 Precompute / Eq. 1), topological order of Sec. 4:
// every row is one add/sub away from an earlier one.  One thread per (group, token).
// ---------------------------------------------------------------------------------------------
//   TOKEN_OUTER false: lut[kg][i][n], tokens contiguous (Sec. 3.3, the layout of the method)
//               true:  lut[n][kg][i], one table per token (the scalar-LUT arrangement; layout ablation of Sec. 5.6)
template <bool TOKEN_OUTER>
__global__ void __launch_bounds__(256) build_lut_kernel(const int8_t* __restrict__ a_q, int G, int N,
                                                        int16_t* __restrict__ lut) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i >= (size_t)G * N) return;
    int n = (int)(i % N);
    int kg = (int)(i / N);
    const int8_t* a = a_q + ((size_t)(n >> 3) * (4 * G) + 4 * kg) * 8 + (n & 7);   // [N/8][K][8]
    int a0 = a[0], a1 = a[8], a2 = a[16], a3 = a[24];
    int16_t* t = TOKEN_OUTER ? lut + ((size_t)n * G + kg) * kRows : lut + ((size_t)kg * kRows) * N + n;
    const size_t row_stride = TOKEN_OUTER ? 1 : (size_t)N;
    int v0 = -a0 - a1 - a2 - a3;                       // row 0, then walk the digits
    for (int d0 = 0; d0 < 3; ++d0) {
        int v1 = v0;
        for (int d1 = 0; d1 < 3; ++d1) {
            int v2 = v1;
            for (int d2 = 0; d2 < 3; ++d2) {
                int v3 = v2;
                for (int d3 = 0; d3 < 3; ++d3) {
                    t[(size_t)(27 * d0 + 9 * d1 + 3 * d2 + d3) * row_stride] = (int16_t)v3;
                    v3 += a3;
                }
                v2 += a2;
            }
            v1 += a1;
        }
        v0 += a0;
    }
}

// ---------------------------------------------------------------------------------------------
// The lookup kernel (Alg. 1 main loop + streamed Precompute, Sec. 3.4).
//
// Roles inside the 16-wave workgroup: waves 0..3 (one per SIMD) only BUILD tables, waves 4..15 only LOOK UP.
// The four LDS slots are used as two halves of two slots each: while the lookup waves read one half, the build
// waves fill the other half with the next two sub-table sets, and one barrier per half-stage hands the halves over.
// The lookups are bound by VALU issue (one address permute + four packed adds per 16-byte table read), the build
// by LDS write bandwidth, so the two overlap well.
//   R       row groups (of 4 output rows) per lookup wave; workgroup tile = up to 48*R rows
//   NEED32  more than 64 lookups per lane: widen INT16 block sums into INT32 every 16 stages
//   MODE    kFast: tables built in LDS from the token-chunked INT8 activations (streamed, the hot path)
//           kFusedQuant: as kFast, but the workgroup first quantises its 8 tokens itself (fp32 rows -> absmax ->
//                        INT8 codes kept in LDS); needs 16 sub-tables per row (8-token tiles)
//           kFromGlobal: LDS slots are filled from a table materialised by vlut_build_lut
// ---------------------------------------------------------------------------------------------
template <int V> using ic = std::integral_constant<int, V>;
template <int I0, int I1, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I0 < I1) {
        f(ic<I0>{});
        static_for<I0 + 1, I1>(f);
    }
}

enum { kFast = 0, kFusedQuant = 1, kFromGlobal = 2 };
constexpr int kBuildWaves = 4;
constexpr int kLookupWaves = kWaves - kBuildWaves;     // 12
constexpr int kRoundRows = kLookupWaves * 4;           // 48 output rows per row-group round of the workgroup

// Issues the table read of lookup number I of half-stage HALF (b-major: I = b*R + r, b = 0,1).  Byte 2*HALF + b of
// the row group's weight dword is the row of slot 2*HALF + b; the lane reads its 16-byte slice (8 INT16 entries).
template <int R, int HALF, int I>
__device__ __forceinline__ i32x4 lookup_read(const unsigned (&w)[R], unsigned lanebase) {
    constexpr int slot = 2 * HALF + I / R, r = I % R;
    constexpr unsigned sel = 0x0c0c0000u | ((4u + (unsigned)slot) << 8);
    const unsigned addr = __builtin_amdgcn_perm(w[r], lanebase, sel);   // idx*256 + slice*16
    return lds_read128<slot * (kSlotBytes / 16)>(addr);
}

template <int R, int I>
__device__ __forceinline__ void lookup_accumulate(s16x2 (&acc16)[R][4], const i32x4 v) {
    constexpr int r = I % R;
    // Written as instructions with the accumulator tied to one register ("+v"): left to the register allocator, the
    // unrolled copies of the stage keep the accumulators in alternating register sets, which doubles their
    // footprint and caps the row groups a wave can hold.
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][0]) : "v"(v.x));
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][1]) : "v"(v.y));
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][2]) : "v"(v.z));
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][3]) : "v"(v.w));
}

// The 2*R lookups of a half-stage, software pipelined in batches of NB: the reads of batch k+1 are in flight while
// the packed INT16 adds of batch k issue (Alg. 1 lines 3-6: one shared index, one vector add over the tokens).
template <int R, int HALF, int NB, int K0>
__device__ __forceinline__ void lookup_batches(const unsigned (&w)[R], unsigned lanebase, s16x2 (&acc16)[R][4],
                                               i32x4 (&cur)[NB]) {
    constexpr int total = 2 * R;
    if constexpr (K0 < total) {
        i32x4 nxt[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) nxt[i] = i32x4{0, 0, 0, 0};
        if constexpr (K0 + NB + 0 < total && NB > 0) nxt[0] = lookup_read<R, HALF, (K0 + NB + 0 < total ? K0 + NB + 0 : 0)>(w, lanebase);
        if constexpr (K0 + NB + 1 < total && NB > 1) nxt[1] = lookup_read<R, HALF, (K0 + NB + 1 < total ? K0 + NB + 1 : 0)>(w, lanebase);
        if constexpr (K0 + NB + 2 < total && NB > 2) nxt[2] = lookup_read<R, HALF, (K0 + NB + 2 < total ? K0 + NB + 2 : 0)>(w, lanebase);
        if constexpr (K0 + NB + 3 < total && NB > 3) nxt[3] = lookup_read<R, HALF, (K0 + NB + 3 < total ? K0 + NB + 3 : 0)>(w, lanebase);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (K0 + 0 < total && NB > 0) lookup_accumulate<R, (K0 + 0 < total ? K0 + 0 : 0)>(acc16, cur[0]);
        if constexpr (K0 + 1 < total && NB > 1) lookup_accumulate<R, (K0 + 1 < total ? K0 + 1 : 0)>(acc16, cur[1]);
        if constexpr (K0 + 2 < total && NB > 2) lookup_accumulate<R, (K0 + 2 < total ? K0 + 2 : 0)>(acc16, cur[2]);
        if constexpr (K0 + 3 < total && NB > 3) lookup_accumulate<R, (K0 + 3 < total ? K0 + 3 : 0)>(acc16, cur[3]);
        __builtin_amdgcn_sched_barrier(0);
        lookup_batches<R, HALF, NB, K0 + NB>(w, lanebase, acc16, nxt);
    }
}

template <int R, int HALF>
__device__ __forceinline__ void lookup_half(const unsigned (&w)[R], unsigned lanebase, s16x2 (&acc16)[R][4]) {
    constexpr int NB = 4;
    constexpr int total = 2 * R;
    i32x4 first[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) first[i] = i32x4{0, 0, 0, 0};
    first[0] = lookup_read<R, HALF, 0>(w, lanebase);
    if constexpr (total > 1) first[1] = lookup_read<R, HALF, 1>(w, lanebase);
    if constexpr (total > 2) first[2] = lookup_read<R, HALF, (total > 2 ? 2 : 0)>(w, lanebase);
    if constexpr (total > 3) first[3] = lookup_read<R, HALF, (total > 3 ? 3 : 0)>(w, lanebase);
    __builtin_amdgcn_sched_barrier(0);
    lookup_batches<R, HALF, NB, 0>(w, lanebase, acc16, first);
}

// Nine table rows that share their two leading digits (b1 = their common part): the third and fourth digits add or
// subtract a2 and a3.  Row offsets 0..8 from dst.
__device__ __forceinline__ void build_rows9(unsigned dst, const s16x2 (&b1)[4], const s16x2 (&a2)[4],
                                            const s16x2 (&a3)[4]) {
    s16x2 u[4], lo[4], hi[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) { u[q] = b1[q] - a2[q]; lo[q] = u[q] - a3[q]; hi[q] = u[q] + a3[q]; }
    lds_write128<0 * 16>(dst, i32x4{as_int(lo[0]), as_int(lo[1]), as_int(lo[2]), as_int(lo[3])});
    lds_write128<1 * 16>(dst, i32x4{as_int(u[0]), as_int(u[1]), as_int(u[2]), as_int(u[3])});
    lds_write128<2 * 16>(dst, i32x4{as_int(hi[0]), as_int(hi[1]), as_int(hi[2]), as_int(hi[3])});
#pragma unroll
    for (int q = 0; q < 4; ++q) { lo[q] = b1[q] - a3[q]; hi[q] = b1[q] + a3[q]; }
    lds_write128<3 * 16>(dst, i32x4{as_int(lo[0]), as_int(lo[1]), as_int(lo[2]), as_int(lo[3])});
    lds_write128<4 * 16>(dst, i32x4{as_int(b1[0]), as_int(b1[1]), as_int(b1[2]), as_int(b1[3])});
    lds_write128<5 * 16>(dst, i32x4{as_int(hi[0]), as_int(hi[1]), as_int(hi[2]), as_int(hi[3])});
#pragma unroll
    for (int q = 0; q < 4; ++q) { u[q] = b1[q] + a2[q]; lo[q] = u[q] - a3[q]; hi[q] = u[q] + a3[q]; }
    lds_write128<6 * 16>(dst, i32x4{as_int(lo[0]), as_int(lo[1]), as_int(lo[2]), as_int(lo[3])});
    lds_write128<7 * 16>(dst, i32x4{as_int(u[0]), as_int(u[1]), as_int(u[2]), as_int(u[3])});
    lds_write128<8 * 16>(dst, i32x4{as_int(hi[0]), as_int(hi[1]), as_int(hi[2]), as_int(hi[3])});
}

template <int R, bool NEED32, int MODE>
__global__ void __launch_bounds__(kThreads) lookup_kernel(const LookupParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // The kernel has no static LDS, so the dynamic segment starts at LDS address 0; table addresses are formed
    // as idx*256 + slice*16 by a byte permute and rely on that.
    if (lds_base_of(smem) != 0u) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction

    // Fetch every launch parameter now, in one batch of scalar loads.  Left alone, the compiler loads only what the
    // early exit below needs and the rest after it, so each workgroup would wait for the argument buffer twice.
    asm volatile("" ::"s"(p.per_xcd), "s"(p.total_tiles), "s"(p.S), "s"(p.tiles_n), "s"(p.Jlog), "s"(p.RGW),
                 "s"(p.stages_per_split), "s"(p.stages_total), "s"(p.K), "s"(p.N), "s"(p.G), "s"(p.KCn), "s"(p.RGtotal),
                 "s"(p.M), "s"(p.ldy), "s"(p.w_scale), "s"(p.packed), "s"(p.a_q), "s"(p.a_scale), "s"(p.y), "s"(p.acc),
                 "s"(p.ws), "s"(p.lut), "s"(p.aligned8), "s"(p.w_rows), "s"(p.x), "s"(p.a_scale_out), "s"(p.ldx),
                 "s"(p.x_vec));

    // ---- which tile (XCD-aware: the 8 XCDs take contiguous ranges of the tile list, so the
    //      workgroups that share a weight tile also share an L2)
    int L = (int)(blockIdx.x & 7) * p.per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= p.per_xcd || L >= p.total_tiles) return;
    const int ks = L % p.S;
    L /= p.S;
    const int nt = L % p.tiles_n;
    const int mt = L / p.tiles_n;

    const int Jlog = p.Jlog;
    const int J = 1 << Jlog;
    const int TClog = 4 - Jlog;          // log2(token chunks per sub-table)
    const int n_tile = 128 >> Jlog;
    const int n0 = nt * n_tile;
    const int rgw0 = mt * p.RGW;          // first row group of this workgroup

    const int l = lane & 15;             // 16-byte slice of the table rows this lane reads or writes
    const int grp = lane >> 4;
    const int j = l >> TClog;            // sub-table selector of the slice
    const int t = l & ((1 << TClog) - 1);   // 8-token chunk of the slice
    const unsigned lanebase = (unsigned)l * 16u;

    const int st_begin = ks * p.stages_per_split;
    const int st_end = min(p.stages_total, st_begin + p.stages_per_split);
    const bool builder = wave < kBuildWaves;          // scalar condition
    const int lw = wave - kBuildWaves;                // index among the lookup waves

    // Output scale of every token of the tile, parked behind the tables (read in the epilogue).
    typedef __attribute__((address_space(3))) float lds_f32;
    lds_f32* scale_lds = (lds_f32*)(unsigned)kTableBytes;
    // Loaded now, stored to LDS only when the K loop is over: nothing at the start of the kernel waits for it.
    float my_scale = 0.0f;
    if (MODE != kFusedQuant && tid < n_tile && n0 + tid < p.N)
        my_scale = p.w_rows ? p.a_scale[n0 + tid] : p.w_scale * p.a_scale[n0 + tid];

    // Fused quantisation (all 16 waves; called once by either role, after its first loads are on their way): lane =
    // token + 8 * quad, a wave reads 8 consecutive float4 of each of the 8 rows per pass.  Absmax over all of K
    // (also when K is split: every split needs the same scale), codes only for this workgroup's K range.
    auto quantise_tile = [&]() {
        typedef __attribute__((address_space(3))) unsigned lds_u32;
        lds_f32* red = (lds_f32*)(unsigned)kFusedRedBase;      // [wave][token]
        const int tok = lane & 7;
        const int kq = wave * 8 + (lane >> 3);
        const int n = n0 + tok;
        const bool live = n < p.N;
        const float* row = p.x + (size_t)(live ? n : 0) * p.ldx;
        const int nquad = p.G;                                 // a float4 of a row = one k-group
        const int q_lo = st_begin * 64, q_hi = min(st_end * 64, nquad);
        auto load4 = [&](int qi) -> f32x4 {
            const float* src = row + 4 * (size_t)qi;
            if (p.x_vec) return *(const f32x4*)src;
            return f32x4{src[0], src[1], src[2], src[3]};
        };
        auto absmax4 = [](float m, const f32x4 v) {
            return fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
        };
        constexpr int NVC = 8;                                 // float4 per thread kept in registers (K <= 4096)
        f32x4 xv[NVC];
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < NVC; ++i) {
            const int qi = kq + 128 * i;
            xv[i] = (live && qi < nquad) ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            amax = absmax4(amax, xv[i]);
        }
        for (int q0 = 128 * NVC; q0 < nquad; q0 += 128 * NVC) {   // longer rows: NVC loads in flight per pass
            f32x4 tv[NVC];
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = q0 + kq + 128 * i;
                tv[i] = (live && qi < nquad) ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < NVC; ++i) amax = absmax4(amax, tv[i]);
        }
        for (int off = 32; off >= 8; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));   // lanes of the same token
        if (lane < 8) red[wave * 8 + lane] = amax;
        wg_barrier_lds();
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v = fmaxf(v, red[w * 8 + tok]);
        const float inv = (v > 0.0f) ? 127.0f / v : 0.0f;      // IEEE divisions, as in quantize_kernel
        const float sc = v / 127.0f;
        if (tid < 8) {                                         // lane = token here
            my_scale = live ? (p.w_rows ? sc : p.w_scale * sc) : 0.0f;
            if (live && mt == 0 && ks == 0 && p.a_scale_out) p.a_scale_out[n] = sc;
        }
        // LDS address of the lane's dword for k-group kq; the address is affine in the k-group (128 groups = 2 stages)
        const int ql0 = kq - q_lo;
        const int a0 = kFusedAqBase + (ql0 >> 6) * kFusedStageBytes +
                       ((ql0 & 3) * 2 + ((tok & 3) >> 1)) * kFusedBlockPitch +   // (slot of the stage, row pair)
                       ((ql0 >> 2) & 15) * 16 + (tok & 1) * 8 + (tok >> 2) * 4;
        auto emit = [&](int qi, const f32x4 xq, int addr) {
            const unsigned e = quad_transpose_codes(quant_codes4(xq, inv), tok);   // 4 tokens of row tok % 4 of the group
            if (qi >= q_lo && qi < q_hi) *(lds_u32*)(unsigned)addr = e;
        };
#pragma unroll
        for (int i = 0; i < NVC; ++i) emit(kq + 128 * i, xv[i], a0 + i * 2 * kFusedStageBytes);
        // the rest of the range is read again; every lane runs the same passes (the quad exchange needs its partners)
        for (int q0 = max(128 * NVC, q_lo & ~127); q0 < q_hi; q0 += 128 * NVC) {
            f32x4 tv[NVC];
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = q0 + kq + 128 * i;
                tv[i] = (live && qi >= q_lo && qi < q_hi) ? load4(qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < NVC; ++i)
                emit(q0 + kq + 128 * i, tv[i], a0 + ((q0 >> 6) + 2 * i) * kFusedStageBytes);
        }
        wg_barrier_lds();
    };

    s16x2 acc16[R][4];
    int acc32[NEED32 ? R : 1][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc16[r][q] = s16x2{0, 0};
    if (NEED32) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc32[r][e] = 0;
    }

    if (builder) {
        // ================================ build role ================================
        // Task of a lane for one half-stage: slot s2 of the half (0/1), slice l, leading digits hh = u (table rows
        // 9u .. 9u+8); the ninth digit pair (rows 72..80) is shared out one row per lane, lane u = 0 takes two.
        const int u = (wave * 4 + grp) & 7;
        const int s2 = (wave * 4 + grp) >> 3;
        const int nb = n0 + 8 * t;                   // first token of the slice
        const int chunk_b = nb >> 3;
        unsigned actA[4][2], actB[4][2];
        bool validA = false, validB = false;

        // Half-stage hs = 2*stage + half holds slots 2*half, 2*half+1 = sub-tables kg = stage*4J + 4j + slot.
        auto fetch_act = [&](int hs, unsigned (&act)[4][2], bool& valid) {
            const int kg = (hs >> 1) * 4 * J + 4 * j + 2 * (hs & 1) + s2;
            valid = (hs < 2 * st_end) && (kg < p.G) && (nb < p.N);
            if (MODE == kFusedQuant) {
                // the codes this workgroup made itself: rows 0,1 and rows 2,3 of the group, 16 bytes each
                const int stl = min((hs >> 1) - st_begin, p.stages_per_split - 1);   // prefetches run past the end
                const unsigned a0 = (unsigned)(kFusedAqBase + stl * kFusedStageBytes +
                                               (2 * (hs & 1) + s2) * 2 * kFusedBlockPitch + j * 16);
                const i32x4 v0 = lds_read128<0>(a0), v1 = lds_read128<kFusedBlockPitch / 16>(a0);
                act[0][0] = (unsigned)v0.x; act[0][1] = (unsigned)v0.y;
                act[1][0] = (unsigned)v0.z; act[1][1] = (unsigned)v0.w;
                act[2][0] = (unsigned)v1.x; act[2][1] = (unsigned)v1.y;
                act[3][0] = (unsigned)v1.z; act[3][1] = (unsigned)v1.w;
            }
            if (MODE == kFast) {
                // 4 activation rows x 8 tokens = 32 contiguous bytes of the token-chunked layout; branch-free
                // (address clamped into the tensor, validity applied at use) so nothing waits on the data early.
                const int kgc = min(kg, p.G - 1);
                const int cc = (nb < p.N) ? chunk_b : 0;
                const i32x4* src = (const i32x4*)(p.a_q + ((size_t)cc * p.Ka + 4 * kgc) * 8);
                const i32x4 v0 = src[0], v1 = src[1];
                act[0][0] = (unsigned)v0.x; act[0][1] = (unsigned)v0.y;
                act[1][0] = (unsigned)v0.z; act[1][1] = (unsigned)v0.w;
                act[2][0] = (unsigned)v1.x; act[2][1] = (unsigned)v1.y;
                act[3][0] = (unsigned)v1.z; act[3][1] = (unsigned)v1.w;
            }
        };

        auto build_half = [&](int hs, unsigned (&act)[4][2], bool valid) {
            const unsigned slot = (unsigned)(2 * (hs & 1) + s2);
            const unsigned dst = slot * kSlotBytes + (unsigned)l * 16u;
            if (MODE == kFromGlobal) {
                const int kg = (hs >> 1) * 4 * J + 4 * j + 2 * (hs & 1) + s2;
                auto copy_row = [&](int row) {
                    i32x4 v = {0, 0, 0, 0};
                    if (kg < p.G && nb < p.N) {
                        const int16_t* src = p.lut + ((size_t)kg * kRows + row) * p.N + nb;
                        if (p.aligned8 && nb + 8 <= p.N) {
                            v = *(const i32x4*)src;
                        } else {
                            int tmp[4] = {0, 0, 0, 0};
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                unsigned hw = (nb + e < p.N) ? (unsigned)(uint16_t)src[e] : 0u;
                                tmp[e >> 1] |= (int)(hw << (16 * (e & 1)));
                            }
                            v = i32x4{tmp[0], tmp[1], tmp[2], tmp[3]};
                        }
                    }
                    lds_write128<0>(dst + (unsigned)row * kRowBytes, v);
                };
#pragma unroll
                for (int i = 0; i < 9; ++i) copy_row(9 * u + i);
                copy_row(72 + u);
                if (u == 0) copy_row(80);
            } else {
                // Every row is one packed add/sub away from an earlier one (topological order, Sec. 4).
                if (!valid) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) { act[c][0] = 0u; act[c][1] = 0u; }
                }
                const short s0 = (short)(u / 3 - 1), s1 = (short)(u % 3 - 1);
                const s16x2 m0 = {s0, s0}, m1 = {s1, s1};
                const short e2 = (short)(u / 3 - 1), e3 = (short)(u % 3 - 1);    // digits (d2,d3) of the extra row 72+u
                const s16x2 x2 = {e2, e2}, x3 = {e3, e3};
                s16x2 a2[4], a3[4], b1[4], ex[4], top[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const s16x2 a0 = unpack_pair(act[0][q >> 1], q & 1);
                    const s16x2 a1 = unpack_pair(act[1][q >> 1], q & 1);
                    a2[q] = unpack_pair(act[2][q >> 1], q & 1);
                    a3[q] = unpack_pair(act[3][q >> 1], q & 1);
                    b1[q] = a0 * m0 + a1 * m1;
                    top[q] = a0 + a1;                               // leading digits (2,2)
                    ex[q] = top[q] + a2[q] * x2 + a3[q] * x3;       // row 72 + 3*d2 + d3 with (d2,d3) = (u/3, u%3)
                }
                build_rows9(dst + (unsigned)(9 * u) * kRowBytes, b1, a2, a3);
                lds_write128<0>(dst + (unsigned)(72 + u) * kRowBytes,
                                i32x4{as_int(ex[0]), as_int(ex[1]), as_int(ex[2]), as_int(ex[3])});
                if (u == 0) {
                    lds_write128<80 * 16>(dst, i32x4{as_int(top[0] + a2[0] + a3[0]), as_int(top[1] + a2[1] + a3[1]),
                                                      as_int(top[2] + a2[2] + a3[2]), as_int(top[3] + a2[3] + a3[3])});
                }
            }
        };

        const int hs0 = 2 * st_begin, hs1 = 2 * st_end;
        if constexpr (MODE == kFusedQuant) quantise_tile();
        if constexpr (MODE == kFromGlobal) {
            if (hs0 < hs1) build_half(hs0, actA, validA);
            wg_barrier_lds();
            for (int hs = hs0; hs < hs1; hs += 2) {
                build_half(hs + 1, actB, validB);     // lookups read half 0 now: fill half 1
                wg_barrier_lds();
                if (hs + 2 < hs1) build_half(hs + 2, actA, validA);   // lookups read half 1 now: fill half 0
                wg_barrier_lds();
            }
        } else {
            // The build waves are few and every barrier waits for them: let them issue first.
            __builtin_amdgcn_s_setprio(3);
            // Rows are computed one half-stage ahead: after a barrier a build wave only has to issue its eleven
            // LDS writes, and it computes the next half-stage's rows while those writes drain.  Activations are
            // fetched four half-stages ahead of their use.
            struct Rows { s16x2 r[9][4], ex[4], last[4]; };
            unsigned act2[4][2], act3[4][2];
            bool valid2 = false, valid3 = false;
            auto compute_rows = [&](unsigned (&act)[4][2], bool valid, Rows& rw) {
                if (!valid) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) { act[c][0] = 0u; act[c][1] = 0u; }
                }
                const short d0 = (short)(u / 3 - 1), d1 = (short)(u % 3 - 1);   // leading digits of rows 9u..9u+8,
                const s16x2 m0 = {d0, d0}, m1 = {d1, d1};                         // and digits (d2,d3) of row 72+u
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const s16x2 a0 = unpack_pair(act[0][q >> 1], q & 1);
                    const s16x2 a1 = unpack_pair(act[1][q >> 1], q & 1);
                    const s16x2 a2 = unpack_pair(act[2][q >> 1], q & 1);
                    const s16x2 a3 = unpack_pair(act[3][q >> 1], q & 1);
                    const s16x2 b1 = a0 * m0 + a1 * m1;
                    const s16x2 top = a0 + a1;                          // leading digits (2,2)
                    const s16x2 lo = b1 - a2, hi = b1 + a2;
                    rw.r[0][q] = lo - a3; rw.r[1][q] = lo; rw.r[2][q] = lo + a3;
                    rw.r[3][q] = b1 - a3; rw.r[4][q] = b1; rw.r[5][q] = b1 + a3;
                    rw.r[6][q] = hi - a3; rw.r[7][q] = hi; rw.r[8][q] = hi + a3;
                    rw.ex[q] = top + a2 * m0 + a3 * m1;                 // row 72 + 3*d2 + d3 with (d2,d3) = (u/3, u%3)
                    rw.last[q] = top + a2 + a3;                         // row 80
                }
                // Pin the finished rows in registers here, so that the arithmetic stays where it is written
                // (between the LDS writes of one half-stage and the barrier) instead of sinking below the barrier.
#pragma unroll
                for (int q = 0; q < 4; ++q) {
#pragma unroll
                    for (int i = 0; i < 9; ++i) asm volatile("" : "+v"(rw.r[i][q]));
                    asm volatile("" : "+v"(rw.ex[q]));
                    asm volatile("" : "+v"(rw.last[q]));
                }
            };
            auto write_rows = [&](int hs, const Rows& rw) {
                const unsigned dst = (unsigned)(2 * (hs & 1) + s2) * kSlotBytes + (unsigned)l * 16u;
                const unsigned dst9 = dst + (unsigned)(9 * u) * kRowBytes;
                static_for<0, 9>([&](auto ic_) {
                    constexpr int i = decltype(ic_)::value;
                    lds_write128<i * 16>(dst9, i32x4{as_int(rw.r[i][0]), as_int(rw.r[i][1]), as_int(rw.r[i][2]), as_int(rw.r[i][3])});
                });
                lds_write128<0>(dst + (unsigned)(72 + u) * kRowBytes,
                                i32x4{as_int(rw.ex[0]), as_int(rw.ex[1]), as_int(rw.ex[2]), as_int(rw.ex[3])});
                if (u == 0) {
                    lds_write128<80 * 16>(dst, i32x4{as_int(rw.last[0]), as_int(rw.last[1]), as_int(rw.last[2]), as_int(rw.last[3])});
                }
            };
            Rows rows;
            // One half-stage: write the rows computed earlier (half-stage hs, if it exists), compute the rows of
            // half-stage hs + 1 from `act_next`, refill that activation buffer, and meet the lookup waves.
            auto step = [&](int hs, unsigned (&act_next)[4][2], bool& valid_next) {
                if (hs < hs1) write_rows(hs, rows);
                compute_rows(act_next, valid_next, rows);
                fetch_act(hs + 5, act_next, valid_next);
                wg_barrier_lds();
            };
            if (hs0 < hs1) {
                fetch_act(hs0, actA, validA);
                fetch_act(hs0 + 1, actB, validB);
                fetch_act(hs0 + 2, act2, valid2);
                fetch_act(hs0 + 3, act3, valid3);
                compute_rows(actA, validA, rows);
                fetch_act(hs0 + 4, actA, validA);
            }
            // half 0 of the first stage: hand it over as soon as it is written, compute the next rows afterwards
            if (hs0 < hs1) write_rows(hs0, rows);
            wg_barrier_lds();
            compute_rows(actB, validB, rows);
            fetch_act(hs0 + 5, actB, validB);
            for (int hs = hs0; hs < hs1; hs += 4) {
                step(hs + 1, act2, valid2);           // lookups read half 0 (hs): fill half 1
                step(hs + 2, act3, valid3);           // lookups read half 1 (hs+1): fill half 0
                step(hs + 3, actA, validA);           // (with an odd number of stages the last two steps only meet
                                                      //  the lookup waves at their two matching barriers)
                step(hs + 4, actB, validB);
            }
            __builtin_amdgcn_s_setprio(0);
        }
    } else {
        // ================================ lookup role ================================
        // Row group r of this wave: its packed tiles start at a wave-uniform address (scalar registers); the lane
        // adds its row (grp) and, per stage, the tile and dword it needs.
        const unsigned char* wbase[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int rgl = r * kLookupWaves + lw;   // r-major: round r of the epilogue covers 48 consecutive rows
            const int rg = rgw0 + rgl;
            const bool valid = (rgl < p.RGW) && (rg < p.RGtotal);
            wbase[r] = p.packed + ((size_t)(valid ? rg : 0) * p.KCn) * 64;
        }
        // Weight dwords (4 lookups each) are fetched one whole stage ahead.  Dword q = st*J + j of each row.
        // Out-of-range cases need no masking: a tile index past the end of K is clamped to the last tile and meets
        // tables built from zero activations, and rows past M are clamped to row group 0 and never stored.
        auto load_weights = [&](int st, unsigned (&wdst)[R]) {
            const int q = st * J + j;
            const int kc = min(q >> 2, p.KCn - 1);
            const unsigned voff = (unsigned)(kc * 64 + grp * 16 + (q & 3) * 4);
#pragma unroll
            for (int r = 0; r < R; ++r) wdst[r] = *(const unsigned*)(wbase[r] + voff);
        };
        auto stage = [&](int st, unsigned (&w)[R], unsigned (&wnext)[R]) {
            load_weights(st + 1, wnext);
            lookup_half<R, 0>(w, lanebase, acc16);
            wg_barrier_lds();
            lookup_half<R, 1>(w, lanebase, acc16);
            wg_barrier_lds();
            if (NEED32 && (((st - st_begin) & 15) == 15)) {   // 16 stages x 4 lookups = block of 64 (Sec. 3.4)
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc32[r][2 * q] += (int)acc16[r][q].x;
                        acc32[r][2 * q + 1] += (int)acc16[r][q].y;
                        acc16[r][q] = s16x2{0, 0};
                    }
            }
        };
        unsigned wa[R], wb[R];
        load_weights(st_begin, wa);
        if constexpr (MODE == kFusedQuant) quantise_tile();
        wg_barrier_lds();                      // half-stage 0 of the first stage is built
        for (int st = st_begin; st < st_end; st += 2) {
            stage(st, wa, wb);
            if (st + 1 < st_end) {
                stage(st + 1, wb, wa);
            } else if (MODE != kFromGlobal) {
                wg_barrier_lds();              // the build waves run in units of two stages
                wg_barrier_lds();
            }
        }
    }

    // ---- epilogue.  Per row group: widen to INT32, add the J partial sums of each token across the 16 lanes of
    // the group with a reduce-scatter (each step halves the tokens a lane keeps), park the sums in LDS as
    // [token][row] and let the whole workgroup write consecutive output rows per token.
    lds_i32* park = (lds_i32*)0u;
    if (tid < n_tile) scale_lds[tid] = my_scale;     // visible after the first barrier below
    const int m0 = rgw0 * 4;
    const int rows_wg = min(p.RGW * 4, p.M - m0);
    // RC = row-group rounds parked per pass.  All R at once when the tile has few tokens (the R independent
    // reduction chains then overlap); two at a time when [tokens][rows] would not fit in LDS.
    auto epilogue = [&](auto rc_tag) {
    constexpr int RC = decltype(rc_tag)::value;
    constexpr int kParkStride = RC * kRoundRows + 4;        // ints per parked token; +4 keeps the writes conflict-free
#pragma unroll
    for (int c0 = 0; c0 < R; c0 += RC) {
        if (!builder) {
#pragma unroll
        for (int rr = 0; rr < RC; ++rr) {
            const int r = c0 + rr;
            if (r < R && Jlog == 4) {
                // both lanes of a pair hold the same total and store it to the same place
                park[(l >> 1) * kParkStride + rr * kRoundRows + lw * 4 + grp] =
                    reduce16<NEED32>(acc16[r], acc32[NEED32 ? r : 0], l);
            } else if (r < R) {
                int v[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[2 * q] = (int)acc16[r][q].x + (NEED32 ? acc32[r][2 * q] : 0);
                    v[2 * q + 1] = (int)acc16[r][q].y + (NEED32 ? acc32[r][2 * q + 1] : 0);
                }
                // Reduce-scatter over the sub-table selector j (the top Jlog bits of the lane's slice index): each
                // step exchanges half of the remaining tokens with the lane whose index differs in one bit.
                int tokoff = 0;
                bool owner = true;
                if (Jlog > 0) {
                    const bool hi = (l & 8) != 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int send = hi ? v[e] : v[e + 4];
                        const int keep = hi ? v[e + 4] : v[e];
                        v[e] = keep + lane_xor16<8>(send);
                    }
                    tokoff += hi ? 4 : 0;
                }
                if (Jlog > 1) {
                    const bool hi = (l & 4) != 0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int send = hi ? v[e] : v[e + 2];
                        const int keep = hi ? v[e + 2] : v[e];
                        v[e] = keep + lane_xor16<4>(send);
                    }
                    tokoff += hi ? 2 : 0;
                }
                if (Jlog > 2) {
                    const bool hi = (l & 2) != 0;
                    const int send = hi ? v[0] : v[1];
                    const int keep = hi ? v[1] : v[0];
                    v[0] = keep + lane_xor16<2>(send);
                    tokoff += hi ? 1 : 0;
                }
                if (Jlog > 3) {
                    v[0] += lane_xor16<1>(v[0]);
                    owner = (l & 1) == 0;
                }
                const int cnt = 8 >> min(Jlog, 3);
                if (owner) {
                    const int col = rr * kRoundRows + lw * 4 + grp;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (e < cnt) park[(8 * t + tokoff + e) * kParkStride + col] = v[e];
                }
            }
        }
        }
        wg_barrier_lds();
        for (int i = tid; i < RC * kRoundRows * n_tile; i += kThreads) {
            const int col = i % (RC * kRoundRows);
            const int nl = i / (RC * kRoundRows);
            const int mrow = c0 * kRoundRows + col;         // row inside the workgroup tile
            const int n = n0 + nl;
            if (mrow < rows_wg && mrow < R * kRoundRows && n < p.N) {
                const int val = park[nl * kParkStride + col];
                const int m = m0 + mrow;
                if (p.S == 1 && !p.partial) {
                    if (p.y) p.y[(size_t)n * p.ldy + m] = (float)val * (p.w_rows ? p.w_rows[m] * scale_lds[nl] : scale_lds[nl]);
                    if (p.acc) p.acc[(size_t)m * p.N + n] = val;
                } else {
                    p.ws[((size_t)(p.slot0 + ks) * p.N + n) * p.M + m] = val;
                }
            }
        }
        wg_barrier_lds();
    }
    };
    if (n_tile * (R * kRoundRows + 4) * 4 <= kTableBytes) epilogue(std::integral_constant<int, R>{});
    else epilogue(std::integral_constant<int, (R > 1 ? 2 : 1)>{});
}

// ---------------------------------------------------------------------------------------------
// Comparison path (not the method): the multiply-add way of Sec. 2.2.1 on the INT8 matrix cores.
// Packed bytes are unpacked to four INT8 weights through an 81-entry table in LDS and multiplied with
// v_mfma_i32_16x16x64_i8.  Activations are first copied to a [tokens][K] layout (k contiguous) so that a
// lane's 16 consecutive k of one token are one 16-byte load.
// ---------------------------------------------------------------------------------------------
// a_q token-chunked [N/8][K][8] -> aT [Npad][Kp], Npad = multiple of 16 >= N, Kp = multiple of 64 >= K, zero padded.
__global__ void __launch_bounds__(256) act_transpose_kernel(const int8_t* __restrict__ a_q, int N, int K, int Npad, int Kp,
                                                            int8_t* __restrict__ aT) {
    const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;     // one dword (4 k) of aT per thread
    const int kq = Kp / 4;
    if (i >= (size_t)Npad * kq) return;
    const int n = (int)(i / kq);
    const int k = (int)(i % kq) * 4;
    unsigned v = 0;
    if (n < N) {
        const int8_t* src = a_q + ((size_t)(n >> 3) * K) * 8 + (n & 7);
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (k + c < K) v |= (unsigned)(uint8_t)src[(size_t)(k + c) * 8] << (8 * c);
    }
    *(unsigned*)(aT + (size_t)n * Kp + k) = v;
}

struct MfmaParams {
    const uint8_t* packed;
    const int8_t* aT;
    const float* a_scale;
    float* y;
    int32_t* acc;
    float w_scale;
    int M, N, Npad, Kp, KCn, RGtotal, ldy;
};

// One workgroup = 4 waves x 16 output rows; each wave multiplies its 16 x Kp weight strip with NT tiles of 16 tokens.
template <int NT>
__global__ void __launch_bounds__(256) mfma_kernel(const MfmaParams p) {
    __shared__ unsigned dec[kRows];            // index -> four INT8 weights (first weight in the low byte)
    const int tid = threadIdx.x;
    if (tid < kRows) {
        const int d0 = tid / 27, d1 = (tid / 9) % 3, d2 = (tid / 3) % 3, d3 = tid % 3;
        dec[tid] = ((unsigned)(d0 - 1) & 0xffu) | (((unsigned)(d1 - 1) & 0xffu) << 8) | (((unsigned)(d2 - 1) & 0xffu) << 16) |
                   (((unsigned)(d3 - 1) & 0xffu) << 24);
    }
    __syncthreads();
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i = lane & 15;                   // row of the A tile / token of the B tile / column of the C tile
    const int kblk = lane >> 4;                // which 16 of the 64 k of a step this lane holds (same for A and B)
    const int m_row = blockIdx.x * 64 + wave * 16 + i;
    const int n0 = blockIdx.y * 16 * NT;
    const int mc = min(m_row, p.RGtotal * 4 - 1);          // rows past the padded matrix read row data that is discarded
    const unsigned char* arow = p.packed + ((size_t)(mc >> 2) * p.KCn) * 64 + (mc & 3) * 16 + kblk * 4;
    const int8_t* brow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) brow[t] = p.aT + (size_t)min(n0 + 16 * t + i, p.Npad - 1) * p.Kp + kblk * 16;
    i32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = i32x4{0, 0, 0, 0};
    // Operands of the next two K steps are in flight while one step is multiplied (loads are clamped to the last
    // step instead of branching; the surplus loads are never used).
    auto load_w = [&](int ks) { return *(const unsigned*)(arow + (size_t)min(ks, p.KCn - 1) * 64); };
    auto load_b = [&](int ks, i32x4 (&b)[NT]) {
#pragma unroll
        for (int t = 0; t < NT; ++t) b[t] = *(const i32x4*)(brow[t] + (size_t)min(ks, p.KCn - 1) * 64);
    };
    auto mul = [&](unsigned w, const i32x4 (&b)[NT]) {
        const i32x4 a = {(int)dec[w & 0xffu], (int)dec[(w >> 8) & 0xffu], (int)dec[(w >> 16) & 0xffu], (int)dec[w >> 24]};
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[t], acc[t], 0, 0, 0);
    };
    unsigned w0 = load_w(0), w1 = load_w(1), w2;
    i32x4 b0[NT], b1[NT], b2[NT];
    load_b(0, b0);
    load_b(1, b1);
    for (int ks = 0; ks < p.KCn; ks += 3) {
        w2 = load_w(ks + 2); load_b(ks + 2, b2);
        mul(w0, b0);
        if (ks + 1 >= p.KCn) break;
        w0 = load_w(ks + 3); load_b(ks + 3, b0);
        mul(w1, b1);
        if (ks + 2 >= p.KCn) break;
        w1 = load_w(ks + 4); load_b(ks + 4, b1);
        mul(w2, b2);
    }
    // C tile: lane (column = token i, row block kblk) holds rows 4*kblk .. 4*kblk+3
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = n0 + 16 * t + i;
        if (n < p.N) {
            const float sc = p.w_scale * p.a_scale[n];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = blockIdx.x * 64 + wave * 16 + 4 * kblk + r;
                if (m < p.M) {
                    const int v = acc[t][r];
                    if (p.y) p.y[(size_t)n * p.ldy + m] = (float)v * sc;
                    if (p.acc) p.acc[(size_t)m * p.N + n] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 1.60-bit packing (g = 5; Sec. 3.3 "Flexible sub-2-bit weight packing"): five weights per byte, 243-row sub-tables.
// Same roles, same 256-byte table rows (16 sub-tables x 8 tokens) and same hand-over by barriers as lookup_kernel;
// what changes: a slot is 243 x 256 B = 62 208 B, so two slots are resident and a half-stage is ONE slot, i.e. one
// byte of the weight dword (bytes 0..3 of a dword use slots 0,1,0,1); a lane builds 9-row groups that share their
// three leading digits (27 groups per sub-table slice, handed out over the 16 lane groups of the build waves in two
// passes); the INT16 block is 48 lookups (bound 51 = floor(32767 / (127*5)), Sec. 3.4).
// ---------------------------------------------------------------------------------------------
constexpr int kRows5 = 243;
constexpr int kSlot5Bytes = kRows5 * kRowBytes;          // 62208
constexpr int kScale5Base = 2 * kSlot5Bytes;             // 124416: output scales of the tile's 8 tokens
constexpr int kLds5Bytes = kScale5Base + 128 * 4;        // 124928
constexpr int kBlockLookups5 = 51;
constexpr int kWidenEvery5 = 12;                         // dword stages between widenings: 48 lookups <= 51

struct Lookup5Params {
    const uint8_t* packed;
    const int8_t* a_q;
    const float* a_scale;
    float* y;
    int32_t* acc;
    int32_t* ws;
    float w_scale;
    int M, K, N, G, KCn, RGtotal, ldy;
    int S, tiles_m, tiles_n, RGW, dstages_total, dstages_per_split, total_tiles, per_xcd;
    int Ka;        // rows per token chunk of the activation tensor a_q points into
    int partial;   // mixed packing: write INT32 sums to ws slots ks also when K is not split
};

// Table read of lookup I (= row group I) of the half-stage that uses byte B of the weight dwords (slot B & 1).
template <int R, int B, int I>
__device__ __forceinline__ i32x4 lookup5_read(const unsigned (&w)[R], unsigned lanebase) {
    constexpr unsigned sel = 0x0c0c0000u | ((4u + (unsigned)B) << 8);
    const unsigned addr = __builtin_amdgcn_perm(w[I], lanebase, sel);   // idx*256 + slice*16
    return lds_read128<(B & 1) * (kSlot5Bytes / 16)>(addr);
}

template <int R, int B, int NB, int K0>
__device__ __forceinline__ void lookup5_batches(const unsigned (&w)[R], unsigned lanebase, s16x2 (&acc16)[R][4],
                                                i32x4 (&cur)[NB]) {
    if constexpr (K0 < R) {
        i32x4 nxt[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) nxt[i] = i32x4{0, 0, 0, 0};
        static_for<0, NB>([&](auto ic_) {
            constexpr int i = decltype(ic_)::value;
            if constexpr (K0 + NB + i < R) nxt[i] = lookup5_read<R, B, (K0 + NB + i < R ? K0 + NB + i : 0)>(w, lanebase);
        });
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NB>([&](auto ic_) {
            constexpr int i = decltype(ic_)::value;
            if constexpr (K0 + i < R) lookup_accumulate<R, (K0 + i < R ? K0 + i : 0)>(acc16, cur[i]);
        });
        __builtin_amdgcn_sched_barrier(0);
        lookup5_batches<R, B, NB, K0 + NB>(w, lanebase, acc16, nxt);
    }
}

// The R lookups of one half-stage (Alg. 1 lines 3-6), software pipelined in batches of four.
template <int R, int B>
__device__ __forceinline__ void lookup5_half(const unsigned (&w)[R], unsigned lanebase, s16x2 (&acc16)[R][4]) {
    constexpr int NB = 4;
    i32x4 first[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) first[i] = i32x4{0, 0, 0, 0};
    static_for<0, NB>([&](auto ic_) {
        constexpr int i = decltype(ic_)::value;
        if constexpr (i < R) first[i] = lookup5_read<R, B, (i < R ? i : 0)>(w, lanebase);
    });
    __builtin_amdgcn_sched_barrier(0);
    lookup5_batches<R, B, NB, 0>(w, lanebase, acc16, first);
}

template <int R, bool NEED32>
__global__ void __launch_bounds__(kThreads) lookup5_kernel(const Lookup5Params p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem5[];
    if (lds_base_of(smem5) != 0u) return;      // table addresses are formed as idx*256 + slice*16 from LDS address 0
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int L = (int)(blockIdx.x & 7) * p.per_xcd + (int)(blockIdx.x >> 3);      // XCD-aware tile order, as in lookup_kernel
    if ((int)(blockIdx.x >> 3) >= p.per_xcd || L >= p.total_tiles) return;
    const int ks = L % p.S;
    L /= p.S;
    const int nt = L % p.tiles_n;
    const int mt = L / p.tiles_n;
    const int n0 = nt * 8;                      // 8 tokens per workgroup (16 sub-tables per table row)
    const int rgw0 = mt * p.RGW;

    const int l = lane & 15;                    // slice = sub-table selector
    const int grp = lane >> 4;
    const unsigned lanebase = (unsigned)l * 16u;
    const int ds_begin = ks * p.dstages_per_split;        // a dword stage = 4 half-stages = 64 groups = 320 weights
    const int ds_end = min(p.dstages_total, ds_begin + p.dstages_per_split);
    const bool builder = wave < kBuildWaves;
    const int lw = wave - kBuildWaves;

    typedef __attribute__((address_space(3))) float lds_f32;
    lds_f32* scale_lds = (lds_f32*)(unsigned)kScale5Base;
    float my_scale = 0.0f;
    if (tid < 8 && n0 + tid < p.N) my_scale = p.w_scale * p.a_scale[n0 + tid];

    s16x2 acc16[R][4];
    int acc32[NEED32 ? R : 1][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc16[r][q] = s16x2{0, 0};
    if (NEED32) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc32[r][e] = 0;
    }

    if (builder) {
        __builtin_amdgcn_s_setprio(3);
        // Tasks of a lane per half-stage: slice l, leading digits (d0,d1,d2) = ua, and = ub when ub < 27.
        const int ua = 4 * wave + grp, ub = 16 + ua;
        const bool has_b = ub < 27;
        const bool tok_valid = n0 < p.N;
        const int chunk = n0 >> 3;
        const int hs0 = 4 * ds_begin, hs1 = 4 * ds_end;
        unsigned actA[5][2], actB[5][2];
        bool validA = false, validB = false;

        // Half-stage hs = 4*dstage + b holds, in slot b & 1, the sub-tables of groups kg = dstage*64 + 4*slice + b.
        auto fetch_act = [&](int hs, unsigned (&act)[5][2], bool& valid) {
            const int kg = (hs >> 2) * 64 + 4 * l + (hs & 3);
            valid = (hs < hs1) && (kg < p.G) && tok_valid;
            const int kgc = min(kg, p.G - 1);               // clamped into the tensor; validity applied at use
            const int cc = tok_valid ? chunk : 0;
            const i32x2* src = (const i32x2*)(p.a_q + ((size_t)cc * p.Ka + 5 * (size_t)kgc) * 8);   // 5 rows x 8 tokens
#pragma unroll
            for (int c = 0; c < 5; ++c) {
                const i32x2 v = src[c];
                act[c][0] = (unsigned)v.x;
                act[c][1] = (unsigned)v.y;
            }
        };
        // Nine rows that share their three leading digits u: base +- a3 +- a4 (topological order of Sec. 4).
        auto build_group = [&](unsigned dst, int u, const s16x2 (&a)[5][4]) {
            const short d0 = (short)(u / 9 - 1), d1 = (short)((u / 3) % 3 - 1), d2 = (short)(u % 3 - 1);
            const s16x2 m0 = {d0, d0}, m1 = {d1, d1}, m2 = {d2, d2};
            s16x2 rows[9][4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const s16x2 base = a[0][q] * m0 + a[1][q] * m1 + a[2][q] * m2;
                const s16x2 lo = base - a[3][q], hi = base + a[3][q];
                rows[0][q] = lo - a[4][q]; rows[1][q] = lo; rows[2][q] = lo + a[4][q];
                rows[3][q] = base - a[4][q]; rows[4][q] = base; rows[5][q] = base + a[4][q];
                rows[6][q] = hi - a[4][q]; rows[7][q] = hi; rows[8][q] = hi + a[4][q];
            }
            const unsigned dst9 = dst + (unsigned)(9 * u) * kRowBytes;
            static_for<0, 9>([&](auto ic_) {
                constexpr int i = decltype(ic_)::value;
                lds_write128<i * 16>(dst9, i32x4{as_int(rows[i][0]), as_int(rows[i][1]), as_int(rows[i][2]), as_int(rows[i][3])});
            });
        };
        auto build_half = [&](int hs, unsigned (&act)[5][2], bool valid) {
            if (!valid) {
#pragma unroll
                for (int c = 0; c < 5; ++c) { act[c][0] = 0u; act[c][1] = 0u; }
            }
            s16x2 a[5][4];
#pragma unroll
            for (int c = 0; c < 5; ++c)
#pragma unroll
                for (int q = 0; q < 4; ++q) a[c][q] = unpack_pair(act[c][q >> 1], q & 1);
            const unsigned dst = (unsigned)(hs & 1) * kSlot5Bytes + (unsigned)l * 16u;
            build_group(dst, ua, a);
            if (has_b) build_group(dst, ub, a);
        };
        if (hs0 < hs1) {
            fetch_act(hs0, actA, validA);
            fetch_act(hs0 + 1, actB, validB);
            build_half(hs0, actA, validA);
            fetch_act(hs0 + 2, actA, validA);
        }
        wg_barrier_lds();
        for (int hs = hs0; hs < hs1; hs += 2) {     // hs1 - hs0 is a multiple of 4
            build_half(hs + 1, actB, validB);       // lookups read slot 0 (hs): fill slot 1
            fetch_act(hs + 3, actB, validB);
            wg_barrier_lds();
            if (hs + 2 < hs1) build_half(hs + 2, actA, validA);   // lookups read slot 1 (hs+1): fill slot 0
            fetch_act(hs + 4, actA, validA);
            wg_barrier_lds();
        }
        __builtin_amdgcn_s_setprio(0);
    } else {
        const unsigned char* wbase[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int rgl = r * kLookupWaves + lw;
            const int rg = rgw0 + rgl;
            const bool valid = (rgl < p.RGW) && (rg < p.RGtotal);
            wbase[r] = p.packed + ((size_t)(valid ? rg : 0) * p.KCn) * 64;
        }
        // Dword q = ds*16 + slice of each row, fetched one dword stage ahead.  A tile index past the end of K is
        // clamped to the last tile and meets tables built from zero activations; rows past M are clamped to row group
        // 0 and never stored.
        auto load_weights = [&](int ds, unsigned (&wdst)[R]) {
            const int q = ds * 16 + l;
            const int kc = min(q >> 2, p.KCn - 1);
            const unsigned voff = (unsigned)(kc * 64 + grp * 16 + (q & 3) * 4);
#pragma unroll
            for (int r = 0; r < R; ++r) wdst[r] = *(const unsigned*)(wbase[r] + voff);
        };
        auto dstage = [&](int ds, unsigned (&w)[R], unsigned (&wnext)[R]) {
            load_weights(ds + 1, wnext);
            lookup5_half<R, 0>(w, lanebase, acc16);
            wg_barrier_lds();
            lookup5_half<R, 1>(w, lanebase, acc16);
            wg_barrier_lds();
            lookup5_half<R, 2>(w, lanebase, acc16);
            wg_barrier_lds();
            lookup5_half<R, 3>(w, lanebase, acc16);
            wg_barrier_lds();
            if (NEED32 && ((ds - ds_begin) % kWidenEvery5 == kWidenEvery5 - 1)) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc32[r][2 * q] += (int)acc16[r][q].x;
                        acc32[r][2 * q + 1] += (int)acc16[r][q].y;
                        acc16[r][q] = s16x2{0, 0};
                    }
            }
        };
        unsigned wa[R], wb[R];
        load_weights(ds_begin, wa);
        wg_barrier_lds();                          // slot 0 of the first dword stage is built
        for (int ds = ds_begin; ds < ds_end; ds += 2) {
            dstage(ds, wa, wb);
            if (ds + 1 < ds_end) dstage(ds + 1, wb, wa);
        }
    }

    // ---- epilogue: reduce the 16 partial sums per token across the lane group, park as [token][row], store rows.
    lds_i32* park = (lds_i32*)0u;
    if (tid < 8) scale_lds[tid] = my_scale;
    constexpr int kParkStride = R * kRoundRows + 4;
    const int m0 = rgw0 * 4;
    const int rows_wg = min(p.RGW * 4, p.M - m0);
    if (!builder) {
#pragma unroll
        for (int r = 0; r < R; ++r)
            park[(l >> 1) * kParkStride + r * kRoundRows + lw * 4 + grp] = reduce16<NEED32>(acc16[r], acc32[NEED32 ? r : 0], l);
    }
    wg_barrier_lds();
    for (int i = tid; i < R * kRoundRows * 8; i += kThreads) {
        const int col = i % (R * kRoundRows);
        const int nl = i / (R * kRoundRows);
        const int n = n0 + nl;
        if (col < rows_wg && n < p.N) {
            const int val = park[nl * kParkStride + col];
            const int m = m0 + col;
            if (p.S == 1 && !p.partial) {
                if (p.y) p.y[(size_t)n * p.ldy + m] = (float)val * scale_lds[nl];
                if (p.acc) p.acc[(size_t)m * p.N + n] = val;
            } else {
                p.ws[((size_t)ks * p.N + n) * p.M + m] = val;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// N <= 2 (one or two parallel tokens: decoding).  The tables of a 256-group chunk of K then take 83 KB (two tokens: an
// entry is one dword = two INT16 sums) or 42 KB (one token: an entry is one INT16), and a workgroup can sweep all of K
// by itself: no split-K partial sums, no second kernel, one barrier pair per chunk.  The waves build a chunk
// together, then all 16 look it up.
//   Tables: NTOK = 2: sub-table kg of the chunk = 81 dwords at kg*324 + idx*4; a build lane (kg, leading digit d0)
//           makes 27 entries and stores them as single dwords.  NTOK = 1: sub-table = 81 INT16 + 1 pad = 41 dwords at
//           kg*164 + idx*2; a build lane owns a whole sub-table.  Consecutive lanes are 27 or 41 dwords apart: odd, so
//           every store of a wave is free of bank conflicts.
//   Lookups: wave w reads the packed tile w of the chunk (16 groups); a lane owns an output row and 16/PARTS of the
//           tile's groups (PARTS lanes per row), RR rows one after the other.  Address = lane constant + idx * entry
//           size, the group's offset is an immediate: 3 VALU instructions per lookup.  With PARTS = 1 all lanes of a
//           read look into the same sub-table, whose dwords lie in distinct banks (equal bank = equal address =
//           broadcast).  Two tokens: INT16 sums inside a chunk (at most 16 lookups), INT32 across chunks; one token:
//           INT32 throughout.  The 16*PARTS partial sums per row are added through LDS at the end.
//   Tiles past the end of K are neither built nor looked up.
// ---------------------------------------------------------------------------------------------
constexpr int kNarrowChunk = 256;                        // k-groups per chunk = 16 packed tiles, one per wave
constexpr int narrow_sub_bytes(int ntok) { return ntok == 2 ? 324 : 164; }
constexpr int narrow_tab_bytes(int ntok) { return kNarrowChunk * narrow_sub_bytes(ntok); }   // 82944 / 41984

struct NarrowParams {
    const uint8_t* packed;
    const int8_t* a_q;
    const float* a_scale;
    const float* w_rows;
    float* y;
    int32_t* acc;
    float w_scale;
    int M, K, N, G, KCn, RGtotal, ldy, chunks;
    // fused quantisation (FUSED): fp32 activations [N][ldx] instead of a_q / a_scale
    const float* x;
    float* a_scale_out;       // optional: the token scales, written by workgroup 0
    int64_t ldx;
    int x_vec;
};
// FUSED keeps, behind the tables, two dwords per k-group (the four codes of token 0 and of token 1) and the 16 x 2
// partial absmax values.
constexpr int narrow_fused_lds_bytes(int ntok, int chunks) { return narrow_tab_bytes(ntok) + chunks * kNarrowChunk * 8 + 128; }
constexpr int narrow_fused_max_chunks(int ntok) {        // 39 (K <= 39936) for two tokens, 59 for one
    return (160 * 1024 - narrow_tab_bytes(ntok) - 128) / (kNarrowChunk * 8);
}

template <int NTOK, int PARTS, int RR, bool FUSED>
__global__ void __launch_bounds__(kThreads) narrow_kernel(const NarrowParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_n[];
    if (lds_base_of(smem_n) != 0u) return;               // table addresses below are absolute LDS addresses
    constexpr int SUB = narrow_sub_bytes(NTOK);           // bytes per sub-table
    constexpr int TAB = narrow_tab_bytes(NTOK);
    constexpr int RPW = 64 / PARTS;                       // rows of one pass of a wave
    constexpr int ROWS = RPW * RR;                        // rows of the workgroup
    constexpr int NBYTES = 16 / PARTS;                    // groups (= bytes of the packed tile row) per lane
    typedef __attribute__((address_space(3))) short lds_i16;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m0 = blockIdx.x * ROWS;

    // ---- build geometry.  Two tokens: thread tid < 768 owns (k-group tid/3, leading digit tid%3) of every chunk;
    //      one token: thread tid < 256 owns k-group tid.
    const bool builds = tid < (NTOK == 2 ? 3 : 1) * kNarrowChunk;
    const int kg_b = NTOK == 2 ? tid / 3 : tid;
    const int d0 = tid - 3 * kg_b;                        // NTOK == 2 only
    // ---- lookup geometry
    const int part = lane / RPW, row_l = lane % RPW;
    const unsigned lane_tab = (unsigned)(wave * 16 + part * NBYTES) * SUB;   // first sub-table of this lane
    const unsigned char* wrow[RR];
    bool row_ok[RR];
#pragma unroll
    for (int rr = 0; rr < RR; ++rr) {
        const int m = m0 + rr * RPW + row_l;
        row_ok[rr] = m < p.M;
        const int mc = row_ok[rr] ? m : 0;
        wrow[rr] = p.packed + ((size_t)(mc >> 2) * p.KCn) * 64 + (mc & 3) * 16 + part * NBYTES;
    }
    int acc32[RR][2];
#pragma unroll
    for (int rr = 0; rr < RR; ++rr) { acc32[rr][0] = 0; acc32[rr][1] = 0; }

    // activations of tokens 0,1 for the four rows of a k-group: bytes 0,1 of a_q[0][4kg + j][*] (chunk 0 of tokens)
    auto fetch_act = [&](int c, unsigned (&a)[4]) {
        const int kg = min(c * kNarrowChunk + kg_b, p.G - 1);          // clamped; validity applied at use
        if constexpr (FUSED) {
            const i32x2 d = *(const __attribute__((address_space(3))) i32x2*)(unsigned)(TAB + kg * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j)                                // {code of token 0, code of token 1} of row j
                a[j] = __builtin_amdgcn_perm((unsigned)d.y, (unsigned)d.x, 0x0c0c0000u | ((4u + j) << 8) | (unsigned)j);
        } else {
            const unsigned short* src = (const unsigned short*)(p.a_q + (size_t)(4 * kg) * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] = src[4 * j];             // 8 bytes per activation row
        }
    };
    typedef unsigned wvec __attribute__((ext_vector_type(4)));
    auto fetch_w = [&](int c, wvec (&w)[RR]) {
        const int tile = min(c * 16 + wave, p.KCn - 1);                // clamped; tiles past the end are not looked up
#pragma unroll
        for (int rr = 0; rr < RR; ++rr) {
            const unsigned char* src = wrow[rr] + (size_t)tile * 64;
            if constexpr (PARTS == 1) {
                const i32x4 v = *(const i32x4*)src;
                w[rr] = wvec{(unsigned)v.x, (unsigned)v.y, (unsigned)v.z, (unsigned)v.w};
            } else if constexpr (PARTS == 2) {
                const i32x2 v = *(const i32x2*)src;
                w[rr] = wvec{(unsigned)v.x, (unsigned)v.y, 0u, 0u};
            } else {
                w[rr] = wvec{*(const unsigned*)src, 0u, 0u, 0u};
            }
        }
    };

    // The loop streams the packed weights from HBM and a chunk takes less than the latency of a load, so the weights
    // are fetched WD chunks ahead (a ring of WD + 1 register sets; fewer for more rows per lane), the activations two.
    constexpr int WD = RR == 1 ? 4 : (RR == 2 ? 2 : 1);
    unsigned act_cur[4] = {0, 0, 0, 0}, act_nxt[4] = {0, 0, 0, 0}, act_nx2[4] = {0, 0, 0, 0};
    wvec w_ring[WD + 1][RR];                               // w_ring[0] = the chunk being looked up
    wvec (&w_cur)[RR] = w_ring[0];
#pragma unroll
    for (int d = 0; d < WD; ++d) fetch_w(d, w_ring[d]);
    float sc[2] = {0.0f, 0.0f};                                        // token scales (FUSED)
    if constexpr (FUSED) {
        // Quantise the one or two rows of x over all of K: thread tid takes the float4 (= k-group) tid + 1024 i.
        typedef __attribute__((address_space(3))) float lds_f32;
        typedef __attribute__((address_space(3))) i32x2 lds_i32x2;
        lds_f32* red = (lds_f32*)(unsigned)(TAB + p.chunks * kNarrowChunk * 8);   // [wave][token]
        lds_i32x2* aq = (lds_i32x2*)(unsigned)TAB;
        const int nquad = p.G;
        auto load4 = [&](int n, int qi) -> f32x4 {
            const float* src = p.x + (size_t)n * p.ldx + 4 * (size_t)qi;
            if (p.x_vec) return *(const f32x4*)src;
            return f32x4{src[0], src[1], src[2], src[3]};
        };
        auto absmax4 = [](float m, const f32x4 v) {
            return fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
        };
        auto codes4 = [](const f32x4 v, float inv) { return (int)quant_codes4(v, inv); };
        constexpr int NVC = 4;                                         // float4 per thread and token kept (K <= 16384)
        f32x4 xv[NTOK][NVC];
        float amax[NTOK];
#pragma unroll
        for (int n = 0; n < NTOK; ++n) {
            amax[n] = 0.0f;
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = tid + kThreads * i;
                xv[n][i] = (n < p.N && qi < nquad) ? load4(n, qi) : f32x4{0.f, 0.f, 0.f, 0.f};
                amax[n] = absmax4(amax[n], xv[n][i]);
            }
            if (n < p.N)
                for (int q0 = kThreads * NVC; q0 < nquad; q0 += kThreads * NVC) {   // NVC loads in flight per pass
                    f32x4 tv[NVC];
#pragma unroll
                    for (int i = 0; i < NVC; ++i) {
                        const int qi = q0 + tid + kThreads * i;
                        tv[i] = qi < nquad ? load4(n, qi) : f32x4{0.f, 0.f, 0.f, 0.f};
                    }
#pragma unroll
                    for (int i = 0; i < NVC; ++i) amax[n] = absmax4(amax[n], tv[i]);
                }
            for (int off = 32; off > 0; off >>= 1) amax[n] = fmaxf(amax[n], __shfl_xor(amax[n], off));
        }
        if (lane == 0) {
#pragma unroll
            for (int n = 0; n < NTOK; ++n) red[wave * 2 + n] = amax[n];
        }
        wg_barrier_lds();
        float inv[NTOK];
#pragma unroll
        for (int n = 0; n < NTOK; ++n) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) v = fmaxf(v, red[w * 2 + n]);
            inv[n] = (v > 0.0f) ? 127.0f / v : 0.0f;                   // IEEE divisions, as in quantize_kernel
            sc[n] = v / 127.0f;
        }
        if (blockIdx.x == 0 && tid < p.N && p.a_scale_out) p.a_scale_out[tid] = tid == 0 ? sc[0] : sc[1];
#pragma unroll
        for (int i = 0; i < NVC; ++i) {
            const int qi = tid + kThreads * i;
            if (qi < nquad) aq[qi] = i32x2{codes4(xv[0][i], inv[0]), NTOK == 2 ? codes4(xv[NTOK - 1][i], inv[NTOK - 1]) : 0};
        }
        for (int q0 = kThreads * NVC; q0 < nquad; q0 += kThreads * NVC) {
            f32x4 tv[NTOK][NVC];
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = q0 + tid + kThreads * i;
#pragma unroll
                for (int n = 0; n < NTOK; ++n)
                    tv[n][i] = (n < p.N && qi < nquad) ? load4(n, qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = q0 + tid + kThreads * i;
                if (qi < nquad)
                    aq[qi] = i32x2{codes4(tv[0][i], inv[0]), NTOK == 2 ? codes4(tv[NTOK - 1][i], inv[NTOK - 1]) : 0};
            }
        }
        wg_barrier_lds();
    }
    if (builds) { fetch_act(0, act_cur); fetch_act(1, act_nxt); }
    for (int c = 0; c < p.chunks; ++c) {
        fetch_w(c + WD, w_ring[WD]);
        if (builds) fetch_act(c + 2, act_nx2);
        // ---------------- build the chunk's tables (topological order of Sec. 4: one add per entry); only the groups
        //                  of real tiles: the padding groups of the last tile get all-zero tables
        if (builds) {
            const int kgg = c * kNarrowChunk + kg_b;
            if (kgg < p.KCn * 16) {
                const bool valid = kgg < p.G;
                if constexpr (NTOK == 2) {
                    s16x2 a[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const unsigned v = valid ? act_cur[j] : 0u;
                        a[j] = s16x2{(short)(signed char)(v & 0xffu), (short)(signed char)((v >> 8) & 0xffu)};
                    }
                    const short s0 = (short)(d0 - 1);
                    const s16x2 base = a[0] * s16x2{s0, s0};
                    lds_i32* dst = (lds_i32*)(unsigned)(kg_b * SUB + d0 * 108);
                    static_for<0, 3>([&](auto c1) {
                        constexpr int d1 = decltype(c1)::value;
                        const s16x2 b1 = d1 == 0 ? base - a[1] : (d1 == 1 ? base : base + a[1]);
                        static_for<0, 3>([&](auto c2) {
                            constexpr int d2 = decltype(c2)::value;
                            const s16x2 b2 = d2 == 0 ? b1 - a[2] : (d2 == 1 ? b1 : b1 + a[2]);
                            dst[9 * d1 + 3 * d2 + 0] = as_int(b2 - a[3]);
                            dst[9 * d1 + 3 * d2 + 1] = as_int(b2);
                            dst[9 * d1 + 3 * d2 + 2] = as_int(b2 + a[3]);
                        });
                    });
                } else {
                    int a[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) a[j] = valid ? (int)(signed char)(act_cur[j] & 0xffu) : 0;
                    int e[82];
                    static_for<0, 3>([&](auto c0) {
                        constexpr int e0 = decltype(c0)::value;
                        const int b0 = e0 == 0 ? -a[0] : (e0 == 1 ? 0 : a[0]);
                        static_for<0, 3>([&](auto c1) {
                            constexpr int d1 = decltype(c1)::value;
                            const int b1 = d1 == 0 ? b0 - a[1] : (d1 == 1 ? b0 : b0 + a[1]);
                            static_for<0, 3>([&](auto c2) {
                                constexpr int d2 = decltype(c2)::value;
                                const int b2 = d2 == 0 ? b1 - a[2] : (d2 == 1 ? b1 : b1 + a[2]);
                                e[27 * e0 + 9 * d1 + 3 * d2 + 0] = b2 - a[3];
                                e[27 * e0 + 9 * d1 + 3 * d2 + 1] = b2;
                                e[27 * e0 + 9 * d1 + 3 * d2 + 2] = b2 + a[3];
                            });
                        });
                    });
                    e[81] = 0;
                    lds_i32* dst = (lds_i32*)(unsigned)(kg_b * SUB);
                    static_for<0, 41>([&](auto ci) {
                        constexpr int i = decltype(ci)::value;      // entries 2i (low half) and 2i + 1 (high half)
                        dst[i] = (int)__builtin_amdgcn_perm((unsigned)e[2 * i + 1], (unsigned)e[2 * i], 0x05040100u);
                    });
                }
            }
        }
        wg_barrier_lds();
        // ---------------- look the chunk up
        if (c * 16 + wave < p.KCn) {                                   // wave-uniform
#pragma unroll
            for (int rr = 0; rr < RR; ++rr) {
                if constexpr (NTOK == 2) {
                    s16x2 acc16 = {0, 0};
                    static_for<0, NBYTES>([&](auto bc) {
                        constexpr int b = decltype(bc)::value;
                        const unsigned idx = (w_cur[rr][b >> 2] >> (8 * (b & 3))) & 0xffu;
                        const unsigned addr = lane_tab + idx * 4u;
                        acc16 += as_s16x2(((const lds_i32*)addr)[b * (SUB / 4)]);
                    });
                    acc32[rr][0] += (int)acc16.x;
                    acc32[rr][1] += (int)acc16.y;
                } else {
                    static_for<0, NBYTES>([&](auto bc) {
                        constexpr int b = decltype(bc)::value;
                        const unsigned idx = (w_cur[rr][b >> 2] >> (8 * (b & 3))) & 0xffu;
                        const unsigned addr = lane_tab + idx * 2u;
                        acc32[rr][0] += (int)((const lds_i16*)addr)[b * (SUB / 2)];
                    });
                }
            }
        }
        wg_barrier_lds();
#pragma unroll
        for (int j = 0; j < 4; ++j) { act_cur[j] = act_nxt[j]; act_nxt[j] = act_nx2[j]; }
#pragma unroll
        for (int d = 0; d < WD; ++d)
#pragma unroll
            for (int rr = 0; rr < RR; ++rr) w_ring[d][rr] = w_ring[d + 1][rr];
    }

    // ---------------- add the 16*PARTS partial sums of every (row, token) through LDS, scale, store
    lds_i32* red = (lds_i32*)0u;                          // [16*PARTS][ROWS][2], reuses the table space
#pragma unroll
    for (int rr = 0; rr < RR; ++rr) {
        const int ri = rr * RPW + row_l;
        const int pi = wave * PARTS + part;
        red[(pi * ROWS + ri) * 2 + 0] = acc32[rr][0];
        red[(pi * ROWS + ri) * 2 + 1] = acc32[rr][1];
    }
    wg_barrier_lds();
    for (int i = tid; i < ROWS * 2; i += kThreads) {
        const int ri = i >> 1, n = i & 1;
        const int m = m0 + ri;
        if (m < p.M && n < p.N) {
            int v = 0;
            for (int pi = 0; pi < 16 * PARTS; ++pi) v += red[(pi * ROWS + ri) * 2 + n];
            const float s_n = FUSED ? (n ? sc[1] : sc[0]) : p.a_scale[n];
            if (p.y) p.y[(size_t)n * p.ldy + m] = (float)v * ((p.w_rows ? p.w_rows[m] : p.w_scale) * s_n);
            if (p.acc) p.acc[(size_t)m * p.N + n] = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Layout ablation (Sec. 5.6, Sec. 3.3): the mpGeMM on a table with the token index outermost, lut[n][kg][i].  A
// lookup then yields one value for one token (1 -> 1), so every (row, group, token) is a 2-byte gather.  A wave takes
// 64 rows of one token (its lanes gather from the 162 bytes of one sub-table at a time); INT32 accumulation.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) token_outer_lookup_kernel(const uint8_t* __restrict__ packed,
                                                                 const int16_t* __restrict__ lut, int M, int N, int G,
                                                                 int KCn, float w_scale, const float* __restrict__ a_scale,
                                                                 float* __restrict__ y, int64_t ldy,
                                                                 int32_t* __restrict__ acc) {
    const int m = blockIdx.x * 64 + (threadIdx.x & 63);
    const int n = blockIdx.y * 4 + (threadIdx.x >> 6);          // uniform per wave
    if (n >= N) return;
    const int mc = m < M ? m : 0;
    const unsigned char* wrow = packed + ((size_t)(mc >> 2) * KCn) * 64 + (mc & 3) * 16;
    const int16_t* tab = lut + (size_t)n * G * kRows;
    int sum = 0;
    for (int kc = 0; kc < KCn; ++kc) {
        const i32x4 w = *(const i32x4*)(wrow + (size_t)kc * 64);   // 16 groups of this row
        const unsigned wd[4] = {(unsigned)w.x, (unsigned)w.y, (unsigned)w.z, (unsigned)w.w};
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            const int kg = kc * 16 + b;
            const unsigned idx = (wd[b >> 2] >> (8 * (b & 3))) & 0xffu;
            if (kg < G) sum += tab[(size_t)kg * kRows + min(idx, (unsigned)(kRows - 1))];   // padding groups (index 40) have no table
        }
    }
    if (m < M) {
        if (y) y[(size_t)n * ldy + m] = (float)sum * (w_scale * a_scale[n]);
        if (acc) acc[(size_t)m * N + n] = sum;
    }
}

// Sum of the split-K partials (any order is exact: integers) + scale step.
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const int32_t* __restrict__ ws, int S, int M, int N,
                                                            float w_scale, const float* __restrict__ w_rows,
                                                            const float* __restrict__ a_scale,
                                                            float* __restrict__ y, int64_t ldy,
                                                            int32_t* __restrict__ acc) {
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i >= (size_t)M * N) return;
    int m = (int)(i % M);
    int n = (int)(i / M);
    int v = 0;
    for (int s = 0; s < S; ++s) v += ws[((size_t)s * N + n) * M + m];
    if (y) y[(size_t)n * ldy + m] = (float)v * ((w_rows ? w_rows[m] : w_scale) * a_scale[n]);
    if (acc) acc[(size_t)m * N + n] = v;
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
struct Plan {
    int Jlog, R, S;
};

thread_local Plan t_forced = {-1, 0, 0};

const int kSupportedR[] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 14};

bool r_supported(int R) {
    for (int v : kSupportedR)
        if (v == R) return true;
    return false;
}

bool shape_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && N >= 1 && K >= 4 && (K % 4) == 0 && M < kMaxDim && K < kMaxDim && N < kMaxDim;
}

struct Derived {
    int G, KCn, RGtotal, n_tile, tiles_n, tiles_m, RGW, stages_total, stages_per_split, total, per_xcd;
    bool need32;
};

Derived derive(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    Derived d;
    d.G = (int)(K / 4);
    d.KCn = (d.G + 15) / 16;
    d.RGtotal = (int)((M + 3) / 4);
    int J = 1 << pl.Jlog;
    d.n_tile = 128 >> pl.Jlog;
    d.tiles_n = (int)((N + d.n_tile - 1) / d.n_tile);
    int cap = kLookupWaves * pl.R;                    // row groups a workgroup can hold
    d.tiles_m = (d.RGtotal + cap - 1) / cap;
    d.RGW = (d.RGtotal + d.tiles_m - 1) / d.tiles_m;  // balanced rows per workgroup
    d.stages_total = (d.G + 4 * J - 1) / (4 * J);
    d.stages_per_split = (d.stages_total + pl.S - 1) / pl.S;
    d.total = d.tiles_m * d.tiles_n * pl.S;
    d.per_xcd = (d.total + 7) / 8;
    d.need32 = d.stages_per_split * 4 > kBlockLookups;
    return d;
}

// Cost model in CU clocks, fitted to microbenchmarks of this chip.  Per stage (4 slots) the lookup waves issue, per
// SIMD, 3 waves x 4 lookups x 5 VALU instructions per row group, next to ~230 VALU instructions of the SIMD's build
// wave; the LDS pipe serves the table reads (~4.3 clk per wave read) and ~83 KB of table writes (~1400 clk).
double plan_cost(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    Derived d = derive(pl, M, K, N);
    double rw = (double)((d.RGW + kLookupWaves - 1) / kLookupWaves);   // row groups of the slowest lookup wave
    // Measured (K-scans at 256 workgroups, cycles of the shader clock): a stage of 64 k-groups costs about
    // 2280 + 283 per row-group round: the table writes and the table reads share one LDS pipe and add up.
    // Outside the K loop: first loads and first build, then the reduction and the stores of every round.
    double stage = 2280.0 + 283.0 * rw;
    double wg = d.stages_per_split * stage + 5900.0 + 840.0 * rw + (d.need32 ? 0.05 * d.stages_per_split * stage : 0.0);
    double rounds = (double)((d.total + 255) / 256);
    double t = rounds * wg;
    if (pl.S > 1) t += 5000.0 + 600.0 * pl.S + (double)pl.S * (double)M * (double)N * 8.0 / (256.0 * 16.0);   // second kernel
    // weight bytes pulled from L2 by all token tiles (256 CUs x ~24 B/clk)
    double traffic = (double)d.tiles_n * (double)d.RGtotal * d.KCn * 64.0 / (256.0 * 24.0);
    return t > traffic ? t : traffic;
}

bool plan_valid(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    if (pl.Jlog < 0 || pl.Jlog > 4 || !r_supported(pl.R) || pl.S < 1 || pl.S > 16) return false;
    Derived d = derive(pl, M, K, N);
    if (d.need32 && pl.R > 6) return false;      // register budget of the INT32 variant
    if (pl.S > d.stages_total) return false;
    return true;
}

Plan search_plan(int64_t M, int64_t K, int64_t N) {
    Plan best = {0, 4, 1};
    double best_cost = 1e300;
    const int Ss[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int Jlog = 0; Jlog <= 4; ++Jlog)
        for (int R : kSupportedR)
            for (int S : Ss) {
                Plan pl = {t_forced.Jlog >= 0 ? t_forced.Jlog : Jlog, t_forced.R > 0 ? t_forced.R : R,
                           t_forced.S > 0 ? t_forced.S : S};
                if (!plan_valid(pl, M, K, N)) continue;
                double c = plan_cost(pl, M, K, N);
                if (c < best_cost) { best_cost = c; best = pl; }
            }
    return best;
}

// Fused quantisation needs 8-token tiles (16 sub-tables per row) and the codes of the workgroup's K range in LDS.
bool fused_plan_valid(const Plan& pl, int64_t M, int64_t K, int64_t N) {
    if (pl.Jlog != 4 || !plan_valid(pl, M, K, N)) return false;
    return derive(pl, M, K, N).stages_per_split <= kFusedMaxStages;
}

bool search_fused_plan(int64_t M, int64_t K, int64_t N, Plan* out) {
    if (t_forced.Jlog >= 0 && t_forced.Jlog != 4) return false;
    bool found = false;
    double best_cost = 1e300;
    const int Ss[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int R : kSupportedR)
        for (int S : Ss) {
            Plan pl = {4, t_forced.R > 0 ? t_forced.R : R, t_forced.S > 0 ? t_forced.S : S};
            if (!fused_plan_valid(pl, M, K, N)) continue;
            double c = plan_cost(pl, M, K, N);
            if (c < best_cost) { best_cost = c; *out = pl; found = true; }
        }
    return found;
}

// The search above costs microseconds of host time; a launch-bound caller repeats a handful of shapes, so the
// last few answers are kept per thread (invalidated by vlut_set_plan).
struct PlanCacheEntry {
    int64_t M, K, N;
    Plan plan;
};
thread_local PlanCacheEntry t_cache[8];
thread_local int t_cache_used = 0, t_cache_next = 0;

Plan choose_plan(int64_t M, int64_t K, int64_t N) {
    for (int i = 0; i < t_cache_used; ++i)
        if (t_cache[i].M == M && t_cache[i].K == K && t_cache[i].N == N) return t_cache[i].plan;
    Plan pl = search_plan(M, K, N);
    t_cache[t_cache_next] = {M, K, N, pl};
    t_cache_next = (t_cache_next + 1) % 8;
    if (t_cache_used < 8) ++t_cache_used;
    return pl;
}

struct FusedCacheEntry {
    int64_t M, K, N;
    Plan plan;
    bool found;
};
thread_local FusedCacheEntry t_fcache[8];
thread_local int t_fcache_used = 0, t_fcache_next = 0;

bool choose_fused_plan(int64_t M, int64_t K, int64_t N, Plan* out) {
    for (int i = 0; i < t_fcache_used; ++i)
        if (t_fcache[i].M == M && t_fcache[i].K == K && t_fcache[i].N == N) {
            *out = t_fcache[i].plan;
            return t_fcache[i].found;
        }
    Plan pl = {4, 1, 1};
    const bool found = search_fused_plan(M, K, N, &pl);
    t_fcache[t_fcache_next] = {M, K, N, pl, found};
    t_fcache_next = (t_fcache_next + 1) % 8;
    if (t_fcache_used < 8) ++t_fcache_used;
    *out = pl;
    return found;
}

template <int R, bool NEED32, int MODE>
int launch_lookup_t(const LookupParams& p, int grid, hipStream_t stream) {
    auto kfn = lookup_kernel<R, NEED32, MODE>;
    constexpr int max_lds = MODE == kFusedQuant ? kFusedMaxLds : kLdsBytes;
    const int lds = MODE == kFusedQuant ? kFusedAqBase + p.stages_per_split * kFusedStageBytes : kLdsBytes;
    if (lds > max_lds) return VLUT_ERR_UNSUPPORTED;
    static bool attr_done = false;   // benign race: the call is idempotent
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, max_lds) != hipSuccess)
            return VLUT_ERR_DEVICE;
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(kThreads), lds, stream, p);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

// The streamed kernels exist for every supported R; the variant that reads a materialised table only for a few
// small R (the launcher maps R down).
template <bool NEED32>
int launch_lookup_r(int R, int mode, const LookupParams& p, int grid, hipStream_t stream) {
    if (mode == kFusedQuant) {
        switch (R) {
        case 1: return launch_lookup_t<1, NEED32, kFusedQuant>(p, grid, stream);
        case 2: return launch_lookup_t<2, NEED32, kFusedQuant>(p, grid, stream);
        case 3: return launch_lookup_t<3, NEED32, kFusedQuant>(p, grid, stream);
        case 4: return launch_lookup_t<4, NEED32, kFusedQuant>(p, grid, stream);
        case 5: return launch_lookup_t<5, NEED32, kFusedQuant>(p, grid, stream);
        case 6: return launch_lookup_t<6, NEED32, kFusedQuant>(p, grid, stream);
        default: break;
        }
        if constexpr (!NEED32) {
            switch (R) {
            case 7: return launch_lookup_t<7, false, kFusedQuant>(p, grid, stream);
            case 8: return launch_lookup_t<8, false, kFusedQuant>(p, grid, stream);
            case 9: return launch_lookup_t<9, false, kFusedQuant>(p, grid, stream);
            case 10: return launch_lookup_t<10, false, kFusedQuant>(p, grid, stream);
            case 11: return launch_lookup_t<11, false, kFusedQuant>(p, grid, stream);
            case 12: return launch_lookup_t<12, false, kFusedQuant>(p, grid, stream);
            case 14: return launch_lookup_t<14, false, kFusedQuant>(p, grid, stream);
            default: break;
            }
        }
        return VLUT_ERR_UNSUPPORTED;
    }
    if (mode == kFast) {
        switch (R) {
        case 1: return launch_lookup_t<1, NEED32, kFast>(p, grid, stream);
        case 2: return launch_lookup_t<2, NEED32, kFast>(p, grid, stream);
        case 3: return launch_lookup_t<3, NEED32, kFast>(p, grid, stream);
        case 4: return launch_lookup_t<4, NEED32, kFast>(p, grid, stream);
        case 5: return launch_lookup_t<5, NEED32, kFast>(p, grid, stream);
        case 6: return launch_lookup_t<6, NEED32, kFast>(p, grid, stream);
        default: break;
        }
        if constexpr (!NEED32) {
            switch (R) {
            case 7: return launch_lookup_t<7, false, kFast>(p, grid, stream);
            case 8: return launch_lookup_t<8, false, kFast>(p, grid, stream);
            case 9: return launch_lookup_t<9, false, kFast>(p, grid, stream);
            case 10: return launch_lookup_t<10, false, kFast>(p, grid, stream);
            case 11: return launch_lookup_t<11, false, kFast>(p, grid, stream);
            case 12: return launch_lookup_t<12, false, kFast>(p, grid, stream);
            case 14: return launch_lookup_t<14, false, kFast>(p, grid, stream);
            default: break;
            }
        }
        return VLUT_ERR_UNSUPPORTED;
    }
    switch (R) {
    case 1: return launch_lookup_t<1, NEED32, kFromGlobal>(p, grid, stream);
    case 2: return launch_lookup_t<2, NEED32, kFromGlobal>(p, grid, stream);
    case 4: return launch_lookup_t<4, NEED32, kFromGlobal>(p, grid, stream);
    default: return VLUT_ERR_UNSUPPORTED;
    }
}

int check_mpgemm_args(const uint8_t* packed, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                      int64_t N, float* y, int64_t ldy, int32_t* acc) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !a_q || !a_scale) return VLUT_ERR_NULL;
    if (!y && !acc) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    return VLUT_OK;
}

// ---- N <= 2 kernel: rows per workgroup (16..256) so that the grid is about one workgroup per CU
struct NarrowPlan {
    int parts, rr, rows, grid, chunks;
};

bool narrow_applies(int64_t N, const void* lut) {
    return N <= 2 && lut == nullptr && t_forced.Jlog < 0 && t_forced.R == 0 && t_forced.S == 0;
}

NarrowPlan narrow_plan(int64_t M, int64_t K) {
    const int64_t want = (M + 255) / 256;
    NarrowPlan np;
    if (want <= 16) np = {4, 1, 16, 0, 0};
    else if (want <= 32) np = {2, 1, 32, 0, 0};
    else if (want <= 64) np = {1, 1, 64, 0, 0};
    else if (want <= 128) np = {1, 2, 128, 0, 0};
    else np = {1, 4, 256, 0, 0};
    np.grid = (int)((M + np.rows - 1) / np.rows);
    np.chunks = (int)((K / 4 + kNarrowChunk - 1) / kNarrowChunk);
    return np;
}

template <int NTOK, int PARTS, int RR, bool FUSED>
int launch_narrow_t(const NarrowParams& p, int grid, hipStream_t stream) {
    auto kfn = narrow_kernel<NTOK, PARTS, RR, FUSED>;
    constexpr int max_lds = FUSED ? 160 * 1024 : narrow_tab_bytes(NTOK);
    const int lds = FUSED ? narrow_fused_lds_bytes(NTOK, p.chunks) : narrow_tab_bytes(NTOK);
    if (lds > max_lds) return VLUT_ERR_UNSUPPORTED;
    static bool attr_done = false;   // benign race: the call is idempotent
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, max_lds) != hipSuccess)
            return VLUT_ERR_DEVICE;
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(kThreads), lds, stream, p);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

template <int NTOK, bool FUSED>
int launch_narrow_n(const NarrowPlan& np, const NarrowParams& p, hipStream_t stream) {
    if (np.parts == 4) return launch_narrow_t<NTOK, 4, 1, FUSED>(p, np.grid, stream);
    if (np.parts == 2) return launch_narrow_t<NTOK, 2, 1, FUSED>(p, np.grid, stream);
    if (np.rr == 1) return launch_narrow_t<NTOK, 1, 1, FUSED>(p, np.grid, stream);
    if (np.rr == 2) return launch_narrow_t<NTOK, 1, 2, FUSED>(p, np.grid, stream);
    return launch_narrow_t<NTOK, 1, 4, FUSED>(p, np.grid, stream);
}

template <bool FUSED>
int launch_narrow(const NarrowPlan& np, const NarrowParams& p, hipStream_t stream) {
    return p.N == 1 ? launch_narrow_n<1, FUSED>(np, p, stream) : launch_narrow_n<2, FUSED>(np, p, stream);
}

std::mutex g_pack_mutex;

// ---- vlut_mpgemm_f32: which kernels run and how the caller's workspace is divided
enum { kF32Narrow = 0, kF32Fused = 1, kF32TwoLaunches = 2 };
struct F32Layout {
    int kind;
    Plan plan;                                   // kF32Fused
    size_t off_scale, off_aq, off_ws, total;     // byte offsets into the workspace
};

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

F32Layout f32_layout(int64_t M, int64_t K, int64_t N) {
    F32Layout L;
    std::memset(&L, 0, sizeof(L));
    const size_t scale_bytes = round256((size_t)N * sizeof(float));
    if (narrow_applies(N, nullptr) && narrow_plan(M, K).chunks <= narrow_fused_max_chunks((int)N)) {
        L.kind = kF32Narrow;
        return L;
    }
    // More than two tokens: measured, quantising inside the lookup kernel loses against a kernel of its own ahead of
    // it (every workgroup reads the whole rows of its 8 tokens and 16 row tiles repeat the work: +5.6 us on the
    // lookup kernel at M = 6912, K = 2560, N = 128, against 3.2 us + the gap between two kernels).  The fused form
    // is therefore only taken when a launch plan is forced (an override selects the kernel too).
    const bool forced = t_forced.Jlog >= 0 || t_forced.R > 0 || t_forced.S > 0;
    const bool fused = forced && choose_fused_plan(M, K, N, &L.plan);
    if (fused) {
        L.kind = kF32Fused;
        if (L.plan.S > 1) {                      // the second kernel reads the scales from memory
            L.off_ws = scale_bytes;
            L.total = L.off_ws + (size_t)L.plan.S * (size_t)M * (size_t)N * sizeof(int32_t);
        }
        return L;
    }
    L.kind = kF32TwoLaunches;                    // quantise into the workspace, then the ordinary path
    L.off_aq = scale_bytes;
    L.off_ws = L.off_aq + round256((size_t)((N + 7) / 8) * (size_t)K * 8);
    const bool narrow = narrow_applies(N, nullptr);
    const Plan pl = narrow ? Plan{4, 1, 1} : choose_plan(M, K, N);
    L.total = L.off_ws + (pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0);
    return L;
}

// ---- 1.60-bit (g = 5) host side
struct Plan5 {
    int R, S;
};
thread_local Plan5 t_forced5 = {0, 0};
const int kSupportedR5[] = {1, 2, 4, 6, 9, 12, 14};

bool shape5_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && N >= 1 && K >= 5 && (K % 5) == 0 && M < kMaxDim && K < kMaxDim && N < kMaxDim;
}

struct Derived5 {
    int G, KCn, RGtotal, tiles_n, tiles_m, RGW, dstages_total, dstages_per_split, total, per_xcd;
    bool need32;
};

Derived5 derive5(const Plan5& pl, int64_t M, int64_t K, int64_t N) {
    Derived5 d;
    d.G = (int)(K / 5);
    d.KCn = (d.G + 15) / 16;
    d.RGtotal = (int)((M + 3) / 4);
    d.tiles_n = (int)((N + 7) / 8);
    int cap = kLookupWaves * pl.R;
    d.tiles_m = (d.RGtotal + cap - 1) / cap;
    d.RGW = (d.RGtotal + d.tiles_m - 1) / d.tiles_m;
    d.dstages_total = (d.G + 63) / 64;
    d.dstages_per_split = (d.dstages_total + pl.S - 1) / pl.S;
    d.total = d.tiles_m * d.tiles_n * pl.S;
    d.per_xcd = (d.total + 7) / 8;
    d.need32 = d.dstages_per_split * 4 > kBlockLookups5;
    return d;
}

bool plan5_valid(const Plan5& pl, int64_t M, int64_t K, int64_t N) {
    bool ok = false;
    for (int v : kSupportedR5) ok = ok || v == pl.R;
    if (!ok || pl.S < 1 || pl.S > 16) return false;
    Derived5 d = derive5(pl, M, K, N);
    if (d.need32 && pl.R > 6) return false;
    return pl.S <= d.dstages_total;
}

Plan5 choose_plan5(int64_t M, int64_t K, int64_t N) {
    Plan5 best = {1, 1};
    double best_cost = 1e300;
    const int Ss[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
    for (int R : kSupportedR5)
        for (int S : Ss) {
            Plan5 pl = {t_forced5.R > 0 ? t_forced5.R : R, t_forced5.S > 0 ? t_forced5.S : S};
            if (!plan5_valid(pl, M, K, N)) continue;
            Derived5 d = derive5(pl, M, K, N);
            double rw = (double)((d.RGW + kLookupWaves - 1) / kLookupWaves);
            // a dword stage = four half-stages; each writes a 62 KB slot and reads it rw times per lookup wave
            double wg = d.dstages_per_split * 4.0 * (1900.0 + 75.0 * rw) + 5900.0 + 840.0 * rw;
            double t = (double)((d.total + 255) / 256) * wg;
            if (pl.S > 1) t += 5000.0 + 600.0 * pl.S;
            if (t < best_cost) { best_cost = t; best = pl; }
        }
    return best;
}

template <int R, bool NEED32>
int launch_lookup5_t(const Lookup5Params& p, int grid, hipStream_t stream) {
    auto kfn = lookup5_kernel<R, NEED32>;
    static bool attr_done = false;   // benign race: the call is idempotent
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, kLds5Bytes) != hipSuccess)
            return VLUT_ERR_DEVICE;
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(kThreads), kLds5Bytes, stream, p);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

template <bool NEED32>
int launch_lookup5_r(int R, const Lookup5Params& p, int grid, hipStream_t stream) {
    switch (R) {
    case 1: return launch_lookup5_t<1, NEED32>(p, grid, stream);
    case 2: return launch_lookup5_t<2, NEED32>(p, grid, stream);
    case 4: return launch_lookup5_t<4, NEED32>(p, grid, stream);
    case 6: return launch_lookup5_t<6, NEED32>(p, grid, stream);
    default: break;
    }
    if constexpr (!NEED32) {
        switch (R) {
        case 9: return launch_lookup5_t<9, false>(p, grid, stream);
        case 12: return launch_lookup5_t<12, false>(p, grid, stream);
        case 14: return launch_lookup5_t<14, false>(p, grid, stream);
        default: break;
        }
    }
    return VLUT_ERR_UNSUPPORTED;
}

}  // namespace

extern "C" {

const char* vlut_status_string(int status) {
    switch (status) {
    case VLUT_OK: return "VLUT_OK";
    case VLUT_ERR_NULL: return "VLUT_ERR_NULL: a required pointer is NULL";
    case VLUT_ERR_SHAPE: return "VLUT_ERR_SHAPE: shape or leading dimension out of range";
    case VLUT_ERR_SMALL_BUFFER: return "VLUT_ERR_SMALL_BUFFER: buffer smaller than required";
    case VLUT_ERR_VALUE: return "VLUT_ERR_VALUE: weight outside {-1,0,+1}";
    case VLUT_ERR_DEVICE: return "VLUT_ERR_DEVICE: HIP call or kernel launch failed";
    case VLUT_ERR_UNSUPPORTED: return "VLUT_ERR_UNSUPPORTED: request not supported by this build";
    default: return "VLUT_ERR_UNKNOWN";
    }
}

int vlut_version(void) { return 100; }

size_t vlut_packed_weight_bytes(int64_t M, int64_t K) {
    if (!shape_ok(M, K, 1)) return 0;
    return (size_t)((M + 3) / 4) * (size_t)((K / 4 + 15) / 16) * 64;
}

size_t vlut_packed_offset(int64_t M, int64_t K, int64_t m, int64_t kg) {
    if (!shape_ok(M, K, 1) || m < 0 || m >= M || kg < 0 || kg >= K / 4) return (size_t)-1;
    size_t KCn = (size_t)((K / 4 + 15) / 16);
    return (((size_t)(m / 4) * KCn + (size_t)(kg / 16)) * 64) + (size_t)(m % 4) * 16 + (size_t)(kg % 16);
}

size_t vlut_act_bytes(int64_t K, int64_t N) {
    if (!shape_ok(1, K, N)) return 0;
    return (size_t)((N + 7) / 8) * (size_t)K * 8;
}

size_t vlut_lut_bytes(int64_t K, int64_t N) {
    if (!shape_ok(1, K, N)) return 0;
    return (size_t)(K / 4) * kRows * (size_t)N * sizeof(int16_t);
}

size_t vlut_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    if (narrow_applies(N, nullptr)) return 0;
    Plan pl = choose_plan(M, K, N);
    return pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
}

int vlut_set_plan(int J, int R, int waves, int split_k) {
    int Jlog = -1;
    if (J != 0) {
        for (int e = 0; e <= 4; ++e)
            if ((1 << e) == J) Jlog = e;
        if (Jlog < 0) return VLUT_ERR_UNSUPPORTED;
    }
    if (R != 0 && !r_supported(R)) return VLUT_ERR_UNSUPPORTED;
    if (waves != 0 && waves != kWaves) return VLUT_ERR_UNSUPPORTED;
    if (split_k < 0 || split_k > 16) return VLUT_ERR_UNSUPPORTED;
    t_forced = {Jlog, R, split_k};
    t_cache_used = 0;
    t_cache_next = 0;
    t_fcache_used = 0;
    t_fcache_next = 0;
    return VLUT_OK;
}

int vlut_query_plan(int64_t M, int64_t K, int64_t N, int* out4) {
    if (!out4) return VLUT_ERR_NULL;
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (narrow_applies(N, nullptr)) {          // the N <= 2 kernel: J reported as 0, R = rows per workgroup
        const NarrowPlan np = narrow_plan(M, K);
        out4[0] = 0; out4[1] = np.rows; out4[2] = 1; out4[3] = np.grid;
        return VLUT_OK;
    }
    Plan pl = choose_plan(M, K, N);
    Derived d = derive(pl, M, K, N);
    out4[0] = 1 << pl.Jlog;
    out4[1] = pl.R;
    out4[2] = pl.S;
    out4[3] = d.total;
    return VLUT_OK;
}

int vlut_pack_weights(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                      void* stream) {
    if (!shape_ok(M, K, 1)) return VLUT_ERR_SHAPE;
    if (!w_ternary || !packed) return VLUT_ERR_NULL;
    size_t need = vlut_packed_weight_bytes(M, K);
    if (packed_bytes < need) return VLUT_ERR_SMALL_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_pack_mutex);
    int zero = 0;
    if (hipMemcpyToSymbolAsync(HIP_SYMBOL(g_pack_error), &zero, sizeof(int), 0, hipMemcpyHostToDevice, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    int G = (int)(K / 4), KCn = (G + 15) / 16, RGtotal = (int)((M + 3) / 4);
    size_t blocks = (need + 255) / 256;
    hipLaunchKernelGGL(pack_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, s, w_ternary, (int)M, K, G, KCn, RGtotal,
                       packed);
    if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    int err = 0;
    if (hipMemcpyFromSymbolAsync(&err, HIP_SYMBOL(g_pack_error), sizeof(int), 0, hipMemcpyDeviceToHost, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return VLUT_ERR_DEVICE;
    return err ? VLUT_ERR_VALUE : VLUT_OK;
}

#ifndef VLUT_QUANT_PER_TOKEN
// measured: the per-token kernel is the faster one except for more than ~2M values in short rows, where its
// single-byte stores cost more than the chunk kernel's serial reads
#define VLUT_QUANT_PER_TOKEN(N, K) (!((N) * (K) >= 2000000 && (K) <= 4096))
#endif
int vlut_quantize_act(const float* x, int64_t N, int64_t K, int64_t ldx, int8_t* a_q, float* a_scale,
                      void* stream) {
    if (!shape_ok(1, K, N)) return VLUT_ERR_SHAPE;
    if (ldx < K) return VLUT_ERR_SHAPE;
    if (!x || !a_q || !a_scale) return VLUT_ERR_NULL;
    if (((uintptr_t)a_q) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    const unsigned chunks = (unsigned)((N + 7) / 8);
    const bool vec = (((uintptr_t)x) % 16 == 0) && (ldx % 4 == 0);
    const size_t lds = (size_t)K * 8;
    const int nquad_per_thread = (int)((K / 4 + 127) / 128);
    auto launch = [&](auto kfn) -> int {
        if (lds > 160 * 1024 - 1024) return VLUT_ERR_UNSUPPORTED;   // the chunk's [K][8] block is staged in LDS
        if (lds > 48 * 1024 &&
            hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return VLUT_ERR_DEVICE;
        hipLaunchKernelGGL(kfn, dim3(chunks), dim3(kQuantThreads), lds, s, x, (int)N, (int)K, ldx, a_q, a_scale);
        return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
    };
    // One workgroup per token (every CU reads one row once) unless the byte stores would dominate
    if (VLUT_QUANT_PER_TOKEN(N, K)) {
        const unsigned blocks = ((chunks + 7) / 8) * 64;
        const int per_thread = (int)((K / 4 + kTokThreads - 1) / kTokThreads);
        auto launch_tok = [&](auto kfn) -> int {
            hipLaunchKernelGGL(kfn, dim3(blocks), dim3(kTokThreads), 0, s, x, (int)N, (int)K, ldx, a_q, a_scale, (int)chunks);
            return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
        };
        if (!vec) return launch_tok(quantize_token_kernel<0, false>);
        if (per_thread <= 4) return launch_tok(quantize_token_kernel<4, true>);
        if (per_thread <= 10) return launch_tok(quantize_token_kernel<10, true>);
        if (per_thread <= 16) return launch_tok(quantize_token_kernel<16, true>);
        return launch_tok(quantize_token_kernel<0, true>);
    }
    if (vec) {
        if (nquad_per_thread <= 5) return launch(quantize_kernel<5, true>);
        if (nquad_per_thread <= 8) return launch(quantize_kernel<8, true>);
        if (nquad_per_thread <= 16) return launch(quantize_kernel<16, true>);
        return launch(quantize_kernel<0, true>);
    }
    return launch(quantize_kernel<0, false>);
}

int vlut_build_lut(const int8_t* a_q, int64_t K, int64_t N, int16_t* lut, size_t lut_bytes, void* stream) {
    if (!shape_ok(1, K, N)) return VLUT_ERR_SHAPE;
    if (!a_q || !lut) return VLUT_ERR_NULL;
    if (lut_bytes < vlut_lut_bytes(K, N)) return VLUT_ERR_SMALL_BUFFER;
    size_t total = (size_t)(K / 4) * (size_t)N;
    hipLaunchKernelGGL(build_lut_kernel<false>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       a_q, (int)(K / 4), (int)N, lut);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

int vlut_build_lut_token_outer(const int8_t* a_q, int64_t K, int64_t N, int16_t* lut, size_t lut_bytes, void* stream) {
    if (!shape_ok(1, K, N)) return VLUT_ERR_SHAPE;
    if (!a_q || !lut) return VLUT_ERR_NULL;
    if (lut_bytes < vlut_lut_bytes(K, N)) return VLUT_ERR_SMALL_BUFFER;
    size_t total = (size_t)(K / 4) * (size_t)N;
    hipLaunchKernelGGL(build_lut_kernel<true>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       a_q, (int)(K / 4), (int)N, lut);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

int vlut_mpgemm_token_outer(const uint8_t* packed, float w_scale, const float* a_scale, const int16_t* lut, int64_t M,
                            int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* stream) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !a_scale || !lut) return VLUT_ERR_NULL;
    if (!y && !acc_or_null) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    const int G = (int)(K / 4), KCn = (G + 15) / 16;
    const dim3 grid((unsigned)((M + 63) / 64), (unsigned)((N + 3) / 4));
    if (grid.y > 65535u) return VLUT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(token_outer_lookup_kernel, grid, dim3(256), 0, (hipStream_t)stream, packed, lut, (int)M, (int)N, G,
                       KCn, w_scale, a_scale, y, ldy, acc_or_null);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

static int mpgemm_impl(const uint8_t* packed, float w_scale, const float* w_rows, const int8_t* a_q, const float* a_scale,
                       const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                       int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    if (((uintptr_t)a_q) % 16 != 0) return VLUT_ERR_UNSUPPORTED;      // the [N/8][K][8] blocks are read 16 bytes at a time
    if (narrow_applies(N, lut_or_null)) {      // one or two tokens: the workgroups sweep all of K, no workspace
        const NarrowPlan np = narrow_plan(M, K);
        NarrowParams q;
        std::memset(&q, 0, sizeof(q));
        q.packed = packed; q.a_q = a_q; q.a_scale = a_scale; q.w_rows = w_rows; q.y = y; q.acc = acc_or_null;
        q.w_scale = w_scale; q.M = (int)M; q.K = (int)K; q.N = (int)N; q.G = (int)(K / 4);
        q.KCn = (int)((K / 4 + 15) / 16); q.RGtotal = (int)((M + 3) / 4); q.ldy = (int)ldy; q.chunks = np.chunks;
        return launch_narrow<false>(np, q, (hipStream_t)stream);
    }
    Plan pl = choose_plan(M, K, N);
    const bool al = lut_or_null && (N % 8 == 0) && (((uintptr_t)lut_or_null) % 16 == 0);
    const int mode = lut_or_null ? kFromGlobal : kFast;
    if (mode != kFast) pl.R = pl.R >= 4 ? 4 : (pl.R >= 2 ? 2 : 1);   // the general-purpose kernels are built for these R only
    Derived d = derive(pl, M, K, N);
    size_t ws_need = pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
    if (ws_need > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < ws_need) return VLUT_ERR_SMALL_BUFFER;
    }
    LookupParams p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.lut = lut_or_null;
    p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)workspace; p.w_scale = w_scale; p.w_rows = w_rows;
    p.M = (int)M; p.K = (int)K; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
    p.Jlog = pl.Jlog; p.S = pl.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
    p.stages_total = d.stages_total; p.stages_per_split = d.stages_per_split;
    p.total_tiles = d.total; p.per_xcd = d.per_xcd;
    p.aligned8 = al ? 1 : 0;
    p.Ka = (int)K;
    hipStream_t s = (hipStream_t)stream;
    int grid = d.per_xcd * 8;
    rc = d.need32 ? launch_lookup_r<true>(pl.R, mode, p, grid, s) : launch_lookup_r<false>(pl.R, mode, p, grid, s);
    if (rc != VLUT_OK) return rc;
    if (pl.S > 1) {
        size_t total = (size_t)M * (size_t)N;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const int32_t*)workspace, pl.S, (int)M, (int)N, w_scale, w_rows, a_scale, y, ldy, acc_or_null);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    return VLUT_OK;
}

int vlut_mpgemm(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale,
                const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    return mpgemm_impl(packed, w_scale, nullptr, a_q, a_scale, lut_or_null, M, K, N, y, ldy, acc_or_null, workspace,
                       workspace_bytes, stream);
}

int vlut_mpgemm_rows(const uint8_t* packed, const float* w_scale_rows, const int8_t* a_q, const float* a_scale,
                     const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                     int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    if (!w_scale_rows) return VLUT_ERR_NULL;
    return mpgemm_impl(packed, 1.0f, w_scale_rows, a_q, a_scale, lut_or_null, M, K, N, y, ldy, acc_or_null, workspace,
                       workspace_bytes, stream);
}

size_t vlut_workspace_bytes_f32(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    return f32_layout(M, K, N).total;
}

int vlut_query_plan_f32(int64_t M, int64_t K, int64_t N, int* out5) {
    if (!out5) return VLUT_ERR_NULL;
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    const F32Layout L = f32_layout(M, K, N);
    out5[4] = L.kind == kF32TwoLaunches ? 0 : 1;
    if (L.kind == kF32Fused) {
        const Derived d = derive(L.plan, M, K, N);
        out5[0] = 1 << L.plan.Jlog; out5[1] = L.plan.R; out5[2] = L.plan.S; out5[3] = d.total;
        return VLUT_OK;
    }
    return vlut_query_plan(M, K, N, out5);
}

int vlut_mpgemm_f32(const uint8_t* packed, float w_scale, const float* w_scale_rows_or_null, const float* x, int64_t ldx,
                    int64_t M, int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null,
                    float* a_scale_out_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    if (!shape_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !x) return VLUT_ERR_NULL;
    if (!y && !acc_or_null) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    if (ldx < K) return VLUT_ERR_SHAPE;
    const F32Layout L = f32_layout(M, K, N);
    if (L.total > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < L.total) return VLUT_ERR_SMALL_BUFFER;
        if (((uintptr_t)workspace) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    }
    hipStream_t s = (hipStream_t)stream;
    const int x_vec = ((((uintptr_t)x) % 16 == 0) && (ldx % 4 == 0)) ? 1 : 0;
    const float* w_rows = w_scale_rows_or_null;
    const float w_one = w_rows ? 1.0f : w_scale;
    char* ws = (char*)workspace;

    if (L.kind == kF32Narrow) {
        const NarrowPlan np = narrow_plan(M, K);
        NarrowParams q;
        std::memset(&q, 0, sizeof(q));
        q.packed = packed; q.w_rows = w_rows; q.y = y; q.acc = acc_or_null; q.w_scale = w_one;
        q.M = (int)M; q.K = (int)K; q.N = (int)N; q.G = (int)(K / 4);
        q.KCn = (int)((K / 4 + 15) / 16); q.RGtotal = (int)((M + 3) / 4); q.ldy = (int)ldy; q.chunks = np.chunks;
        q.x = x; q.ldx = ldx; q.x_vec = x_vec; q.a_scale_out = a_scale_out_or_null;
        return launch_narrow<true>(np, q, s);
    }
    if (L.kind == kF32TwoLaunches) {
        float* scales = a_scale_out_or_null ? a_scale_out_or_null : (float*)(ws + L.off_scale);
        int8_t* a_q = (int8_t*)(ws + L.off_aq);
        int rc = vlut_quantize_act(x, N, K, ldx, a_q, scales, stream);
        if (rc != VLUT_OK) return rc;
        return mpgemm_impl(packed, w_one, w_rows, a_q, scales, nullptr, M, K, N, y, ldy, acc_or_null, ws + L.off_ws,
                           L.total - L.off_ws, stream);
    }
    const Plan pl = L.plan;
    const Derived d = derive(pl, M, K, N);
    float* scales = a_scale_out_or_null;
    if (pl.S > 1 && !scales) scales = (float*)(ws + L.off_scale);
    LookupParams p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.x = x; p.ldx = ldx; p.x_vec = x_vec; p.a_scale_out = scales; p.Ka = (int)K;
    p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)(ws + L.off_ws); p.w_scale = w_one; p.w_rows = w_rows;
    p.M = (int)M; p.K = (int)K; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
    p.Jlog = pl.Jlog; p.S = pl.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
    p.stages_total = d.stages_total; p.stages_per_split = d.stages_per_split;
    p.total_tiles = d.total; p.per_xcd = d.per_xcd;
    const int grid = d.per_xcd * 8;
    int rc = d.need32 ? launch_lookup_r<true>(pl.R, kFusedQuant, p, grid, s)
                      : launch_lookup_r<false>(pl.R, kFusedQuant, p, grid, s);
    if (rc != VLUT_OK) return rc;
    if (pl.S > 1) {
        size_t total = (size_t)M * (size_t)N;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const int32_t*)(ws + L.off_ws), pl.S, (int)M, (int)N, w_one, w_rows, (const float*)scales, y,
                           ldy, acc_or_null);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    return VLUT_OK;
}

// ---- 1.60-bit packing (g = 5)
size_t vlut_packed_weight_bytes_g5(int64_t M, int64_t K) {
    if (!shape5_ok(M, K, 1)) return 0;
    return (size_t)((M + 3) / 4) * (size_t)((K / 5 + 15) / 16) * 64;
}

size_t vlut_packed_offset_g5(int64_t M, int64_t K, int64_t m, int64_t kg) {
    if (!shape5_ok(M, K, 1) || m < 0 || m >= M || kg < 0 || kg >= K / 5) return (size_t)-1;
    size_t KCn = (size_t)((K / 5 + 15) / 16);
    return (((size_t)(m / 4) * KCn + (size_t)(kg / 16)) * 64) + (size_t)(m % 4) * 16 + (size_t)(kg % 16);
}

int vlut_pack_weights_g5(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                         void* stream) {
    if (!shape5_ok(M, K, 1)) return VLUT_ERR_SHAPE;
    if (!w_ternary || !packed) return VLUT_ERR_NULL;
    size_t need = vlut_packed_weight_bytes_g5(M, K);
    if (packed_bytes < need) return VLUT_ERR_SMALL_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_pack_mutex);
    int zero = 0;
    if (hipMemcpyToSymbolAsync(HIP_SYMBOL(g_pack_error), &zero, sizeof(int), 0, hipMemcpyHostToDevice, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    int G = (int)(K / 5), KCn = (G + 15) / 16, RGtotal = (int)((M + 3) / 4);
    size_t blocks = (need + 255) / 256;
    hipLaunchKernelGGL(pack_kernel<5>, dim3((unsigned)blocks), dim3(256), 0, s, w_ternary, (int)M, K, G, KCn, RGtotal,
                       packed);
    if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    int err = 0;
    if (hipMemcpyFromSymbolAsync(&err, HIP_SYMBOL(g_pack_error), sizeof(int), 0, hipMemcpyDeviceToHost, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return VLUT_ERR_DEVICE;
    return err ? VLUT_ERR_VALUE : VLUT_OK;
}

size_t vlut_workspace_bytes_g5(int64_t M, int64_t K, int64_t N) {
    if (!shape5_ok(M, K, N)) return 0;
    Plan5 pl = choose_plan5(M, K, N);
    return pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
}

int vlut_set_plan_g5(int R, int split_k) {
    if (R != 0) {
        bool ok = false;
        for (int v : kSupportedR5) ok = ok || v == R;
        if (!ok) return VLUT_ERR_UNSUPPORTED;
    }
    if (split_k < 0 || split_k > 16) return VLUT_ERR_UNSUPPORTED;
    t_forced5 = {R, split_k};
    return VLUT_OK;
}

int vlut_query_plan_g5(int64_t M, int64_t K, int64_t N, int* out3) {
    if (!out3) return VLUT_ERR_NULL;
    if (!shape5_ok(M, K, N)) return VLUT_ERR_SHAPE;
    Plan5 pl = choose_plan5(M, K, N);
    Derived5 d = derive5(pl, M, K, N);
    out3[0] = pl.R; out3[1] = pl.S; out3[2] = d.total;
    return VLUT_OK;
}

int vlut_mpgemm_g5(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                   int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* workspace, size_t workspace_bytes,
                   void* stream) {
    if (!shape5_ok(M, K, N)) return VLUT_ERR_SHAPE;
    if (!packed || !a_q || !a_scale) return VLUT_ERR_NULL;
    if (!y && !acc_or_null) return VLUT_ERR_NULL;
    if (y && (ldy < M || ldy > INT32_MAX)) return VLUT_ERR_SHAPE;
    if (((uintptr_t)a_q) % 8 != 0) return VLUT_ERR_UNSUPPORTED;       // 5 rows x 8 tokens are read 8 bytes at a time
    Plan5 pl = choose_plan5(M, K, N);
    if (!plan5_valid(pl, M, K, N)) return VLUT_ERR_UNSUPPORTED;
    Derived5 d = derive5(pl, M, K, N);
    size_t ws_need = pl.S > 1 ? (size_t)pl.S * (size_t)M * (size_t)N * sizeof(int32_t) : 0;
    if (ws_need > 0) {
        if (!workspace) return VLUT_ERR_NULL;
        if (workspace_bytes < ws_need) return VLUT_ERR_SMALL_BUFFER;
    }
    Lookup5Params p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.y = y; p.acc = acc_or_null; p.ws = (int32_t*)workspace;
    p.w_scale = w_scale;
    p.M = (int)M; p.K = (int)K; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
    p.S = pl.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
    p.dstages_total = d.dstages_total; p.dstages_per_split = d.dstages_per_split;
    p.total_tiles = d.total; p.per_xcd = d.per_xcd;
    p.Ka = (int)K;
    hipStream_t s = (hipStream_t)stream;
    int grid = d.per_xcd * 8;
    int rc = d.need32 ? launch_lookup5_r<true>(pl.R, p, grid, s) : launch_lookup5_r<false>(pl.R, p, grid, s);
    if (rc != VLUT_OK) return rc;
    if (pl.S > 1) {
        size_t total = (size_t)M * (size_t)N;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const int32_t*)workspace, pl.S, (int)M, (int)N, w_scale, (const float*)nullptr, a_scale, y, ldy,
                           acc_or_null);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    return VLUT_OK;
}

// ---- mixed 1.60-bit / 2-bit packing (Sec. 3.3 "Flexible sub-2-bit weight packing")
int64_t vlut_mixed_k5(int64_t K) {
    if (K < 4 || (K % 4) != 0) return -1;
    return (K / 20) * 20;
}

size_t vlut_packed_weight_bytes_mixed(int64_t M, int64_t K) {
    if (!shape_ok(M, K, 1)) return 0;
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    return (K5 > 0 ? vlut_packed_weight_bytes_g5(M, K5) : 0) + (K4 > 0 ? vlut_packed_weight_bytes(M, K4) : 0);
}

int vlut_pack_weights_mixed(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                            void* stream) {
    if (!shape_ok(M, K, 1)) return VLUT_ERR_SHAPE;
    if (!w_ternary || !packed) return VLUT_ERR_NULL;
    if (packed_bytes < vlut_packed_weight_bytes_mixed(M, K)) return VLUT_ERR_SMALL_BUFFER;
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    const size_t bytes5 = K5 > 0 ? vlut_packed_weight_bytes_g5(M, K5) : 0;
    const size_t bytes4 = K4 > 0 ? vlut_packed_weight_bytes(M, K4) : 0;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_pack_mutex);
    int zero = 0;
    if (hipMemcpyToSymbolAsync(HIP_SYMBOL(g_pack_error), &zero, sizeof(int), 0, hipMemcpyHostToDevice, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    const int RGtotal = (int)((M + 3) / 4);
    if (K5 > 0) {
        const int G = (int)(K5 / 5), KCn = (G + 15) / 16;
        hipLaunchKernelGGL(pack_kernel<5>, dim3((unsigned)((bytes5 + 255) / 256)), dim3(256), 0, s, w_ternary, (int)M, K, G,
                           KCn, RGtotal, packed);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    if (K4 > 0) {
        const int G = (int)(K4 / 4), KCn = (G + 15) / 16;
        hipLaunchKernelGGL(pack_kernel<4>, dim3((unsigned)((bytes4 + 255) / 256)), dim3(256), 0, s, w_ternary + K5, (int)M, K,
                           G, KCn, RGtotal, packed + bytes5);
        if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    }
    int err = 0;
    if (hipMemcpyFromSymbolAsync(&err, HIP_SYMBOL(g_pack_error), sizeof(int), 0, hipMemcpyDeviceToHost, s) != hipSuccess)
        return VLUT_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return VLUT_ERR_DEVICE;
    return err ? VLUT_ERR_VALUE : VLUT_OK;
}

// The two parts as launches of the kernels above in partial-sum mode, then one exact INT32 sum + scale step.
// Workspace: [S5 + S4][N][M] INT32.
static bool mixed_plans(int64_t M, int64_t K, int64_t N, Plan5* p5, Plan* p4) {
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    if (K5 > 0) {
        *p5 = choose_plan5(M, K5, N);
        if (!plan5_valid(*p5, M, K5, N)) return false;
    } else {
        *p5 = Plan5{0, 0};
    }
    *p4 = K4 > 0 ? choose_plan(M, K4, N) : Plan{0, 0, 0};
    return true;
}

size_t vlut_workspace_bytes_mixed(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    Plan5 p5;
    Plan p4;
    if (!mixed_plans(M, K, N, &p5, &p4)) return 0;
    return (size_t)(p5.S + p4.S) * (size_t)M * (size_t)N * sizeof(int32_t);
}

int vlut_mpgemm_mixed(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                      int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* workspace, size_t workspace_bytes,
                      void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    if (((uintptr_t)a_q) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    const int64_t K5 = vlut_mixed_k5(K), K4 = K - K5;
    Plan5 pl5;
    Plan pl4;
    if (!mixed_plans(M, K, N, &pl5, &pl4)) return VLUT_ERR_UNSUPPORTED;
    const size_t need = (size_t)(pl5.S + pl4.S) * (size_t)M * (size_t)N * sizeof(int32_t);
    if (!workspace) return VLUT_ERR_NULL;
    if (workspace_bytes < need) return VLUT_ERR_SMALL_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    if (K5 > 0) {
        const Derived5 d = derive5(pl5, M, K5, N);
        Lookup5Params p;
        std::memset(&p, 0, sizeof(p));
        p.packed = packed; p.a_q = a_q; p.a_scale = a_scale; p.ws = (int32_t*)workspace; p.w_scale = w_scale;
        p.M = (int)M; p.K = (int)K5; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
        p.S = pl5.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
        p.dstages_total = d.dstages_total; p.dstages_per_split = d.dstages_per_split;
        p.total_tiles = d.total; p.per_xcd = d.per_xcd;
        p.Ka = (int)K; p.partial = 1;
        const int grid = d.per_xcd * 8;
        rc = d.need32 ? launch_lookup5_r<true>(pl5.R, p, grid, s) : launch_lookup5_r<false>(pl5.R, p, grid, s);
        if (rc != VLUT_OK) return rc;
    }
    if (K4 > 0) {
        const Derived d = derive(pl4, M, K4, N);
        LookupParams p;
        std::memset(&p, 0, sizeof(p));
        p.packed = packed + (K5 > 0 ? vlut_packed_weight_bytes_g5(M, K5) : 0);
        p.a_q = a_q + (size_t)K5 * 8;                      // activation rows K5 .. K-1 of every token chunk
        p.a_scale = a_scale; p.ws = (int32_t*)workspace; p.w_scale = w_scale;
        p.M = (int)M; p.K = (int)K4; p.N = (int)N; p.G = d.G; p.KCn = d.KCn; p.RGtotal = d.RGtotal; p.ldy = (int)ldy;
        p.Jlog = pl4.Jlog; p.S = pl4.S; p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.RGW = d.RGW;
        p.stages_total = d.stages_total; p.stages_per_split = d.stages_per_split;
        p.total_tiles = d.total; p.per_xcd = d.per_xcd;
        p.Ka = (int)K; p.partial = 1; p.slot0 = pl5.S;
        const int grid = d.per_xcd * 8;
        rc = d.need32 ? launch_lookup_r<true>(pl4.R, kFast, p, grid, s) : launch_lookup_r<false>(pl4.R, kFast, p, grid, s);
        if (rc != VLUT_OK) return rc;
    }
    const size_t total = (size_t)M * (size_t)N;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       (const int32_t*)workspace, pl5.S + pl4.S, (int)M, (int)N, w_scale, (const float*)nullptr, a_scale, y,
                       ldy, acc_or_null);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

size_t vlut_mfma_workspace_bytes(int64_t M, int64_t K, int64_t N) {
    if (!shape_ok(M, K, N)) return 0;
    return (size_t)((N + 15) / 16 * 16) * (size_t)((K + 63) / 64 * 64);
}

int vlut_mpgemm_mfma(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale,
                     const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                     int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_mpgemm_args(packed, a_q, a_scale, M, K, N, y, ldy, acc_or_null);
    if (rc != VLUT_OK) return rc;
    if (lut_or_null) return VLUT_ERR_UNSUPPORTED;
    if (!workspace) return VLUT_ERR_NULL;
    if (workspace_bytes < vlut_mfma_workspace_bytes(M, K, N)) return VLUT_ERR_SMALL_BUFFER;
    if (((uintptr_t)workspace) % 16 != 0) return VLUT_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    MfmaParams p;
    std::memset(&p, 0, sizeof(p));
    p.packed = packed; p.aT = (const int8_t*)workspace; p.a_scale = a_scale; p.y = y; p.acc = acc_or_null;
    p.w_scale = w_scale; p.M = (int)M; p.N = (int)N; p.Npad = (int)((N + 15) / 16 * 16); p.Kp = (int)((K + 63) / 64 * 64);
    p.KCn = (int)((K / 4 + 15) / 16); p.RGtotal = (int)((M + 3) / 4); p.ldy = (int)ldy;
    const size_t dwords = (size_t)p.Npad * (p.Kp / 4);
    hipLaunchKernelGGL(act_transpose_kernel, dim3((unsigned)((dwords + 255) / 256)), dim3(256), 0, s, a_q, (int)N, (int)K, p.Npad,
                       p.Kp, (int8_t*)workspace);
    if (hipGetLastError() != hipSuccess) return VLUT_ERR_DEVICE;
    const unsigned gx = (unsigned)((M + 63) / 64);
    // Tokens per workgroup (16, 32 or 64): the widest tile that still gives about four workgroups per CU, since the
    // kernel hides memory latency with resident waves only.
    const unsigned g64 = (unsigned)((p.Npad + 63) / 64), g32 = (unsigned)((p.Npad + 31) / 32), g16 = (unsigned)(p.Npad / 16);
    if (N > 32 && (size_t)gx * g64 >= 1024) hipLaunchKernelGGL(mfma_kernel<4>, dim3(gx, g64), dim3(256), 0, s, p);
    else if (N > 16 && (size_t)gx * g32 >= 1024) hipLaunchKernelGGL(mfma_kernel<2>, dim3(gx, g32), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(mfma_kernel<1>, dim3(gx, g16), dim3(256), 0, s, p);
    return hipGetLastError() == hipSuccess ? VLUT_OK : VLUT_ERR_DEVICE;
}

}  // extern "C"
