// Kernels that prepare operands: offline weight packing (Sec. 3.3), activation quantisation + transposition (Sec. 3.4,
// Sec. 3.3), the table materialised in device memory (Alg. 1 Precompute / Eq. 1).
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

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
    amax = wave_max_f32(amax);
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
// The same quantiser as two kernels, for inputs of a few million values: reading x twice costs less than either the
// single-byte stores of quantize_token_kernel or the few workgroups of quantize_kernel.
//   absmax_token_kernel    one workgroup per token: amax[n] = max_k |x[n][k]|
//   quantize_chunk_kernel  one workgroup per (chunk of 8 tokens, range of K): a thread reads the same four k of the 8
//                          rows, quantises, transposes the bytes in registers and stores the 32 bytes [4 k][8 tokens]
//                          of the token-chunked layout with two 16-byte stores (full lines per wave)
// Same decisions in fp32 as the other two kernels (amax, IEEE divisions, rint, clamp), hence the same bits.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__global__ void __launch_bounds__(kTokThreads) absmax_token_kernel(const float* __restrict__ x, int N, int K, int64_t ldx,
                                                                   float* __restrict__ amax_out) {
    __shared__ float red[kTokThreads / 64];
    const int tid = threadIdx.x;
    const int n = blockIdx.x;
    if (n >= N) return;
    const float* row = x + (size_t)n * ldx;
    const int nquad = K >> 2;
    float amax = 0.0f;
    for (int q0 = 0; q0 < nquad; q0 += kTokThreads * 8) {       // eight loads in flight per thread and pass
        f32x4 xv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int qi = q0 + tid + kTokThreads * i;
            const float* src = row + 4 * (size_t)(qi < nquad ? qi : 0);
            xv[i] = qi < nquad ? (VEC ? *(const f32x4*)src : f32x4{src[0], src[1], src[2], src[3]}) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            amax = fmaxf(fmaxf(amax, fmaxf(fabsf(xv[i].x), fabsf(xv[i].y))), fmaxf(fabsf(xv[i].z), fabsf(xv[i].w)));
    }
    amax = wave_max_f32(amax);
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    if (tid == 0) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < kTokThreads / 64; ++w) v = fmaxf(v, red[w]);
        amax_out[n] = v;
    }
}

// 4 x 4 byte transpose: in[r] holds bytes (r,0..3); out[c] holds bytes (0..3, c).
__device__ __forceinline__ void transpose_bytes4(const unsigned (&in)[4], unsigned (&out)[4]) {
    const unsigned t01l = __builtin_amdgcn_perm(in[1], in[0], 0x05010400u), t01h = __builtin_amdgcn_perm(in[1], in[0], 0x07030602u);
    const unsigned t23l = __builtin_amdgcn_perm(in[3], in[2], 0x05010400u), t23h = __builtin_amdgcn_perm(in[3], in[2], 0x07030602u);
    out[0] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
}

template <bool VEC>
__global__ void __launch_bounds__(kTokThreads) quantize_chunk_kernel(const float* __restrict__ x, int N, int K, int64_t ldx,
                                                                     const float* __restrict__ amax,
                                                                     int8_t* __restrict__ a_q, float* __restrict__ a_scale,
                                                                     int quads_per_block) {
    __shared__ float s_inv[8];
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x;
    if (tid < 8) {
        const int n = chunk * 8 + tid;
        const float v = n < N ? amax[n] : 0.0f;
        s_inv[tid] = (v > 0.0f) ? 127.0f / v : 0.0f;           // IEEE divisions, as in the other quantisers
        if (n < N && blockIdx.y == 0) a_scale[n] = v / 127.0f;
    }
    __syncthreads();
    float inv[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) inv[t] = s_inv[t];
    const int nquad = K >> 2;
    const int q_begin = blockIdx.y * quads_per_block;
    const int q_end = min(nquad, q_begin + quads_per_block);
    int8_t* dst = a_q + (size_t)chunk * K * 8;
    for (int qi = q_begin + tid; qi < q_end; qi += kTokThreads) {
        unsigned c[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int n = chunk * 8 + t;
            const float* src = x + (size_t)(n < N ? n : 0) * ldx + 4 * (size_t)qi;
            const f32x4 v = n < N ? (VEC ? *(const f32x4*)src : f32x4{src[0], src[1], src[2], src[3]}) : f32x4{0.f, 0.f, 0.f, 0.f};
            c[t] = n < N ? quant_codes4(v, inv[t]) : 0u;         // tokens past N: zeros
        }
        unsigned lo[4], hi[4];                                   // lo[k] = tokens 0-3 of k, hi[k] = tokens 4-7
        const unsigned c_lo[4] = {c[0], c[1], c[2], c[3]}, c_hi[4] = {c[4], c[5], c[6], c[7]};
        transpose_bytes4(c_lo, lo);
        transpose_bytes4(c_hi, hi);
        i32x4* o = (i32x4*)(dst + (size_t)qi * 32);
        o[0] = i32x4{(int)lo[0], (int)hi[0], (int)lo[1], (int)hi[1]};
        o[1] = i32x4{(int)lo[2], (int)hi[2], (int)lo[3], (int)hi[3]};
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

}  // namespace
