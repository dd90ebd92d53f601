// The lookup kernel of the layout ablation (token-outermost table) and the split-K sum + scale step.
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

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

// Sum of the split-K partials (any order is exact: integers) + scale step.  A thread takes VEC (1 or 4) consecutive
// output rows of one token; the scales are requested first and up to sixteen partial sums at once, so that the kernel
// is one memory round trip (a loop that adds the partial sums one by one waits for every load in turn, and scales
// fetched after the sum wait once more).  VEC = 4 needs M % 4 == 0 and 16-byte aligned ws, y rows and w_rows.
template <int VEC>
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const int32_t* __restrict__ ws, int S, int M, int N,
                                                            float w_scale, const float* __restrict__ w_rows,
                                                            const float* __restrict__ a_scale,
                                                            float* __restrict__ y, int64_t ldy,
                                                            int32_t* __restrict__ acc) {
    static_assert(VEC == 1 || VEC == 4, "one row or four rows per thread");
    const int Mv = M / VEC;
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (i >= (size_t)Mv * N) return;
    const int m = (int)(i % Mv) * VEC;
    const int n = (int)(i / Mv);
    const float as = y ? a_scale[n] : 0.0f;
    float wr[VEC];
    if constexpr (VEC == 1) {
        wr[0] = (y && w_rows) ? w_rows[m] : w_scale;
    } else {
        const f32x4 w4 = (y && w_rows) ? *(const f32x4*)(w_rows + m) : f32x4{w_scale, w_scale, w_scale, w_scale};
        wr[0] = w4.x; wr[1] = w4.y; wr[2] = w4.z; wr[3] = w4.w;
    }
    constexpr int NB = VEC == 1 ? 16 : 8;                   // partial sums in flight
    int v[VEC] = {};
    for (int s0 = 0; s0 < S; s0 += NB) {
        int part[NB][VEC];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int32_t* src = ws + ((size_t)min(s0 + k, S - 1) * N + n) * M + m;   // clamped; masked below
            if constexpr (VEC == 1) {
                part[k][0] = *src;
            } else {
                const i32x4 q = *(const i32x4*)src;
                part[k][0] = q.x; part[k][1] = q.y; part[k][2] = q.z; part[k][3] = q.w;
            }
        }
#pragma unroll
        for (int k = 0; k < NB; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] += (s0 + k < S) ? part[k][e] : 0;
    }
    if (y) {
        float* dst = y + (size_t)n * ldy + m;
        if constexpr (VEC == 1) {
            dst[0] = (float)v[0] * (wr[0] * as);
        } else {
            *(f32x4*)dst = f32x4{(float)v[0] * (wr[0] * as), (float)v[1] * (wr[1] * as), (float)v[2] * (wr[2] * as),
                                 (float)v[3] * (wr[3] * as)};
        }
    }
    if (acc) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[(size_t)(m + e) * N + n] = v[e];
    }
}

}  // namespace
