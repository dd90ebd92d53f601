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
    // Sixteen partial sums are requested at once (a loop that adds them one by one waits for every load in turn,
    // S memory round trips instead of one).
    int v = 0;
    for (int s0 = 0; s0 < S; s0 += 16) {
        int part[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) part[k] = (s0 + k < S) ? ws[((size_t)(s0 + k) * N + n) * M + m] : 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) v += part[k];
    }
    if (y) y[(size_t)n * ldy + m] = (float)v * ((w_rows ? w_rows[m] : w_scale) * a_scale[n]);
    if (acc) acc[(size_t)m * N + n] = v;
}

}  // namespace
