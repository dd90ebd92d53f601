// The comparison path on the INT8 matrix cores (the multiply-add way of Sec. 2.2.1).
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

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

}  // namespace
