// The comparison path on the INT8 matrix cores (the multiply-add way of Sec. 2.2.1).
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------------
// Comparison path (not the method): the multiply-add way of Sec. 2.2.1 on the INT8 matrix cores, written as a
// tiled GEMM.  A workgroup (4 waves) owns 128 output rows x BN tokens.  Per K step of 64 values it
//   - unpacks its 128 x 16 packed bytes to 128 x 64 INT8 weights ONCE, through an 81-entry table in LDS, into an LDS
//     tile (a thread unpacks 8 bytes of one row),
//   - stages the BN x 64 INT8 activations from the token-chunked layout into an LDS tile with k contiguous per token
//     (a thread transposes the bytes of 4 k x 8 tokens with byte permutes),
// and every wave multiplies its 32 rows with all BN tokens: 2 x BN/16 v_mfma_i32_16x16x64_i8 per step, operands read
// from the tiles 16 bytes per lane.  Tile rows are pitched 80 bytes, so that the 16 lanes of an operand read hit
// distinct banks.  The LDS tiles are double buffered and the global loads run three steps ahead in registers; one
// LDS-only barrier per step.  K can be split over workgroups (partial sums to the workspace, summed by
// splitk_reduce_kernel) so that small token counts still fill the device.
// ---------------------------------------------------------------------------------------------
constexpr int kMfRows = 128;      // output rows per workgroup
constexpr int kMfPitch = 80;      // bytes per tile row: 64 values + 16 bytes of padding

struct MfmaParams {
    const uint8_t* packed;
    const int8_t* a_q;
    const float* a_scale;
    float* y;
    int32_t* acc;
    int32_t* ws;
    float w_scale;
    int M, K, N, KCn, RGtotal, ldy, chunks;
    int S, steps_per_split, tiles_m, tiles_n;
    int out_vec;              // y (or the partial-sum slots) can be written four rows at a time
};

template <int BN>
__global__ void __launch_bounds__(256) mfma_kernel(const MfmaParams p) {
    static_assert(BN == 16 || BN == 32 || BN == 64 || BN == 128, "tokens per workgroup");
    constexpr int NT = BN / 16;                       // token tiles of 16 per wave
    __shared__ unsigned dec[kRows];                   // index -> four INT8 weights (first weight in the low byte)
    __shared__ __attribute__((aligned(16))) unsigned char wt[2][kMfRows * kMfPitch];
    __shared__ __attribute__((aligned(16))) unsigned char at[2][BN * kMfPitch];
    const int tid = threadIdx.x;
    if (tid < kRows) {
        const int d0 = tid / 27, d1 = (tid / 9) % 3, d2 = (tid / 3) % 3, d3 = tid % 3;
        dec[tid] = ((unsigned)(d0 - 1) & 0xffu) | (((unsigned)(d1 - 1) & 0xffu) << 8) | (((unsigned)(d2 - 1) & 0xffu) << 16) |
                   (((unsigned)(d3 - 1) & 0xffu) << 24);
    }
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i = lane & 15;                   // row of the A tile / token of the B tile / column of the C tile
    const int kblk = lane >> 4;                // which 16 of the 64 k of a step this lane holds (same for A and B)

    int L = blockIdx.x;
    const int ks = L % p.S;
    L /= p.S;
    const int nt = L % p.tiles_n;
    const int mt = L / p.tiles_n;
    const int m0 = mt * kMfRows, n0 = nt * BN;
    const int step0 = ks * p.steps_per_split;
    const int step1 = min(p.KCn, step0 + p.steps_per_split);

    // ---- staging roles
    // weights: thread = (row of the tile, half of its 16 packed bytes)
    const int w_row = tid >> 1, w_half = tid & 1;
    const int w_rg = min((m0 + w_row) >> 2, p.RGtotal - 1);      // rows past the padded matrix read data that is never stored
    const unsigned char* w_src = p.packed + ((size_t)w_rg * p.KCn) * 64 + ((m0 + w_row) & 3) * 16 + w_half * 8;
    // activations: thread = (token chunk of the tile, quad of k): 4 k x 8 tokens = 32 contiguous bytes
    const int a_c = tid >> 4, a_q4 = tid & 15;
    const bool a_thread = a_c < BN / 8;
    const int a_chunk = (n0 >> 3) + a_c;
    const bool a_chunk_ok = a_thread && a_chunk < p.chunks;
    const int8_t* a_src = p.a_q + ((size_t)(a_chunk_ok ? a_chunk : 0) * p.K) * 8;

    // Global loads run three K steps ahead of their use, in three register sets that rotate (the loop is unrolled by
    // three so that every set has a fixed name).
    struct Staged { i32x2 w; i32x4 a[2]; };
    auto load_global = [&](int step, Staged& r) {
        const int st = min(step, p.KCn - 1);                     // steps past the end are loaded (clamped) and never used
        r.w = *(const i32x2*)(w_src + (size_t)st * 64);
        const int k = st * 64 + 4 * a_q4;
        const bool ok = a_chunk_ok && k < p.K;                   // K % 4 == 0: a quad is inside K or past it
        const i32x4* src = (const i32x4*)(a_src + (size_t)(ok ? k : 0) * 8);
        r.a[0] = ok ? src[0] : i32x4{0, 0, 0, 0};
        r.a[1] = ok ? src[1] : i32x4{0, 0, 0, 0};
    };
    auto stage = [&](int buf, const Staged& r) {
        const unsigned w0 = (unsigned)r.w.x, w1 = (unsigned)r.w.y;
        const i32x4 lo = {(int)dec[w0 & 0xffu], (int)dec[(w0 >> 8) & 0xffu], (int)dec[(w0 >> 16) & 0xffu], (int)dec[w0 >> 24]};
        const i32x4 hi = {(int)dec[w1 & 0xffu], (int)dec[(w1 >> 8) & 0xffu], (int)dec[(w1 >> 16) & 0xffu], (int)dec[w1 >> 24]};
        i32x4* wdst = (i32x4*)(wt[buf] + w_row * kMfPitch + w_half * 32);
        wdst[0] = lo;
        wdst[1] = hi;
        if (a_thread) {
            // in: [k][tokens 0-3], [k][4-7], [k+1][0-3], [k+1][4-7] | [k+2].., [k+3]..; out: per token the bytes of k..k+3
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const unsigned d0 = (unsigned)(h ? r.a[0].y : r.a[0].x), d1 = (unsigned)(h ? r.a[0].w : r.a[0].z);
                const unsigned d2 = (unsigned)(h ? r.a[1].y : r.a[1].x), d3 = (unsigned)(h ? r.a[1].w : r.a[1].z);
                const unsigned t01l = __builtin_amdgcn_perm(d1, d0, 0x05010400u), t01h = __builtin_amdgcn_perm(d1, d0, 0x07030602u);
                const unsigned t23l = __builtin_amdgcn_perm(d3, d2, 0x05010400u), t23h = __builtin_amdgcn_perm(d3, d2, 0x07030602u);
                unsigned* adst = (unsigned*)(at[buf] + (8 * a_c + 4 * h) * kMfPitch + 4 * a_q4);
                adst[0 * (kMfPitch / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
                adst[1 * (kMfPitch / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
                adst[2 * (kMfPitch / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
                adst[3 * (kMfPitch / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
            }
        }
    };

    i32x4 acc[2][NT];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[rt][t] = i32x4{0, 0, 0, 0};

    Staged s0, s1, s2;
    load_global(step0, s0);
    load_global(step0 + 1, s1);
    load_global(step0 + 2, s2);
    __syncthreads();                               // the decode table is complete
    stage(0, s0);
    load_global(step0 + 3, s0);
    wg_barrier_lds();
    int buf = 0;
    // one K step: multiply the tile in `buf`, stage the next step's operands (loaded two steps ago) into the other
    // buffer, refill their registers three steps ahead
    auto iterate = [&](int step, Staged& next) {
        const unsigned char* wbase = wt[buf] + (wave * 32 + i) * kMfPitch + kblk * 16;
        const unsigned char* abase = at[buf] + i * kMfPitch + kblk * 16;
        const i32x4 a0 = *(const i32x4*)wbase, a1 = *(const i32x4*)(wbase + 16 * kMfPitch);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const i32x4 b = *(const i32x4*)(abase + t * 16 * kMfPitch);
            acc[0][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b, acc[0][t], 0, 0, 0);
            acc[1][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b, acc[1][t], 0, 0, 0);
        }
        if (step + 1 < step1) {
            stage(buf ^ 1, next);
            load_global(step + 4, next);
        }
        wg_barrier_lds();                          // orders the LDS tiles only: the loads just issued stay in flight
        buf ^= 1;
    };
    for (int step = step0; step < step1; step += 3) {
        iterate(step, s1);
        if (step + 1 < step1) iterate(step + 1, s2);
        if (step + 2 < step1) iterate(step + 2, s0);
    }

    // C tile: lane (column = token i, row block kblk) holds rows 4*kblk .. 4*kblk+3 of each 16 x 16 product
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = n0 + 16 * t + i;
        if (n >= p.N) continue;
        const float sc = (p.S == 1 && p.y) ? p.w_scale * p.a_scale[n] : 0.0f;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int m = m0 + wave * 32 + rt * 16 + 4 * kblk;
            if (m >= p.M) continue;
            const i32x4 v = acc[rt][t];
            const int val[4] = {v.x, v.y, v.z, v.w};
            const int cnt = min(4, p.M - m);
            if (p.S == 1) {
                if (p.y) {
                    float* dst = p.y + (size_t)n * p.ldy + m;
                    if (cnt == 4 && p.out_vec) {
                        *(f32x4*)dst = f32x4{(float)val[0] * sc, (float)val[1] * sc, (float)val[2] * sc, (float)val[3] * sc};
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (r < cnt) dst[r] = (float)val[r] * sc;
                    }
                }
                if (p.acc) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (r < cnt) p.acc[(size_t)(m + r) * p.N + n] = val[r];
                }
            } else {
                int32_t* dst = p.ws + ((size_t)ks * p.N + n) * p.M + m;
                if (cnt == 4 && p.out_vec) {
                    *(i32x4*)dst = v;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (r < cnt) dst[r] = val[r];
                }
            }
        }
    }
}

}  // namespace
