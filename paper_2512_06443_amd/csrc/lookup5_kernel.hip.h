// The kernel for the 1.60-bit packing (g = 5, 243-row tables; Sec. 3.3, Sec. 3.4).
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

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

constexpr int kBuildWaves5 = 4;                        // waves 0..3 build, 4..15 look up
constexpr int kLookupWaves5 = kWaves - kBuildWaves5;   // 12
constexpr int kRoundRows5 = kLookupWaves5 * 4;         // 48 output rows per row-group round of the workgroup

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
    int out_vec;   // y (or the partial-sum slots) can be written four rows at a time
};

// Table read of lookup I (= row group I) of the half-stage that uses byte B of the weight dwords (slot B & 1).
template <int R, int B, int I>
__device__ __forceinline__ i32x4 lookup5_read(const unsigned (&w)[R], unsigned lanebase) {
    constexpr unsigned sel = 0x0c0c0000u | ((4u + (unsigned)B) << 8);
    const unsigned addr = __builtin_amdgcn_perm(w[I], lanebase, sel);   // idx*256 + slice*16
    return lds_read128<(B & 1) * (kSlot5Bytes / 16)>(addr);
}

// Adds the 8 entries of one table read to the row group's packed INT16 accumulators (Alg. 1 lines 3-6).
template <int R, int I>
__device__ __forceinline__ void lookup_accumulate(s16x2 (&acc16)[R][4], const i32x4 v) {
    constexpr int r = I % R;
    // instructions with the accumulator tied to one register ("+v"): the unrolled copies of a stage must not keep
    // the accumulators in alternating register sets
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][0]) : "v"(v.x));
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][1]) : "v"(v.y));
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][2]) : "v"(v.z));
    asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(acc16[r][3]) : "v"(v.w));
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
    // table addresses are formed as idx*256 + slice*16 from LDS address 0; the host checks that the kernel has no
    // static LDS before the first launch and refuses to launch otherwise, so this branch is never taken
    if (lds_base_of(smem5) != 0u) return;
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
    const bool builder = wave < kBuildWaves5;
    const int lw = wave - kBuildWaves5;

    typedef __attribute__((address_space(3))) float lds_f32;
    lds_f32* scale_lds = (lds_f32*)(unsigned)kScale5Base;
    float my_scale = 0.0f;
    if (tid < 8 && n0 + tid < p.N) my_scale = p.a_scale[n0 + tid];   // times w_scale at the end: no wait here

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
            const int rgl = r * kLookupWaves5 + lw;
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
    if (tid < 8) scale_lds[tid] = p.w_scale * my_scale;
    constexpr int kParkStride = R * kRoundRows5 + 4;
    const int m0 = rgw0 * 4;
    const int rows_wg = min(p.RGW * 4, p.M - m0);
    if (!builder) {
#pragma unroll
        for (int r = 0; r < R; ++r)
            park[(l >> 1) * kParkStride + r * kRoundRows5 + lw * 4 + grp] = reduce16<NEED32>(acc16[r], acc32[NEED32 ? r : 0], l);
    }
    wg_barrier_lds();
    if (p.out_vec) {
        // four consecutive rows of one token per thread: one 16-byte read of the parked sums, one 16-byte store
        for (int i = tid; i < R * (kRoundRows5 / 4) * 8; i += kThreads) {
            const int col = 4 * (i % (R * (kRoundRows5 / 4)));
            const int nl = i / (R * (kRoundRows5 / 4));
            const int n = n0 + nl;
            if (col < rows_wg && n < p.N) {
                const i32x4 v4 = *(const lds_i32x4*)(park + nl * kParkStride + col);
                const int val[4] = {v4.x, v4.y, v4.z, v4.w};
                const int m = m0 + col;
                const int cnt = min(4, rows_wg - col);
                if (p.S == 1 && !p.partial) {
                    if (p.y) {
                        const float sn = scale_lds[nl];
                        float* dsty = p.y + (size_t)n * p.ldy + m;
                        if (cnt == 4) {
                            *(f32x4*)dsty = f32x4{(float)val[0] * sn, (float)val[1] * sn, (float)val[2] * sn, (float)val[3] * sn};
                        } else {
#pragma unroll
                            for (int e = 0; e < 3; ++e)
                                if (e < cnt) dsty[e] = (float)val[e] * sn;
                        }
                    }
                    if (p.acc) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (e < cnt) p.acc[(size_t)(m + e) * p.N + n] = val[e];
                    }
                } else {
                    int32_t* dstw = p.ws + ((size_t)ks * p.N + n) * p.M + m;
                    if (cnt == 4) {
                        *(i32x4*)dstw = v4;
                    } else {
#pragma unroll
                        for (int e = 0; e < 3; ++e)
                            if (e < cnt) dstw[e] = val[e];
                    }
                }
            }
        }
    } else
    for (int i = tid; i < R * kRoundRows5 * 8; i += kThreads) {
        const int col = i % (R * kRoundRows5);
        const int nl = i / (R * kRoundRows5);
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

}  // namespace
