// The kernel for a few tokens (decoding), two tokens per workgroup.
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------------
// One or two parallel tokens per workgroup (decoding).  The tables of a 256-group chunk of K then take 83 KB (two tokens: an
// entry is one dword = two INT16 sums) or 45 KB (one token: an entry is one INT16), and a workgroup can sweep all of K
// by itself: no split-K partial sums, no second kernel.  Two tokens: the waves build a chunk, barrier, all 16 look it
// up, barrier.  One token: the tables fit twice, so the build waves fill chunk c + 1 and then join the others in
// looking chunk c up, one barrier per chunk.
//   Tables: NTOK = 2: sub-table kg of the chunk = 81 dwords at kg*324 + idx*4; a build lane (kg, leading digit d0)
//           makes 27 entries and stores them as single dwords; consecutive lanes are 27 dwords apart: odd, so every
//           store of a wave is free of bank conflicts.  NTOK = 1: sub-table = 81 INT16 + 7 pads = 44 dwords at
//           kg*176 + idx*2; a build lane owns a whole sub-table and stores it 16 bytes at a time; consecutive lanes
//           are 11 such units apart (odd): the 16 lanes of a store pass cover the 64 banks once.
//   Lookups: wave w reads the packed tile w of the chunk (16 groups); a lane owns an output row and 16/PARTS of the
//           tile's groups (PARTS lanes per row), RR rows one after the other.  Address = lane constant + idx * entry
//           size, the group's offset is an immediate: 2.5 VALU instructions per lookup.  With PARTS = 1 all lanes of a
//           read look into the same sub-table, whose dwords lie in distinct banks (equal bank = equal address =
//           broadcast).  Two tokens: INT16 sums inside a chunk (at most 16 lookups), INT32 across chunks; one token:
//           INT32 throughout.  The 16*PARTS partial sums per row are added through LDS at the end.
//   Tiles past the end of K are neither built nor looked up.
//   More than two tokens: the grid holds one copy of the row tiles per token pair (workgroup = row tile + gx8 * pair,
//   gx8 = the row tiles rounded up to a multiple of 8, so that the workgroups that stream the same weights sit on the
//   same XCD and share its L2); every pair is an independent two-token problem.
// ---------------------------------------------------------------------------------------------
constexpr int kNarrowChunk = 256;                        // k-groups per chunk = 16 packed tiles, one per wave
constexpr int narrow_sub_bytes(int ntok) { return ntok == 2 ? 324 : 176; }
constexpr int narrow_buffers(int ntok) { return ntok == 2 ? 1 : 2; }
constexpr int narrow_tab_bytes(int ntok) { return narrow_buffers(ntok) * kNarrowChunk * narrow_sub_bytes(ntok); }   // 82944 / 90112

struct NarrowParams {
    const uint8_t* packed;
    const int8_t* a_q;
    const float* a_scale;
    const float* w_rows;
    float* y;
    int32_t* acc;
    float w_scale;
    int M, K, N, G, KCn, RGtotal, ldy, chunks;
    int gridx, gx8;           // row tiles, and the stride between the token pairs' copies of them in blockIdx.x
    // fused quantisation (FUSED): fp32 activations [N][ldx] instead of a_q / a_scale
    const float* x;
    float* a_scale_out;       // optional: the token scales, written by workgroup 0
    int64_t ldx;
    int x_vec;
};
// FUSED keeps, behind the tables, two dwords per k-group (the four codes of token 0 and of token 1) and the 16 x 2
// partial absmax values.
constexpr int narrow_fused_lds_bytes(int ntok, int chunks) { return narrow_tab_bytes(ntok) + chunks * kNarrowChunk * 8 + 128; }
constexpr int narrow_fused_max_chunks(int ntok) {        // 39 (K <= 39936) for two tokens, 35 (K <= 35840) for one
    return (160 * 1024 - narrow_tab_bytes(ntok) - 128) / (kNarrowChunk * 8);
}

template <int NTOK, int PARTS, int RR, bool FUSED>
__global__ void __launch_bounds__(kThreads) narrow_kernel(const NarrowParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_n[];
    // table addresses below are absolute LDS addresses; the host checks that the kernel has no static LDS before
    // the first launch and refuses to launch otherwise, so this branch is never taken
    if (lds_base_of(smem_n) != 0u) return;
    static_assert(PARTS == 1 || PARTS == 2, "a row's 16 groups of a tile belong to one lane or to two");
    constexpr int SUB = narrow_sub_bytes(NTOK);           // bytes per sub-table
    constexpr int BUFS = narrow_buffers(NTOK);            // table buffers: one token's tables fit twice
    constexpr int BUF = kNarrowChunk * SUB;               // bytes of one buffer
    constexpr int TAB = narrow_tab_bytes(NTOK);
    constexpr int RPW = 64 / PARTS;                       // rows of one pass of a wave
    constexpr int ROWS = RPW * RR;                        // rows of the workgroup
    constexpr int NBYTES = 16 / PARTS;                    // groups (= bytes of the packed tile row) per lane
    typedef __attribute__((address_space(3))) short lds_i16;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pair = (int)blockIdx.x / p.gx8, bx = (int)blockIdx.x - pair * p.gx8;
    if (bx >= p.gridx) return;                            // padding of the row tiles to a multiple of 8 (uniform)
    const int t0 = 2 * pair;                              // first token of this workgroup
    const int Nl = min(2, p.N - t0);                      // its tokens: 1 or 2
    const int m0 = bx * ROWS;

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

    // activations of the workgroup's two tokens for the four rows of a k-group: two bytes of a_q[t0/8][4kg + j][*]
    // The activations of a k-group are fetched raw and taken apart when its tables are built (no wait at the fetch):
    // FUSED: the two dwords of codes the prologue left in LDS; else the 32 bytes a_q[t0/8][4kg .. 4kg+3][0..7] as two
    // 16-byte loads, consecutive lanes consecutive addresses (2-byte loads of the one token pair, 32 bytes apart,
    // cost the load unit of the CU more than the build itself).
    constexpr int AW = FUSED ? 2 : 8;
    auto fetch_act = [&](int c, unsigned (&raw)[AW]) {
        const int kg = min(c * kNarrowChunk + kg_b, p.G - 1);          // clamped; validity applied at use
        if constexpr (FUSED) {
            const i32x2 d = *(const __attribute__((address_space(3))) i32x2*)(unsigned)(TAB + kg * 8);
            raw[0] = (unsigned)d.x;
            raw[1] = (unsigned)d.y;
        } else {
            const int8_t* src = p.a_q + (size_t)(t0 >> 3) * p.K * 8 + (size_t)(4 * kg) * 8;
            const i32x4 v0 = *(const i32x4*)src, v1 = *(const i32x4*)(src + 16);
            raw[0] = (unsigned)v0.x; raw[1] = (unsigned)v0.y; raw[2] = (unsigned)v0.z; raw[3] = (unsigned)v0.w;
            raw[4] = (unsigned)v1.x; raw[5] = (unsigned)v1.y; raw[6] = (unsigned)v1.z; raw[7] = (unsigned)v1.w;
        }
    };
    // a[j] = {code of the first token, code of the second token} of row j of the k-group, in the low 16 bits
    auto decode_act = [&](const unsigned (&raw)[AW], unsigned (&a)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (FUSED) {
                a[j] = __builtin_amdgcn_perm(raw[1], raw[0], 0x0c0c0000u | ((4u + j) << 8) | (unsigned)j);
            } else {                                                   // bytes t0 % 8 and t0 % 8 + 1 of the row's eight
                const unsigned long long row8 = ((unsigned long long)raw[2 * j + 1] << 32) | raw[2 * j];
                a[j] = (unsigned)(row8 >> (8 * (t0 & 7))) & 0xffffu;
            }
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
            } else {
                const i32x2 v = *(const i32x2*)src;
                w[rr] = wvec{(unsigned)v.x, (unsigned)v.y, 0u, 0u};
            }
        }
    };

    // The loop streams the packed weights from HBM: they are fetched WD chunks ahead (a ring of WD + 1 register sets),
    // the activations two or three.  One chunk ahead measured best for every tile shape (2 to 4 chunks ahead cost
    // 3-8 %: a row has only a few chunks, and more loads in flight at the start delay the first ones).
    // Loads complete in the order of their issue, and the first table build needs the activations only: they (or the
    // fp32 rows they are made from, and the scales of the epilogue) are requested ahead of the weights, so that
    // quantisation and the first build run while the weights are still on their way from HBM.
    constexpr int WD = 1;
    unsigned act_cur[AW] = {}, act_nxt[AW] = {}, act_nx2[AW] = {};
    wvec w_ring[WD + 1][RR];                               // w_ring[0] = the chunk being looked up
    wvec (&w_cur)[RR] = w_ring[0];
    const int nquad = p.G;
    auto load4 = [&](int n, int qi) -> f32x4 {
        const float* src = p.x + (size_t)(t0 + n) * p.ldx + 4 * (size_t)qi;
        if (p.x_vec) return *(const f32x4*)src;
        return f32x4{src[0], src[1], src[2], src[3]};
    };
    constexpr int NVC = 4;                                             // float4 per thread and token kept (K <= 16384)
    f32x4 xv[NTOK][NVC];
    if constexpr (FUSED) {
#pragma unroll
        for (int n = 0; n < NTOK; ++n)
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = tid + kThreads * i;
                xv[n][i] = (n < Nl && qi < nquad) ? load4(n, qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
    } else if (builds) {
        fetch_act(0, act_cur);
        fetch_act(1, act_nxt);
        if constexpr (BUFS == 2) fetch_act(2, act_nx2);
    }
    // the epilogue's scales: thread tid < 2 * ROWS finishes output (row tid / 2, token tid % 2)
    const int out_m = m0 + (tid >> 1), out_n = tid & 1;
    const bool out_ok = tid < ROWS * 2 && out_m < p.M && out_n < Nl;
    float out_w = p.w_scale, out_a = 1.0f;                 // multiplied at the very end: no wait for them here
    if (out_ok) {
        if (p.w_rows) out_w = p.w_rows[out_m];
        if constexpr (!FUSED) out_a = p.a_scale[t0 + out_n];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 0; d < WD; ++d) fetch_w(d, w_ring[d]);
    __builtin_amdgcn_sched_barrier(0);
    float vmax[2] = {0.0f, 0.0f};                                      // absmax of the tokens (FUSED)
    if constexpr (FUSED) {
        // Quantise the one or two rows of x over all of K: thread tid takes the float4 (= k-group) tid + 1024 i.
        typedef __attribute__((address_space(3))) float lds_f32;
        typedef __attribute__((address_space(3))) i32x2 lds_i32x2;
        lds_f32* red = (lds_f32*)(unsigned)(TAB + p.chunks * kNarrowChunk * 8);   // [wave][token]
        lds_i32x2* aq = (lds_i32x2*)(unsigned)TAB;
        auto absmax4 = [](float m, const f32x4 v) {
            return fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
        };
        auto codes4 = [](const f32x4 v, float inv) { return (int)quant_codes4(v, inv); };
        // All 16 waves run this prologue at once, four to a SIMD: its length is its instruction count, so whatever a
        // whole wave has no data for (float4 slots past the end of the row, the second token of a one-token pair)
        // is skipped by wave-uniform branches.
        bool slot_live[NVC];
#pragma unroll
        for (int i = 0; i < NVC; ++i) slot_live[i] = kThreads * i + wave * 64 < nquad;
        float amax[NTOK];
#pragma unroll
        for (int n = 0; n < NTOK; ++n) {
            amax[n] = 0.0f;
            if (n >= Nl) continue;
#pragma unroll
            for (int i = 0; i < NVC; ++i)
                if (slot_live[i]) amax[n] = absmax4(amax[n], xv[n][i]);
            if (n < Nl)
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
            amax[n] = wave_max_f32(amax[n]);
        }
        if (lane == 0) {
#pragma unroll
            for (int n = 0; n < NTOK; ++n) red[wave * 2 + n] = amax[n];
        }
        wg_barrier_lds();
        float inv[NTOK];
#pragma unroll
        for (int n = 0; n < NTOK; ++n) {
            const float v = row_max_f32(red[(lane & 15) * 2 + n]);     // the 16 waves' results, one per lane of a row
            inv[n] = (v > 0.0f) ? 127.0f / v : 0.0f;                   // IEEE division, as in quantize_kernel
            vmax[n] = v;                                               // the scale v / 127 is divided out where it is used
        }
        if (bx == 0 && tid < Nl && p.a_scale_out) p.a_scale_out[t0 + tid] = (tid == 0 ? vmax[0] : vmax[1]) / 127.0f;
#pragma unroll
        for (int i = 0; i < NVC; ++i) {
            if (!slot_live[i]) continue;
            const int qi = tid + kThreads * i;
            i32x2 cd = i32x2{codes4(xv[0][i], inv[0]), 0};
            if constexpr (NTOK == 2) {
                if (Nl == 2) cd.y = codes4(xv[NTOK - 1][i], inv[NTOK - 1]);
            }
            if (qi < nquad) aq[qi] = cd;
            if constexpr (NTOK == 1) {
                if (i == 0) act_cur[0] = (unsigned)cd.x;               // k-group tid: what this lane builds of chunk 0
            }
        }
        for (int q0 = kThreads * NVC; q0 < nquad; q0 += kThreads * NVC) {
            f32x4 tv[NTOK][NVC];
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = q0 + tid + kThreads * i;
#pragma unroll
                for (int n = 0; n < NTOK; ++n)
                    tv[n][i] = (n < Nl && qi < nquad) ? load4(n, qi) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < NVC; ++i) {
                const int qi = q0 + tid + kThreads * i;
                if (qi < nquad)
                    aq[qi] = i32x2{codes4(tv[0][i], inv[0]), NTOK == 2 ? codes4(tv[NTOK - 1][i], inv[NTOK - 1]) : 0};
            }
        }
        // Two tokens: the build lanes read other lanes' codes next.  One token: a build lane starts with the codes
        // it has just made itself, and the barrier after the first build publishes the rest.
        if constexpr (NTOK == 2) wg_barrier_lds();
    }
    // ---------------- build the tables of chunk cb (topological order of Sec. 4: one add per entry); only the groups
    //                  of real tiles: the padding groups of the last tile get all-zero tables
    auto do_build = [&](int cb, const unsigned (&raw)[AW]) {
        const int kgg = cb * kNarrowChunk + kg_b;
        if (kgg >= p.KCn * 16) return;
        const bool valid = kgg < p.G;
        unsigned act[4];
        decode_act(raw, act);
        const unsigned buf = (unsigned)((cb & (BUFS - 1)) * BUF);
        if constexpr (NTOK == 2) {
            s16x2 a[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned v = valid ? act[j] : 0u;
                a[j] = s16x2{(short)(signed char)(v & 0xffu), (short)(signed char)((v >> 8) & 0xffu)};
            }
            const short s0 = (short)(d0 - 1);
            const s16x2 base = a[0] * s16x2{s0, s0};
            lds_i32* dst = (lds_i32*)(buf + (unsigned)(kg_b * SUB + d0 * 108));
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
            // One token: entry idx = 27 d0 + 9 d1 + 3 d2 + d3 is A[idx / 9] + B[idx % 9] with A = (d0-1) x0 + (d1-1) x1
            // and B = (d2-1) x2 + (d3-1) x3.  Entries are made two at a time (packed INT16, idx even | idx + 1): a
            // pair inside a block of nine is A (both halves) + {B[r], B[r+1]}, a pair across two blocks is
            // {A[q], A[q+1]} + {B[8], B[0]}: one packed add per pair, stored four entries at a time.
            int x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] = valid ? (int)(signed char)(act[j] & 0xffu) : 0;
            int A[9], Bv[9];
            A[4] = 0; A[1] = -x[0]; A[7] = x[0]; A[3] = -x[1]; A[5] = x[1];
            A[0] = A[1] - x[1]; A[2] = A[1] + x[1]; A[6] = x[0] - x[1]; A[8] = x[0] + x[1];
            Bv[4] = 0; Bv[1] = -x[2]; Bv[7] = x[2]; Bv[3] = -x[3]; Bv[5] = x[3];
            Bv[0] = Bv[1] - x[3]; Bv[2] = Bv[1] + x[3]; Bv[6] = x[2] - x[3]; Bv[8] = x[2] + x[3];
            auto pk = [](int lo, int hi) {
                return as_s16x2((int)__builtin_amdgcn_perm((unsigned)hi, (unsigned)lo, 0x05040100u));
            };
            s16x2 Bp[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) Bp[r] = pk(Bv[r], Bv[r + 1]);
            const s16x2 Bx = pk(Bv[8], Bv[0]);
            s16x2 P[44];
            static_for<0, 41>([&](auto ci) {
                constexpr int i = decltype(ci)::value, q = (2 * i) / 9, r = (2 * i) % 9;
                if constexpr (r < 8) P[i] = pk(A[q], A[q]) + Bp[r];
                else P[i] = pk(A[q], A[q < 8 ? q + 1 : q]) + Bx;       // i = 40: entry 80 and a pad
            });
            P[41] = P[42] = P[43] = s16x2{0, 0};
            lds_i32x4* dst = (lds_i32x4*)(buf + (unsigned)(kg_b * SUB));   // lanes 44 dwords apart: conflict-free
            static_for<0, 11>([&](auto cj) {
                constexpr int j = decltype(cj)::value;
                dst[j] = i32x4{as_int(P[4 * j]), as_int(P[4 * j + 1]), as_int(P[4 * j + 2]), as_int(P[4 * j + 3])};
            });
        }
    };
    // ---------------- look chunk c up (the weights in w_cur)
    // Addresses of two lookups from one dword of four indices: the two bytes are widened to 16-bit fields by one
    // byte permute, and a multiply-add with a 16-bit operand select turns each field into field * entry size + lane
    // base: 2.5 instead of 3 VALU instructions per lookup (with the add of the value read).
    auto two_addresses = [&](unsigned w4, auto b_tag, unsigned tab, unsigned& addr0, unsigned& addr1) {
        constexpr int b0 = decltype(b_tag)::value;                     // even: bytes b0 % 4 and b0 % 4 + 1 of w4
        constexpr unsigned sel = 0x0c000c00u | ((unsigned)((b0 + 1) & 3) << 16) | (unsigned)(b0 & 3);
        const unsigned two = __builtin_amdgcn_perm(0u, w4, sel);
        if constexpr (NTOK == 2) {
            asm("v_mad_u32_u16 %0, %1, 4, %2" : "=v"(addr0) : "v"(two), "v"(tab));
            asm("v_mad_u32_u16 %0, %1, 4, %2 op_sel:[1,0,0,0]" : "=v"(addr1) : "v"(two), "v"(tab));
        } else {
            asm("v_mad_u32_u16 %0, %1, 2, %2" : "=v"(addr0) : "v"(two), "v"(tab));
            asm("v_mad_u32_u16 %0, %1, 2, %2 op_sel:[1,0,0,0]" : "=v"(addr1) : "v"(two), "v"(tab));
        }
    };
    auto do_lookup = [&](int c) {
        if (c * 16 + wave >= p.KCn) return;                            // wave-uniform
        const unsigned tab = lane_tab + (unsigned)((c & (BUFS - 1)) * BUF);
#pragma unroll
        for (int rr = 0; rr < RR; ++rr) {
            if constexpr (NTOK == 2) {
                s16x2 acc16 = {0, 0};
                static_for<0, NBYTES / 2>([&](auto pc) {
                    constexpr int b = 2 * decltype(pc)::value;
                    unsigned addr0, addr1;
                    two_addresses(w_cur[rr][b >> 2], ic<b>{}, tab, addr0, addr1);
                    acc16 += as_s16x2(((const lds_i32*)addr0)[b * (SUB / 4)]);
                    acc16 += as_s16x2(((const lds_i32*)addr1)[(b + 1) * (SUB / 4)]);
                });
                acc32[rr][0] += (int)acc16.x;
                acc32[rr][1] += (int)acc16.y;
            } else {
                static_for<0, NBYTES / 2>([&](auto pc) {
                    constexpr int b = 2 * decltype(pc)::value;
                    unsigned addr0, addr1;
                    two_addresses(w_cur[rr][b >> 2], ic<b>{}, tab, addr0, addr1);
                    acc32[rr][0] += (int)((const lds_i16*)addr0)[b * (SUB / 2)];
                    acc32[rr][0] += (int)((const lds_i16*)addr1)[(b + 1) * (SUB / 2)];
                });
            }
        }
    };
    auto rotate = [&]() {
#pragma unroll
        for (int j = 0; j < AW; ++j) { act_cur[j] = act_nxt[j]; act_nxt[j] = act_nx2[j]; }
    };
    auto rotate_w = [&]() {
#pragma unroll
        for (int d = 0; d < WD; ++d)
#pragma unroll
            for (int rr = 0; rr < RR; ++rr) w_ring[d][rr] = w_ring[d + 1][rr];
    };

    // Activations: from global memory they are requested two or three chunks ahead (act_cur always belongs to the
    // next chunk to build); FUSED reads the codes in LDS right before the build.  The build waves issue at raised
    // priority: the others wait for their tables.
    if constexpr (BUFS == 2) {
        // One token: two table buffers, so the build waves fill chunk c + 1 while every wave (they too, afterwards)
        // looks chunk c up: one barrier per chunk.
        if (builds) {
            __builtin_amdgcn_s_setprio(3);
            do_build(0, act_cur);
            __builtin_amdgcn_s_setprio(0);
            if constexpr (!FUSED) rotate();
        }
        wg_barrier_lds();
        for (int c = 0; c < p.chunks; ++c) {
            fetch_w(c + WD, w_ring[WD]);
            if (builds) {
                __builtin_amdgcn_s_setprio(3);
                if constexpr (FUSED) {
                    if (c + 1 < p.chunks) {
                        fetch_act(c + 1, act_cur);
                        do_build(c + 1, act_cur);
                    }
                } else {
                    fetch_act(c + 3, act_nx2);
                    if (c + 1 < p.chunks) do_build(c + 1, act_cur);
                    rotate();
                }
                __builtin_amdgcn_s_setprio(0);
            }
            do_lookup(c);
            wg_barrier_lds();                  // chunk c + 1 is built, and nobody reads chunk c any more
            rotate_w();
        }
    } else {
        for (int c = 0; c < p.chunks; ++c) {
            fetch_w(c + WD, w_ring[WD]);
            if (builds) {
                if constexpr (FUSED) fetch_act(c, act_cur);
                else fetch_act(c + 2, act_nx2);
                do_build(c, act_cur);
            }
            wg_barrier_lds();
            do_lookup(c);
            wg_barrier_lds();
            if constexpr (!FUSED) rotate();
            rotate_w();
        }
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
    if (out_ok) {                                         // all partial sums requested before the first add
        int part_v[16 * PARTS];
#pragma unroll
        for (int pi = 0; pi < 16 * PARTS; ++pi) part_v[pi] = red[pi * ROWS * 2 + tid];
        int v = 0;
#pragma unroll
        for (int pi = 0; pi < 16 * PARTS; ++pi) v += part_v[pi];
        if constexpr (FUSED) out_a = (out_n ? vmax[1] : vmax[0]) / 127.0f;
        if (p.y) p.y[(size_t)(t0 + out_n) * p.ldy + out_m] = (float)v * (out_w * out_a);
        if (p.acc) p.acc[(size_t)out_m * p.N + t0 + out_n] = v;
    }
}

}  // namespace
