// The main kernel: streamed LDS table build + lookup-accumulate + scale epilogue for g = 4 (Alg. 1, Sec. 3.4).
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

namespace {

// ---------------------------------------------------------------------------------------------
// The lookup kernel (Alg. 1 main loop + streamed Precompute, Sec. 3.4).
//
// Roles inside the 16-wave workgroup: waves 0..BW-1 (BW = 4, 2 or 1) only BUILD tables, the other LW = 16 - BW only
// LOOK UP.  Fewer build waves mean more output rows per table (workgroup tile = 4*LW*R rows) and less repeated work
// in the build (a build lane then makes the rows of 4/BW leading digit pairs from one unpacking of its activations),
// but a longer build per half-stage, which only large R hides.
// The four LDS slots are used as two halves of two slots each: while the lookup waves read one half, the build
// waves fill the other half with the next two sub-table sets, and one barrier per half-stage hands the halves over.
// Table entries and block accumulators are words of two INT16 values each (word_lo / word_hi), so that one
// three-operand 32-bit add accumulates the entries of two lookups: per lookup one address permute, one 16-byte
// table read and two adds.
// Workgroups are persistent: the launch has at most one per compute unit, and each walks through its share of the
// output tiles (row tile x token tile x K split).  With 8-token tiles the lookup waves finish a tile on their own
// (cross-lane sums, transposition through a private patch of LDS, stores) while the build waves already fetch the
// activations and build the first tables of the next tile.
//   R       row groups (of 4 output rows) per lookup wave; workgroup tile = up to 4*LW*R rows
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

// The two table reads of row group RR in half-stage HALF (slots 2*HALF and 2*HALF + 1): bytes 2*HALF and 2*HALF + 1 of
// the row group's weight dword are the table rows; the lane reads its 16-byte slice (8 entries) of each.
template <int R, int HALF, int RR>
__device__ __forceinline__ void lookup_read_pair(const unsigned (&w)[R], unsigned lanebase, i32x4& a, i32x4& b) {
    constexpr unsigned selA = 0x0c0c0000u | ((4u + (unsigned)(2 * HALF)) << 8);
    constexpr unsigned selB = 0x0c0c0000u | ((4u + (unsigned)(2 * HALF + 1)) << 8);
    const unsigned addrA = __builtin_amdgcn_perm(w[RR], lanebase, selA);   // idx*256 + slice*16
    const unsigned addrB = __builtin_amdgcn_perm(w[RR], lanebase, selB);
    a = lds_read128<(2 * HALF) * (kSlotBytes / 16)>(addrA);
    b = lds_read128<(2 * HALF + 1) * (kSlotBytes / 16)>(addrB);
}

// Adds the entries of two lookups to the row group's accumulators: entries and accumulators are words of two INT16
// values (see word_lo / word_hi), so one three-operand 32-bit add does four INT16 additions (Alg. 1 lines 3-6: one
// shared index, one vector add over the tokens).
template <int R, int RR>
__device__ __forceinline__ void lookup_accumulate_pair(int (&accw)[R][4], const i32x4 a, const i32x4 b) {
    // Written as instructions with the accumulator tied to one register ("+v"): left to the register allocator, the
    // unrolled copies of the stage keep the accumulators in alternating register sets, which doubles their
    // footprint and caps the row groups a wave can hold.
    asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(accw[RR][0]) : "v"(a.x), "v"(b.x));
    asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(accw[RR][1]) : "v"(a.y), "v"(b.y));
    asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(accw[RR][2]) : "v"(a.z), "v"(b.z));
    asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(accw[RR][3]) : "v"(a.w), "v"(b.w));
}

// The 2*R lookups of a half-stage as a rolling pipeline over the row groups: the reads of D row groups are in flight
// while the adds of the oldest one issue.
template <int R, int HALF>
__device__ __forceinline__ void lookup_half(const unsigned (&w)[R], unsigned lanebase, int (&accw)[R][4]) {
    constexpr int D = R > 14 ? 2 : 3;   // row groups (pairs of table reads) in flight; the widest instances have registers for two
    i32x4 bufA[D], bufB[D];
    static_for<0, D>([&](auto ic_) {
        constexpr int i = decltype(ic_)::value;
        if constexpr (i < R) lookup_read_pair<R, HALF, (i < R ? i : 0)>(w, lanebase, bufA[i], bufB[i]);
    });
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, R>([&](auto ic_) {
        constexpr int i = decltype(ic_)::value;
        lookup_accumulate_pair<R, i>(accw, bufA[i % D], bufB[i % D]);
        if constexpr (i + D < R) lookup_read_pair<R, HALF, (i + D < R ? i + D : 0)>(w, lanebase, bufA[i % D], bufB[i % D]);
        __builtin_amdgcn_sched_barrier(0);
    });
}

// The kernel's argument struct, read field by field from the kernel-argument segment (scalar loads).
typedef const __attribute__((address_space(4))) LookupParams* LookupKernelArgs;
__device__ __forceinline__ LookupParams read_lookup_params(LookupKernelArgs a) {
    LookupParams r;
    r.packed = a->packed;
    r.a_q = a->a_q;
    r.a_scale = a->a_scale;
    r.w_rows = a->w_rows;
    r.lut = a->lut;
    r.y = a->y;
    r.acc = a->acc;
    r.ws = a->ws;
    r.w_scale = a->w_scale;
    r.M = a->M;
    r.K = a->K;
    r.N = a->N;
    r.G = a->G;
    r.KCn = a->KCn;
    r.RGtotal = a->RGtotal;
    r.ldy = a->ldy;
    r.Jlog = a->Jlog;
    r.S = a->S;
    r.tiles_m = a->tiles_m;
    r.tiles_n = a->tiles_n;
    r.RGW = a->RGW;
    r.stages_total = a->stages_total;
    r.stages_per_split = a->stages_per_split;
    r.total_tiles = a->total_tiles;
    r.per_xcd = a->per_xcd;
    r.aligned8 = a->aligned8;
    r.Ka = a->Ka;
    r.partial = a->partial;
    r.slot0 = a->slot0;
    r.x = a->x;
    r.a_scale_out = a->a_scale_out;
    r.ldx = a->ldx;
    r.x_vec = a->x_vec;
    r.out_vec = a->out_vec;
    r.magic_S = a->magic_S;
    r.magic_tiles_n = a->magic_tiles_n;
    return r;
}

template <int R, bool NEED32, int MODE, int BW>
__global__ void __launch_bounds__(kThreads) lookup_kernel(const LookupParams launch_params) {
    constexpr int kBuildWaves = BW;
    constexpr int kLookupWaves = kWaves - BW;
    constexpr int kRoundRows = kLookupWaves * 4;     // output rows per row-group round of the workgroup
    constexpr int kUPerLane = 4 / BW;                // leading digit pairs (table rows 9u..9u+8) per build lane
    static_assert(BW == 4 || BW == 2 || BW == 1, "build waves");
    static_assert(MODE != kFromGlobal || BW == 4, "the materialised-table variant keeps four build waves");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // The kernel has no static LDS, so the dynamic segment starts at LDS address 0; table addresses are formed
    // as idx*256 + slice*16 by a byte permute and rely on that.  The host verifies it (static LDS size of the
    // kernel == 0) before the first launch and refuses to launch otherwise, so this branch is never taken.
    if (lds_base_of(smem) != 0u) return;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);   // wave-uniform by construction

    // The launch parameters live in a local copy that is filled from the kernel-argument segment (the struct is the
    // kernel's only argument, at offset 0): once here, in one batch of scalar loads (the argument buffer is cold,
    // and left alone the compiler would fetch its cache lines one after the other, where each is first needed), and
    // again after the K loop of every tile through a pointer the optimiser cannot see through.  So the parameters
    // need no registers during the K loop, and the loads that bring them back are hidden behind the epilogue.
    (void)launch_params;
    const LookupKernelArgs kernel_args = (LookupKernelArgs)__builtin_amdgcn_kernarg_segment_ptr();
    LookupParams p = read_lookup_params(kernel_args);
    asm volatile("" ::"s"(p.per_xcd), "s"(p.total_tiles), "s"(p.S), "s"(p.tiles_n), "s"(p.Jlog), "s"(p.RGW),
                 "s"(p.stages_per_split), "s"(p.stages_total), "s"(p.K), "s"(p.N), "s"(p.G), "s"(p.KCn),
                 "s"(p.RGtotal), "s"(p.M), "s"(p.ldy), "s"(p.w_scale), "s"(p.packed), "s"(p.a_q), "s"(p.a_scale),
                 "s"(p.y), "s"(p.acc), "s"(p.ws), "s"(p.lut), "s"(p.aligned8), "s"(p.w_rows), "s"(p.x),
                 "s"(p.a_scale_out), "s"(p.ldx), "s"(p.x_vec), "s"(p.out_vec), "s"(p.Ka), "s"(p.slot0),
                 "s"(p.magic_S), "s"(p.magic_tiles_n));

    const bool builder = wave < kBuildWaves;          // scalar condition
    const int lw = wave - kBuildWaves;                // index among the lookup waves

    typedef __attribute__((address_space(3))) float lds_f32;
    lds_f32* scale_lds = (lds_f32*)(unsigned)kTableBytes;   // output scale of every token of the tile, behind the tables

    // ---- the tiles of this workgroup.  The grid is one workgroup per compute unit (or fewer); the 8 XCDs take
    //      contiguous ranges of the tile list (workgroups that share a weight tile also share an L2), and inside
    //      a range the workgroups of the XCD take tiles round robin.  The trip count is the same for every wave of the
    //      workgroup, and so is the number of barriers either role passes per tile.
    const int xcd = (int)(blockIdx.x & 7), wg_in_xcd = (int)(blockIdx.x >> 3), wgs_per_xcd = (int)(gridDim.x >> 3);
    const int tiles_here = min(p.per_xcd, p.total_tiles - xcd * p.per_xcd);
    for (int ti = wg_in_xcd; ti < tiles_here; ti += wgs_per_xcd) {
    // The lane's coordinates, from a copy of the thread index the optimiser cannot see through: everything derived
    // from them is then computed per tile, where it is used, instead of once before the tile loop and held in
    // registers (or spilled) across the K loop.
    int tid = (int)threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int Jlog = p.Jlog;
    const int J = 1 << Jlog;
    const int TClog = 4 - Jlog;          // log2(token chunks per sub-table)
    const int n_tile = 128 >> Jlog;
    const int lane = tid & 63;
    const int l = lane & 15;             // 16-byte slice of the table rows this lane reads or writes
    const int grp = lane >> 4;
    const int j = l >> TClog;            // sub-table selector of the slice
    const int t = l & ((1 << TClog) - 1);   // 8-token chunk of the slice
    const unsigned lanebase = (unsigned)l * 16u;
    // With 8-token tiles (16 sub-tables per table row) every lookup wave owns consecutive row groups and writes its
    // own results (no workgroup barrier after the K loop), so the build waves go straight on to the next tile of the
    // workgroup and its first tables are ready when the lookup waves arrive.  Otherwise row groups are dealt round
    // robin and the whole workgroup transposes and writes the tile.
    const bool own_rows = Jlog == 4;
    const int rg_per_wave = (p.RGW + kLookupWaves - 1) / kLookupWaves;
    // Tile index -> (K split, token tile, row tile).  The two divisions are multiplications by floor(2^32 / d)
    // (from the host) with one correction step: the product's high word is the quotient or one less.
    auto divide = [](unsigned x, unsigned d, unsigned magic, unsigned& q, unsigned& r) {
        q = __umulhi(x, magic);
        r = x - q * d;
        if (r >= d) { ++q; r -= d; }
    };
    unsigned L1, uks, umt, unt;
    divide((unsigned)(xcd * p.per_xcd + ti), (unsigned)p.S, p.magic_S, L1, uks);
    divide(L1, (unsigned)p.tiles_n, p.magic_tiles_n, umt, unt);
    const int ks = (int)uks, nt = (int)unt, mt = (int)umt;
    const int n0 = nt * n_tile;
    const int rgw0 = mt * p.RGW;          // first row group of this workgroup
    const int st_begin = ks * p.stages_per_split;
    const int st_end = min(p.stages_total, st_begin + p.stages_per_split);

    // The token scales are loaded at the start of a tile and stored to LDS after the tile's first barrier (by then
    // every wave has finished the stores of the previous tile, which read them); the epilogue reads them many
    // barriers later.  tid < n_tile <= 128 are lanes of build waves.
    float my_scale = 0.0f;
    if (MODE != kFusedQuant && tid < n_tile && n0 + tid < p.N) my_scale = p.a_scale[n0 + tid];
    auto publish_scales = [&]() {
        if (tid < n_tile) scale_lds[tid] = (MODE != kFusedQuant && !p.w_rows) ? p.w_scale * my_scale : my_scale;
    };

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

    int accw[R][4];                       // block sums: two INT16 sums per word (word_lo / word_hi)
    int acc32[NEED32 ? R : 1][8];
    // (the 16-lane reduction of the own-rows epilogue takes biased halves when there are no INT32 partial sums)
    const int acc_zero = (own_rows && !NEED32) ? kBiasedZero : 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) accw[r][q] = acc_zero;
    if (NEED32) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc32[r][e] = 0;
    }

    if (builder) {
        // ================================ build role ================================
        // Task of a lane for one half-stage: slot s2 of the half (0/1), slice l, and kUPerLane leading digit pairs
        // u = u0 .. u0+kUPerLane-1 (table rows 9u .. 9u+8 each); the ninth digit pair (rows 72..80) is shared out one
        // row per u, and the lane with u = 0 also takes row 80.
        constexpr int kGroupsPerSlot = 2 * BW;        // 16-lane groups that share a slot
        const int s2 = (wave * 4 + grp) / kGroupsPerSlot;
        const int u0 = ((wave * 4 + grp) % kGroupsPerSlot) * kUPerLane;
        const int u = u0;                            // (kFromGlobal: one digit pair per lane)
        const int nb = n0 + 8 * t;                   // first token of the slice
        const int chunk_b = nb >> 3;
        unsigned actA[4][2] = {}, actB[4][2] = {};       // (initialised: otherwise they count as carried from tile to tile)
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

        // kFromGlobal only: copies the lane's rows of half-stage hs from the materialised table (bit-packed INT16
        // pairs there, words here)
        auto build_half = [&](int hs) {
            const unsigned slot = (unsigned)(2 * (hs & 1) + s2);
            const unsigned dst = slot * kSlotBytes + (unsigned)l * 16u;
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
                lds_write128<0>(dst + (unsigned)row * kRowBytes,
                                i32x4{packed_to_word(v.x), packed_to_word(v.y), packed_to_word(v.z), packed_to_word(v.w)});
            };
#pragma unroll
            for (int i = 0; i < 9; ++i) copy_row(9 * u + i);
            copy_row(72 + u);
            if (u == 0) copy_row(80);
        };

        const int hs0 = 2 * st_begin, hs1 = 2 * st_end;
        if constexpr (MODE == kFusedQuant) quantise_tile();
        if constexpr (MODE == kFromGlobal) {
            if (hs0 < hs1) build_half(hs0);
            wg_barrier_lds();
            publish_scales();
            for (int hs = hs0; hs < hs1; hs += 2) {
                build_half(hs + 1);                   // lookups read half 0 now: fill half 1
                wg_barrier_lds();
                if (hs + 2 < hs1) build_half(hs + 2);                 // lookups read half 1 now: fill half 0
                wg_barrier_lds();
            }
        } else {
            // The build waves are few and every barrier waits for them: let them issue first.
            __builtin_amdgcn_s_setprio(3);
            // After a barrier a build wave makes the tables of the half the lookup waves have just left: it unpacks
            // its activations (fetched four half-stages earlier) into words once and then, for each of its digit
            // pairs, computes a table row and writes it at once, so that arithmetic and LDS writes interleave and only
            // a few rows are ever live.  Every row is one add or subtract away from an earlier one (topological
            // order, Sec. 4); the arithmetic is plain 32-bit on words of two entries each (|word| < 2^23 for an
            // activation, so the 24-bit multiplies by the digits -1, 0, +1 are exact).
            unsigned act2[4][2] = {}, act3[4][2] = {};
            bool valid2 = false, valid3 = false;
            auto build_rows = [&](int hs, unsigned (&act)[4][2], bool valid) {
                if (!valid) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) { act[c][0] = 0u; act[c][1] = 0u; }
                }
                const unsigned dst = (unsigned)(2 * (hs & 1) + s2) * kSlotBytes + (unsigned)l * 16u;
                int a0[4], a1[4], a2[4], a3[4], top[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    a0[q] = unpack_word(act[0][q >> 1], q & 1);
                    a1[q] = unpack_word(act[1][q >> 1], q & 1);
                    a2[q] = unpack_word(act[2][q >> 1], q & 1);
                    a3[q] = unpack_word(act[3][q >> 1], q & 1);
                    top[q] = a0[q] + a1[q];                             // leading digits (2,2)
                }
                auto put = [&](unsigned addr, auto off_tag, const int (&v)[4]) {
                    lds_write128<decltype(off_tag)::value>(addr, i32x4{v[0], v[1], v[2], v[3]});
                };
                static_for<0, kUPerLane>([&](auto ui_) {
                    constexpr int ui = decltype(ui_)::value;
                    const int uu = u0 + ui;
                    const int m0 = uu / 3 - 1, m1 = uu % 3 - 1;   // leading digits of rows 9uu..9uu+8 = digits (d2,d3) of row 72+uu
                    const unsigned dst9 = dst + (unsigned)(9 * uu) * kRowBytes;
                    int b1[4], lo[4], hi[4], t[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) b1[q] = __mul24(a0[q], m0) + __mul24(a1[q], m1);
                    put(dst9, ic<4 * 16>{}, b1);
#pragma unroll
                    for (int q = 0; q < 4; ++q) lo[q] = b1[q] - a2[q];
                    put(dst9, ic<1 * 16>{}, lo);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = lo[q] - a3[q];
                    put(dst9, ic<0 * 16>{}, t);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = lo[q] + a3[q];
                    put(dst9, ic<2 * 16>{}, t);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = b1[q] - a3[q];
                    put(dst9, ic<3 * 16>{}, t);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = b1[q] + a3[q];
                    put(dst9, ic<5 * 16>{}, t);
#pragma unroll
                    for (int q = 0; q < 4; ++q) hi[q] = b1[q] + a2[q];
                    put(dst9, ic<7 * 16>{}, hi);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = hi[q] - a3[q];
                    put(dst9, ic<6 * 16>{}, t);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = hi[q] + a3[q];
                    put(dst9, ic<8 * 16>{}, t);
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = top[q] + __mul24(a2[q], m0) + __mul24(a3[q], m1);
                    put(dst + (unsigned)(72 + uu) * kRowBytes, ic<0>{}, t);   // row 72 + 3*d2 + d3
                });
                if (u0 == 0) {
                    int t[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) t[q] = top[q] + a2[q] + a3[q];
                    put(dst, ic<80 * 16>{}, t);                          // row 80
                }
            };
            // One half-stage: build the tables of half-stage hs from `act` (if that half-stage exists), refill the
            // activation buffer four half-stages ahead, and meet the lookup waves.
            auto step = [&](int hs, unsigned (&act)[4][2], bool& valid) {
                if (hs < hs1) build_rows(hs, act, valid);
                fetch_act(hs + 4, act, valid);
                wg_barrier_lds();
            };
            if (hs0 < hs1) {
                fetch_act(hs0, actA, validA);
                fetch_act(hs0 + 1, actB, validB);
                fetch_act(hs0 + 2, act2, valid2);
                fetch_act(hs0 + 3, act3, valid3);
            }
            // half 0 of the first stage, handed over as soon as it is written
            step(hs0, actA, validA);
            publish_scales();
            for (int hs = hs0; hs < hs1; hs += 4) {
                step(hs + 1, actB, validB);           // lookups read half 0 (hs): fill half 1
                step(hs + 2, act2, valid2);           // lookups read half 1 (hs+1): fill half 0
                step(hs + 3, act3, valid3);           // (with an odd number of stages the last two steps only meet
                                                      //  the lookup waves at their two matching barriers)
                step(hs + 4, actA, validA);
            }
            __builtin_amdgcn_s_setprio(0);
        }
    } else {
        // ================================ lookup role ================================
        // Row group r of this wave: its packed tiles start at a wave-uniform address (scalar registers); the lane
        // adds its row (grp) and, per stage, the tile and dword it needs.
        // The wave's row groups are first, first + step, ... : consecutive ones when the wave writes its own rows,
        // else dealt round robin over the lookup waves (round r of the epilogue then covers consecutive rows).
        // nvalid of them lie inside the tile and the matrix; the others repeat the last valid one and are never
        // stored.  Few scalar instructions per row group: this runs before the tile's first barrier.
        const unsigned char* wbase[R];
        {
            const int first = own_rows ? lw * rg_per_wave : lw;
            const int lim = min(p.RGW, p.RGtotal - rgw0) - first;           // existing row groups from `first` on
            int nvalid = own_rows ? min(lim, rg_per_wave) : (lim + kLookupWaves - 1) / kLookupWaves;
            nvalid = max(0, min(nvalid, R));
            const unsigned last = (unsigned)max(nvalid - 1, 0);
            const unsigned tile_bytes = (unsigned)p.KCn * 64u;               // packed bytes of a row group
            const unsigned step_bytes = own_rows ? tile_bytes : tile_bytes * (unsigned)kLookupWaves;   // < 2^28
            const unsigned char* base0 = p.packed + (size_t)(rgw0 + (nvalid > 0 ? first : 0)) * tile_bytes;
#pragma unroll
            for (int r = 0; r < R; ++r) wbase[r] = base0 + min((unsigned)r, last) * step_bytes;      // < 2^32
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
            lookup_half<R, 0>(w, lanebase, accw);
            wg_barrier_lds();
            lookup_half<R, 1>(w, lanebase, accw);
            wg_barrier_lds();
            if (NEED32 && (((st - st_begin) & 15) == 15)) {   // 16 stages x 4 lookups = block of 64 (Sec. 3.4)
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc32[r][2 * q] += word_lo(accw[r][q]);
                        acc32[r][2 * q + 1] += word_hi(accw[r][q]);
                        accw[r][q] = 0;
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
    // [token][row] and write consecutive output rows per token.
    {   // the parameters again, for this epilogue and the next tile
        LookupKernelArgs again = kernel_args;
        asm volatile("" : "+s"(again));
        p = read_lookup_params(again);
    }
    const int m0 = rgw0 * 4;
    const int rows_wg = min(p.RGW * 4, p.M - m0);
    // What the stores need:
    float* const out_y = p.y;
    int32_t* const out_acc = p.acc;
    int32_t* const out_ws = p.ws + (size_t)(p.slot0 + ks) * p.N * p.M;
    const float* const w_rows = p.w_rows;
    const int out_ldy = p.ldy, out_N = p.N, out_M = p.M;
    const bool final_out = p.S == 1 && !p.partial, out_vec = p.out_vec != 0;
    // The lane's coordinates again, from a copy of the thread index the optimiser cannot see through: otherwise every
    // address below is computed before the tile loop and held in registers (or spilled) across the K loop.
    int tid_e = tid;
    asm volatile("" : "+v"(tid_e));
    const int lane_e = tid_e & 63, l_e = lane_e & 15, grp_e = lane_e >> 4, t_e = l_e & ((1 << TClog) - 1);
    // Four consecutive rows of one token (INT32 sums `v4`, rows m .. m + cnt - 1, token n with tile-local index nl).
    auto store_quad = [&](const i32x4 v4, int m, int cnt, int n, int nl) {
        const int val[4] = {v4.x, v4.y, v4.z, v4.w};
        if (final_out) {
            if (out_y) {
                const float sn = scale_lds[nl];
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = (float)val[e] * ((w_rows && e < cnt) ? w_rows[m + e] * sn : sn);
                float* dsty = out_y + (size_t)n * out_ldy + m;
                if (cnt == 4) {
                    *(f32x4*)dsty = f32x4{o[0], o[1], o[2], o[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 3; ++e)
                        if (e < cnt) dsty[e] = o[e];
                }
            }
            if (out_acc) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (e < cnt) out_acc[(size_t)(m + e) * out_N + n] = val[e];
            }
        } else {
            int32_t* dstw = out_ws + (size_t)n * out_M + m;
            if (cnt == 4) {
                *(i32x4*)dstw = v4;
            } else {
#pragma unroll
                for (int e = 0; e < 3; ++e)
                    if (e < cnt) dstw[e] = val[e];
            }
        }
    };
    auto store_one = [&](int val, int m, int n, int nl) {
        if (final_out) {
            if (out_y) out_y[(size_t)n * out_ldy + m] = (float)val * (w_rows ? w_rows[m] * scale_lds[nl] : scale_lds[nl]);
            if (out_acc) out_acc[(size_t)m * out_N + n] = val;
        } else {
            out_ws[(size_t)n * out_M + m] = val;
        }
    };
    if (own_rows) {
        // Every lookup wave on its own: its R row groups are 4R consecutive rows; the totals go through a private
        // patch of LDS (in the second half of the table slots: the build waves, already at work on the next tile,
        // write only the first half before the next barrier) and come back as runs of consecutive rows per token.
        // LDS operations of one wave complete in order, so the wave only waits for its own writes.
        if (!builder) {
            // ints per parked token: four times an odd number >= R, so that the 8 tokens x 4 rows a wave writes at
            // once fall into 32 distinct banks (4R + 4 = 64 at R = 15 put all tokens into the same four)
            constexpr int kOwnStride = 4 * (R | 1);
            lds_i32* own = (lds_i32*)(unsigned)(2 * kSlotBytes + lw * (8 * kOwnStride * 4));
#pragma unroll
            for (int r = 0; r < R; ++r)   // both lanes of a pair hold the same total and store it to the same place
                own[(l_e >> 1) * kOwnStride + 4 * r + grp_e] = reduce16w<NEED32>(accw[r], acc32[NEED32 ? r : 0], l_e);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            const int mrow0 = lw * rg_per_wave * 4;                       // first row of this wave inside the tile
            const int rows_w = min(rg_per_wave * 4, rows_wg - mrow0);     // <= 0: nothing to write
            if (out_vec) {
                for (int it = lane_e; it < 8 * R; it += 64) {
                    const int q = it % R, nl = it / R;
                    const int n = n0 + nl;
                    if (4 * q < rows_w && n < out_N)
                        store_quad(*(const lds_i32x4*)(own + nl * kOwnStride + 4 * q), m0 + mrow0 + 4 * q,
                                   min(4, rows_w - 4 * q), n, nl);
                }
            } else {
                for (int it = lane_e; it < 8 * 4 * R; it += 64) {
                    const int col = it % (4 * R), nl = it / (4 * R);
                    const int n = n0 + nl;
                    if (col < rows_w && n < out_N) store_one(own[nl * kOwnStride + col], m0 + mrow0 + col, n, nl);
                }
            }
        }
    } else {
    lds_i32* park = (lds_i32*)0u;
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
            if (r < R) {
                int v[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[2 * q] = word_lo(accw[r][q]) + (NEED32 ? acc32[r][2 * q] : 0);
                    v[2 * q + 1] = word_hi(accw[r][q]) + (NEED32 ? acc32[r][2 * q + 1] : 0);
                }
                // Reduce-scatter over the sub-table selector j (the top Jlog bits of the lane_e's slice index): each
                // step exchanges half of the remaining tokens with the lane_e whose index differs in one bit.
                int tokoff = 0;
                if (Jlog > 0) {
                    const bool hi = (l_e & 8) != 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int send = hi ? v[e] : v[e + 4];
                        const int keep = hi ? v[e + 4] : v[e];
                        v[e] = keep + lane_xor16<8>(send);
                    }
                    tokoff += hi ? 4 : 0;
                }
                if (Jlog > 1) {
                    const bool hi = (l_e & 4) != 0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int send = hi ? v[e] : v[e + 2];
                        const int keep = hi ? v[e + 2] : v[e];
                        v[e] = keep + lane_xor16<4>(send);
                    }
                    tokoff += hi ? 2 : 0;
                }
                if (Jlog > 2) {
                    const bool hi = (l_e & 2) != 0;
                    const int send = hi ? v[0] : v[1];
                    const int keep = hi ? v[1] : v[0];
                    v[0] = keep + lane_xor16<2>(send);
                    tokoff += hi ? 1 : 0;
                }
                const int cnt = 8 >> Jlog;      // Jlog <= 3 here
                const int col = rr * kRoundRows + lw * 4 + grp_e;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e < cnt) park[(8 * t_e + tokoff + e) * kParkStride + col] = v[e];
            }
        }
        }
        wg_barrier_lds();
        if (out_vec) {
            // four consecutive rows of one token per thread: one 16-byte read of the parked sums, one 16-byte store
            for (int i = tid_e; i < RC * (kRoundRows / 4) * n_tile; i += kThreads) {
                const int col = 4 * (i % (RC * (kRoundRows / 4)));
                const int nl = i / (RC * (kRoundRows / 4));
                const int mrow = c0 * kRoundRows + col;     // row inside the workgroup tile
                const int n = n0 + nl;
                if (mrow < rows_wg && mrow < R * kRoundRows && n < out_N)
                    store_quad(*(const lds_i32x4*)(park + nl * kParkStride + col), m0 + mrow, min(4, rows_wg - mrow), n, nl);
            }
        } else
        for (int i = tid_e; i < RC * kRoundRows * n_tile; i += kThreads) {
            const int col = i % (RC * kRoundRows);
            const int nl = i / (RC * kRoundRows);
            const int mrow = c0 * kRoundRows + col;         // row inside the workgroup tile
            const int n = n0 + nl;
            if (mrow < rows_wg && mrow < R * kRoundRows && n < out_N) store_one(park[nl * kParkStride + col], m0 + mrow, n, nl);
        }
        wg_barrier_lds();
    }
    };
    if (n_tile * (R * kRoundRows + 4) * 4 <= kTableBytes) epilogue(std::integral_constant<int, R>{});
    else epilogue(std::integral_constant<int, (R > 1 ? 2 : 1)>{});
    }
    }   // tiles of this workgroup
}

}  // namespace
