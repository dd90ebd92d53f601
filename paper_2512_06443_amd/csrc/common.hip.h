// Types, constants, launch parameters of the main lookup kernel and the small device helpers (LDS access, DPP
// lane exchanges, the LDS-only barrier) shared by the kernels.
// Part of the single translation unit vlut.hip (included there, in this order).
#pragma once

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
constexpr int kFusedMaxR = 14;   // the quantising variant holds more live state per wave
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
    int out_vec;              // y (or the partial-sum slots) can be written four rows at a time
    unsigned magic_S, magic_tiles_n;   // floor(2^32 / S), floor(2^32 / tiles_n) (0xffffffff for a divisor of 1): set by the launcher
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
// Value of lane l ^ 8 where the result is not the operand of an addition the exchange could be folded into: every
// lane has a source lane, so the value itself serves as the fill value and no register has to be zeroed first.
__device__ __forceinline__ int lane_xor8_plain(int x) { return __builtin_amdgcn_update_dpp(x, x, 0x128, 0xF, 0xF, false); }
// Value of lane l ^ 7 (row_half_mirror reverses each group of 8 lanes): a one-instruction partner whose bit 2 differs.
__device__ __forceinline__ int lane_xor7(int x) { return __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false); }

// Maximum over each row of 16 lanes, in every lane of the row: four exchanges by data parallel primitives (no LDS
// traffic).
__device__ __forceinline__ float row_max_f32(float v) {
    v = fmaxf(v, __builtin_bit_cast(float, lane_xor16<1>(__builtin_bit_cast(int, v))));
    v = fmaxf(v, __builtin_bit_cast(float, lane_xor16<2>(__builtin_bit_cast(int, v))));
    v = fmaxf(v, __builtin_bit_cast(float, lane_xor7(__builtin_bit_cast(int, v))));      // quads are uniform by now
    return fmaxf(v, __builtin_bit_cast(float, lane_xor16<8>(__builtin_bit_cast(int, v))));
}
// Maximum over the 64 lanes of a wave, in every lane: the four row results meet through scalar registers.
__device__ __forceinline__ float wave_max_f32(float v) {
    const int iv = __builtin_bit_cast(int, row_max_f32(v));
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

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

// ---- two INT16 values in one 32-bit word, "carry-compensated": word = 65536 * hi + lo as a plain integer (the
// stored high half is hi - 1 when lo is negative).  Sums of such words, formed with ordinary 32-bit additions (also
// the three-operand ones), are 65536 * sum(hi) + sum(lo) exactly, and both sums are recovered as long as each stays
// inside INT16 -- which is what the block bound of Sec. 3.4 guarantees for up to 64 lookups of |entry| <= 508.
// The main lookup kernel keeps its LDS table entries and its block accumulators in this form: one v_add3_u32 then
// adds the entries of two lookups (four INT16 values) to an accumulator.
__device__ __forceinline__ int word_lo(int w) { return (int)(short)w; }
__device__ __forceinline__ int word_hi(int w) { return (w - (int)(short)w) >> 16; }
// Bytes 2h and 2h+1 of x (two INT8 activations of neighbouring tokens) as one such word.
__device__ __forceinline__ int unpack_word(unsigned x, int h) {
    const int lo = (int)(signed char)(x >> (16 * h));
    const int hi = (int)(signed char)(x >> (16 * h + 8));
    return (int)((unsigned)hi << 16) + lo;
}
// A bit-packed INT16 pair (low half = first value) as such a word.
__device__ __forceinline__ int packed_to_word(int p) { return p + (int)((unsigned)((int)(short)p >> 15) << 16); }

__device__ __forceinline__ s16x2 as_s16x2(int v) { return __builtin_bit_cast(s16x2, v); }
__device__ __forceinline__ int as_int(s16x2 v) { return __builtin_bit_cast(int, v); }

// Two INT8 values (bytes 2h and 2h+1 of x) -> sign-extended packed INT16 pair.
__device__ __forceinline__ s16x2 unpack_pair(unsigned x, int h) {
    unsigned sel = h ? 0x070c060cu : 0x050c040cu;   // {0, byte, 0, byte}: value in the high byte of each half
    s16x2 v = as_s16x2((int)__builtin_amdgcn_perm(x, 0u, sel));
    return v >> (short)8;                            // arithmetic shift per half
}

// Start value of a word accumulator whose halves are kept biased by +32768 each (see reduce16w): with at most 64
// lookups of |entry| <= 508 per block both halves stay inside [256, 65280].
constexpr int kBiasedZero = (int)0x80008000u;

// reduce16 for accumulators in word form: lane l ends with the total of token l >> 1.  Without INT32 partial sums
// (WIDE == false) the words must have started at kBiasedZero.
template <bool WIDE>
__device__ __forceinline__ int reduce16w(const int (&aw)[4], const int (&a32)[8], int l) {
    const bool hi3 = (l & 8) != 0, hi2 = (l & 4) != 0, hi1 = (l & 2) != 0;
    int w[4];
    if constexpr (!WIDE) {
        // Here the accumulators started at kBiasedZero instead of 0: both halves carry +32768, so they are plain
        // unsigned 16-bit fields (no borrow between them) and come apart with a mask and a shift; the 16 biases of a
        // total are taken off at the end.
        const unsigned kA = (unsigned)(hi3 ? aw[2] : aw[0]), kB = (unsigned)(hi3 ? aw[3] : aw[1]);
        const unsigned rA = (unsigned)lane_xor8_plain(hi3 ? aw[0] : aw[2]);
        const unsigned rB = (unsigned)lane_xor8_plain(hi3 ? aw[1] : aw[3]);
        w[0] = (int)((kA & 0xffffu) + (rA & 0xffffu));
        w[1] = (int)((kA >> 16) + (rA >> 16));
        w[2] = (int)((kB & 0xffffu) + (rB & 0xffffu));
        w[3] = (int)((kB >> 16) + (rB >> 16));
    } else {
        int v[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[2 * q] = word_lo(aw[q]) + a32[2 * q];
            v[2 * q + 1] = word_hi(aw[q]) + a32[2 * q + 1];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (hi3 ? v[e + 4] : v[e]) + lane_xor16<8>(hi3 ? v[e] : v[e + 4]);
    }
    const int x0 = (hi2 ? w[2] : w[0]) + lane_xor7(hi2 ? w[0] : w[2]);
    const int x1 = (hi2 ? w[3] : w[1]) + lane_xor7(hi2 ? w[1] : w[3]);
    const int y1 = (hi1 ? x1 : x0) + lane_xor16<2>(hi1 ? x0 : x1);
    return (y1 - (WIDE ? 0 : 16 * 32768)) + lane_xor16<1>(y1);
}

}  // namespace
