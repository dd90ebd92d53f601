/*
 * CPU oracle for the ternary x INT8 mixed-precision GEMM of the Vec-LUT paper.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call into this
 * file; it exists so that tests, the smoke check and the bench's host-baseline
 * leg have an independent definition of every result.  It shares no code,
 * header, table or constant with the HIP library.
 *
 * The method is lossless (Sec. 3.4 "INT16-INT32 hierarchical accumulation":
 * no clipping, no scaling, no numerical error), so the result of the lookup
 * path has a plain definition, O = W x A (Table 2), and the oracle is that
 * definition written out as a triple loop.  The table T is a public
 * intermediate of the library, so it has a definition here too: Eq. 1, every
 * row the dot product of its decoded pattern with the group's activations.
 *
 * Every function here is pinned by tests/test_oracle_pins.py against facts the
 * paper prints or the mathematics fixes; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_VALUE 1
#define ORACLE_OVERFLOW 2

/* Number of table rows for a group of g ternary weights: 3^g (Sec. 2.1.3, 81 for g = 4). */
static int pow3(int e) {
    int p = 1;
    for (int i = 0; i < e; ++i) p *= 3;
    return p;
}

/*
 * Sign that table row i applies to the j-th activation row of a group
 * (Alg. 1, function GetSign: a base-3 digit of i, minus one).
 *
 * Which digit belongs to which row: the printed pseudo-code counts digits from
 * the least significant one, but the worked example in Sec. 3.2
 * (i = 23 = 0*27 + 2*9 + 1*3 + 2 -> (0,2,1,2) -> (-1,+1,0,+1) -> row value
 * -A[0] + A[1] + A[3]) gives row 0 the MOST significant digit.  The example
 * prints concrete values, so it decides: row j (0-based) uses digit g-1-j.
 */
int oracle_get_sign(int i, int j, int g) {
    int trit = (i / pow3(g - 1 - j)) % 3;
    return trit - 1;
}

/*
 * Offline packing (Sec. 3.3 "Tile-contiguous packed weight layout", Fig. 5
 * caption: the table row index equals the decimal value of the packed byte).
 * idx[m][kg] = sum_j (W[m][g*kg+j] + 1) * 3^(g-1-j); plain row-major [M][K/g].
 */
int oracle_pack_indices(const int8_t *W, int64_t M, int64_t K, int g, uint8_t *idx) {
    int64_t G = K / g;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t kg = 0; kg < G; ++kg) {
            int v = 0;
            for (int j = 0; j < g; ++j) {
                int w = W[m * K + kg * g + j];
                if (w < -1 || w > 1) return ORACLE_BAD_VALUE;
                v = v * 3 + (w + 1);
            }
            idx[m * G + kg] = (uint8_t)v;
        }
    return ORACLE_OK;
}

/* Independent decoder of the same index (peels digits from the least significant end). */
int oracle_unpack_indices(const uint8_t *idx, int64_t M, int64_t K, int g, int8_t *W) {
    int64_t G = K / g;
    int rows = pow3(g);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t kg = 0; kg < G; ++kg) {
            int v = idx[m * G + kg];
            if (v >= rows) return ORACLE_BAD_VALUE;
            for (int j = g - 1; j >= 0; --j) {
                W[m * K + kg * g + j] = (int8_t)(v % 3 - 1);
                v /= 3;
            }
        }
    return ORACLE_OK;
}

/*
 * Per-token symmetric INT8 quantisation (Sec. 3.4: activations are quantised
 * per token, symmetrically, to INT8; the block-size bound there divides by
 * max(INT8) = 127, so -128 is never a code).  The paper gives no formula; the
 * reading, in fp32 because this floating-point step decides integers:
 *   amax = max_k |x[n][k]|, s_n = amax / 127, inv = 127 / amax (0 if amax == 0),
 *   q = clamp(round-half-even(x * inv), -127, 127).
 * Input x is feature-contiguous [N][ldx]; output q is token-contiguous [K][N]
 * (Sec. 3.3 "Token-contiguous LUT layout" applies to A as well).
 */
void oracle_quantize(const float *x, int64_t N, int64_t K, int64_t ldx, int8_t *q, float *s) {
    for (int64_t n = 0; n < N; ++n) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(x[n * ldx + k]);
            if (a > amax) amax = a;
        }
        float scale = amax / 127.0f; /* built with -ffp-contract=off, no fast-math */
        float inv = (amax > 0.0f) ? 127.0f / amax : 0.0f;
        s[n] = scale;
        for (int64_t k = 0; k < K; ++k) {
            float prod = x[n * ldx + k] * inv; /* one rounded fp32 multiply */
            float r = nearbyintf(prod);                 /* default mode: ties to even */
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            q[k * N + n] = (int8_t)r;
        }
    }
}

/*
 * The definition of the result (Table 2, O = W x A; Sec. 3.4: INT32 outputs):
 *   acc[m][n] = sum_k W[m][k] * q[k][n].
 * Loop order m, k, n.  Exactness is checked in 64 bits: any |acc| that does
 * not fit INT32 is reported instead of wrapped.
 */
int oracle_gemm_acc(const int8_t *W, const int8_t *q, int64_t M, int64_t K, int64_t N, int32_t *acc) {
    int status = ORACLE_OK;
#pragma omp parallel for schedule(static) reduction(max : status)
    for (int64_t m = 0; m < M; ++m) {
        int64_t *row = (int64_t *)calloc((size_t)N, sizeof(int64_t));
        for (int64_t k = 0; k < K; ++k) {
            int w = W[m * K + k];
            if (w < -1 || w > 1) status = ORACLE_BAD_VALUE;
            for (int64_t n = 0; n < N; ++n) row[n] += (int64_t)w * (int64_t)q[k * N + n];
        }
        for (int64_t n = 0; n < N; ++n) {
            if (row[n] > INT32_MAX || row[n] < INT32_MIN) status = ORACLE_OVERFLOW;
            acc[m * N + n] = (int32_t)row[n];
        }
        free(row);
    }
    return status;
}

/*
 * Scale step (Table 1 has a "Scale" column; the paper never writes it out).
 * Dequantised value of the integer sum: y[n][m] = acc[m][n] * w_scale * s[n],
 * evaluated in fp64, written feature-contiguous [N][ldy] (Sec. 3.3 "Fused
 * activation and output transformation": the framework side is feature-first).
 */
void oracle_epilogue(const int32_t *acc, int64_t M, int64_t N, float w_scale, const float *s,
                     double *y, int64_t ldy) {
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m)
            y[n * ldy + m] = (double)acc[m * N + n] * ((double)w_scale * (double)s[n]);
}

/*
 * Vector table T of shape [K/g][3^g][N], N contiguous (Sec. 3.3), INT16 entries
 * (Sec. 3.4 step i), written as what Eq. 1 defines: row i of sub-table kg is the
 * plain dot product of the ternary pattern that index i encodes (decoded with
 * oracle_unpack_indices, the same decoder the packing round trip uses) with the
 * g activation rows of the group,
 *   T[kg][i][n] = sum_{j<g} pattern_i[j] * q[g*kg + j][n].
 */
void oracle_build_lut(const int8_t *q, int64_t K, int64_t N, int g, int16_t *T) {
    int rows = pow3(g);
    int64_t G = K / g;
    for (int64_t kg = 0; kg < G; ++kg)
        for (int i = 0; i < rows; ++i) {
            uint8_t code = (uint8_t)i;
            int8_t pattern[8];
            oracle_unpack_indices(&code, 1, g, g, pattern);
            for (int64_t n = 0; n < N; ++n) {
                int dot = 0;
                for (int j = 0; j < g; ++j) dot += pattern[j] * q[(size_t)(kg * g + j) * N + n];
                T[((size_t)kg * rows + i) * N + n] = (int16_t)dot;
            }
        }
}

/*
 * Eq. 2 written out per output element: O[m][n] = sum_kg T[kg][idx[m][kg]][n].
 * Kept only so that tests can check "lookups into the oracle's table give the
 * plain product of Table 2"; it is not the timed baseline.
 */
void oracle_lookup_accumulate(const uint8_t *idx, const int16_t *T, int64_t M, int64_t K, int64_t N,
                              int g, int32_t *acc) {
    int rows = pow3(g);
    int64_t G = K / g;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t sum = 0;
            for (int64_t kg = 0; kg < G; ++kg) sum += T[((size_t)kg * rows + idx[m * G + kg]) * N + n];
            acc[m * N + n] = (int32_t)sum;
        }
}

/* Threads the parallel loop above will use (reported next to the host-baseline timing). */
int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
