/* CPU oracle for the GEMM -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * The plain definition, nothing else:
 *     C[i][j] = sum_{k=0}^{K-1} a[i][k] * b[k][j]
 * with the already-quantised inputs decoded exactly to double and accumulated in double in
 * natural k order (the dense GEMM workloads of the paper's Sec. 4.1), and, when scales are
 * given, the block-scaled form
 *     C[i][j] = sum_{kb} sA[i/bs][kb] * sB[j/bs][kb] * ( sum_{k in block kb} a[i][k] * b[k][j] )
 * (the block-wise scaled FP8 GEMM of Sec. 4.1; scales here are fp32 as this build's workload fixes;
 * A's scales may also be one per row and k block).
 *
 * Only the loop over output elements is spread over threads; every output is an independent
 * serial sum.  The number formats are decoded from their definitions:
 *   bf16  = upper 16 bits of IEEE binary32;
 *   e4m3  = OCP FP8 E4M3 (bias 7, subnormals, no infinities, S.1111.111 = NaN, max 448);
 *   f16   = IEEE binary16 (the fused MoE layer of Sec. 4.1 is an FP16 layer).
 * This file shares nothing with the GPU library.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 1, ORACLE_FP8_E4M3 = 2, ORACLE_F16 = 4 };

static double dec_bf16(uint16_t h) {
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits; exponent 0 = subnormals, 31 = inf / NaN */
static double dec_f16(uint16_t h) {
    int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m / 1024.0, -14);
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return s ? -v : v;
}

static double dec_e4m3(uint8_t c) {
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* e4m3 has 256 codes: the value of each, by dec_e4m3, looked up instead of decoded again for every product */
static double load(const void* p, int64_t idx, int dtype, const double* e4m3_values) {
    if (dtype == ORACLE_BF16) return dec_bf16(((const uint16_t*)p)[idx]);
    if (dtype == ORACLE_F16) return dec_f16(((const uint16_t*)p)[idx]);
    return e4m3_values[((const uint8_t*)p)[idx]];
}

int axe_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* A: logical (M,K), element (i,k) at A[i*a_sm + k*a_sk]; B: logical (K,N), element (k,j) at
 * B[k*b_sk + j*b_sn] (strides in elements).  sA: row-major (ceil(M/bs_am), ceil(K/bs)) floats or
 * NULL (bs_am = rows of A that share a scale: bs for square blocks, 1 for one scale per row and
 * k block, the usual choice for activations); sB: row-major (ceil(N/bs), ceil(K/bs)) floats or NULL
 * (both or neither).
 * out: row-major (nrows, ncols) doubles holding C[rows[r]][cols[c]]. */
int axe_oracle_gemm(int dtype, int64_t M, int64_t N, int64_t K,
                    const void* A, int64_t a_sm, int64_t a_sk,
                    const void* B, int64_t b_sk, int64_t b_sn,
                    const float* sA, const float* sB, int64_t bs, int64_t bs_am,
                    const int64_t* rows, int64_t nrows, const int64_t* cols, int64_t ncols,
                    double* out) {
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP8_E4M3 && dtype != ORACLE_F16) return -1;
    if ((sA == 0) != (sB == 0)) return -2;
    if (sA && (bs <= 0 || bs_am <= 0)) return -3;
    (void)M; (void)N;
    int64_t nkb = sA ? (K + bs - 1) / bs : 0;
    double v8[256];
    for (int c = 0; c < 256; ++c) v8[c] = dec_e4m3((uint8_t)c);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        for (int64_t c = 0; c < ncols; ++c) {
            int64_t i = rows[r], j = cols[c];
            double acc = 0.0;
            if (!sA) {
                for (int64_t k = 0; k < K; ++k)
                    acc += load(A, i * a_sm + k * a_sk, dtype, v8) * load(B, k * b_sk + j * b_sn, dtype, v8);
            } else {
                for (int64_t kb = 0; kb < nkb; ++kb) {
                    double part = 0.0;
                    int64_t k1 = (kb + 1) * bs < K ? (kb + 1) * bs : K;
                    for (int64_t k = kb * bs; k < k1; ++k)
                        part += load(A, i * a_sm + k * a_sk, dtype, v8) * load(B, k * b_sk + j * b_sn, dtype, v8);
                    acc += (double)sA[(i / bs_am) * nkb + kb] * (double)sB[(j / bs) * nkb + kb] * part;
                }
            }
            out[r * ncols + c] = acc;
        }
    }
    return 0;
}
